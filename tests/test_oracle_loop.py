"""Pins of the loop oracle (oracle/loop.py) against what the paper fixes for the adaptive
transmission schedule (Sec. 3.2, Sec. 4.1): the worked numbers N = 8 / h = 12, the initial
priority of never-synchronised fragments, the overdue rule of Algorithm 2 and the bounded
staleness it is there to guarantee.  CPU only."""
import math

import numpy as np
import torch

from paper_2504_17672_amd import synth


def make_run(ref, wl, gamma, T_c, T_s, steps, seed=0, closed=True):
    from oracle.loop import RefLoop
    st = {k: v.numpy() for k, v in synth.make_state(wl, "cpu", seed=seed).items()}
    hp = ref.hparams(wl.tau, wl.H, wl.lam, wl.eta, wl.mu)
    loop = RefLoop(wl.frags, hp, gamma, T_c, T_s)
    send_buf = st["delta_g"] if closed else np.zeros_like(st["delta_g"])
    g = torch.Generator().manual_seed(1234 + seed)
    log = []
    for t in range(1, steps + 1):
        drift = torch.empty(wl.n_total).normal_(0.0, 1e-4, generator=g).numpy()
        st["theta_m"] += drift  # the worker's local training step
        if not closed:
            for p in loop.due(t):
                o, l = wl.frags[p]
                st["delta_g"][o:o + l] = torch.empty(l).normal_(0.0, 1e-3, generator=g).numpy()
        before_tb, before_R = list(loop.t_b), loop.R.copy()
        flying_before = list(loop.in_flight)
        rec, sent = loop.step(t, st["theta_m"], st["theta_m_send"], st["theta_g"], st["momentum"], st["delta_g"],
                              send_buf)
        log.append(dict(t=t, received=rec, sent=sent, t_b_before=before_tb, R_before=before_R,
                        flying_before=flying_before, t_b=list(loop.t_b), I_p=list(loop.I_p), R=loop.R.copy()))
    return loop, st, log


def test_paper_setup_gives_eight_syncs_per_period(ref):
    """Sec. 4.1: K = 4, H = 100, tau = 5, gamma = 0.4 -> 8 synchronisations per H steps."""
    wl = synth.Workload("paper", (3000, 2500, 2000, 1500), tau=5, H=100)
    loop, st, log = make_run(ref, wl, 0.4, 1.0, 5.0, 300)
    assert (loop.N, loop.h) == (8, 12)
    assert sum(1 for e in log if e["sent"] >= 0 and e["t"] <= 100) == 8
    assert sum(1 for e in log if e["sent"] >= 0) == 300 // 12
    assert [e["t"] for e in log if e["sent"] >= 0][:8] == [12, 24, 36, 48, 60, 72, 84, 96]
    # never-synchronised fragments have R = infinity: the first K sends are 0, 1, 2, 3
    assert [e["sent"] for e in log if e["sent"] >= 0][:4] == [0, 1, 2, 3]
    # every send arrives exactly tau steps later, with I_p = t_p - t_{p,b}
    sent_at = {}
    for e in log:
        for p in e["received"]:
            assert sent_at[p] + 5 == e["t"]
            assert e["I_p"][p] == sent_at[p] - e["t_b_before"][p]
            assert e["t_b"][p] == e["t"] and math.isfinite(e["R"][p]) and e["R"][p] > 0
            del sent_at[p]
        if e["sent"] >= 0:
            assert e["sent"] not in sent_at
            sent_at[e["sent"]] = e["t"]


def test_every_send_is_algorithm_2_on_the_current_scores(ref):
    wl = synth.Workload("alg2", (900, 800, 700, 600, 500), tau=3, H=60)
    loop, st, log = make_run(ref, wl, 0.5, 1.0, 3.0, 400, closed=False)
    assert loop.h == 6
    n_overdue = 0
    for e in log:
        if e["t"] % 6:
            assert e["sent"] == -1
            continue
        # state the decision saw: after this step's receives
        t_b = list(e["t_b_before"])
        R = e["R_before"].copy()
        flying = [f >= 0 for f in e["flying_before"]]
        for p in e["received"]:
            t_b[p], R[p], flying[p] = e["t"], e["R"][p], False
        elig = [p for p in range(5) if not flying[p]]
        overdue = [p for p in elig if e["t"] - t_b[p] >= 60]
        if overdue:
            want = overdue[0]
            n_overdue += 1
        else:
            want = max(elig, key=lambda p: (R[p], -p))
        assert e["sent"] == want, e["t"]
    assert n_overdue > 0  # the overdue branch was exercised


def test_staleness_stays_bounded(ref):
    """Algorithm 2's first loop exists so that no fragment lags far behind H."""
    wl = synth.Workload("stale", (500,) * 6, tau=4, H=48)
    loop, st, log = make_run(ref, wl, 1.0, 1.0, 8.0, 600)  # N = K = 6, h = 8
    assert (loop.N, loop.h) == (6, 8)
    worst = max(e["t"] - tb for e in log for tb in e["t_b"])
    assert worst <= 48 + 6 * 8 + 4
    sends = [e["sent"] for e in log if e["sent"] >= 0]
    assert set(sends) == set(range(6))


def test_overlap_longer_than_send_interval_keeps_in_flight_fragments_out(ref):
    wl = synth.Workload("deep", (400,) * 5, tau=30, H=50)
    loop, st, log = make_run(ref, wl, 1.0, 1.0, 5.0, 300)  # N = 10, h = 5: up to 5 fragments in flight
    assert (loop.N, loop.h) == (10, 5)
    flying = {}
    max_flying = 0
    for e in log:
        for p in e["received"]:
            assert flying.pop(p) + 30 == e["t"]
        if e["sent"] >= 0:
            assert e["sent"] not in flying
            flying[e["sent"]] = e["t"]
        max_flying = max(max_flying, len(flying))
    assert max_flying == 5
    assert any(e["t"] % 5 == 0 and e["sent"] == -1 for e in log)  # nothing eligible: no send


def test_moving_average_replans(ref):
    from oracle.loop import RefLoop
    hp = ref.hparams(5, 100)
    loop = RefLoop([(0, 10)] * 1 + [(10, 10), (20, 10), (30, 10)], hp, 0.4, 1.0, 5.0)
    assert (loop.N, loop.h) == (8, 12)
    loop.observe(1.0, 2.5, 1.0)      # beta = 1: the sample replaces the average
    assert (loop.N, loop.h) == (16, 6)
    loop.observe(1.0, 7.5, 0.5)      # T_s = 5.0 again
    assert abs(loop.T_s - 5.0) < 1e-15 and (loop.N, loop.h) == (8, 12)
    loop.observe(1.0, 1000.0, 1.0)   # no capacity: N falls back to K (Eq. 9)
    assert (loop.N, loop.h) == (4, 25)
