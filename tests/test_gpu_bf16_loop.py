"""GPU parity of the 16-bit entry points beyond the contiguous fused step: bf16 local parameters on
strided shards (cocodc_sync_step_bf16_segmented), in one loop event (cocodc_sync_event_bf16) and
through the Sec. 3.2 loop (cocodc_loop_step_bf16), each against the oracle's function of the same
name.  Every stored value, 16-bit ones included, must be bit-identical (both sides round the same
fp64 value once); scores to the tight bar; selections and event logs identical.  Needs an MI355X."""
import random

import numpy as np
import pytest
import torch

from paper_2504_17672_amd import synth

import parity_util as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2504_17672_amd import binding
    assert torch.cuda.is_available()
    return binding


def _u16(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16).copy()


def _half_state(n, tau, H, seed, amplified=False, view_off=0):
    """fp32 global buffers and bf16 local ones on the device, and the same bytes on the host."""
    base = synth.Workload("half", (n + view_off,), tau=tau, H=H)
    st = synth.make_state(base, "cuda", seed=seed, amplified=amplified)
    dev = {k: (v.to(torch.bfloat16) if k in ("theta_m", "theta_m_send") else v.clone())[view_off:] for k, v in st.items()}
    host = {k: (_u16(v) if v.dtype == torch.bfloat16 else v.cpu().numpy().copy()) for k, v in dev.items()}
    return dev, host


def _same_buffers(dev, host):
    for k, v in dev.items():
        g = _u16(v) if v.dtype == torch.bfloat16 else v.cpu().numpy()
        if g.dtype == np.float32:
            assert np.array_equal(g.view(np.uint32), host[k].view(np.uint32)), k
        else:
            assert np.array_equal(g, host[k]), k


def _pg_buffers(n, fill=0x7FC1):
    pg = torch.full((n,), fill, dtype=torch.int32, device="cuda").to(torch.int16).view(torch.bfloat16)
    return pg, np.full(n, fill, np.uint16)


# ------------------------------------------------------------------ strided shards
def _segmented_case(B, ref, segs, K, n, I_p, t_b, budget, tau=5, H=100, seed=0, amplified=False, view_off=0, **hpkw):
    print(f"case bf16 segmented S={len(segs)} K={K} n={n} view_off={view_off} amplified={amplified} hp={hpkw}", flush=True)
    dev, host = _half_state(n, tau, H, seed, amplified, view_off)
    ghp, rhp = B.hparams(tau, H, **hpkw), ref.hparams(tau, H, **hpkw)
    ws = B.new_workspace_segmented(len(segs), K, n)
    out = U.gpu_outputs(K)
    pg, h_pg = _pg_buffers(n)
    rc = B.cocodc_sync_step_bf16_segmented(segs, K, n, dev["theta_m"], dev["theta_m_send"], dev["theta_g"],
                                           dev["momentum"], dev["delta_g"], pg, I_p, t_b, 1000, budget, ghp, out["R"],
                                           out["sel"], out["n_sel"], out["sums"], ws)
    assert rc == 0, B.cocodc_status_string(rc)
    torch.cuda.synchronize()
    ro = ref.sync_step_bf16_segmented(segs, K, host["theta_m"], host["theta_m_send"], host["theta_g"], host["momentum"],
                                      host["delta_g"], h_pg, I_p, t_b, 1000, budget, rhp)
    assert ro["rc"] == 0
    _same_buffers(dev, host)
    assert np.array_equal(_u16(pg), h_pg)
    Rg, Rr = out["R"].cpu().numpy(), ro["R"]
    fin = np.isfinite(Rr)
    assert np.array_equal(np.isposinf(Rg), np.isposinf(Rr))
    assert U.rel_err(Rg[fin], Rr[fin]) <= U.SCORE_TOL_TIGHT
    ok = np.isfinite(ro["sums"])
    assert U.rel_err(out["sums"].cpu().numpy()[ok], ro["sums"][ok]) <= U.SCORE_TOL_TIGHT
    out["sel_list"] = out["sel"][:int(out["n_sel"].item())].cpu().tolist()
    U.compare_selection(out, ro, synth.Bookkeeping(t_g=1000, t_b=list(t_b), I_p=list(I_p)), H)
    print("   ok; selected", out["sel_list"], flush=True)
    return out


def test_bf16_on_the_papers_strided_shards(B, ref):
    """Sec. 4.1 as the paper runs it: 12 layers (125M dimensions) in K = 4 strided shards, bf16 local
    parameters; both 16-bit formats of the outgoing pseudo-gradient."""
    segs, n = synth.strided_segments(12, 768, 2048, 4)
    out = _segmented_case(B, ref, segs, 4, n, [12, 24, 36, 12], [988, 976, 964, 988], 2)
    assert len(out["sel_list"]) == 2
    segs, n = synth.strided_segments(12, 96, 256, 4)
    _segmented_case(B, ref, segs, 4, n, [12, 24, 36, 12], [988, 976, 964, 988], 3, pg_format=1)
    _segmented_case(B, ref, segs, 4, n, [12, 24, 36, 12], [988, 976, 964, 988], 3, tau=2, H=1, amplified=True)
    _segmented_case(B, ref, segs, 4, n, [12, 0, 36, 12], [988, 976, 100, 988], 4, merge_mode=1, alpha=0.3, score_src=1,
                    norm_kind=1)


@pytest.mark.parametrize("view_off", [0, 1])
def test_bf16_shuffled_pieces_with_tables_in_the_workspace(B, ref, view_off):
    """70 pieces in 6 shards, listed in random order, unaligned, one shard without a piece: more than
    the kernel arguments hold, so the tables go through the workspace; view_off 1 makes every base
    2 bytes (bf16) or 4 bytes (fp32) off a 16-byte boundary (element-wise kernel variant)."""
    rng = random.Random(19)
    segs, off, K = [], 3, 6
    for j in range(70):
        ln = rng.choice([1, 5, 2047, 2048, 4097, rng.randrange(1, 9000)])
        segs.append((off, ln, rng.choice([0, 1, 2, 4, 5])))
        off += ln + rng.choice([0, 1, 7])
    rng.shuffle(segs)
    _segmented_case(B, ref, segs, K, off + 5, [3, 1, 9, 2, 0, 5], [990, 999, 100, 950, 996, 980], 3, seed=7,
                    view_off=view_off)
    _segmented_case(B, ref, segs, K, off + 5, [3, 1, 9, 2, 4, 5], [990, 999, 997, 950, 996, 980], 6, seed=8,
                    view_off=view_off, pg_format=1, tau=2, H=1, amplified=True)


# ------------------------------------------------------------------ one loop event
def test_bf16_event_random_masks(B, ref):
    """30 random events: K from 1 to 24, arrived / in-flight marks, odd sizes, every merge mode, both
    pseudo-gradient formats, old scores (infinities, a NaN) that must survive untouched."""
    rng = random.Random(78)
    for case in range(30):
        K = rng.choice([1, 2, 4, 9, 24])
        sizes = tuple(rng.choice([0, 1, 5, 2048, 4097, rng.randrange(1, 20000)]) for _ in range(K))
        wl = synth.Workload(f"event16-{case}", sizes, tau=rng.choice([0, 2, 5]), H=rng.choice([1, 3, 100]))
        n_alloc = max(wl.n_total, 1) + 16
        mask = [int(rng.random() < rng.choice([0.0, 0.3, 1.0])) for _ in range(K)]
        if case % 2:
            mask = [m | (2 if rng.random() < 0.4 else 0) for m in mask]
        merge_mode = rng.choice([0, 0, 1, 2])
        hpk = dict(lam=rng.choice([0.0, 0.5, 3.0]), nesterov=rng.choice([0, 1]), drift_sign=rng.choice([1, -1]),
                   score_src=rng.choice([0, 1]), norm_kind=rng.choice([1, 2]), merge_mode=merge_mode, alpha=0.5,
                   delta_src=rng.choice([0, 1]) if merge_mode == 0 else 0, pg_format=rng.choice([0, 1]))
        view_off = rng.choice([0, 0, 1])
        print(f"case event16 #{case} K={K} n={n_alloc} mask={mask} tau={wl.tau} H={wl.H} view_off={view_off} hp={hpk}",
              flush=True)
        dev, host = _half_state(n_alloc, wl.tau, wl.H, case, amplified=rng.random() < 0.5, view_off=view_off)
        ghp, rhp = B.hparams(wl.tau, wl.H, **hpk), ref.hparams(wl.tau, wl.H, **hpk)
        I_p = [rng.choice([0, 1, 7, 30]) for _ in range(K)]
        t_b = [1000 - rng.choice([0, 1, 2, 3, 99, 100, 500]) for _ in range(K)]
        budget = rng.randrange(0, K + 2)
        R0 = np.array([rng.choice([np.inf, 0.0, 0.5, 2.0, rng.random(), np.nan if K > 3 and rng.random() < 0.1 else 1.5])
                       for _ in range(K)])
        R_dev = torch.from_numpy(R0.copy()).cuda()
        sums_dev = torch.full((K, 4), -3.0, dtype=torch.float64, device="cuda")
        out = U.gpu_outputs(K)
        pg, h_pg = _pg_buffers(n_alloc)
        ws = B.new_workspace(K, n_alloc)
        rc = B.cocodc_sync_event_bf16(wl.frags, n_alloc, mask, dev["theta_m"], dev["theta_m_send"], dev["theta_g"],
                                      dev["momentum"], dev["delta_g"], pg, I_p, t_b, 1000, budget, ghp, R_dev,
                                      out["sel"], out["n_sel"], sums_dev, ws)
        assert rc == 0, B.cocodc_status_string(rc)
        torch.cuda.synchronize()
        R_ref = R0.copy()
        sums_ref = np.full((K, 4), -3.0)
        ro = ref.sync_event_bf16(wl.frags, mask, host["theta_m"], host["theta_m_send"], host["theta_g"],
                                 host["momentum"], host["delta_g"], h_pg, I_p, t_b, 1000, budget, rhp, R_ref,
                                 sums=sums_ref)
        assert ro["rc"] == 0
        _same_buffers(dev, host)
        assert np.array_equal(_u16(pg), h_pg)
        Rg = R_dev.cpu().numpy()
        arrived = np.array([m & 1 for m in mask], bool)
        assert np.array_equal(Rg[~arrived].view(np.uint64), R0[~arrived].view(np.uint64))
        fin = arrived & np.isfinite(R_ref)
        assert np.array_equal(np.isposinf(Rg[arrived]), np.isposinf(R_ref[arrived]))
        assert np.array_equal(np.isnan(Rg[arrived]), np.isnan(R_ref[arrived]))
        assert U.rel_err(Rg[fin], R_ref[fin]) <= U.SCORE_TOL_TIGHT
        sg = sums_dev.cpu().numpy()
        assert np.array_equal(sg[~arrived], sums_ref[~arrived])
        ok = arrived[:, None] & np.isfinite(sums_ref)
        assert U.rel_err(sg[ok], sums_ref[ok]) <= U.SCORE_TOL_TIGHT
        n_sel = int(out["n_sel"].item())
        assert n_sel == min(budget, sum(1 for m in mask if not m & 2))
        got = out["sel"][:n_sel].cpu().tolist()
        rc_o, order = ref.select_fragments(Rg, t_b, 1000, wl.H, K)
        assert rc_o == 0 and got == [q for q in order.tolist() if not mask[q] & 2][:n_sel]
        if not np.isnan(R_ref).any():
            assert got == ro["sel"].tolist()


# ------------------------------------------------------------------ the loop
def _loop_case(B, ref, n, tau, H, gamma, T_c, T_s, steps, frags=None, segs=None, K=None, lazy=False, seed=0, **hpkw):
    from oracle.loop import RefLoop
    print(f"case loop16 n={n} K={K or len(frags)} S={len(segs) if segs else '-'} steps={steps} lazy={lazy} hp={hpkw}",
          flush=True)
    dev, host = _half_state(n, tau, H, seed)
    ghp, rhp = B.hparams(tau, H, **hpkw), ref.hparams(tau, H, **hpkw)
    if segs is None:
        K = len(frags)
        rc, loop = B.cocodc_loop_create(frags, n, ghp, gamma, T_c, T_s)
        rloop = RefLoop(frags, rhp, gamma, T_c, T_s, half=True)
        ws = B.new_workspace(K, n)
        pieces = [[f] for f in frags]
    else:
        rc, loop = B.cocodc_loop_create_segmented(segs, K, n, ghp, gamma, T_c, T_s)
        rloop = RefLoop(None, rhp, gamma, T_c, T_s, segs=segs, K=K, half=True)
        ws = B.new_workspace_segmented(len(segs), K, n)
        pieces = rloop.pieces
    assert rc == 0
    R = torch.zeros(K, dtype=torch.float64, device="cuda")
    sel = torch.zeros(K, dtype=torch.int32, device="cuda")
    n_sel = torch.zeros(1, dtype=torch.int32, device="cuda")
    assert B.cocodc_loop_reset_scores(loop, R) == 0
    out, h_out = _pg_buffers(n)
    bufs = B.loop_buffers(dev["theta_m"], dev["theta_m_send"], dev["theta_g"], dev["momentum"], dev["delta_g"], out,
                          R, sel, n_sel, ws)
    g = torch.Generator(device="cuda").manual_seed(177 + seed)
    n_sent = n_received = 0
    try:
        for t in range(1, steps + 1):
            # the worker's local step, in bf16: the harness rounds once per step, the same bytes go to both sides
            drift = torch.empty(n, device="cuda").normal_(0.0, 1e-3, generator=g)
            dev["theta_m"].copy_((dev["theta_m"].float() + drift).to(torch.bfloat16))
            host["theta_m"][:] = _u16(dev["theta_m"])
            rc, due = B.cocodc_loop_due(loop, t)
            assert rc == 0 and due == rloop.due(t)
            for p in due:   # the all-reduce hands back an fp32 average
                for o, l in pieces[p]:
                    fresh = torch.empty(l, device="cuda").normal_(0.0, 1e-3, generator=g)
                    dev["delta_g"][o:o + l] = fresh
                    host["delta_g"][o:o + l] = fresh.cpu().numpy()
            rc, rec, sent = B.cocodc_loop_step_bf16(loop, t, bufs)
            assert rc == 0, B.cocodc_status_string(rc)
            rrec, rsent = rloop.step(t, host["theta_m"], host["theta_m_send"], host["theta_g"], host["momentum"],
                                     host["delta_g"], h_out)
            assert rec == rrec, (t, rec, rrec)
            assert sent in (-1, B.COCODC_LOOP_SENT_PENDING)
            if rsent >= 0:
                assert sent == B.COCODC_LOOP_SENT_PENDING, (t, sent, rsent)
            if not lazy:
                if sent == B.COCODC_LOOP_SENT_PENDING:
                    assert B.cocodc_loop_last_sent(loop) == (0, t, rsent), (t, rsent)
                else:
                    assert rsent == -1
                rc, t_b, I_p, fl = B.cocodc_loop_state(loop)
                assert (t_b, I_p, fl) == (rloop.t_b, rloop.I_p, rloop.in_flight)
            n_sent += rsent >= 0
            n_received += len(rec)
        rc, t_b, I_p, fl = B.cocodc_loop_state(loop)
        assert (t_b, I_p, fl) == (rloop.t_b, rloop.I_p, rloop.in_flight)
        torch.cuda.synchronize()
        _same_buffers(dev, host)
        assert np.array_equal(_u16(out), h_out)
        Rg = R.cpu().numpy()
        fin = np.isfinite(rloop.R)
        assert np.array_equal(np.isposinf(Rg), np.isposinf(rloop.R))
        assert U.rel_err(Rg[fin], rloop.R[fin]) <= U.SCORE_TOL_TIGHT
    finally:
        B.cocodc_loop_destroy(loop)
    print(f"   {n_sent} sends, {n_received} receives, plan N={rloop.N} h={rloop.h}", flush=True)
    return n_sent, n_received


@pytest.mark.parametrize("pg_format", [0, 1])
def test_bf16_loop_on_the_papers_setup(B, ref, pg_format):
    """Sec. 4.1 in full: 12 layers in K = 4 strided shards, H = 100, tau = 5, gamma = 0.4 (8 syncs per
    period), bf16 local parameters, the pseudo-gradient on the wire in either 16-bit format."""
    segs, n = synth.strided_segments(12, 96, 256, 4)
    n_sent, n_rec = _loop_case(B, ref, n, 5, 100, 0.4, 1.0, 5.0, 250, segs=segs, K=4, pg_format=pg_format)
    assert n_sent == 250 // 12 and n_rec >= n_sent - 1


def test_bf16_loop_contiguous_fragments_never_asking(B, ref):
    """Contiguous fragments of awkward sizes (several tiles, one element, none); nobody reads the send
    decisions back, the schedule does so itself when it needs them; h == tau in the second run."""
    wl = synth.Workload("loop16", (70001, 1, 0, 33000, 4097), tau=3, H=40)
    n_sent, _ = _loop_case(B, ref, wl.n_total, 3, 40, 1.0, 1.0, 4.0, 260, frags=wl.frags, lazy=True, pg_format=1)
    assert n_sent >= 260 // 4 - 1
    wl = synth.Workload("loop16-h-eq-tau", (30000, 25000, 20001, 15000), tau=5, H=100)
    _loop_case(B, ref, wl.n_total, 5, 100, 1.0, 1.0, 5.0, 300, frags=wl.frags)


def test_bf16_loop_many_pieces_deep_overlap(B, ref):
    """70 shuffled pieces in 6 shards (tables through the workspace) with an overlap longer than the send
    interval, so that several shards are in flight at once."""
    rng = random.Random(29)
    segs, off, K = [], 3, 6
    for j in range(70):
        ln = rng.choice([1, 5, 2047, 2048, 4097, rng.randrange(1, 9000)])
        segs.append((off, ln, rng.choice([0, 1, 2, 4, 5])))
        off += ln + rng.choice([0, 1, 7])
    rng.shuffle(segs)
    _loop_case(B, ref, off + 5, 11, 30, 1.0, 1.0, 3.0, 200, segs=segs, K=K)
    _loop_case(B, ref, off + 5, 11, 30, 1.0, 1.0, 3.0, 200, segs=segs, K=K, lazy=True, pg_format=1)


def test_bf16_loop_on_buffers_large_enough_for_the_wide_tiles(B, ref):
    """More than 2^24 elements: 4 096-element tiles in the 16-bit event and in the 16-bit walk over the chosen
    fragment."""
    wl = synth.Workload("loop16-wide-tiles", (6000000, 5000001, 4999999, 1500003), tau=5, H=100)
    assert wl.n_total > 1 << 24 and B.cocodc_tile_elements(wl.n_total) == 4096
    n_sent, n_rec = _loop_case(B, ref, wl.n_total, 5, 100, 0.4, 1.0, 5.0, 110, frags=wl.frags, pg_format=1)
    assert n_sent == 110 // 12 and n_rec == n_sent - 1


@pytest.mark.parametrize("seed", range(2))
def test_random_bf16_segmented_cases(B, ref, seed):
    """The seeded random sweep of the fp32 entry points (random tables with empty and one-element fragments, gaps,
    any base alignment, every hyper-parameter switch, buffers beyond 2^24 elements) through the 16-bit segmented
    step: every fragment cut into random pieces, the pieces of all fragments shuffled, both wire formats."""
    from test_gpu_random_sweep import _random_case
    rng = random.Random(3000 + seed)
    for case in range(20):
        c = _random_case(rng)
        K = len(c["frags"])
        segs = []
        for p, (o, l) in enumerate(c["frags"]):
            cuts = sorted(rng.randrange(0, l + 1) for _ in range(rng.choice([0, 0, 1, 2, 5]))) if l else []
            edges = [0] + cuts + [l]
            segs += [(o + a, b - a, p) for a, b in zip(edges, edges[1:])]
        rng.shuffle(segs)
        n_alloc = c["n"] + ((1 << 24) if c["pad_big"] else 0) + 8
        hpk = dict(c["hp"], pg_format=rng.choice([0, 1]))
        tau, H = hpk.pop("tau"), hpk.pop("H")
        print(f"case bf16 segmented random seed={seed} #{case} S={len(segs)} K={K} n={n_alloc} "
              f"view_off={c['view_off']} amplified={c['amplified']} budget={c['budget']} hp={hpk}", flush=True)
        dev, host = _half_state(n_alloc, tau, H, seed * 100 + case, c["amplified"], c["view_off"])
        ghp, rhp = B.hparams(tau, H, **hpk), ref.hparams(tau, H, **hpk)
        ws = B.new_workspace_segmented(len(segs), K, n_alloc)
        out = U.gpu_outputs(K)
        pg, h_pg = _pg_buffers(n_alloc)
        rc = B.cocodc_sync_step_bf16_segmented(segs, K, n_alloc, dev["theta_m"], dev["theta_m_send"], dev["theta_g"],
                                               dev["momentum"], dev["delta_g"], pg, c["I_p"], c["t_b"], 1000,
                                               c["budget"], ghp, out["R"], out["sel"], out["n_sel"], out["sums"], ws)
        assert rc == 0, B.cocodc_status_string(rc)
        torch.cuda.synchronize()
        ro = ref.sync_step_bf16_segmented(segs, K, host["theta_m"], host["theta_m_send"], host["theta_g"],
                                          host["momentum"], host["delta_g"], h_pg, c["I_p"], c["t_b"], 1000,
                                          c["budget"], rhp)
        assert ro["rc"] == 0
        _same_buffers(dev, host)
        assert np.array_equal(_u16(pg), h_pg)
        Rg, Rr = out["R"].cpu().numpy(), ro["R"]
        fin = np.isfinite(Rr)
        assert np.array_equal(np.isposinf(Rg), np.isposinf(Rr)) and np.array_equal(np.isnan(Rg), np.isnan(Rr))
        assert U.rel_err(Rg[fin], Rr[fin]) <= U.SCORE_TOL_TIGHT
        ok = np.isfinite(ro["sums"])
        assert U.rel_err(out["sums"].cpu().numpy()[ok], ro["sums"][ok]) <= U.SCORE_TOL_TIGHT
        out["sel_list"] = out["sel"][:int(out["n_sel"].item())].cpu().tolist()
        assert len(out["sel_list"]) == min(c["budget"], K)
        if not np.isnan(Rr).any():
            U.compare_selection(out, ro, synth.Bookkeeping(t_g=1000, t_b=c["t_b"], I_p=c["I_p"]), H)


def test_bf16_segmented_event_random_masks(B, ref):
    """cocodc_sync_event_bf16_segmented: 24 random events on shuffled segment tables (the paper's configuration in
    one call per event: strided shards, bf16 local parameters), marks for arrived and in-flight shards, both wire
    formats; stored values bit-identical, untouched scores preserved, selection identical."""
    from test_gpu_random_sweep import _random_case
    rng = random.Random(5000)
    for case in range(24):
        c = _random_case(rng)
        K = len(c["frags"])
        segs = []
        for p, (o, l) in enumerate(c["frags"]):
            cuts = sorted(rng.randrange(0, l + 1) for _ in range(rng.choice([0, 0, 1, 2, 5]))) if l else []
            edges = [0] + cuts + [l]
            segs += [(o + a, b - a, p) for a, b in zip(edges, edges[1:])]
        rng.shuffle(segs)
        n_alloc = c["n"] + ((1 << 24) if c["pad_big"] else 0) + 8
        mask = [int(rng.random() < rng.choice([0.0, 0.3, 1.0])) for _ in range(K)]
        if case % 2:
            mask = [m | (2 if rng.random() < 0.4 else 0) for m in mask]
        hpk = dict(c["hp"], pg_format=rng.choice([0, 1]))
        tau, H = hpk.pop("tau"), hpk.pop("H")
        print(f"case bf16 segmented event #{case} S={len(segs)} K={K} n={n_alloc} mask={mask} "
              f"view_off={c['view_off']} hp={hpk}", flush=True)
        dev, host = _half_state(n_alloc, tau, H, 700 + case, c["amplified"], c["view_off"])
        ghp, rhp = B.hparams(tau, H, **hpk), ref.hparams(tau, H, **hpk)
        R0 = np.array([rng.choice([np.inf, 0.0, 0.5, 2.0, rng.random(), np.nan if K > 3 and rng.random() < 0.1 else 1.5])
                       for _ in range(K)])
        R_dev = torch.from_numpy(R0.copy()).cuda()
        sums_dev = torch.full((K, 4), -3.0, dtype=torch.float64, device="cuda")
        out = U.gpu_outputs(K)
        pg, h_pg = _pg_buffers(n_alloc)
        ws = B.new_workspace_segmented(len(segs), K, n_alloc)
        rc = B.cocodc_sync_event_bf16_segmented(segs, K, n_alloc, mask, dev["theta_m"], dev["theta_m_send"],
                                                dev["theta_g"], dev["momentum"], dev["delta_g"], pg, c["I_p"], c["t_b"],
                                                1000, c["budget"], ghp, R_dev, out["sel"], out["n_sel"], sums_dev, ws)
        assert rc == 0, B.cocodc_status_string(rc)
        torch.cuda.synchronize()
        R_ref, sums_ref = R0.copy(), np.full((K, 4), -3.0)
        ro = ref.sync_event_bf16_segmented(segs, K, mask, host["theta_m"], host["theta_m_send"], host["theta_g"],
                                           host["momentum"], host["delta_g"], h_pg, c["I_p"], c["t_b"], 1000,
                                           c["budget"], rhp, R_ref, sums=sums_ref)
        assert ro["rc"] == 0
        _same_buffers(dev, host)
        assert np.array_equal(_u16(pg), h_pg)
        Rg = R_dev.cpu().numpy()
        arrived = np.array([m & 1 for m in mask], bool)
        assert np.array_equal(Rg[~arrived].view(np.uint64), R0[~arrived].view(np.uint64))
        fin = arrived & np.isfinite(R_ref)
        assert np.array_equal(np.isposinf(Rg[arrived]), np.isposinf(R_ref[arrived]))
        assert np.array_equal(np.isnan(Rg[arrived]), np.isnan(R_ref[arrived]))
        assert U.rel_err(Rg[fin], R_ref[fin]) <= U.SCORE_TOL_TIGHT
        sg = sums_dev.cpu().numpy()
        assert np.array_equal(sg[~arrived], sums_ref[~arrived])
        ok = arrived[:, None] & np.isfinite(sums_ref)
        assert U.rel_err(sg[ok], sums_ref[ok]) <= U.SCORE_TOL_TIGHT
        n_sel = int(out["n_sel"].item())
        assert n_sel == min(c["budget"], sum(1 for m in mask if not m & 2))
        got = out["sel"][:n_sel].cpu().tolist()
        rc_o, order = ref.select_fragments(Rg, c["t_b"], 1000, H, K)
        assert rc_o == 0 and got == [q for q in order.tolist() if not mask[q] & 2][:n_sel]
        if not np.isnan(R_ref).any() and not np.isnan(Rg).any():
            assert got == ro["sel"].tolist()
