"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element,
on the same seeded synthetic inputs.  Needs an MI355X: run with -m gpu.
"""
import math

import numpy as np
import pytest
import torch

from paper_2504_17672_amd import synth

import parity_util as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2504_17672_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return binding


def _hp_pair(B, ref, wl, **kw):
    args = dict(lam=wl.lam, eta=wl.eta, mu=wl.mu)
    args.update(kw)
    return B.hparams(wl.tau, wl.H, **args), ref.hparams(wl.tau, wl.H, **args)


def _fused_case(B, ref, wl, seed=0, variant="regular", pg="separate", amplified=False, pad=0, tight=True,
                budget=None, **hpkw):
    print(f"case {wl.name} K={wl.K} n={wl.n_total} seed={seed} variant={variant} pg={pg} "
          f"amplified={amplified} hp={hpkw}", flush=True)
    st = synth.make_state(wl, "cuda", seed=seed, pad=pad, amplified=amplified)
    bk = synth.bookkeeping(wl, variant)
    ghp, rhp = _hp_pair(B, ref, wl, **hpkw)
    budget = wl.budget if budget is None else budget
    host = U.host_copy(st)
    n_alloc = wl.n_total + pad
    ws = B.new_workspace(wl.K, n_alloc)
    go = U.run_gpu_fused(B, wl.frags, n_alloc, st, bk, budget, ghp, ws, pg=pg)
    host_dg_before = host["delta_g"].copy()
    ro = U.run_ref_fused(ref, wl.frags, host, bk, budget, rhp)
    if pg == "alias":
        # the oracle wrote its pseudo-gradient to a separate buffer; the GPU overwrote delta_g
        assert np.array_equal(st["delta_g"][wl.n_total:].cpu().numpy(), host_dg_before[wl.n_total:])
    obs = U.compare_fused(st, go, host, ro, wl.frags, tight=tight)
    assert np.array_equal(st["theta_m_send"].cpu().numpy(), host["theta_m_send"])
    if pg != "alias":
        assert np.array_equal(st["delta_g"].cpu().numpy(), host_dg_before)
    if pg == "separate":
        outside = np.ones(n_alloc, bool)
        for off, ln in wl.frags:
            outside[off:off + ln] = False
        assert np.all(go["pg"].cpu().numpy()[outside] == 555.0)
    obs["margin"] = U.compare_selection(go, ro, bk, wl.H)
    assert len(go["sel_list"]) == min(budget, wl.K)
    print("   observed", {k: (f"{v:.3g}" if isinstance(v, float) else v) for k, v in obs.items()},
          "sel", go["sel_list"], flush=True)
    return obs, go, ro


# ------------------------------------------------------------------ configured workloads
def test_tiny_config(B, ref):
    wl = synth.WORKLOADS["tiny"]
    obs, go, ro = _fused_case(B, ref, wl, seed=0)
    assert len(go["sel_list"]) == 1
    _fused_case(B, ref, wl, seed=0, variant="mixed")


@pytest.mark.parametrize("name", ["125M-mini", "350M-mini", "1.3B-mini", "7B-mini"])
def test_mini_workloads(B, ref, name):
    wl = synth.MINI_WORKLOADS[name]
    _fused_case(B, ref, wl, seed=0)
    _fused_case(B, ref, wl, seed=1, variant="mixed", pg="alias")


def test_lambda_sweep_and_amplified_variant(B, ref):
    wl = synth.MINI_WORKLOADS["350M-mini"]
    for lam in wl.lam_sweep:
        _fused_case(B, ref, wl, seed=0, lam=lam)
    # with the configured distributions the cubic term is below fp32 resolution; amplify it
    amp = synth.Workload("350M-mini-amp", wl.frag_lengths, tau=2, H=1, budget=2)
    outs = {}
    for lam in wl.lam_sweep:
        obs, go, ro = _fused_case(B, ref, amp, seed=0, amplified=True, lam=lam)
        outs[lam] = ro["theta_m64"]
    assert np.max(np.abs(outs[1.0] - outs[0.0])) > 1e-2


@pytest.mark.parametrize("name", ["125M", "350M"])
def test_full_size_every_element(B, ref, name):
    wl = synth.WORKLOADS[name]
    _fused_case(B, ref, wl, seed=0)


# ------------------------------------------------------------------ shapes and edge cases
EDGE_TABLES = {
    "K1": [(0, 70001)],
    "odd_lengths": [(0, 1), (1, 2), (3, 3), (6, 5), (11, 16383), (16394, 16385), (32779, 7)],
    "unaligned_with_gaps": [(5, 1000), (1013, 3), (1030, 40000), (41031, 16384), (60001, 1)],
    "empty_fragments": [(0, 0), (0, 5000), (5000, 0), (5000, 33000), (38000, 0)],
    "out_of_order": [(50000, 20000), (0, 17), (17, 49983)],
    "tile_boundaries": [(16383, 2), (16385, 16383), (32768, 16384), (49152, 1), (49153, 16383 + 16384)],
}


@pytest.mark.parametrize("table", sorted(EDGE_TABLES))
def test_edge_tables(B, ref, table):
    frags = EDGE_TABLES[table]
    n_total = max(o + l for o, l in frags)

    base = synth.Workload(table, (n_total,), tau=5, H=100)
    st = synth.make_state(base, "cuda", seed=3, pad=9)
    bk = synth.Bookkeeping(t_g=1000, t_b=[1000 - 7 * (1 + p % 3) for p in range(len(frags))],
                           I_p=[7 * (1 + p % 3) for p in range(len(frags))])
    ghp, rhp = B.hparams(5, 100), ref.hparams(5, 100)
    for view_off in (0, 1):  # 1: base pointers only 4-byte aligned -> element-wise kernel variant
        print(f"case {table} view_off={view_off}", flush=True)
        s = {k: v.clone()[view_off:] for k, v in st.items()}
        fr = [(max(o - view_off, 0), l if o >= view_off else max(l - (view_off - o), 0)) for o, l in frags]
        n_alloc = s["theta_m"].numel()
        host = U.host_copy(s)
        ws = B.new_workspace(len(fr), n_alloc)
        go = U.run_gpu_fused(B, fr, n_alloc, s, bk, 2, ghp, ws)
        ro = U.run_ref_fused(ref, fr, host, bk, 2, rhp)
        U.compare_fused(s, go, host, ro, fr)
        U.compare_selection(go, ro, bk, 100)


def test_hand_computed_element_in_binary_fractions(B):
    """The element worked out by hand in tests/test_oracle_pins.py (every operand and intermediate
    an exact binary fraction), through the GPU library alone:
      eta = mu = 1/2, theta_g = 1, m = 1/4, delta_g = 1/2, theta_m = 1, theta_send = 3/2, tau = 4,
      H = 8, lambda = 1/2, I_p = 4  ->  m' = 5/8, G = 19/32, theta_m' = 8931/8192, pg = 0, R = 1/8."""
    from fractions import Fraction as F
    hp = B.hparams(4, 8, lam=0.5, eta=0.5, mu=0.5)
    n = 8   # the element sits at index 5 of a small buffer; the rest must stay untouched
    mk = lambda v: torch.full((n,), 9.0, device="cuda").index_fill_(0, torch.tensor([5], device="cuda"), v)
    tm, ts, tg, m, dg = mk(1.0), mk(1.5), mk(1.0), mk(0.25), mk(0.5)
    pg = torch.full((n,), 7.0, device="cuda")
    out = U.gpu_outputs(1)
    ws = B.new_workspace(1, n)
    assert B.cocodc_sync_step([(5, 1)], n, tm, ts, tg, m, dg, pg, [4], [96], 100, 1, hp, out["R"], out["sel"],
                              out["n_sel"], out["sums"], ws) == 0
    torch.cuda.synchronize()
    assert F(m[5].item()) == F(5, 8) and F(tg[5].item()) == F(19, 32) and F(tm[5].item()) == F(8931, 8192)
    assert pg[5].item() == 0.0 and F(out["R"][0].item()) == F(1, 8)
    assert [F(v) for v in out["sums"][0].tolist()] == [F(1, 4), F(1, 2), F(1, 4), F(1, 2)]
    assert out["n_sel"].item() == 1 and out["sel"][0].item() == 0
    keep = [i for i in range(n) if i != 5]
    for t, v in ((tm, 9.0), (tg, 9.0), (m, 9.0), (pg, 7.0)):
        assert (t[keep] == v).all()


def test_stream_mix_measurement_aid(B):
    """The measurement kernel's output is defined (a += b, c += e, d += e, f = b + c on the elements
    of the fragments, nothing elsewhere), so that what bench.py times is known to have run."""
    n = (1 << 24) + 5000
    frags = [(3, 70001), (80000, 4096 * 3), ((1 << 24) + 1, 4000)]
    g = torch.Generator(device="cuda").manual_seed(5)
    a, b, c, d, e, f = (torch.randn(n, device="cuda", generator=g) for _ in range(6))
    want = [a.clone(), c.clone(), d.clone(), f.clone()]
    for o, l in frags:
        sl = slice(o, o + l)
        want[0][sl] = a[sl] + b[sl]
        want[1][sl] = c[sl] + e[sl]
        want[2][sl] = d[sl] + e[sl]
        want[3][sl] = b[sl] + c[sl]
    ws = B.new_workspace(len(frags), n)
    assert B.cocodc_debug_stream_mix(frags, n, a, b, c, d, e, f, ws) == 0
    torch.cuda.synchronize()
    for got, w in zip((a, c, d, f), want):
        assert torch.equal(got, w)
    assert B.cocodc_debug_stream_mix(frags, n, a, a, c, d, e, f, ws) == -7   # overlapping buffers


def test_maximum_number_of_fragments(B, ref):
    """1024 fragments (the most a table may hold): lengths from 0 to a few tiles, gaps, budget 100,
    some fragments overdue and some never synchronised; scores, ranks and every element."""
    import random
    rng = random.Random(7)
    frags, off = [], 2
    for p in range(1024):
        ln = rng.choice([0, 1, 3, 4, 257, 2047, 2048, 2049, 4097, rng.randrange(1, 9000)])
        frags.append((off, ln))
        off += ln + rng.choice([0, 0, 1, 5])
    n_total = off + 3
    base = synth.Workload("k1024", (n_total,), tau=5, H=100)
    st = synth.make_state(base, "cuda", seed=8)
    bk = synth.Bookkeeping(t_g=1000, t_b=[1000 - (p * 13) % 120 for p in range(1024)],
                           I_p=[(p * 7) % 11 for p in range(1024)])   # every 11th: never synchronised
    ghp, rhp = B.hparams(5, 100), ref.hparams(5, 100)
    host = U.host_copy(st)
    ws = B.new_workspace(1024, n_total)
    print(f"case k1024 n={n_total}", flush=True)
    go = U.run_gpu_fused(B, frags, n_total, st, bk, 100, ghp, ws)
    ro = U.run_ref_fused(ref, frags, host, bk, 100, rhp)
    U.compare_fused(st, go, host, ro, frags)
    U.compare_selection(go, ro, bk, 100)
    assert len(go["sel_list"]) == 100


@pytest.mark.parametrize("view_off", [0, 1])
def test_odd_tables_in_a_large_buffer(B, ref, view_off):
    """Buffers of 2^24 elements or more are walked in 4096-element tiles (smaller ones in
    2048-element tiles): unaligned fragments across those boundaries, both kernel variants."""
    n_total = (1 << 24) + 70001
    frags = [(5, 100000), (16384 * 7 - 1, 2), (16384 * 9 + 1, 16383), (16384 * 11, 16384), (16384 * 20 + 3, 3 * 16384 + 1),
             (4096 * 93 - 1, 2), (4096 * 95 + 1, 4095), ((1 << 24) + 1, 70000)]
    base = synth.Workload("large-odd", (n_total,), tau=5, H=100)
    st = synth.make_state(base, "cuda", seed=4, pad=9)
    bk = synth.Bookkeeping(t_g=1000, t_b=[1000 - 7 * (1 + p % 3) for p in range(len(frags))],
                           I_p=[7 * (1 + p % 3) for p in range(len(frags))])
    ghp, rhp = B.hparams(5, 100), ref.hparams(5, 100)
    s = {k: v[view_off:] for k, v in st.items()}
    fr = [(o - view_off, l) for o, l in frags]
    n_alloc = s["theta_m"].numel()
    assert B.cocodc_tile_elements(n_alloc) == 4096
    host = U.host_copy(s)
    ws = B.new_workspace(len(fr), n_alloc)
    go = U.run_gpu_fused(B, fr, n_alloc, s, bk, 2, ghp, ws)
    ro = U.run_ref_fused(ref, fr, host, bk, 2, rhp)
    U.compare_fused(s, go, host, ro, fr)
    U.compare_selection(go, ro, bk, 100)


def test_budget_at_least_k_and_zero(B, ref):
    wl = synth.Workload("b", (3000, 2000, 1000, 500), tau=5, H=100)
    for budget in (0, 4, 9):
        obs, go, ro = _fused_case(B, ref, wl, seed=5, budget=budget)
        assert len(go["sel_list"]) == min(budget, 4)


@pytest.mark.parametrize("hpkw", [
    dict(nesterov=0), dict(drift_sign=-1), dict(merge_mode=1, alpha=0.3), dict(merge_mode=2),
    dict(score_src=1), dict(norm_kind=1), dict(score_src=1, norm_kind=1), dict(lam=0.0), dict(mu=0.0, eta=1.0),
    dict(delta_src=1), dict(delta_src=1, nesterov=0, drift_sign=-1),
])
def test_hyper_parameter_switches(B, ref, hpkw):
    wl = synth.Workload("hp", (40000, 33333, 12345), tau=5, H=100, budget=2)
    _fused_case(B, ref, wl, seed=6, **hpkw)
    amp = synth.Workload("hp-amp", (40000, 33333, 12345), tau=2, H=1, budget=2)
    _fused_case(B, ref, amp, seed=6, amplified=True, **hpkw)


@pytest.mark.parametrize("mode", [1, 2])
def test_baseline_merges_without_send_time_record(B, ref, mode):
    """Eq. 3 / blocking merge with theta_m_send = NULL: 32-byte pass, drift sums zero."""
    wl = synth.Workload("nosend", (50001, 16384, 3, 70000), tau=5, H=100, budget=2)
    bk = synth.bookkeeping(wl)
    st = synth.make_state(wl, "cuda", seed=12)
    host = U.host_copy(st)
    ghp = B.hparams(5, 100, merge_mode=mode, alpha=0.4)
    rhp = ref.hparams(5, 100, merge_mode=mode, alpha=0.4)
    ws = B.new_workspace(wl.K, wl.n_total)
    out = U.gpu_outputs(wl.K)
    pg = torch.full_like(st["delta_g"], 555.0)
    send_before = st["theta_m_send"].clone()
    assert B.cocodc_sync_step(wl.frags, wl.n_total, st["theta_m"], None, st["theta_g"], st["momentum"],
                              st["delta_g"], pg, bk.I_p, bk.t_b, bk.t_g, 2, ghp, out["R"], out["sel"],
                              out["n_sel"], out["sums"], ws) == 0
    torch.cuda.synchronize()
    out["pg"] = pg
    out["sel_list"] = out["sel"][:int(out["n_sel"].item())].cpu().tolist()
    h_pg = np.full(wl.n_total, 555.0, np.float32)
    ro = ref.sync_step(wl.frags, host["theta_m"], None, host["theta_g"], host["momentum"], host["delta_g"], h_pg,
                       bk.I_p, bk.t_b, bk.t_g, 2, rhp, shadow=True)
    ro["pg"] = h_pg
    U.compare_fused(st, out, host, ro, wl.frags)
    U.compare_selection(out, ro, bk, 100)
    assert torch.equal(out["sums"][:, 2:], torch.zeros_like(out["sums"][:, 2:]))
    assert torch.equal(st["theta_m_send"], send_before)
    # single-step entry point without the record
    tm = torch.from_numpy(U.host_copy(synth.make_state(wl, "cuda", seed=12))["theta_m"]).cuda()
    assert B.cocodc_delay_compensate(wl.frags, wl.n_total, tm, None, st["theta_g"], ghp, ws) == 0
    torch.cuda.synchronize()
    assert torch.equal(tm, st["theta_m"])
    # Algorithm 1 and drift scoring refuse to run without it
    assert B.cocodc_delay_compensate(wl.frags, wl.n_total, tm, None, st["theta_g"], B.hparams(5, 100), ws) \
        == B.COCODC_ERR_NULL
    assert B.cocodc_sync_step(wl.frags, wl.n_total, st["theta_m"], None, st["theta_g"], st["momentum"],
                              st["delta_g"], pg, bk.I_p, bk.t_b, bk.t_g, 2, B.hparams(5, 100, merge_mode=mode, score_src=1),
                              out["R"], out["sel"], out["n_sel"], out["sums"], ws) == B.COCODC_ERR_NULL


def test_tau_zero_drops_the_correction(B, ref):
    wl = synth.Workload("tau0", (40000, 12345), tau=0, H=3, budget=1)
    _fused_case(B, ref, wl, seed=7, amplified=True)


def test_special_values_propagate(B, ref):
    """Denormals, zeros, huge values, infinities and NaN go through both paths alike."""
    n = 4096
    wl = synth.Workload("special", (n,), tau=5, H=100, budget=1)
    st = synth.make_state(wl, "cuda", seed=8)
    specials = torch.tensor([0.0, -0.0, 1e-45, -1e-40, 1e-38, 3e38, -3e38, float("inf"), float("-inf"),
                             float("nan"), 1.0, -1.0], device="cuda")
    g = torch.Generator(device="cuda").manual_seed(9)
    for k in ("theta_m", "theta_g", "momentum", "delta_g", "theta_m_send"):
        idx = torch.randint(0, n, (64,), generator=g, device="cuda")
        val = specials[torch.randint(0, specials.numel(), (64,), generator=g, device="cuda")]
        st[k][idx] = val
    bk = synth.bookkeeping(wl)
    ghp, rhp = B.hparams(5, 100), ref.hparams(5, 100)
    host = U.host_copy(st)
    ws = B.new_workspace(1, n)
    go = U.run_gpu_fused(B, wl.frags, n, st, bk, 1, ghp, ws)
    ro = U.run_ref_fused(ref, wl.frags, host, bk, 1, rhp)
    for k in ("theta_m", "theta_g", "momentum"):
        g_, r_ = st[k].cpu().numpy(), host[k]
        assert np.array_equal(np.isnan(g_), np.isnan(r_)), k
        ok = ~np.isnan(r_)
        assert np.array_equal(g_[ok], r_[ok]), k  # incl. infinities, signed zeros aside from -0 == 0
    assert np.array_equal(go["pg"].cpu().numpy().view(np.uint32)[~np.isnan(ro["pg"])],
                          ro["pg"].view(np.uint32)[~np.isnan(ro["pg"])])
    assert math.isnan(go["R"].cpu().numpy()[0]) == math.isnan(ro["R"][0])


# ------------------------------------------------------------------ single-step entry points
def test_primitives_match_oracle_and_fused_bit_for_bit(B, ref):
    wl = synth.Workload("prim", (50001, 16384, 3, 70000), tau=5, H=100, budget=2)
    bk = synth.bookkeeping(wl, "mixed")
    for amplified in (False, True):
        tau, H = (2, 1) if amplified else (wl.tau, wl.H)
        ghp, rhp = B.hparams(tau, H), ref.hparams(tau, H)
        st = synth.make_state(wl, "cuda", seed=11, amplified=amplified)
        n = wl.n_total
        ws = B.new_workspace(wl.K, n)
        # fused
        f = {k: v.clone() for k, v in st.items()}
        fo = U.run_gpu_fused(B, wl.frags, n, f, bk, 2, ghp, ws)
        # sequence of single-step calls
        s = {k: v.clone() for k, v in st.items()}
        h = U.host_copy(st)
        pg = torch.zeros(n, device="cuda")
        send = torch.zeros(n, device="cuda")
        assert B.cocodc_pseudograd(wl.frags, n, s["theta_g"], s["theta_m"], pg, send, ws) == 0
        assert torch.equal(send, s["theta_m"])
        h_pg = np.zeros(n, np.float32)
        ref.pseudograd(wl.frags, h["theta_g"], h["theta_m"], h_pg)
        assert np.array_equal(pg.cpu().numpy(), h_pg)
        assert B.cocodc_outer_nesterov(wl.frags, n, s["theta_g"], s["momentum"], s["delta_g"], ghp, ws) == 0
        ref.outer_nesterov(wl.frags, h["theta_g"], h["momentum"], h["delta_g"], rhp)
        assert U.rel_err(s["theta_g"].cpu().numpy(), h["theta_g"]) <= U.REL_TOL_TIGHT
        assert U.rel_err(s["momentum"].cpu().numpy(), h["momentum"]) <= U.REL_TOL_TIGHT
        assert B.cocodc_delay_compensate(wl.frags, n, s["theta_m"], s["theta_m_send"], s["theta_g"], ghp, ws) == 0
        ref.delay_compensate(wl.frags, h["theta_m"], h["theta_m_send"], h["theta_g"], rhp)
        assert U.rel_err(s["theta_m"].cpu().numpy(), h["theta_m"]) <= 2 * U.REL_TOL_TIGHT
        for kind in (2, 1):
            R = torch.zeros(wl.K, dtype=torch.float64, device="cuda")
            S = torch.zeros(wl.K, dtype=torch.float64, device="cuda")
            assert B.cocodc_fragment_scores(wl.frags, n, s["delta_g"], bk.I_p, kind, R, S, ws) == 0
            rc, hR, hS = ref.fragment_scores(wl.frags, h["delta_g"], bk.I_p, kind)
            fin = np.isfinite(hR)
            assert np.array_equal(np.isposinf(R.cpu().numpy()), np.isposinf(hR))
            assert U.rel_err(R.cpu().numpy()[fin], hR[fin]) <= U.SCORE_TOL_TIGHT
            assert U.rel_err(S.cpu().numpy(), hS) <= U.SCORE_TOL_TIGHT
            if kind == 2:
                R2 = R.clone()
        sel = torch.full((wl.K,), -1, dtype=torch.int32, device="cuda")
        n_sel = torch.zeros(1, dtype=torch.int32, device="cuda")
        assert B.cocodc_select_fragments(wl.K, R2, bk.t_b, bk.t_g, H, 2, sel, n_sel, ws) == 0
        torch.cuda.synchronize()
        # fused == sequence, bit for bit
        for k in ("theta_m", "theta_g", "momentum"):
            assert torch.equal(f[k], s[k]), k
        assert torch.equal(fo["pg"], pg)
        assert torch.equal(fo["R"], R2)
        assert fo["sel_list"] == sel[:int(n_sel.item())].cpu().tolist()


def test_selection_only_large_k_ties_inf_nan(B, ref):
    rng = np.random.default_rng(0)
    for K in (1, 2, 63, 64, 65, 257, 1024):
        vals = np.array([0.0, 0.5, 1.0, 2.0, math.inf, math.nan])
        R = vals[rng.integers(0, vals.size, K)]
        if K > 8:
            R[: K // 2] = rng.random(K // 2)
        t_g, H = 10_000, 100
        t_b = (t_g - rng.integers(1, 150, K)).tolist()
        ws = B.new_workspace(K, 0)
        for budget in (0, 1, 3, K // 2, K, K + 5):
            Rd = torch.from_numpy(R).cuda()
            sel = torch.full((K,), -7, dtype=torch.int32, device="cuda")
            n_sel = torch.zeros(1, dtype=torch.int32, device="cuda")
            assert B.cocodc_select_fragments(K, Rd, t_b, t_g, H, budget, sel, n_sel, ws) == 0
            torch.cuda.synchronize()
            rc, want = ref.select_fragments(R, t_b, t_g, H, budget)
            n = int(n_sel.item())
            assert n == min(budget, K)
            assert sel[:n].cpu().tolist() == want.tolist(), (K, budget)
            assert torch.all(sel[n:] == -7)


def test_selection_under_byte_budget(B, ref):
    rng = np.random.default_rng(1)
    for K in (1, 3, 24, 65, 1024):
        vals = np.array([0.0, 0.5, 1.0, 2.0, math.inf, math.nan])
        R = vals[rng.integers(0, vals.size, K)]
        if K > 8:
            R[: K // 2] = rng.random(K // 2)
        t_g, H = 10_000, 100
        t_b = (t_g - rng.integers(1, 150, K)).tolist()
        sizes = rng.integers(0, 1 << 30, K).tolist()
        ws = B.new_workspace(K, 0)
        for budget in (0, 1 << 29, 1 << 31, (1 << 30) * (K // 2), 1 << 62):
            Rd = torch.from_numpy(R).cuda()
            sel = torch.full((K,), -7, dtype=torch.int32, device="cuda")
            n_sel = torch.zeros(1, dtype=torch.int32, device="cuda")
            assert B.cocodc_select_fragments_bytes(K, Rd, t_b, t_g, H, sizes, budget, sel, n_sel, ws) == 0
            torch.cuda.synchronize()
            rc, want = ref.select_fragments_bytes(R, t_b, t_g, H, sizes, budget)
            n = int(n_sel.item())
            assert sel[:n].cpu().tolist() == want.tolist(), (K, budget)
            assert torch.all(sel[n:] == -7)
    assert B.cocodc_select_fragments_bytes(2, Rd, t_b[:2], t_g, H, None, 5, sel, n_sel, ws) == B.COCODC_ERR_NULL


# ------------------------------------------------------------------ determinism
def test_bitwise_reproducible_and_independent_of_launch_shape(B, ref):
    wl = synth.MINI_WORKLOADS["1.3B-mini"]
    bk = synth.bookkeeping(wl)
    ghp = B.hparams(wl.tau, wl.H)
    st = synth.make_state(wl, "cuda", seed=2)
    ws = B.new_workspace(wl.K, wl.n_total)
    results = []
    old = B.cocodc_set_blocks_per_cu(0)
    try:
        for bpc in (0, 0, 1, 3, 8):
            B.cocodc_set_blocks_per_cu(bpc)
            s = {k: v.clone() for k, v in st.items()}
            o = U.run_gpu_fused(B, wl.frags, wl.n_total, s, bk, wl.budget, ghp, ws)
            results.append((s, o))
    finally:
        B.cocodc_set_blocks_per_cu(old)
    s0, o0 = results[0]
    for s, o in results[1:]:
        for k in ("theta_m", "theta_g", "momentum"):
            assert torch.equal(s[k], s0[k])
        assert torch.equal(o["R"], o0["R"]) and torch.equal(o["sums"], o0["sums"])
        assert o["sel_list"] == o0["sel_list"]


@pytest.mark.parametrize("name", ["tiny", "125M-mini", "7B-mini"])
def test_tables_in_kernel_arguments_equal_uploaded_tables(B, name):
    """Tables of up to 32 segments and fragments travel inside the kernel arguments instead of being
    written to the workspace first: the fused step, the single steps and the selection give the very
    same bits either way (7B-mini has exactly 32 fragments, the largest table that takes this path)."""
    wl = synth.WORKLOADS[name] if name in synth.WORKLOADS else synth.MINI_WORKLOADS[name]
    bk = synth.bookkeeping(wl, "mixed")
    ghp = B.hparams(wl.tau, wl.H)
    st = synth.make_state(wl, "cuda", seed=9)
    n, K = wl.n_total, wl.K
    ws = B.new_workspace(K, n)
    results = []
    old = B.cocodc_set_tables_in_args(1)
    try:
        for in_args in (1, 0, 1):
            B.cocodc_set_tables_in_args(in_args)
            s = {k: v.clone() for k, v in st.items()}
            o = U.run_gpu_fused(B, wl.frags, n, s, bk, wl.budget, ghp, ws)
            # the single steps on a second copy
            t = {k: v.clone() for k, v in st.items()}
            pg, send = torch.zeros(n, device="cuda"), torch.zeros(n, device="cuda")
            R, S = (torch.zeros(K, dtype=torch.float64, device="cuda") for _ in range(2))
            sel = torch.full((K,), -1, dtype=torch.int32, device="cuda")
            n_sel = torch.zeros(1, dtype=torch.int32, device="cuda")
            assert B.cocodc_pseudograd(wl.frags, n, t["theta_g"], t["theta_m"], pg, send, ws) == 0
            assert B.cocodc_outer_nesterov(wl.frags, n, t["theta_g"], t["momentum"], t["delta_g"], ghp, ws) == 0
            assert B.cocodc_delay_compensate(wl.frags, n, t["theta_m"], t["theta_m_send"], t["theta_g"], ghp, ws) == 0
            assert B.cocodc_fragment_scores(wl.frags, n, t["delta_g"], bk.I_p, 2, R, S, ws) == 0
            assert B.cocodc_select_fragments(K, R, bk.t_b, bk.t_g, wl.H, wl.budget, sel, n_sel, ws) == 0
            torch.cuda.synchronize()
            results.append((s, o, t, pg, send, R, S, sel, n_sel))
    finally:
        B.cocodc_set_tables_in_args(old)
    s0, o0, t0, pg0, send0, R0, S0, sel0, n_sel0 = results[0]
    for s, o, t, pg, send, R, S, sel, n_sel in results[1:]:
        for k in ("theta_m", "theta_g", "momentum"):
            assert torch.equal(s[k], s0[k]) and torch.equal(t[k], t0[k]) and torch.equal(s[k], t[k]), k
        assert torch.equal(o["pg"], o0["pg"]) and torch.equal(pg, pg0) and torch.equal(send, send0)
        assert torch.equal(o["R"], o0["R"]) and torch.equal(o["sums"], o0["sums"]) and o["sel_list"] == o0["sel_list"]
        assert torch.equal(R, R0) and torch.equal(S, S0) and torch.equal(sel, sel0) and torch.equal(n_sel, n_sel0)
        assert torch.equal(R, o["R"])


def test_scores_do_not_depend_on_buffer_alignment(B):
    """The same fragment table over the same values at bases that are 16-byte aligned, 4 bytes off
    and 8 bytes off: stored values, raw sums, scores and selection are bit-identical."""
    wl = synth.MINI_WORKLOADS["125M-mini"]
    bk = synth.bookkeeping(wl)
    ghp = B.hparams(wl.tau, wl.H)
    st = synth.make_state(wl, "cuda", seed=6)
    ws = B.new_workspace(wl.K, wl.n_total)
    results = []
    for shift in (0, 1, 2, 3, 4):
        s = {}
        for k, v in st.items():
            buf = torch.empty(wl.n_total + 8, device="cuda")
            buf[shift:shift + wl.n_total].copy_(v)
            s[k] = buf[shift:shift + wl.n_total]
            assert s[k].data_ptr() % 16 == (4 * shift) % 16
        o = U.run_gpu_fused(B, wl.frags, wl.n_total, s, bk, wl.budget, ghp, ws)
        results.append((s, o))
    s0, o0 = results[0]
    for s, o in results[1:]:
        for k in ("theta_m", "theta_g", "momentum"):
            assert torch.equal(s[k], s0[k])
        assert torch.equal(o["pg"], o0["pg"])
        assert torch.equal(o["R"], o0["R"]) and torch.equal(o["sums"], o0["sums"])
        assert o["sel_list"] == o0["sel_list"]


def test_concurrent_calls_from_threads_on_their_own_streams(B, ref):
    """Calls that use different workspaces may run at the same time: four host threads, each on a
    stream of its own with its own buffers and workspace, 20 steps each; every thread's final state
    equals the one the same 20 steps give when run alone."""
    import threading
    wl = synth.MINI_WORKLOADS["1.3B-mini"]
    bk = synth.bookkeeping(wl)
    ghp = B.hparams(wl.tau, wl.H)
    n_threads, n_steps = 4, 20

    def run(seed, stream, box):
        st = synth.make_state(wl, "cuda", seed=seed)
        ws = B.new_workspace(wl.K, wl.n_total)
        out = U.gpu_outputs(wl.K)
        pg = torch.empty_like(st["delta_g"])
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            for _ in range(n_steps):
                rc = B.cocodc_sync_step(wl.frags, wl.n_total, st["theta_m"], st["theta_m_send"], st["theta_g"],
                                        st["momentum"], st["delta_g"], pg, bk.I_p, bk.t_b, bk.t_g, wl.budget, ghp,
                                        out["R"], out["sel"], out["n_sel"], out["sums"], ws, stream=stream)
                if rc != 0:
                    box["rc"] = rc
                    return
            stream.synchronize()
        box.update(rc=0, st=st, out=out, pg=pg)

    alone = []
    for t in range(n_threads):
        box = {}
        run(100 + t, torch.cuda.Stream(), box)
        assert box["rc"] == 0
        alone.append(box)
    together = [{} for _ in range(n_threads)]
    threads = [threading.Thread(target=run, args=(100 + t, torch.cuda.Stream(), together[t])) for t in range(n_threads)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    for a, b in zip(alone, together):
        assert b.get("rc") == 0
        for k in ("theta_m", "theta_g", "momentum"):
            assert torch.equal(a["st"][k], b["st"][k]), k
        assert torch.equal(a["pg"], b["pg"])
        assert torch.equal(a["out"]["R"], b["out"]["R"]) and torch.equal(a["out"]["sel"], b["out"]["sel"])


# ------------------------------------------------------------------ consecutive syncs
def test_hundred_consecutive_syncs_heavy_tailed_drift(B, ref):
    """1.3B-shaped run (reduced width): both sides evolve their own state in lock-step."""
    wl = synth.MINI_WORKLOADS["1.3B-mini"]
    for score_src in (0, 1):
        ghp, rhp = _hp_pair(B, ref, wl, score_src=score_src)
        st = synth.make_state(wl, "cuda", seed=0)
        host = U.host_copy(st)
        bk = synth.bookkeeping(wl)
        ws = B.new_workspace(wl.K, wl.n_total)
        log = U.SelectionLog()
        for k in range(wl.n_syncs):
            if k > 0:
                synth.next_sync_inputs(wl, st, 0, k)
                # the oracle side receives the same fresh inputs, applied to ITS OWN state
                drift = (st["theta_m"] - st["theta_m_send"]).cpu().numpy()
                host["theta_m_send"][:] = host["theta_m"]
                host["theta_m"] += drift
                host["delta_g"][:] = st["delta_g"].cpu().numpy()
            go = U.run_gpu_fused(B, wl.frags, wl.n_total, st, bk, wl.budget, ghp, ws, pg=None)
            ro = U.run_ref_fused(ref, wl.frags, host, bk, wl.budget, rhp, pg=False, shadow=(k in (0, 9, 99)))
            margin = U.compare_selection(go, ro, bk, wl.H, frag_lengths=wl.frag_lengths, log=log)
            if k in (0, 9, 99):
                obs = U.compare_fused(st, go, host, ro, wl.frags, tight=False, check_pg=False)
                print(f"   sync {k + 1} score_src={score_src} observed",
                      {a: (f"{b:.3g}" if isinstance(b, float) else b) for a, b in obs.items()},
                      f"margin {margin:.3g}", flush=True)
            bk = synth.advance_bookkeeping(wl, bk, ro["sel"].tolist())
        print(f"   score_src={score_src}: {log}", flush=True)
        assert log.ambiguous == 0 and log.compared == wl.n_syncs


# ------------------------------------------------------------------ error paths that need a device
def test_rejected_calls_touch_nothing(B, ref):
    wl = synth.Workload("err", (1000, 1000), tau=5, H=100, budget=1)
    st = synth.make_state(wl, "cuda", seed=1)
    keep = {k: v.clone() for k, v in st.items()}
    bk = synth.bookkeeping(wl)
    o = U.gpu_outputs(2)
    ws = B.new_workspace(2, wl.n_total)
    hp = B.hparams(5, 100)

    def call(frags=wl.frags, hp=hp, budget=1, ws=ws, wsb=None, tm=st["theta_m"], pg=None, n=wl.n_total):
        return B.cocodc_sync_step(frags, n, tm, st["theta_m_send"], st["theta_g"], st["momentum"],
                                  st["delta_g"], pg, bk.I_p, bk.t_b, bk.t_g, budget, hp, o["R"], o["sel"],
                                  o["n_sel"], o["sums"], ws, wsb)
    assert call(frags=[(0, 1500), (1000, 1000)]) == B.COCODC_ERR_RANGE
    assert call(frags=[(0, 1000), (1000, 1001)]) == B.COCODC_ERR_RANGE
    assert call(hp=B.hparams(-1, 100)) == B.COCODC_ERR_RANGE
    assert call(hp=B.hparams(5, 0)) == B.COCODC_ERR_RANGE
    assert call(hp=B.hparams(5, 100, lam=float("nan"))) == B.COCODC_ERR_NONFINITE
    assert call(budget=-1) == B.COCODC_ERR_RANGE
    assert call(wsb=64) == B.COCODC_ERR_WORKSPACE
    assert call(ws=None) == B.COCODC_ERR_NULL
    assert call(tm=None) == B.COCODC_ERR_NULL
    assert call(tm=st["theta_g"]) == B.COCODC_ERR_ALIAS
    assert call(pg=st["momentum"]) == B.COCODC_ERR_ALIAS
    assert call(pg=st["delta_g"][4:], n=wl.n_total - 4,
                frags=[(0, 1000), (1000, 996)]) == B.COCODC_ERR_ALIAS  # partial overlap
    assert call(tm=st["theta_m"].data_ptr() + 2) == B.COCODC_ERR_ALIGN
    torch.cuda.synchronize()
    for k in keep:
        assert torch.equal(keep[k], st[k]), k
    assert call() == 0
    torch.cuda.synchronize()
    assert not torch.equal(keep["theta_m"], st["theta_m"])
