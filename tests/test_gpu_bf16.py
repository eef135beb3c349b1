"""GPU parity of the bf16 variant (bf16 local parameters, fp32 global state) against the
oracle's bf16 functions.  bf16 outputs must be bit-identical (both sides round the same fp64
value once); the stated bar for them is one bf16 rounding, 2^-8 relative.  Needs an MI355X."""
import numpy as np
import pytest
import torch

from paper_2504_17672_amd import synth

import parity_util as U

pytestmark = pytest.mark.gpu
BF16_TOL = 2.0 ** -8  # half a unit in the last place of an 8-bit significand


@pytest.fixture(scope="module")
def B():
    from paper_2504_17672_amd import binding
    assert torch.cuda.is_available()
    return binding


def _u16(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16).copy()


def _widen(u16):
    return torch.from_numpy(u16.view(np.int16)).view(torch.bfloat16).float().numpy().astype(np.float64)


def _case(B, ref, wl, seed=0, variant="regular", amplified=False, view_off=0, pg=True, send=True, budget=None, **hpkw):
    print(f"case bf16 {wl.name} K={wl.K} n={wl.n_total} seed={seed} amplified={amplified} view_off={view_off} "
          f"hp={hpkw}", flush=True)
    st = synth.make_state(wl, "cuda", seed=seed, amplified=amplified, pad=view_off + 8)
    n = wl.n_total
    dev = {k: (v.to(torch.bfloat16) if k in ("theta_m", "theta_m_send") else v.clone())[view_off:view_off + n + 8]
           for k, v in st.items()}
    if amplified:  # include specials among the bf16 inputs
        dev["theta_m"][5] = float("inf")
        dev["theta_m"][6] = 1e-40
        dev["theta_m_send"][7] = -3e38
    bk = synth.bookkeeping(wl, variant)
    args = dict(lam=wl.lam, eta=wl.eta, mu=wl.mu)
    args.update(hpkw)
    ghp, rhp = B.hparams(wl.tau, wl.H, **args), ref.hparams(wl.tau, wl.H, **args)
    budget = wl.budget if budget is None else budget
    host = {k: (_u16(v) if v.dtype == torch.bfloat16 else v.cpu().numpy().copy()) for k, v in dev.items()}
    n_alloc = n + 8
    ws = B.new_workspace(wl.K, n_alloc)
    out = U.gpu_outputs(wl.K)
    pg_dev = torch.full((n_alloc,), 555.0, device="cuda").to(torch.bfloat16) if pg else None
    rc = B.cocodc_sync_step_bf16(wl.frags, n_alloc, dev["theta_m"], dev["theta_m_send"] if send else None,
                                 dev["theta_g"], dev["momentum"], dev["delta_g"], pg_dev, bk.I_p, bk.t_b, bk.t_g,
                                 budget, ghp, out["R"], out["sel"], out["n_sel"], out["sums"], ws)
    assert rc == 0, B.cocodc_status_string(rc)
    torch.cuda.synchronize()
    h_pg = _u16(torch.full((n_alloc,), 555.0).to(torch.bfloat16)) if pg else None
    ro = ref.sync_step_bf16(wl.frags, host["theta_m"], host["theta_m_send"] if send else None, host["theta_g"],
                            host["momentum"], host["delta_g"], h_pg, bk.I_p, bk.t_b, bk.t_g, budget, rhp, shadow=True)
    assert ro["rc"] == 0
    mask = np.zeros(n_alloc, bool)
    for o, l in wl.frags:
        mask[o:o + l] = True
    # fp32 master copies: bit-identical, and within the stated bar of the fp64 value
    for k in ("theta_g", "momentum"):
        g = dev[k].cpu().numpy()
        same = (g == host[k]) | (np.isnan(g) & np.isnan(host[k]))
        assert same.all(), k
        fin = mask & np.isfinite(ro[k + "64"])
        assert U.rel_err(g[fin], ro[k + "64"][fin]) <= U.REL_TOL
    # bf16 outputs: identical bit patterns; within one bf16 rounding of the fp64 value
    g_tm = _u16(dev["theta_m"])
    assert np.array_equal(g_tm, host["theta_m"])
    fin = mask & np.isfinite(ro["theta_m64"]) & (np.abs(ro["theta_m64"]) > 1e-37) & (np.abs(ro["theta_m64"]) < 3e38)
    assert U.rel_err(_widen(g_tm)[fin], ro["theta_m64"][fin]) <= BF16_TOL
    if pg:
        assert np.array_equal(_u16(pg_dev), h_pg)
    if send:
        assert np.array_equal(_u16(dev["theta_m_send"]), host["theta_m_send"])
    Rg, Rr = out["R"].cpu().numpy(), ro["R"]
    finR = np.isfinite(Rr)
    assert np.array_equal(np.isposinf(Rg), np.isposinf(Rr)) and np.array_equal(np.isnan(Rg), np.isnan(Rr))
    assert U.rel_err(Rg[finR], Rr[finR]) <= U.SCORE_TOL_TIGHT
    sg = out["sums"].cpu().numpy()
    ok = np.isfinite(ro["sums"])
    assert U.rel_err(sg[ok], ro["sums"][ok]) <= U.SCORE_TOL_TIGHT
    n_sel = int(out["n_sel"].item())
    out["sel_list"] = out["sel"][:n_sel].cpu().tolist()
    if not np.isnan(Rr).any():
        U.compare_selection(out, ro, bk, wl.H)
    print("   ok; selected", out["sel_list"], flush=True)
    return out, ro


@pytest.mark.parametrize("name", ["125M-mini", "1.3B-mini", "7B-mini"])
def test_bf16_mini_workloads(B, ref, name):
    wl = synth.MINI_WORKLOADS[name]
    _case(B, ref, wl, seed=0)
    _case(B, ref, wl, seed=1, variant="mixed", pg=False)


def test_bf16_amplified_specials_and_switches(B, ref):
    wl = synth.Workload("bf16-amp", (40000, 33333, 12345), tau=2, H=1, budget=2)
    _case(B, ref, wl, seed=3, amplified=True)
    _case(B, ref, wl, seed=3, amplified=True, nesterov=0, drift_sign=-1)
    _case(B, ref, wl, seed=3, amplified=True, delta_src=1)
    _case(B, ref, wl, seed=4, merge_mode=1, alpha=0.3, send=False)
    _case(B, ref, wl, seed=4, merge_mode=2)
    wl0 = synth.Workload("bf16-tau0", (40000, 12345), tau=0, H=3, budget=1)
    _case(B, ref, wl0, seed=5)


@pytest.mark.parametrize("view_off", [0, 1, 3])
def test_bf16_odd_tables_and_alignments(B, ref, view_off):
    """Unaligned fragment offsets, gaps, an empty fragment; view_off 1 and 3 make the bf16 bases
    2-byte and 6-byte aligned only (element-wise kernel variant)."""
    from types import SimpleNamespace
    frags = [(5, 1000), (1013, 3), (1030, 40000), (41031, 16384), (60001, 1), (60002, 0), (60010, 9991)]
    data_wl = synth.Workload("bf16-odd-data", (70001,), tau=5, H=100)
    w = SimpleNamespace(name="bf16-odd", K=7, n_total=70001, frags=frags, tau=5, H=100, lam=0.5, eta=0.7, mu=0.9,
                        budget=3, h=14)
    orig = synth.make_state
    try:
        synth.make_state = lambda _wl, dev, **kw: orig(data_wl, dev, **kw)
        _case(B, ref, w, seed=6, view_off=view_off)
    finally:
        synth.make_state = orig


def test_bf16_full_125m_every_element(B, ref):
    _case(B, ref, synth.WORKLOADS["125M"], seed=0)


# ------------------------------------------------------------------ IEEE binary16 pseudo-gradient
@pytest.mark.parametrize("name", ["125M-mini", "7B-mini"])
def test_f16_pseudograd_mini_workloads(B, ref, name):
    wl = synth.MINI_WORKLOADS[name]
    _case(B, ref, wl, seed=0, pg_format=1)
    _case(B, ref, wl, seed=1, variant="mixed", pg_format=1, view_off=1)


def test_f16_pseudograd_amplified_specials_and_switches(B, ref):
    wl = synth.Workload("f16-amp", (40000, 33333, 12345), tau=2, H=1, budget=2)
    _case(B, ref, wl, seed=3, amplified=True, pg_format=1)
    _case(B, ref, wl, seed=3, amplified=True, nesterov=0, drift_sign=-1, delta_src=1, pg_format=1)
    _case(B, ref, wl, seed=4, merge_mode=1, alpha=0.3, send=False, pg_format=1)
    _case(B, ref, wl, seed=4, merge_mode=2, pg_format=1, view_off=3)
    _case(B, ref, wl, seed=5, pg=False, pg_format=1)


def test_f16_rounding_on_the_gpu_every_pattern_ties_and_double_rounding_traps(B, ref):
    """cocodc_pseudograd_bf16 with pg_format = binary16 on differences chosen to sit on, just above and just
    below every kind of rounding boundary: every binary16 value itself, the midpoint of every pair of
    neighbours (a tie), midpoints moved by one binary32 step, and midpoints moved by an amount far below
    binary32 resolution (a conversion that went through binary32 and rounded twice would get those wrong).
    The GPU and the oracle (pinned to exact arithmetic) must agree on every bit."""
    pat = np.arange(0x7C00, dtype=np.uint16)                       # every finite non-negative binary16
    val = pat.view(np.float16).astype(np.float64)
    nxt = np.append(val[1:], 65536.0)                                 # the value the next pattern has / would have
    mid = (val + nxt) / 2                                             # exact: 12 significant bits
    mid32 = mid.astype(np.float32)
    assert np.array_equal(mid32.astype(np.float64), mid)
    tg_parts, tm_parts = [], []

    def add(tg32, tm_value):
        tg_parts.append(tg32.astype(np.float32))
        tm_parts.append(np.full(tg32.size, tm_value, np.float32))
    add(val.astype(np.float32), 0.0)                                  # the values themselves
    add(mid32, 0.0)                                                   # exact ties
    add(np.nextafter(mid32, np.float32(np.inf)), 0.0)                 # one binary32 step above / below a tie
    add(np.nextafter(mid32, np.float32(-np.inf)), 0.0)
    for k in (-30, -40, -60, -100):                                   # tie -+ 2^k: not a binary32 number
        add(mid32, 2.0 ** k)
        add(mid32, -(2.0 ** k))
    add(np.array([65504, 65519.99, 65520, 65521, 1e30, np.inf, np.nan, 2.0 ** -25, 2.0 ** -26, 1e-40, 0.0],
                 np.float32), 0.0)
    tg = np.concatenate(tg_parts)
    tm = np.concatenate(tm_parts)
    tg = np.concatenate([tg, -tg])
    tm = np.concatenate([tm, -tm])
    n = tg.size
    tm_bf16 = torch.from_numpy(tm).to(torch.bfloat16)
    assert torch.equal(tm_bf16.float(), torch.from_numpy(tm))         # the offsets are bf16 numbers
    d_tg, d_tm = torch.from_numpy(tg).cuda(), tm_bf16.cuda()
    pg = torch.zeros(n, dtype=torch.int16, device="cuda")
    ws = B.new_workspace(1, n)
    print(f"case f16 rounding n={n}", flush=True)
    assert B.cocodc_pseudograd_bf16([(0, n)], n, d_tg, d_tm, pg, None, ws, pg_format=B.COCODC_PG_F16) == 0
    torch.cuda.synchronize()
    h_pg = np.zeros(n, np.uint16)
    assert ref.pseudograd_bf16([(0, n)], tg, _u16(tm_bf16), h_pg, None, pg_format=1) == 0
    got = pg.cpu().numpy().view(np.uint16)
    bad = np.nonzero(got != h_pg)[0]
    assert bad.size == 0, [(float(tg[i]), float(tm[i]), hex(got[i]), hex(h_pg[i])) for i in bad[:5]]
    # and the bf16 format of the same differences (the default of the same call)
    assert B.cocodc_pseudograd_bf16([(0, n)], n, d_tg, d_tm, pg, None, ws) == 0
    torch.cuda.synchronize()
    assert ref.pseudograd_bf16([(0, n)], tg, _u16(tm_bf16), h_pg, None) == 0
    assert np.array_equal(pg.cpu().numpy().view(np.uint16), h_pg)


def test_bf16_pseudograd_entry_point(B, ref):
    wl = synth.Workload("bf16-pg", (50001, 16384, 3, 70000), tau=5, H=100)
    st = synth.make_state(wl, "cuda", seed=8)
    n = wl.n_total
    tm = st["theta_m"].to(torch.bfloat16)
    pg = torch.zeros(n, device="cuda", dtype=torch.bfloat16)
    send = torch.zeros(n, device="cuda", dtype=torch.bfloat16)
    ws = B.new_workspace(wl.K, n)
    frags = wl.frags[1:]
    assert B.cocodc_pseudograd_bf16(frags, n, st["theta_g"], tm, pg, send, ws) == 0
    torch.cuda.synchronize()
    h_pg, h_send = np.zeros(n, np.uint16), np.zeros(n, np.uint16)
    assert ref.pseudograd_bf16(frags, st["theta_g"].cpu().numpy(), _u16(tm), h_pg, h_send) == 0
    assert np.array_equal(_u16(pg), h_pg) and np.array_equal(_u16(send), h_send)
    assert B.cocodc_pseudograd_bf16(frags, n, st["theta_g"], tm, pg, None, ws) == 0
    assert B.cocodc_pseudograd_bf16(frags, n, st["theta_g"], tm, pg, send, ws, pg_format=B.COCODC_PG_F16) == 0
    torch.cuda.synchronize()
    assert ref.pseudograd_bf16(frags, st["theta_g"].cpu().numpy(), _u16(tm), h_pg, h_send, pg_format=1) == 0
    assert np.array_equal(pg.view(torch.int16).cpu().numpy().view(np.uint16), h_pg)
    assert np.array_equal(_u16(send), h_send)
    assert B.cocodc_pseudograd_bf16(frags, n, st["theta_g"], tm, pg, None, ws, pg_format=7) == B.COCODC_ERR_RANGE
    assert B.cocodc_pseudograd_bf16(frags, n, st["theta_g"], tm, tm, None, ws) == B.COCODC_ERR_ALIAS
    assert B.cocodc_pseudograd_bf16(frags, n, st["theta_g"], tm.data_ptr() + 1, pg, None, ws) == B.COCODC_ERR_ALIGN


@pytest.mark.parametrize("seed", range(2))
def test_bf16_random_cases(B, ref, seed):
    """Seeded random fragment sizes, base alignments and hyper-parameter switches."""
    import random
    rng = random.Random(3000 + seed)
    for case in range(20):
        K = rng.choice([1, 2, 3, 7, 20])
        sizes = tuple(rng.choice([0, 1, 3, 4, 5, 1000, 2047, 2048, 2049, 4096, 4101, rng.randrange(1, 25000)])
                      for _ in range(K))
        if sum(sizes) == 0:
            sizes = sizes + (17,)
        merge_mode = rng.choice([0, 0, 0, 1, 2])
        score_src = rng.choice([0, 0, 1])
        wl = synth.Workload(f"bf16-rnd-{seed}-{case}", sizes, tau=rng.choice([0, 1, 2, 5, 50]),
                            H=rng.choice([1, 3, 100, 1000]), budget=rng.randrange(0, len(sizes) + 1))
        _case(B, ref, wl, seed=seed * 100 + case, amplified=rng.random() < 0.4, view_off=rng.choice([0, 1, 2, 3, 4]),
              pg=rng.random() < 0.8, send=(merge_mode == 0 or score_src == 1 or rng.random() < 0.5),
              variant=rng.choice(["regular", "mixed"]) if len(sizes) > 1 else "regular",
              lam=rng.choice([0.0, 0.5, 1.0, 3.0]), eta=rng.choice([0.7, 1.0]), mu=rng.choice([0.9, 0.0]),
              nesterov=rng.choice([1, 0]), drift_sign=rng.choice([1, -1]), score_src=score_src,
              norm_kind=rng.choice([2, 1]), merge_mode=merge_mode, alpha=rng.choice([1.0, 0.5]),
              delta_src=rng.choice([0, 1]) if merge_mode == 0 else 0, pg_format=rng.choice([0, 0, 1]))
