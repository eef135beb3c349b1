"""GPU parity of the segmented entry points (fragments = strided sets of layers, Sec. 4.1)
against the oracle's segmented functions.  Needs an MI355X."""
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


def _case(B, ref, segs, K, n, I_p, t_b, t_g, budget, tau=5, H=100, seed=0, amplified=False, view_off=0, **hpkw):
    print(f"case segmented S={len(segs)} K={K} n={n} view_off={view_off} amplified={amplified} hp={hpkw}", flush=True)
    base = synth.Workload("seg", (n + view_off,), tau=tau, H=H)
    st = {k: v[view_off:] for k, v in synth.make_state(base, "cuda", seed=seed, amplified=amplified).items()}
    host = U.host_copy(st)
    ghp, rhp = B.hparams(tau, H, **hpkw), ref.hparams(tau, H, **hpkw)
    ws = B.new_workspace_segmented(len(segs), K, n)
    out = U.gpu_outputs(K)
    pg = torch.full((n,), 555.0, device="cuda")
    rc = B.cocodc_sync_step_segmented(segs, K, n, st["theta_m"], st["theta_m_send"], st["theta_g"], st["momentum"],
                                      st["delta_g"], pg, I_p, t_b, t_g, budget, ghp, out["R"], out["sel"],
                                      out["n_sel"], out["sums"], ws)
    assert rc == 0, B.cocodc_status_string(rc)
    torch.cuda.synchronize()
    out["pg"] = pg
    out["sel_list"] = out["sel"][:int(out["n_sel"].item())].cpu().tolist()
    h_pg = np.full(n, 555.0, np.float32)
    ro = ref.sync_step_segmented(segs, K, host["theta_m"], host["theta_m_send"], host["theta_g"], host["momentum"],
                                 host["delta_g"], h_pg, I_p, t_b, t_g, budget, rhp, shadow=True)
    assert ro["rc"] == 0
    ro["pg"] = h_pg
    frags = [(o, l) for o, l, _ in segs]
    obs = U.compare_fused(st, out, host, ro, frags)
    outside = np.ones(n, bool)
    for o, l in frags:
        outside[o:o + l] = False
    assert np.all(pg.cpu().numpy()[outside] == 555.0)
    bk = synth.Bookkeeping(t_g=t_g, t_b=list(t_b), I_p=list(I_p))
    U.compare_selection(out, ro, bk, H)
    # the scores-only entry point gives the same R and raw sums
    R2 = torch.zeros(K, dtype=torch.float64, device="cuda")
    S2 = torch.zeros(K, dtype=torch.float64, device="cuda")
    assert B.cocodc_fragment_scores_segmented(segs, K, n, st["delta_g"], I_p, 2, R2, S2, ws) == 0
    torch.cuda.synchronize()
    if hpkw.get("score_src", 0) == 0 and hpkw.get("norm_kind", 2) == 2:
        assert torch.equal(R2, out["R"])
    assert torch.equal(S2, out["sums"][:, 0].contiguous())
    print("   observed", {k: (f"{v:.3g}" if isinstance(v, float) else v) for k, v in obs.items()},
          "sel", out["sel_list"], flush=True)
    return out


def test_paper_strided_shards_full_125m_dims(B, ref):
    """12 layers of the 125M dimensions in 4 strided shards (shard k = layers k, k+4, k+8)."""
    segs, n = synth.strided_segments(12, 768, 2048, 4)
    out = _case(B, ref, segs, 4, n, [12, 24, 36, 12], [988, 976, 964, 988], 1000, 2)
    assert len(out["sel_list"]) == 2


def test_strided_shards_amplified_and_switches(B, ref):
    segs, n = synth.strided_segments(12, 96, 256, 4)
    _case(B, ref, segs, 4, n, [12, 24, 36, 12], [988, 976, 964, 988], 1000, 3, tau=2, H=1, amplified=True)
    _case(B, ref, segs, 4, n, [12, 24, 36, 12], [988, 976, 964, 988], 1000, 3, score_src=1, norm_kind=1)
    _case(B, ref, segs, 4, n, [12, 0, 36, 12], [988, 976, 100, 988], 1000, 4, merge_mode=1, alpha=0.3)


@pytest.mark.parametrize("view_off", [0, 1])
def test_adversarial_segment_tables(B, ref, view_off):
    segs = [(70001, 3, 2), (5, 1000, 0), (1013, 3, 1), (1030, 40000, 0), (41031, 16384, 1), (60001, 1, 0),
            (16383 + 41031 + 2, 0, 1), (65000, 5001, 4)]  # fragment 3 has no segment; listed out of order
    n = 70010
    _case(B, ref, segs, 5, n, [7, 14, 21, 7, 0], [990, 980, 970, 100, 990], 1000, 3, view_off=view_off)


@pytest.mark.parametrize("n_total_pad", [0, 1 << 24])
def test_maximum_number_of_segments(B, ref, n_total_pad):
    """4096 segments (the most a table may hold) in shuffled order over 300 fragments, every fifth one
    empty, lengths from 1 element to several tiles: every workgroup has to find its segment among
    thousands of records, runs of records without tiles included.  With both tile sizes."""
    import random
    rng = random.Random(11)
    S, K = 4096, 300
    segs, off = [], 3
    for j in range(S):
        if j % 5 == 4:
            ln = 0
        else:
            ln = rng.choice([1, 2, 3, 5, 64, 700, 2047, 2048, 2049, 4095, 4096, 4097, rng.randrange(1, 13000)])
        segs.append((off, ln, rng.randrange(K)))
        off += ln + rng.choice([0, 0, 1, 3, 4096])
    n_used = off + 5
    rng.shuffle(segs)
    I_p = [1 + p % 7 for p in range(K)]
    t_b = [1000 - (p * 37) % 150 for p in range(K)]
    n = n_used + n_total_pad
    assert B.cocodc_tile_elements(n) == (4096 if n_total_pad else 2048)
    _case(B, ref, segs, K, n, I_p, t_b, 1000, 17, seed=5)


def test_segmented_equals_contiguous_on_gpu(B, ref):
    wl = synth.MINI_WORKLOADS["125M-mini"]
    bk = synth.bookkeeping(wl)
    st = synth.make_state(wl, "cuda", seed=3)
    a = {k: v.clone() for k, v in st.items()}
    b = {k: v.clone() for k, v in st.items()}
    ghp = B.hparams(wl.tau, wl.H)
    ws = B.new_workspace(wl.K, wl.n_total)
    oa = U.run_gpu_fused(B, wl.frags, wl.n_total, a, bk, wl.budget, ghp, ws)
    segs = [(o, l, p) for p, (o, l) in enumerate(wl.frags)]
    ob = U.gpu_outputs(wl.K)
    pg = torch.full_like(b["delta_g"], 555.0)
    ws2 = B.new_workspace_segmented(len(segs), wl.K, wl.n_total)
    assert B.cocodc_sync_step_segmented(segs, wl.K, wl.n_total, b["theta_m"], b["theta_m_send"], b["theta_g"],
                                        b["momentum"], b["delta_g"], pg, bk.I_p, bk.t_b, bk.t_g, wl.budget, ghp,
                                        ob["R"], ob["sel"], ob["n_sel"], ob["sums"], ws2) == 0
    torch.cuda.synchronize()
    for k in a:
        assert torch.equal(a[k], b[k])
    assert torch.equal(oa["pg"], pg) and torch.equal(oa["R"], ob["R"]) and torch.equal(oa["sums"], ob["sums"])
    assert torch.equal(oa["sel"], ob["sel"])


def test_segmented_rejections(B):
    n = 4096
    base = 0x10000000
    tm, ts, tg, m, dg, R, sel, ns, ws = (base + i * 0x100000 for i in range(9))
    hp = B.hparams(5, 100)
    wsb = B.cocodc_workspace_bytes_segmented(3, 2, n)
    assert wsb > 0 and B.cocodc_workspace_bytes_segmented(5000, 2, n) == 0

    def call(segs, K=2, S=None, wsb=wsb):
        return B.cocodc_sync_step_segmented(segs, K, n, tm, ts, tg, m, dg, None, [1] * K, [0] * K, 10, 1, hp, R, sel, ns,
                                            None, ws, wsb, stream=0, S=S)
    assert call([(0, 10, 0), (5, 10, 1)]) == B.COCODC_ERR_RANGE
    assert call([(0, 10, 2)]) == B.COCODC_ERR_RANGE
    assert call([(4090, 10, 0)]) == B.COCODC_ERR_RANGE
    assert call(None, S=2) == B.COCODC_ERR_NULL
    assert call([(0, 10, 0)] * 1, wsb=64) == B.COCODC_ERR_WORKSPACE


def test_segmented_event_random_masks(B, ref):
    """cocodc_sync_event_segmented: 30 random events on random segment tables (fragments cut into shuffled
    pieces, empty fragments, unaligned bases, buffers beyond 2^24 elements, every hyper-parameter switch),
    shards marked arrived and / or in flight, old scores with infinities and a NaN that must survive untouched."""
    import random
    from test_gpu_random_sweep import _random_case
    rng = random.Random(4000)
    for case in range(30):
        c = _random_case(rng)
        K = len(c["frags"])
        segs = []
        for p, (o, l) in enumerate(c["frags"]):
            cuts = sorted(rng.randrange(0, l + 1) for _ in range(rng.choice([0, 0, 1, 2, 5]))) if l else []
            edges = [0] + cuts + [l]
            segs += [(o + a, b - a, p) for a, b in zip(edges, edges[1:])]
        rng.shuffle(segs)
        n_alloc = c["n"] + ((1 << 24) if c["pad_big"] else 0)
        mask = [int(rng.random() < rng.choice([0.0, 0.3, 1.0])) for _ in range(K)]
        if case % 2:
            mask = [m | (2 if rng.random() < 0.4 else 0) for m in mask]
        hpk = dict(c["hp"])
        tau, H = hpk.pop("tau"), hpk.pop("H")
        print(f"case segmented event #{case} S={len(segs)} K={K} n={n_alloc} mask={mask} view_off={c['view_off']} "
              f"hp={c['hp']}", flush=True)
        base = synth.Workload("rnd", (n_alloc + c["view_off"],), tau=tau, H=H)
        st = {k: v[c["view_off"]:] for k, v in
              synth.make_state(base, "cuda", seed=500 + case, amplified=c["amplified"]).items()}
        host = U.host_copy(st)
        ghp, rhp = B.hparams(tau, H, **hpk), ref.hparams(tau, H, **hpk)
        R0 = np.array([rng.choice([np.inf, 0.0, 0.5, 2.0, rng.random(), np.nan if K > 3 and rng.random() < 0.1 else 1.5])
                       for _ in range(K)])
        R_dev = torch.from_numpy(R0.copy()).cuda()
        sums_dev = torch.full((K, 4), -3.0, dtype=torch.float64, device="cuda")
        out = U.gpu_outputs(K)
        pg = torch.full((n_alloc,), 555.0, device="cuda")
        ws = B.new_workspace_segmented(len(segs), K, n_alloc)
        rc = B.cocodc_sync_event_segmented(segs, K, n_alloc, mask, st["theta_m"], st["theta_m_send"], st["theta_g"],
                                           st["momentum"], st["delta_g"], pg, c["I_p"], c["t_b"], 1000, c["budget"],
                                           ghp, R_dev, out["sel"], out["n_sel"], sums_dev, ws)
        assert rc == 0, B.cocodc_status_string(rc)
        torch.cuda.synchronize()
        R_ref, sums_ref = R0.copy(), np.full((K, 4), -3.0)
        h_pg = np.full(n_alloc, 555.0, np.float32)
        ro = ref.sync_event_segmented(segs, K, mask, host["theta_m"], host["theta_m_send"], host["theta_g"],
                                      host["momentum"], host["delta_g"], h_pg, c["I_p"], c["t_b"], 1000, c["budget"],
                                      rhp, R_ref, sums=sums_ref)
        assert ro["rc"] == 0
        for k in ("theta_m", "theta_g", "momentum", "theta_m_send", "delta_g"):
            assert np.array_equal(st[k].cpu().numpy().view(np.uint32), host[k].view(np.uint32)), k
        assert np.array_equal(pg.cpu().numpy().view(np.uint32), h_pg.view(np.uint32))
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
