"""The 350M, 1.3B and 7B fragment sets at the full width their configurations state, in the
buffer layout and launch configuration that bench.py times, with EVERY element of every fragment
through the CPU oracle.

The oracle used here is its chunk-parallel variant (cocodc_ref_sync_step_mt): the same per-element
function as the definitional single-threaded loop, pinned to it in tests/test_oracle_pins.py; only
the order in which a fragment's partial sums are added differs (chunks of 65536 elements).  Stored
fp32 values are compared bit for bit on the GPU (the oracle's output is uploaded fragment by
fragment), which implies the stated bar of 1e-5 relative to the oracle's fp64 value: the stored
value is that fp64 value rounded once.  Scores and sums: <= 1e-8 relative (stated bar 1e-5).
Selections: identical indices (parity_util.compare_selection).

Host memory stays modest: one fragment (or, for the 100-sync run, one worker state) at a time.
Every test prints its wall time; the whole file is budgeted at about four minutes on an MI355X.
"""
import time

import numpy as np
import pytest
import torch

from paper_2504_17672_amd import layout as L
from paper_2504_17672_amd import synth

import parity_util as U

pytestmark = pytest.mark.gpu

IN_PLACE = ("theta_m", "theta_g", "momentum")
NAMES = ("theta_m", "theta_m_send", "theta_g", "momentum", "delta_g")


@pytest.fixture(scope="module")
def B():
    from paper_2504_17672_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return binding


def _threads():
    import os
    n = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    env = os.environ.get("OMP_NUM_THREADS")
    return max(1, min(n, int(env)) if env and env.isdigit() else n)


def _checksum(t):
    return t.view(torch.int32).sum(dtype=torch.int64).item()


def _bench_layout(B, wl, arena_fraction=0.8):
    """The six buffers as bench.py places them (one allocation, stride found by its set-up probe)."""
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    arena, carved, stride, _ = L.tuned_spaced_buffers(wl.n_total, wl.frags, "cuda",
                                                      max_arena_bytes=int(free * arena_fraction))
    names = NAMES + ("pg",)
    return arena, dict(zip(names, carved)), stride


class FragmentChecker:
    """Runs one fragment through the oracle on pinned staging buffers and compares the GPU's stored
    values with the oracle's, bit for bit, on the device."""

    def __init__(self, ref, max_len):
        self.ref = ref
        self.host = {k: U.pinned(max_len) for k in NAMES + ("pg",)}
        self.dev = torch.empty(max_len, dtype=torch.float32, device="cuda")
        self.threads = _threads()

    def check(self, frag_len, inputs, gpu_after, gpu_pg, I_p, t_b, t_g, rhp, label):
        """inputs: dict name -> device tensor (frag_len) of the values BEFORE the step;
        gpu_after: dict name -> device tensor of theta_m / theta_g / momentum AFTER it."""
        h = {k: self.host[k][:frag_len] for k in self.host}
        for k in NAMES:
            h[k].copy_(inputs[k])
        torch.cuda.synchronize()
        hn = {k: v.numpy() for k, v in h.items()}
        out = self.ref.sync_step([(0, frag_len)], hn["theta_m"], hn["theta_m_send"], hn["theta_g"], hn["momentum"],
                                 hn["delta_g"], hn["pg"], [I_p], [t_b], t_g, 1, rhp, n_threads=self.threads)
        assert out["rc"] == 0
        for k in IN_PLACE:
            if not U.bits_equal(gpu_after[k], h[k], self.dev):
                raise AssertionError((label, k, U.mismatch_report(gpu_after[k], h[k], self.dev)))
        if gpu_pg is not None and not U.bits_equal(gpu_pg, h["pg"], self.dev):
            raise AssertionError((label, "pg", U.mismatch_report(gpu_pg, h["pg"], self.dev)))
        return out["R"][0], out["sums"][0]


def _compare_scores(Rg, sums_g, R_ref, sums_ref):
    fin = np.isfinite(R_ref)
    assert np.array_equal(np.isposinf(Rg), np.isposinf(R_ref))
    e_R = U.rel_err(Rg[fin], R_ref[fin]) if fin.any() else 0.0
    e_S = U.rel_err(sums_g, sums_ref)
    assert e_R <= U.REL_TOL and e_S <= U.REL_TOL
    assert e_R <= U.SCORE_TOL_TIGHT and e_S <= U.SCORE_TOL_TIGHT, (e_R, e_S)
    return e_R, e_S


def _one_sync_every_fragment(B, ref, wl, st, record, pg, bk, ghp, rhp, checker, label, budget=None, H=None):
    """One fused step over all fragments in one call, then every fragment through the oracle.  The
    values the step overwrote are drawn again from the recorded generator states."""
    n, K = wl.n_total, wl.K
    budget = wl.budget if budget is None else budget
    H = wl.H if H is None else H   # the period the hyper-parameters carry (Algorithm 2's overdue test)
    before = {k: _checksum(st[k]) for k in ("theta_m_send", "delta_g")}
    pg.fill_(555.0)
    out = U.gpu_outputs(K)
    ws = B.new_workspace(K, n)
    rc = B.cocodc_sync_step(wl.frags, n, st["theta_m"], st["theta_m_send"], st["theta_g"], st["momentum"],
                            st["delta_g"], pg, bk.I_p, bk.t_b, bk.t_g, budget, ghp, out["R"], out["sel"], out["n_sel"],
                            out["sums"], ws)
    assert rc == 0, B.cocodc_status_string(rc)
    torch.cuda.synchronize()
    for k, v in before.items():
        assert _checksum(st[k]) == v, f"{k} was modified"
    R_ref, sums_ref = np.zeros(K), np.zeros((K, 4))
    scratch = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    for p, (off, ln) in enumerate(wl.frags):
        inputs = {k: synth.original_slice(record, k, off, off + ln, "cuda", scratch) for k in IN_PLACE}
        inputs["theta_m_send"] = st["theta_m_send"][off:off + ln]
        inputs["delta_g"] = st["delta_g"][off:off + ln]
        after = {k: st[k][off:off + ln] for k in IN_PLACE}
        R_ref[p], sums_ref[p] = checker.check(ln, inputs, after, pg[off:off + ln], bk.I_p[p], bk.t_b[p], bk.t_g, rhp,
                                              f"{label} fragment {p}")
    e_R, e_S = _compare_scores(out["R"].cpu().numpy(), out["sums"].cpu().numpy(), R_ref, sums_ref)
    rc, want = ref.select_fragments(R_ref, bk.t_b, bk.t_g, H, budget)
    assert rc == 0
    n_sel = int(out["n_sel"].item())
    go = dict(R=out["R"], sel_list=out["sel"][:n_sel].cpu().tolist())
    margin = U.compare_selection(go, dict(R=R_ref, sel=want), bk, H, frag_lengths=wl.frag_lengths)
    return dict(R=e_R, sums=e_S, margin=margin, sel=go["sel_list"])


# ------------------------------------------------------------------ config 5: 7B, all 32 fragments
def test_7b_every_element_of_all_fragments(B, ref):
    t0 = time.perf_counter()
    wl = synth.WORKLOADS["7B"]
    arena, bufs, stride = _bench_layout(B, wl)
    print(f"case 7B full width K={wl.K} n={wl.n_total} layout=tuned stride={stride / 2**30:.0f} GiB", flush=True)
    record = {}
    st = synth.make_state(wl, "cuda", seed=0, buffers=bufs, record=record)
    bk = synth.bookkeeping(wl)
    ghp, rhp = B.hparams(wl.tau, wl.H, wl.lam, wl.eta, wl.mu), ref.hparams(wl.tau, wl.H, wl.lam, wl.eta, wl.mu)
    checker = FragmentChecker(ref, max(wl.frag_lengths))
    obs = _one_sync_every_fragment(B, ref, wl, st, record, bufs["pg"], bk, ghp, rhp, checker, "7B")
    print(f"   all {wl.K} fragments ({wl.n_total} parameters) bit-identical to the oracle; observed {obs}; "
          f"wall {time.perf_counter() - t0:.1f} s", flush=True)


def test_7b_in_eight_strided_shards_every_element(B, ref):
    """bench.py --strided-shards 8 at full width: the 7B set's layers in 8 strided shards (Sec. 4.1: shard k =
    layers k, k + 8, ...) on the layer-ordered buffers, one segmented fused call, every segment through the
    oracle; a shard's raw sums are its segments' sums added in the order listed."""
    t0 = time.perf_counter()
    wl = synth.WORKLOADS["7B"]
    n, Ks = wl.n_total, 8
    segs, n_seg = synth.strided_segments(*wl.model, Ks)
    assert n_seg == n
    arena, bufs, stride = _bench_layout(B, wl)
    print(f"case 7B strided full width K={Ks} S={len(segs)} n={n} stride={stride / 2**30:.0f} GiB", flush=True)
    record = {}
    st = synth.make_state(wl, "cuda", seed=0, buffers=bufs, record=record)
    pg = bufs["pg"]
    pg.fill_(555.0)
    h = max(1, wl.H // Ks)
    I_p = [h * (1 + p % 3) for p in range(Ks)]
    t_g = 10 * wl.H
    t_b = [t_g - i for i in I_p]
    ghp, rhp = B.hparams(wl.tau, wl.H, wl.lam, wl.eta, wl.mu), ref.hparams(wl.tau, wl.H, wl.lam, wl.eta, wl.mu)
    out = U.gpu_outputs(Ks)
    ws = B.new_workspace_segmented(len(segs), Ks, n)
    rc = B.cocodc_sync_step_segmented(segs, Ks, n, st["theta_m"], st["theta_m_send"], st["theta_g"], st["momentum"],
                                      st["delta_g"], pg, I_p, t_b, t_g, 2, ghp, out["R"], out["sel"], out["n_sel"],
                                      out["sums"], ws)
    assert rc == 0, B.cocodc_status_string(rc)
    torch.cuda.synchronize()
    checker = FragmentChecker(ref, max(l for _, l, _ in segs))
    scratch = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    sums_ref = np.zeros((Ks, 4))
    covered = 0
    for j, (off, ln, p) in enumerate(segs):
        inputs = {k: synth.original_slice(record, k, off, off + ln, "cuda", scratch) for k in IN_PLACE}
        inputs["theta_m_send"] = st["theta_m_send"][off:off + ln]
        inputs["delta_g"] = st["delta_g"][off:off + ln]
        after = {k: st[k][off:off + ln] for k in IN_PLACE}
        _, sums = checker.check(ln, inputs, after, pg[off:off + ln], 1, t_b[p], t_g, rhp, f"7B strided segment {j}")
        sums_ref[p] += sums
        covered += ln
    assert covered == n
    R_ref = np.sqrt(sums_ref[:, 0]) / np.array(I_p, dtype=np.float64)
    e_R, e_S = _compare_scores(out["R"].cpu().numpy(), out["sums"].cpu().numpy(), R_ref, sums_ref)
    rc, want = ref.select_fragments(R_ref, t_b, t_g, wl.H, 2)
    assert rc == 0
    go = dict(R=out["R"], sel_list=out["sel"][:int(out["n_sel"].item())].cpu().tolist())
    bk = synth.Bookkeeping(t_g=t_g, t_b=t_b, I_p=I_p)
    margin = U.compare_selection(go, dict(R=R_ref, sel=want), bk, wl.H)
    print(f"   all {len(segs)} segments bit-identical to the oracle; scores {e_R:.2e}, sums {e_S:.2e}, margin {margin}; "
          f"selected {go['sel_list']}; wall {time.perf_counter() - t0:.1f} s", flush=True)


def test_7b_bf16_every_element_of_all_fragments(B, ref):
    """The bf16 variant at the width and in the placement bench.py --bf16 times: bf16 local parameters and
    send-time record converted in place in the tuned layout, one fused call over all 32 fragments, then every
    fragment through the oracle's bf16 step; every stored value (bf16 and fp32) bit-identical."""
    t0 = time.perf_counter()
    wl = synth.WORKLOADS["7B"]
    n, K = wl.n_total, wl.K
    arena, bufs, stride = _bench_layout(B, wl)
    print(f"case 7B bf16 full width K={K} n={n} layout=tuned stride={stride / 2**30:.0f} GiB", flush=True)
    record = {}
    st = synth.make_state(wl, "cuda", seed=0, buffers=bufs, record=record)
    for name in ("theta_m", "theta_m_send"):       # each bf16 buffer takes the first half of its fp32 slot
        src = st[name]
        dst = src.view(torch.bfloat16)
        for lo in range(0, n, 1 << 28):
            hi = min(n, lo + (1 << 28))
            dst[lo:hi].copy_(src[lo:hi].to(torch.bfloat16))   # the target lies below its source: safe in ascending order
        st[name] = dst[:n]
    pg = bufs["pg"].view(torch.bfloat16)[:n]
    pg.fill_(555.0)
    bk = synth.bookkeeping(wl)
    ghp, rhp = B.hparams(wl.tau, wl.H, wl.lam, wl.eta, wl.mu), ref.hparams(wl.tau, wl.H, wl.lam, wl.eta, wl.mu)
    i16 = lambda t: t.view(torch.int16)  # noqa: E731
    before = {"theta_m_send": i16(st["theta_m_send"]).sum(dtype=torch.int64).item(), "delta_g": _checksum(st["delta_g"])}
    out = U.gpu_outputs(K)
    ws = B.new_workspace(K, n)
    rc = B.cocodc_sync_step_bf16(wl.frags, n, st["theta_m"], st["theta_m_send"], st["theta_g"], st["momentum"],
                                 st["delta_g"], pg, bk.I_p, bk.t_b, bk.t_g, wl.budget, ghp, out["R"], out["sel"],
                                 out["n_sel"], out["sums"], ws)
    assert rc == 0, B.cocodc_status_string(rc)
    torch.cuda.synchronize()
    assert i16(st["theta_m_send"]).sum(dtype=torch.int64).item() == before["theta_m_send"]
    assert _checksum(st["delta_g"]) == before["delta_g"]
    m = max(wl.frag_lengths)
    h32 = {k: U.pinned(m) for k in ("theta_g", "momentum", "delta_g")}
    h16 = {k: U.pinned(m, torch.int16) for k in ("theta_m", "theta_m_send", "pg")}
    d32 = torch.empty(m, dtype=torch.float32, device="cuda")
    d16 = torch.empty(m, dtype=torch.int16, device="cuda")
    scratch = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    R_ref, sums_ref = np.zeros(K), np.zeros((K, 4))
    from concurrent.futures import ThreadPoolExecutor
    threads = _threads()
    pool = ThreadPoolExecutor(max_workers=threads)
    for p, (off, ln) in enumerate(wl.frags):
        h16["theta_m"][:ln].copy_(i16(synth.original_slice(record, "theta_m", off, off + ln, "cuda", scratch)
                                      .to(torch.bfloat16)))
        h16["theta_m_send"][:ln].copy_(i16(st["theta_m_send"][off:off + ln]))
        for k in ("theta_g", "momentum"):
            h32[k][:ln].copy_(synth.original_slice(record, k, off, off + ln, "cuda", scratch))
        h32["delta_g"][:ln].copy_(st["delta_g"][off:off + ln])
        torch.cuda.synchronize()
        u16 = {k: v[:ln].numpy().view(np.uint16) for k, v in h16.items()}
        f32 = {k: v[:ln].numpy() for k, v in h32.items()}
        # the oracle's bf16 step has no threaded form: the fragment is cut into pieces that run side by side on
        # the same host arrays (element-wise work on disjoint ranges), and the pieces' raw sums are added in order
        cuts = np.linspace(0, ln, threads + 1).astype(np.int64)
        pieces = [(int(a), int(b - a)) for a, b in zip(cuts[:-1], cuts[1:])]

        def piece(fr):
            return ref.sync_step_bf16([fr], u16["theta_m"], u16["theta_m_send"], f32["theta_g"], f32["momentum"],
                                      f32["delta_g"], u16["pg"], [1], [bk.t_b[p]], bk.t_g, 0, rhp)
        outs = list(pool.map(piece, pieces))
        assert all(o["rc"] == 0 for o in outs)
        sums_ref[p] = np.sum([o["sums"][0] for o in outs], axis=0)
        R_ref[p] = np.sqrt(sums_ref[p][0]) / bk.I_p[p] if bk.I_p[p] > 0 else np.inf
        for k, g in (("theta_m", st["theta_m"]), ("pg", pg)):
            d16[:ln].copy_(h16[k][:ln])
            assert torch.equal(i16(g[off:off + ln]), d16[:ln]), (p, k)
        for k in ("theta_g", "momentum"):
            if not U.bits_equal(st[k][off:off + ln], h32[k], d32):
                raise AssertionError((p, k, U.mismatch_report(st[k][off:off + ln], h32[k], d32)))
    pool.shutdown()
    e_R, e_S = _compare_scores(out["R"].cpu().numpy(), out["sums"].cpu().numpy(), R_ref, sums_ref)
    rc, want = ref.select_fragments(R_ref, bk.t_b, bk.t_g, wl.H, wl.budget)
    assert rc == 0
    go = dict(R=out["R"], sel_list=out["sel"][:int(out["n_sel"].item())].cpu().tolist())
    margin = U.compare_selection(go, dict(R=R_ref, sel=want), bk, wl.H, frag_lengths=wl.frag_lengths)
    print(f"   all {K} fragments bit-identical to the oracle's bf16 step; scores {e_R:.2e}, sums {e_S:.2e}, "
          f"margin {margin}; selected {go['sel_list']}; wall {time.perf_counter() - t0:.1f} s", flush=True)


# ------------------------------------------------------------------ config 3: 350M, lambda sweep
def test_350m_lambda_sweep_and_amplified_variant_at_full_width(B, ref):
    t0 = time.perf_counter()
    wl = synth.WORKLOADS["350M"]
    arena, bufs, stride = _bench_layout(B, wl, arena_fraction=0.5)
    checker = FragmentChecker(ref, max(wl.frag_lengths))
    outs = {}
    for amplified in (False, True):
        tau, H = (2, 1) if amplified else (wl.tau, wl.H)
        for lam in wl.lam_sweep:
            print(f"case 350M full width lambda={lam} amplified={amplified} stride={stride / 2**30:.0f} GiB", flush=True)
            record = {}
            st = synth.make_state(wl, "cuda", seed=0, buffers=bufs, record=record, amplified=amplified)
            bk = synth.bookkeeping(wl)
            ghp, rhp = B.hparams(tau, H, lam, wl.eta, wl.mu), ref.hparams(tau, H, lam, wl.eta, wl.mu)
            obs = _one_sync_every_fragment(B, ref, wl, st, record, bufs["pg"], bk, ghp, rhp, checker,
                                           f"350M lambda={lam} amplified={amplified}", H=H)
            print(f"   observed {obs}", flush=True)
            if amplified:
                outs[lam] = st["theta_m"][:1 << 22].clone()
    # the amplified variant is there so that the cubic term of Eq. 7 is visible in fp32 at all,
    # and it is linear in lambda (Eq. 7): theta(1) - theta(0) = 2 (theta(.5) - theta(0)) up to rounding
    d1 = (outs[1.0].double() - outs[0.0].double())
    d5 = (outs[0.5].double() - outs[0.0].double())
    assert d1.abs().max().item() > 1e-2
    assert (d1 - 2 * d5).abs().max().item() <= 4e-7 * max(1.0, outs[1.0].abs().max().item())
    print(f"   wall {time.perf_counter() - t0:.1f} s", flush=True)


# ------------------------------------------------------------------ config 4: 1.3B, 100 consecutive syncs
def _consecutive_syncs(B, ref, wl, n_syncs, score_src, check_at, t0):
    """GPU and oracle evolve their own state in lock-step from the same fresh inputs (drift and new
    global pseudo-gradient of every sync, drawn on the GPU and copied to the host while the oracle
    works on the previous sync).  Selections compared at every sync, all buffers at `check_at`."""
    n, K = wl.n_total, wl.K
    arena, bufs, stride = _bench_layout(B, wl, arena_fraction=0.6)
    print(f"case 1.3B full width {n_syncs} syncs score_src={score_src} K={K} n={n} stride={stride / 2**30:.0f} GiB",
          flush=True)
    st = synth.make_state(wl, "cuda", seed=0, buffers=bufs)
    pg = bufs["pg"]
    ghp = B.hparams(wl.tau, wl.H, wl.lam, wl.eta, wl.mu, score_src=score_src)
    rhp = ref.hparams(wl.tau, wl.H, wl.lam, wl.eta, wl.mu, score_src=score_src)
    threads = _threads()
    # the oracle's own state in ordinary host memory; three pinned buffers rotate between "the global
    # pseudo-gradient the oracle is reading" and "the next sync's inputs being copied out"
    host = {k: torch.empty(n, dtype=torch.float32) for k in NAMES + ("pg",) if k != "delta_g"}
    pin = U.pinned_block(3, n)
    host["delta_g"] = pin[0]
    nxt_host = dict(drift=pin[1], delta_g=pin[2])
    for k in NAMES:
        host[k].copy_(st[k])
    # the next sync's inputs: drawn on the device, copied out on a side stream
    nxt_dev = dict(drift=torch.empty(n, device="cuda"), delta_g=torch.empty(n, device="cuda"))
    side = torch.cuda.Stream()
    copied = torch.cuda.Event()
    cmp = U.DeviceComparer()
    ws = B.new_workspace(K, n)
    out = U.gpu_outputs(K)
    bk = synth.bookkeeping(wl)
    log = U.SelectionLog()
    torch.cuda.synchronize()
    for k in range(n_syncs):
        rc = B.cocodc_sync_step(wl.frags, n, st["theta_m"], st["theta_m_send"], st["theta_g"], st["momentum"],
                                st["delta_g"], pg, bk.I_p, bk.t_b, bk.t_g, wl.budget, ghp, out["R"], out["sel"],
                                out["n_sel"], out["sums"], ws)
        assert rc == 0, B.cocodc_status_string(rc)
        if k + 1 < n_syncs:   # draw sync k+1's inputs and start copying them out
            synth.draw_sync_inputs(wl, "cuda", 0, k + 1, nxt_dev["drift"], nxt_dev["delta_g"])
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                nxt_host["drift"].copy_(nxt_dev["drift"], non_blocking=True)
                nxt_host["delta_g"].copy_(nxt_dev["delta_g"], non_blocking=True)
                copied.record(side)
        hn = {a: b.numpy() for a, b in host.items()}
        ro = ref.sync_step(wl.frags, hn["theta_m"], hn["theta_m_send"], hn["theta_g"], hn["momentum"], hn["delta_g"],
                           hn["pg"], bk.I_p, bk.t_b, bk.t_g, wl.budget, rhp, n_threads=threads)
        assert ro["rc"] == 0
        torch.cuda.synchronize()
        n_sel = int(out["n_sel"].item())
        go = dict(R=out["R"], sel_list=out["sel"][:n_sel].cpu().tolist())
        margin = U.compare_selection(go, ro, bk, wl.H, frag_lengths=wl.frag_lengths, log=log, allow_ambiguous=True)
        e_R, e_S = _compare_scores(out["R"].cpu().numpy(), out["sums"].cpu().numpy(), ro["R"], ro["sums"])
        if k + 1 in check_at:
            for name in IN_PLACE + ("theta_m_send", "delta_g", "pg"):
                dev = pg if name == "pg" else st[name]
                bad = cmp.mismatches(dev, host[name])
                assert bad == 0, (f"sync {k + 1}", name, f"{bad} of {n} stored values differ from the oracle's")
            print(f"   sync {k + 1}: all buffers bit-identical; R {e_R:.2g} sums {e_S:.2g} margin {margin:.3g} "
                  f"sel {go['sel_list']}  t+{time.perf_counter() - t0:.0f} s", flush=True)
        bk = synth.advance_bookkeeping(wl, bk, ro["sel"].tolist())
        if k + 1 < n_syncs:
            # both sides: the previous output becomes the send-time record, the local parameters move by
            # the fresh drift (one fp32 addition each side), the fresh global pseudo-gradient arrives
            st["theta_m_send"].copy_(st["theta_m"])
            st["theta_m"].add_(nxt_dev["drift"])
            st["delta_g"].copy_(nxt_dev["delta_g"])
            copied.synchronize()
            host["theta_m_send"], host["theta_m"] = host["theta_m"], host["theta_m_send"]   # no copy: swap roles
            torch.add(host["theta_m_send"], nxt_host["drift"], out=host["theta_m"])
            host["delta_g"], nxt_host["delta_g"] = nxt_host["delta_g"], host["delta_g"]
    print(f"   score_src={score_src}: {log}", flush=True)
    assert log.compared == n_syncs and log.ambiguous == 0
    return log


def test_1_3b_hundred_consecutive_syncs_at_full_width(B, ref):
    t0 = time.perf_counter()
    wl = synth.WORKLOADS["1.3B"]
    assert wl.n_syncs == 100 and wl.drift == "student_t3"
    _consecutive_syncs(B, ref, wl, wl.n_syncs, 0, (1, 10, 100), t0)
    print(f"   wall {time.perf_counter() - t0:.1f} s", flush=True)


def test_1_3b_ten_syncs_ranked_by_the_heavy_tailed_drift(B, ref):
    """score_src = 1: the ranking is driven by the Student-t drift itself."""
    t0 = time.perf_counter()
    wl = synth.WORKLOADS["1.3B"]
    _consecutive_syncs(B, ref, wl, 10, 1, (1, 10), t0)
    print(f"   wall {time.perf_counter() - t0:.1f} s", flush=True)
