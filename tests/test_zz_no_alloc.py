"""cocodc_sync_step_noalloc (the fused step with its scratch in a fixed array inside the library)
against cocodc_sync_step with a caller-provided workspace: every output bit for bit, on two calls
in a row, the second on a smaller input (so the array still holds the first call's table and
partial sums), then a third that is larger again.  Runs last in the suite and also alone."""
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


def _both(B, wl, seed, variant, hp, budget):
    """One step through each entry point from identical inputs; returns the two result sets."""
    bk = synth.bookkeeping(wl, variant)
    n, K = wl.n_total, wl.K
    res = []
    for which in ("workspace", "noalloc"):
        st = synth.make_state(wl, "cuda", seed=seed)
        out = U.gpu_outputs(K)
        pg = torch.full((n,), 555.0, device="cuda")
        if which == "workspace":
            ws = B.new_workspace(K, n)
            rc = B.cocodc_sync_step(wl.frags, n, st["theta_m"], st["theta_m_send"], st["theta_g"], st["momentum"],
                                    st["delta_g"], pg, bk.I_p, bk.t_b, bk.t_g, budget, hp, out["R"], out["sel"],
                                    out["n_sel"], out["sums"], ws)
        else:
            rc = B.cocodc_sync_step_noalloc(wl.frags, n, st["theta_m"], st["theta_m_send"], st["theta_g"],
                                            st["momentum"], st["delta_g"], pg, bk.I_p, bk.t_b, bk.t_g, budget, hp,
                                            out["R"], out["sel"], out["n_sel"], out["sums"])
        assert rc == 0, (which, B.cocodc_status_string(rc))
        torch.cuda.synchronize()
        res.append((st, out, pg))
    return res


def _assert_identical(a, b):
    (sa, oa, pa), (sb, ob, pb) = a, b
    for k in ("theta_m", "theta_m_send", "theta_g", "momentum", "delta_g"):
        assert torch.equal(sa[k].view(torch.int32), sb[k].view(torch.int32)), k
    assert torch.equal(pa.view(torch.int32), pb.view(torch.int32))
    assert torch.equal(oa["R"].view(torch.int64), ob["R"].view(torch.int64))
    assert torch.equal(oa["sums"].view(torch.int64), ob["sums"].view(torch.int64))
    assert torch.equal(oa["sel"], ob["sel"]) and torch.equal(oa["n_sel"], ob["n_sel"])


def test_noalloc_equals_workspace_entry_point_on_consecutive_calls(B):
    big = synth.Workload("noalloc-big", (1 << 24, 70001, 3, 5000000), tau=5, H=100, budget=2)   # 4096-element tiles
    small = synth.Workload("noalloc-small", (50001, 16384, 0, 7), tau=2, H=1, budget=3)        # 2048-element tiles
    hp_a, hp_b = B.hparams(5, 100), B.hparams(2, 1, lam=3.0, score_src=1, norm_kind=1)
    for i, (wl, hp, variant) in enumerate(((big, hp_a, "regular"), (small, hp_b, "mixed"), (big, hp_a, "mixed"))):
        print(f"case noalloc call {i + 1}: {wl.name} K={wl.K} n={wl.n_total} variant={variant}", flush=True)
        a, b = _both(B, wl, seed=20 + i, variant=variant, hp=hp, budget=wl.budget)
        _assert_identical(a, b)
        assert int(b[1]["n_sel"].item()) == min(wl.budget, wl.K)


def test_noalloc_rejects_what_does_not_fit(B):
    """A call whose table and partial sums would not fit the fixed array is refused before any
    launch (the pointers are never dereferenced)."""
    n = 1 << 34   # 17e9 elements: 4 Mi tiles of 32 bytes = 128 MiB of partial sums
    assert B.cocodc_workspace_bytes(1, n) > B.COCODC_NOALLOC_SCRATCH_BYTES
    fake = 0x10000000
    rc = B.cocodc_sync_step_noalloc([(0, n)], n, fake, fake + (1 << 40), fake + (2 << 40), fake + (3 << 40),
                                    fake + (4 << 40), None, [1], [0], 10, 1, B.hparams(5, 100), fake + (5 << 40),
                                    fake + (5 << 40) + 4096, fake + (5 << 40) + 8192, None, stream=0)
    assert rc == B.COCODC_ERR_WORKSPACE
    assert B.cocodc_sync_step_noalloc([(0, 16)], 16, None, None, None, None, None, None, [1], [0], 10, 1,
                                      B.hparams(5, 100), None, None, None, None, stream=0) == B.COCODC_ERR_NULL


@pytest.mark.parametrize("K", [4, 40])
def test_noalloc_records_into_a_graph(B, K):
    """The callers this entry point is for: a step recorded into a HIP graph (the first call on the
    GPU, which looks the array's address up, is made before the capture) and replayed between eager work;
    every replay must give what the eager cocodc_sync_step chain gives.  K = 40 takes the path that writes
    the table into the array with small upload kernels, K = 4 the one that passes it in the kernel arguments."""
    wl = synth.Workload(f"noalloc-graph-{K}", tuple(30000 + 777 * (p % 5) for p in range(K)), tau=5, H=100, budget=3)
    n = wl.n_total
    bk = synth.bookkeeping(wl, "mixed")
    hp = B.hparams(wl.tau, wl.H)
    init = synth.make_state(wl, "cuda", seed=31)
    work = {k: v.clone() for k, v in init.items()}
    pg = torch.zeros(n, device="cuda")
    out = U.gpu_outputs(K)

    def call_noalloc():
        B.check(B.cocodc_sync_step_noalloc(wl.frags, n, work["theta_m"], work["theta_m_send"], work["theta_g"],
                                           work["momentum"], work["delta_g"], pg, bk.I_p, bk.t_b, bk.t_g, wl.budget, hp,
                                           out["R"], out["sel"], out["n_sel"], out["sums"]))
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call_noalloc()                                  # outside the capture: address look-up, warm-up
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        call_noalloc()
    ref_state = {k: v.clone() for k, v in init.items()}
    ref_pg = torch.zeros(n, device="cuda")
    ref_out = U.gpu_outputs(K)
    ref_ws = B.new_workspace(K, n)
    for k in work:
        work[k].copy_(init[k])
    print(f"case noalloc graph K={K} n={n}", flush=True)
    for replay in range(4):
        B.check(B.cocodc_sync_step(wl.frags, n, ref_state["theta_m"], ref_state["theta_m_send"], ref_state["theta_g"],
                                   ref_state["momentum"], ref_state["delta_g"], ref_pg, bk.I_p, bk.t_b, bk.t_g,
                                   wl.budget, hp, ref_out["R"], ref_out["sel"], ref_out["n_sel"], ref_out["sums"], ref_ws))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in work:
            assert torch.equal(work[k], ref_state[k]), (replay, k)
        assert torch.equal(pg, ref_pg)
        assert torch.equal(out["R"], ref_out["R"]) and torch.equal(out["sums"], ref_out["sums"])
        assert torch.equal(out["sel"], ref_out["sel"]) and torch.equal(out["n_sel"], ref_out["n_sel"])
        torch.empty(1 << 20, device="cuda").normal_().mul_(2.0)   # unrelated eager kernels between the replays
