"""The fused step records into a HIP graph (no memcpy, memset or synchronisation is issued by
the call) and every replay gives the eager result.  Replays are interleaved with eager work and
synchronisations, and each one is checked.  Needs an MI355X."""
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


@pytest.mark.parametrize("name", ["tiny", "125M-mini"])
def test_graph_replays_match_eager(B, name):
    wl = synth.WORKLOADS.get(name) or synth.MINI_WORKLOADS[name]
    n, K = wl.n_total, wl.K
    bk = synth.bookkeeping(wl, "mixed")
    hp = B.hparams(wl.tau, wl.H)
    init = synth.make_state(wl, "cuda", seed=0)
    work = {k: v.clone() for k, v in init.items()}     # buffers the graph is bound to
    pg = torch.zeros(n, device="cuda")
    out = U.gpu_outputs(K)
    ws = B.new_workspace(K, n)

    def call(st, pg_, o, w):
        B.check(B.cocodc_sync_step(wl.frags, n, st["theta_m"], st["theta_m_send"], st["theta_g"], st["momentum"],
                                   st["delta_g"], pg_, bk.I_p, bk.t_b, bk.t_g, wl.budget, hp, o["R"], o["sel"],
                                   o["n_sel"], o["sums"], w))

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(work, pg, out, ws)                        # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        call(work, pg, out, ws)

    # eager reference chain on separate buffers: step k applied to the state after step k-1
    ref_state = {k: v.clone() for k, v in init.items()}
    ref_pg = torch.zeros(n, device="cuda")
    ref_out = U.gpu_outputs(K)
    ref_ws = B.new_workspace(K, n)
    for k in work:
        work[k].copy_(init[k])
    for replay in range(4):
        call(ref_state, ref_pg, ref_out, ref_ws)       # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in work:
            assert torch.equal(work[k], ref_state[k]), (replay, k)
        assert torch.equal(pg, ref_pg)
        assert torch.equal(out["R"], ref_out["R"]) and torch.equal(out["sums"], ref_out["sums"])
        assert torch.equal(out["sel"], ref_out["sel"]) and torch.equal(out["n_sel"], ref_out["n_sel"])
        junk = torch.empty(1 << 20, device="cuda").normal_()  # unrelated eager kernels
        junk.mul_(2.0)
