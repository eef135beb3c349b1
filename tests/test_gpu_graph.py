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


def _capture_and_check(call, init, make_extra, replays=4):
    """`call(state, extra)` enqueues one library call.  Captures it on one set of buffers, then checks every
    replay, bit for bit, against the same call issued eagerly on a second set (step k on the state after
    step k-1), with eager work and synchronisations between the replays."""
    work = {k: v.clone() for k, v in init.items()}
    extra = make_extra()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(work, extra)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        call(work, extra)
    ref_state = {k: v.clone() for k, v in init.items()}
    ref_extra = make_extra()
    for k in work:
        work[k].copy_(init[k])
    for k in extra:
        if k != "ws":
            extra[k].copy_(ref_extra[k])
    for replay in range(replays):
        call(ref_state, ref_extra)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in work:
            assert torch.equal(work[k].view(torch.uint8), ref_state[k].view(torch.uint8)), (replay, k)
        for k in extra:
            if k != "ws":
                assert torch.equal(extra[k].view(torch.uint8), ref_extra[k].view(torch.uint8)), (replay, k)
        junk = torch.empty(1 << 20, device="cuda").normal_()
        junk.mul_(2.0)


def test_graph_replays_of_the_16_bit_step_on_many_segments(B):
    """cocodc_sync_step_bf16_segmented with 70 pieces: the tables do not fit the kernel arguments, so the
    captured call also contains the launches that write them to the workspace."""
    import random
    rng = random.Random(3)
    segs, off, K = [], 3, 6
    for j in range(70):
        ln = rng.choice([1, 5, 2047, 2048, 4097, rng.randrange(1, 9000)])
        segs.append((off, ln, rng.choice([0, 1, 2, 4, 5])))
        off += ln + rng.choice([0, 1, 7])
    rng.shuffle(segs)
    n = off + 5
    st = synth.make_state(synth.Workload("g", (n,), tau=5, H=100), "cuda", seed=2)
    init = {k: (v.to(torch.bfloat16) if k in ("theta_m", "theta_m_send") else v) for k, v in st.items()}
    hp = B.hparams(5, 100, pg_format=1)
    I_p, t_b = [3, 1, 9, 2, 0, 5], [990, 999, 100, 950, 996, 980]

    def make_extra():
        e = U.gpu_outputs(K)
        e["pg"] = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
        e["ws"] = B.new_workspace_segmented(len(segs), K, n)
        return e

    def call(s, e):
        B.check(B.cocodc_sync_step_bf16_segmented(segs, K, n, s["theta_m"], s["theta_m_send"], s["theta_g"],
                                                  s["momentum"], s["delta_g"], e["pg"], I_p, t_b, 1000, 3, hp, e["R"],
                                                  e["sel"], e["n_sel"], e["sums"], e["ws"]))
    _capture_and_check(call, init, make_extra)


def test_graph_replays_of_a_loop_event(B):
    """cocodc_sync_event: two fragments arrive, one is in flight, the scores are read and written."""
    wl = synth.MINI_WORKLOADS["125M-mini"]
    n, K = wl.n_total, wl.K
    init = synth.make_state(wl, "cuda", seed=4)
    hp = B.hparams(wl.tau, wl.H)
    mask = [0] * K
    mask[1], mask[K - 1], mask[2] = 1, 1, 2
    I_p, t_b = [7] * K, [1000 - 3 * p for p in range(K)]
    R0 = torch.tensor([float("inf") if p % 4 == 0 else 0.25 * p for p in range(K)], dtype=torch.float64)

    def make_extra():
        e = U.gpu_outputs(K)
        e["R"] = R0.clone().cuda()
        e["pg"] = torch.zeros(n, device="cuda")
        e["ws"] = B.new_workspace(K, n)
        return e

    def call(s, e):
        B.check(B.cocodc_sync_event(wl.frags, n, mask, s["theta_m"], s["theta_m_send"], s["theta_g"], s["momentum"],
                                    s["delta_g"], e["pg"], I_p, t_b, 1000, 2, hp, e["R"], e["sel"], e["n_sel"],
                                    e["sums"], e["ws"]))
    _capture_and_check(call, init, make_extra)
