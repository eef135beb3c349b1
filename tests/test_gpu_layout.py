"""The buffer placement helpers (paper_2504_17672_amd/layout.py) hand out buffers that do not overlap, lie
where they say, and work as arguments of the fused step (checked against the oracle).  Needs an MI355X."""
import numpy as np
import pytest
import torch

from paper_2504_17672_amd import layout as L
from paper_2504_17672_amd import synth

import parity_util as U

pytestmark = pytest.mark.gpu
NAMES = ("theta_m", "theta_m_send", "theta_g", "momentum", "delta_g", "pg")


@pytest.fixture(scope="module")
def B():
    from paper_2504_17672_amd import binding
    assert torch.cuda.is_available()
    return binding


def _disjoint_inside(arena, bufs, n):
    lo, hi = arena.data_ptr(), arena.data_ptr() + arena.numel()
    spans = sorted((b.data_ptr(), b.data_ptr() + 4 * n) for b in bufs)
    assert all(b.numel() == n and b.dtype == torch.float32 and b.data_ptr() % 256 == 0 for b in bufs)
    assert spans[0][0] >= lo and spans[-1][1] <= hi
    assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))


def _step_matches_oracle(B, ref, wl, bufs):
    st = synth.make_state(wl, "cuda", seed=3, buffers=dict(zip(NAMES, bufs)))
    host = U.host_copy(st)
    bk = synth.bookkeeping(wl, "mixed")
    out = U.gpu_outputs(wl.K)
    ws = B.new_workspace(wl.K, wl.n_total)
    pg = bufs[5]
    B.check(B.cocodc_sync_step(wl.frags, wl.n_total, st["theta_m"], st["theta_m_send"], st["theta_g"], st["momentum"],
                               st["delta_g"], pg, bk.I_p, bk.t_b, bk.t_g, wl.budget, B.hparams(wl.tau, wl.H), out["R"],
                               out["sel"], out["n_sel"], out["sums"], ws))
    torch.cuda.synchronize()
    h_pg = np.zeros(wl.n_total, np.float32)
    ro = ref.sync_step(wl.frags, host["theta_m"], host["theta_m_send"], host["theta_g"], host["momentum"],
                       host["delta_g"], h_pg, bk.I_p, bk.t_b, bk.t_g, wl.budget, ref.hparams(wl.tau, wl.H))
    assert ro["rc"] == 0
    for k in ("theta_m", "theta_g", "momentum"):
        assert np.array_equal(st[k].cpu().numpy(), host[k]), k
    assert np.array_equal(pg.cpu().numpy(), h_pg)
    assert out["sel"][:int(out["n_sel"].item())].cpu().tolist() == ro["sel"].tolist()


def test_region_buffers(B, ref):
    wl = synth.MINI_WORKLOADS["125M-mini"]
    n, GiB = wl.n_total, 1 << 30
    torch.cuda.empty_cache()
    free, total = torch.cuda.mem_get_info()
    print(f"case region_buffers n={n} free {free / GiB:.1f} of {total / GiB:.1f} GiB", flush=True)
    arena, bufs, offs = L.region_buffers(n, (0, 0, 0, 1, 1, 2), "cuda", arena_fraction=0.9)
    try:
        _disjoint_inside(arena, bufs, n)
        assert [b.data_ptr() - arena.data_ptr() for b in bufs] == offs
        start = total - free
        for r, o in zip((0, 0, 0, 1, 1, 2), offs):       # where a bottom-up mapping would put them
            assert r * (96 << 30) <= o + start and o + start + 4 * n <= (r + 1) * (96 << 30)
        _step_matches_oracle(B, ref, wl, bufs)
        with pytest.raises(ValueError):
            L.region_buffers(30 << 30, (0, 0, 0, 0, 1, 2), "cuda")   # four 120 GiB buffers do not fit one third
    finally:
        del bufs, arena
        torch.cuda.empty_cache()


def test_compact_fast_buffers_and_spaced_buffers(B, ref):
    wl = synth.MINI_WORKLOADS["125M-mini"]
    n = wl.n_total
    print(f"case compact_fast_buffers n={n}", flush=True)
    arena, bufs, seen = L.compact_fast_buffers(n, wl.frags, "cuda", ballast_gib=(0, 1), good_gbps=1e9)
    try:
        assert set(seen) == {0, 1} and all(v > 0 for v in seen.values())
        assert arena.numel() == 6 * ((4 * n + 255) // 256 * 256)     # the footprint is the buffers alone
        _disjoint_inside(arena, bufs, n)
        _step_matches_oracle(B, ref, wl, bufs)
    finally:
        del bufs, arena
        torch.cuda.empty_cache()
    arena, bufs = L.spaced_buffers(n, 6, "cuda", stride_bytes=1 << 30)
    try:
        _disjoint_inside(arena, bufs, n)
        assert bufs[1].data_ptr() - bufs[0].data_ptr() == 1 << 30
        _step_matches_oracle(B, ref, wl, bufs)
    finally:
        del bufs, arena
        torch.cuda.empty_cache()
