"""Where the flat buffers are put in the device memory (no paper counterpart; advisory: every entry point
of the library accepts any placement).  On MI355X the fused step runs up to 18 % faster when the buffers it
writes do not all lie within the same 96 GiB third of the device memory (the single steps likewise: written
buffers in different thirds, buffers that are only read together), and a few percent faster still when the
buffers are spread over all three.  Which physical memory an allocation gets cannot be asked for, so
the helpers here place by measurement: they time a few launches of the fused step on candidate placements at
set-up and keep the fastest.  They use torch for the allocations and the timing events, nothing else."""
from .binding import (check, cocodc_layout_stride_bytes, cocodc_sync_step, hparams, new_workspace)


def spaced_buffers(n_total, count, device="cuda", stride_bytes=None):
    """`count` flat fp32 buffers of n_total elements carved out of one device allocation, their
    bases cocodc_layout_stride_bytes(n_total) apart (less if the free device memory does not
    allow it).  Returns (arena, [buffers]); keep the arena alive as long as the buffers are
    used.  Memory between the buffers is free for other data."""
    import torch
    nbytes = 4 * int(n_total)
    if stride_bytes is None:
        GiB = 1 << 30
        free, _ = torch.cuda.mem_get_info(device)
        fit = (int(free * 0.92) - nbytes) // (count - 1) // GiB * GiB
        stride = max(min(cocodc_layout_stride_bytes(n_total), fit), (nbytes + 255) // 256 * 256)
    else:
        stride = int(stride_bytes)
    assert stride % 16 == 0 and stride >= nbytes
    arena = torch.empty((count - 1) * stride + nbytes, dtype=torch.uint8, device=device)
    return arena, [arena[k * stride:k * stride + nbytes].view(torch.float32) for k in range(count)]


class _FusedStepTimer:
    """Times a few launches of the fused step (or of step(buffers)) on candidate buffers: the
    measurement behind the layout helpers below."""

    def __init__(self, n_total, frags, device, step=None):
        import torch
        self.torch, self.n, self.frags, self.step = torch, int(n_total), frags, step
        K = len(frags)
        self.ws = new_workspace(K, n_total, device)
        self.R = torch.zeros(K, dtype=torch.float64, device=device)
        self.sel = torch.zeros(K, dtype=torch.int32, device=device)
        self.n_sel = torch.zeros(1, dtype=torch.int32, device=device)
        self.hp = hparams(5, 100)
        self.ones = [1] * K
        self.start, self.stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def ms(self, b):
        """Best of three launches after one warm-up, in milliseconds."""
        best = float("inf")
        for it in range(4):
            self.start.record()
            if self.step is not None:
                self.step(b)
            else:
                check(cocodc_sync_step(self.frags, self.n, b[0], b[1], b[2], b[3], b[4], b[5] if len(b) > 5 else None,
                                       self.ones, self.ones, 2, 1, self.hp, self.R, self.sel, self.n_sel, None, self.ws))
            self.stop.record()
            self.torch.cuda.synchronize()
            if it:
                best = min(best, self.start.elapsed_time(self.stop))
        return best


def compact_fast_buffers(n_total, frags, device="cuda", count=6, ballast_gib=(0, 16, 48, 88, 128, 176, 208),
                         good_gbps=6200.0, bytes_per_param=36, verbose=None, step=None):
    """`count` flat fp32 buffers of n_total elements back to back in one allocation of their own
    size, placed by trial: the fused step runs 15 % faster when its buffers do not all lie in the
    same third of the device memory, and which physical memory an allocation gets depends on what
    else is allocated at that moment (the driver composes it from power-of-two blocks).  So the
    allocation is made after a temporary ballast allocation of each size in `ballast_gib` in turn,
    timed with a few launches of the fused step (or of step(buffers)) on zero-filled memory, and
    the first one that reaches good_gbps (algorithmic bytes_per_param * n_total / time) is kept,
    else the best seen; the ballast is freed again, so the footprint is the buffers alone.
    Returns (arena, [buffers], {ballast_GiB: GB/s})."""
    import torch
    GiB = 1 << 30
    nbytes = (4 * int(n_total) + 255) // 256 * 256
    timer = _FusedStepTimer(n_total, frags, device, step)
    seen, kept = {}, None

    def carve(arena):
        return [arena[k * nbytes:k * nbytes + 4 * int(n_total)].view(torch.float32) for k in range(count)]
    for gib in ballast_gib:
        free, _ = torch.cuda.mem_get_info(device)
        if gib * GiB + count * nbytes > int(free * 0.97):
            continue
        ballast = torch.empty(gib * GiB, dtype=torch.uint8, device=device) if gib else None
        arena = torch.empty(count * nbytes, dtype=torch.uint8, device=device)
        for off in range(0, arena.numel(), 8 * GiB):
            arena[off:off + 8 * GiB].zero_()
        gbps = bytes_per_param * int(n_total) / (timer.ms(carve(arena)) * 1e-3) / 1e9
        seen[gib] = round(gbps, 0)
        if verbose:
            verbose(f"ballast {gib} GiB: {gbps:.0f} GB/s")
        better = kept is None or gbps > kept[0]
        if better:
            old, kept = kept, (gbps, arena)
            del old
        else:
            del arena
        del ballast
        torch.cuda.empty_cache()   # the ballast (and a rejected candidate) go back to the driver
        if gbps >= good_gbps:
            break
    assert kept is not None, "not enough free device memory for the buffers"
    return kept[1], carve(kept[1]), seen


def tuned_spaced_buffers(n_total, frags, device="cuda", count=6, max_arena_bytes=None, verbose=None, step=None):
    """Like spaced_buffers, but picks the stride by measurement: the best of the candidate
    strides that fit into one allocation of at most max_arena_bytes (default: 92 % of the free
    device memory), each timed with a few launches of the fused step on zero-filled memory.
    Which strides are fastest depends on where the allocation lands (a placement is fast when
    the buffers do not all lie within the same 96 GiB third of the device memory, and a few
    percent faster still when they are spread over all three), so this is done once per
    allocation, at set-up.  A caller whose hot call is not the fused step passes step(buffers),
    a function that enqueues that call (or sequence of calls) on the `count` candidate buffers;
    it is timed instead (the single steps prefer other strides than the fused step does).
    Returns (arena, [buffers], stride_bytes, {stride_GiB: ms})."""
    import torch
    GiB = 1 << 30
    nbytes = 4 * int(n_total)
    if max_arena_bytes is None:
        free, _ = torch.cuda.mem_get_info(device)
        max_arena_bytes = int(free * 0.92)
    back_to_back = (nbytes + GiB - 1) // GiB * GiB   # the smallest stride on the 1 GiB grid
    lo = max(13 * GiB, back_to_back)
    hi = (max_arena_bytes - nbytes) // (count - 1) // GiB * GiB
    base = cocodc_layout_stride_bytes(n_total)
    if hi < lo:
        arena, bufs = spaced_buffers(n_total, count, device)
        return arena, bufs, base, {}
    # every 2 GiB from 13 GiB on (where the fast placements start), and below that every 1 GiB from
    # back-to-back on, so that the probe also tells how small an arena still runs fast
    cands = sorted(set(range(lo, hi + 1, 2 * GiB)) | set(range(back_to_back, lo, GiB)) |
                   ({base} if lo <= base <= hi else set()))
    arena = torch.empty((count - 1) * cands[-1] + nbytes, dtype=torch.uint8, device=device)
    for off in range(0, arena.numel(), 8 * GiB):
        arena[off:off + 8 * GiB].zero_()
    timer = _FusedStepTimer(n_total, frags, device, step)
    timings = {}
    for stride in cands:
        b = [arena[k * stride:k * stride + nbytes].view(torch.float32) for k in range(count)]
        best = timer.ms(b)
        timings[stride / GiB] = best
        if verbose:
            verbose(f"stride {stride / GiB:.0f} GiB: {best:.3f} ms")
    stride = int(min(timings, key=timings.get) * GiB)
    bufs = [arena[k * stride:k * stride + nbytes].view(torch.float32) for k in range(count)]
    return arena, bufs, stride, timings


# Region (third of the device memory) of theta_m, theta_m_send, theta_g, momentum, delta_g and the
# pseudo-gradient buffer that served every entry point well in the enumeration of all assignments
# (bench.py --region-probe): the written buffers are not all in one region, the buffers that the
# send step reads (theta_g, theta_m) share one and the ones it writes lie elsewhere.
DEFAULT_REGIONS = (0, 0, 0, 1, 1, 2)
REGION_BYTES = 96 << 30


def region_buffers(n_total, regions=DEFAULT_REGIONS, device="cuda", arena_fraction=0.95):
    """len(regions) flat fp32 buffers of n_total elements, buffer i inside the regions[i]-th third
    (96 GiB) of the device memory: one allocation of arena_fraction of the free memory is made and
    the buffers are carved out of it at offsets that fall into the wanted thirds IF the allocation
    maps onto the device memory from its bottom upwards in one piece.  That held for an allocation
    of 95 % of the memory made first in a fresh process (the speed steps of bench.py
    --placement-probe sit at the same offsets in every run), and nothing guarantees it: treat the
    result as a candidate placement and time it.  The rest of the allocation is free for the
    caller's other data.  Returns (arena, [buffers], [offsets in bytes])."""
    import torch
    GiB = 1 << 30
    nbytes = (4 * int(n_total) + 255) // 256 * 256
    free, total = torch.cuda.mem_get_info(device)
    start = total - free                           # where the allocation begins if memory is handed out bottom-up
    arena_bytes = int(free * arena_fraction) // GiB * GiB
    slot = (nbytes + GiB - 1) // GiB * GiB + GiB   # buffers of one region lie a whole GiB apart
    offsets, used = [], {}
    for r in regions:
        k = used.get(r, 0)
        used[r] = k + 1
        lo = max(r * REGION_BYTES - start, 0) + 2 * GiB   # 2 GiB clear of the region's lower end
        off = (lo + k * slot) // 256 * 256
        if off + nbytes > min((r + 1) * REGION_BYTES - start, arena_bytes):
            raise ValueError(f"region {r} cannot hold {used[r]} buffers of {nbytes / GiB:.1f} GiB")
        offsets.append(off)
    arena = torch.empty(arena_bytes, dtype=torch.uint8, device=device)
    bufs = [arena[o:o + 4 * int(n_total)].view(torch.float32) for o in offsets]
    return arena, bufs, offsets
