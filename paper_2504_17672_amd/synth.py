"""Seeded synthetic workloads: fragment layouts, hyper-parameters and input tensors.

This module is the ONE piece shared by the GPU tests, the CPU oracle tests, the smoke check
and the benchmark.  It holds no arithmetic of the method itself: only shapes, value
distributions and step bookkeeping.  It depends on torch alone (never on the HIP library,
never on the oracle).

The inputs stand in for the paper's workload (Sec. 4.1: a 12-layer, ~150M-parameter
Llama-style decoder split into K = 4 shards, H = 100, tau = 5, lambda = 0.5).  The path is
data-oblivious (element-wise arithmetic plus per-fragment sums), so only the fragment sizes
and the value distributions matter; no dataset or trained weights are involved.

Layout rule (all model-shaped workloads): a decoder layer has 4*d*d attention weights,
3*d*ffn SwiGLU weights and two RMSNorm vectors of d; the tied embedding (vocab*d) and the
final norm (d) are attached to fragment 0; fragments are contiguous and in layer order.
"""
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import torch

VOCAB = 32000


@dataclass(frozen=True)
class Workload:
    name: str
    frag_lengths: Tuple[int, ...]
    tau: int
    H: int
    lam: float = 0.5
    eta: float = 0.7
    mu: float = 0.9
    budget: int = 1
    drift: str = "normal"  # "normal" | "student_t3"
    lam_sweep: Tuple[float, ...] = ()
    n_syncs: int = 1
    model: Tuple[int, int, int] = ()  # (n_layers, d, ffn) of model-shaped workloads

    @property
    def K(self) -> int:
        return len(self.frag_lengths)

    @property
    def n_total(self) -> int:
        return sum(self.frag_lengths)

    @property
    def frags(self) -> List[Tuple[int, int]]:
        out, off = [], 0
        for n in self.frag_lengths:
            out.append((off, n))
            off += n
        return out

    @property
    def h(self) -> int:
        """Steps between two sends when every fragment is sent once per H (Eq. 10 with N = K)."""
        return max(1, self.H // self.K)


def layer_params(d: int, ffn: int) -> int:
    return 4 * d * d + 3 * d * ffn + 2 * d


def llama_fragments(n_layers: int, d: int, ffn: int, layers_per_fragment: int) -> Tuple[int, ...]:
    assert n_layers % layers_per_fragment == 0
    k = n_layers // layers_per_fragment
    per = layers_per_fragment * layer_params(d, ffn)
    lens = [per] * k
    lens[0] += VOCAB * d + d
    return tuple(lens)


def _scaled(name, n_layers, d, ffn, lpf, **kw) -> Workload:
    return Workload(name=name, frag_lengths=llama_fragments(n_layers, d, ffn, lpf), model=(n_layers, d, ffn), **kw)


def strided_segments(n_layers: int, d: int, ffn: int, n_shards: int):
    """The strided sharding of the paper's experiments (Sec. 4.1: 12 layers, 4 shards of about 3
    layers each, taken with a stride) on a layer-ordered flat buffer
    [embedding + final norm | layer 0 | layer 1 | ...]: shard k owns layers k, k + n_shards, ...;
    the embedding block goes with shard 0.  Returns [(offset, length, fragment), ...] in buffer
    order and the total number of elements."""
    segs = [(0, VOCAB * d + d, 0)]
    off = VOCAB * d + d
    per = layer_params(d, ffn)
    for layer in range(n_layers):
        segs.append((off, per, layer % n_shards))
        off += per
    return segs, off


WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", (262144,) * 4, tau=5, H=100, budget=1),
    "125M": _scaled("125M", 12, 768, 2048, 1, tau=10, H=100, budget=3),
    "350M": _scaled("350M", 24, 1024, 2816, 3, tau=20, H=200, budget=2,
                    lam_sweep=(0.0, 0.25, 0.5, 1.0)),
    "1.3B": _scaled("1.3B", 24, 2048, 5632, 1, tau=50, H=500, budget=6, drift="student_t3",
                    n_syncs=100),
    "7B": _scaled("7B", 32, 4096, 11008, 1, tau=100, H=1000, budget=4),
}

# Reduced copies with the same fragment structure (K, fragment-0 bulge, hyper-parameters)
# for tests that run the CPU oracle on every element or over many consecutive syncs.
MINI_WORKLOADS: Dict[str, Workload] = {
    "125M-mini": _scaled("125M-mini", 12, 96, 256, 1, tau=10, H=100, budget=3),
    "350M-mini": _scaled("350M-mini", 24, 64, 176, 3, tau=20, H=200, budget=2,
                         lam_sweep=(0.0, 0.25, 0.5, 1.0)),
    "1.3B-mini": _scaled("1.3B-mini", 24, 128, 352, 1, tau=50, H=500, budget=6,
                         drift="student_t3", n_syncs=100),
    "7B-mini": _scaled("7B-mini", 32, 128, 344, 1, tau=100, H=1000, budget=4),
}

_BUFFER_IDS = {"theta_m": 1, "theta_g": 2, "momentum": 3, "delta_g": 4, "drift": 5}
SIGMA = {"theta_m": 0.02, "theta_g": 0.02, "momentum": 0.02, "delta_g": 1e-3, "drift": 1e-4}


def _gen(device, seed: int, buffer: str, sync_index: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + _BUFFER_IDS[buffer]) * 1000003 + int(sync_index))
    return g


def fill_normal(out: torch.Tensor, sigma: float, gen: torch.Generator, chunk: int = 1 << 28, states=None):
    """In-place N(0, sigma) fill, in chunks so no full-size temporary is needed.  `states` (a list,
    optional) receives (first element, number of elements, generator state) of every chunk, from which
    refill_chunk can draw the same chunk again later."""
    flat = out.view(-1)
    for lo in range(0, flat.numel(), chunk):
        sl = flat[lo:lo + chunk]
        if states is not None:
            states.append((lo, sl.numel(), gen.get_state()))
        sl.normal_(0.0, sigma, generator=gen)
    return out


def _student_t3_chunk(sl: torch.Tensor, scale: float, gen: torch.Generator):
    n = sl.numel()
    z = torch.empty(n, dtype=torch.float32, device=sl.device).normal_(generator=gen)
    chi = torch.zeros(n, dtype=torch.float32, device=sl.device)
    tmp = torch.empty(n, dtype=torch.float32, device=sl.device)
    for _ in range(3):
        tmp.normal_(generator=gen)
        chi.addcmul_(tmp, tmp)
    chi.div_(3.0).sqrt_()
    sl.copy_(z.div_(chi).mul_(scale))


def fill_student_t3(out: torch.Tensor, scale: float, gen: torch.Generator, chunk: int = 1 << 26, states=None):
    """In-place Student-t(nu=3) * scale: z / sqrt((a^2 + b^2 + c^2) / 3) from four normals."""
    flat = out.view(-1)
    for lo in range(0, flat.numel(), chunk):
        sl = flat[lo:lo + chunk]
        if states is not None:
            states.append((lo, sl.numel(), gen.get_state()))
        _student_t3_chunk(sl, scale, gen)
    return out


def refill_chunk(out: torch.Tensor, kind: str, sigma: float, state) -> torch.Tensor:
    """Draws one recorded chunk again (same generator state, same number of elements, hence the same
    values) into `out`, a tensor of exactly that chunk's length.  kind: "normal" | "student_t3"."""
    gen = torch.Generator(device=out.device)
    gen.set_state(state)
    if kind == "normal":
        out.normal_(0.0, sigma, generator=gen)
    elif kind == "student_t3":
        _student_t3_chunk(out, sigma, gen)
    else:
        raise ValueError(kind)
    return out


def fill_drift(out: torch.Tensor, kind: str, gen: torch.Generator, sigma: float = SIGMA["drift"], states=None):
    if kind == "normal":
        return fill_normal(out, sigma, gen, states=states)
    if kind == "student_t3":
        return fill_student_t3(out, sigma, gen, states=states)
    raise ValueError(kind)


def make_state(wl: Workload, device, seed: int = 0, pad: int = 0, amplified: bool = False, buffers=None,
               record=None):
    """The five resident buffers of one worker just before a sync is applied.

    theta_m_send is derived so that "drift since send" = theta_m - theta_m_send:
    theta_m_send = fp32(theta_m - drift).  With amplified=True every buffer is drawn from
    N(0, 0.5), which makes the cubic term of Eq. 7 large enough to survive fp32 rounding
    (meant to be used with small tau and H).  `pad` extra elements are allocated (and filled
    with a sentinel) after the last fragment so tests can verify nothing outside the
    fragment table is written.  `buffers` (optional) maps each of the five names to a
    preallocated fp32 tensor of n_total + pad elements to fill instead of allocating.
    `record` (a dict, optional) receives, per buffer that the sync step overwrites ("theta_m",
    "theta_g", "momentum"), the (kind, sigma, chunk states) from which original_slice can draw any
    part of that buffer's initial contents again.
    """
    n = wl.n_total

    def alloc(name):
        if buffers is not None:
            t = buffers[name]
            assert t.dtype == torch.float32 and t.numel() == n + pad
            return t
        return torch.empty(n + pad, dtype=torch.float32, device=device)

    st = {}
    for name in ("theta_m", "theta_g", "momentum", "delta_g"):
        t = alloc(name)
        sigma = 0.5 if amplified else SIGMA[name]
        states = [] if record is not None else None
        fill_normal(t[:n], sigma, _gen(device, seed, name, 0), states=states)
        if record is not None:
            record[name] = ("normal", sigma, states)
        if pad:
            t[n:] = 777.0
        st[name] = t
    send = alloc("theta_m_send")
    g = _gen(device, seed, "drift", 0)
    if amplified:
        fill_normal(send[:n], 0.5, g)
    else:
        fill_drift(send[:n], wl.drift, g)
    torch.sub(st["theta_m"][:n], send[:n], out=send[:n])
    if pad:
        send[n:] = 777.0
    st["theta_m_send"] = send
    return st


def original_slice(record, name: str, lo: int, hi: int, device, scratch=None) -> torch.Tensor:
    """Elements [lo, hi) of buffer `name` as make_state(record=...) first filled it, drawn again chunk
    by chunk (for checks at sizes where no copy of the initial state can be kept)."""
    kind, sigma, states = record[name]
    out = torch.empty(hi - lo, dtype=torch.float32, device=device)
    for c_lo, c_n, state in states:
        a, b = max(lo, c_lo), min(hi, c_lo + c_n)
        if a >= b:
            continue
        tmp = scratch[:c_n] if scratch is not None and scratch.numel() >= c_n else \
            torch.empty(c_n, dtype=torch.float32, device=device)
        refill_chunk(tmp, kind, sigma, state)
        out[a - lo:b - lo].copy_(tmp[a - c_lo:b - c_lo])
    return out


def draw_sync_inputs(wl: Workload, device, seed: int, sync_index: int, drift_out: torch.Tensor,
                     delta_g_out: torch.Tensor):
    """The fresh inputs of sync `sync_index` >= 1 of a consecutive-sync run, into caller-provided
    buffers: the local drift since the previous sync and the newly arrived global pseudo-gradient
    (the same values next_sync_inputs draws)."""
    n = wl.n_total
    fill_drift(drift_out[:n], wl.drift, _gen(device, seed, "drift", sync_index))
    fill_normal(delta_g_out[:n], SIGMA["delta_g"], _gen(device, seed, "delta_g", sync_index))


def next_sync_inputs(wl: Workload, st, seed: int, sync_index: int):
    """Advance a state to the next sync of a consecutive-sync run (sync_index >= 1):
    the previous output becomes the send-time record, the local parameters move by a fresh
    drift, and a fresh delayed global pseudo-gradient arrives."""
    n = wl.n_total
    st["theta_m_send"][:n].copy_(st["theta_m"][:n])
    drift = torch.empty(n, dtype=torch.float32, device=st["theta_m"].device)
    fill_drift(drift, wl.drift, _gen(st["theta_m"].device, seed, "drift", sync_index))
    st["theta_m"][:n].add_(drift)
    del drift
    fill_normal(st["delta_g"][:n], SIGMA["delta_g"],
                _gen(st["theta_m"].device, seed, "delta_g", sync_index))
    return st


@dataclass
class Bookkeeping:
    """Per-fragment step counters of the adaptive-transmission schedule (Sec. 3.2)."""
    t_g: int
    t_b: List[int] = field(default_factory=list)
    I_p: List[int] = field(default_factory=list)


def bookkeeping(wl: Workload, variant: str = "regular") -> Bookkeeping:
    """regular: I_p = h*(1 + p mod 3), nobody overdue.
    mixed: additionally the last fragment is overdue (t_g - t_b = H) and fragment 1 has
    never completed a sync (I_p = 0)."""
    t_g = 10 * wl.H
    I_p = [wl.h * (1 + p % 3) for p in range(wl.K)]
    t_b = [t_g - i for i in I_p]
    if variant == "mixed":
        t_b[wl.K - 1] = t_g - wl.H
        if wl.K > 1:
            I_p[1] = 0
    elif variant != "regular":
        raise ValueError(variant)
    return Bookkeeping(t_g=t_g, t_b=t_b, I_p=I_p)


def advance_bookkeeping(wl: Workload, bk: Bookkeeping, selected) -> Bookkeeping:
    """One scheduling interval later: the selected fragments complete a sync now."""
    t_g = bk.t_g + wl.h
    t_b, I_p = list(bk.t_b), list(bk.I_p)
    for p in selected:
        p = int(p)
        I_p[p] = t_g - t_b[p]
        t_b[p] = t_g
    return Bookkeeping(t_g=t_g, t_b=t_b, I_p=I_p)
