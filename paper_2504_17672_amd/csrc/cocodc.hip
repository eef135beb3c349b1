// cocodc.hip -- gfx950 (MI355X) C ABI of the CoCoDC outer-synchronisation path: the one
// translation unit of the library.  cocodc_device.h holds the device code, cocodc_host.h the
// validation, tile planning and launch helpers, cocodc_loop.h the Sec. 3.2 loop; this file holds
// the build switches and the entry points declared in cocodc.h.
//
// One streaming pass per call.  Every kernel walks the same list of TILES: a tile is the
// part of one segment of a fragment that falls into one aligned window of 2^tile_shift elements
// of the flat buffers, so a tile never straddles two fragments and, inside a tile, element
// indices that are multiples of 4 are 16-byte aligned whenever the buffer bases are.  A
// workgroup of 256 threads (4 wavefronts of 64) loads its whole tile with 128-bit accesses
// (COCODC_DEPTH per stream and lane in flight), computes in fp64 registers with one rounding
// per stored value, stores and ends.  Per-fragment sums (paper Eq. 11) are produced as one fp64
// partial per tile (lane -> wavefront shuffle -> LDS -> tile slot) and combined by a second
// kernel in a fixed order, so scores are bit-reproducible and independent of the launch shape.
//
// No MFMA: nothing on this path is a contraction; the bound is HBM bandwidth
// (20 B read + 16 B written per parameter in the fused step).
//
// Compile with -ffp-contract=off: no multiply-add may be contracted, so that the fused kernel,
// the single-step kernels and a plain fp64 evaluation of the same expressions round identically.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <mutex>
#include <vector>

#include "cocodc.h"

// Build switches.  The defaults are the fastest measured; the others exist so that the
// alternatives can be built and timed again (-DNAME=value on the hipcc line).
//   COCODC_TILE          elements per tile of large buffers (power of two >= 1024)
//   COCODC_THREADS       threads per workgroup of the streaming kernels
//   COCODC_DEPTH         128-bit accesses per stream and lane in flight
//                        (TILE == THREADS * 4 * DEPTH: a workgroup handles its tile in one step)
//   COCODC_NT_LOAD/STORE nontemporal loads / stores (1) or plain ones (0)
//   COCODC_EXACT_DIV     fp64 division as the oracle does it (1: bit-identical results) or a
//                        multiplication by a precomputed reciprocal (0: last-bit differences)
//   COCODC_WAVES_PER_EU  occupancy hint for the streaming kernels (0: none)
#ifndef COCODC_TILE
#define COCODC_TILE 4096
#endif
#ifndef COCODC_THREADS
#define COCODC_THREADS 256
#endif
#ifndef COCODC_DEPTH
#define COCODC_DEPTH 4
#endif
#ifndef COCODC_NT_LOAD
#define COCODC_NT_LOAD 1
#endif
#ifndef COCODC_EXACT_DIV
#define COCODC_EXACT_DIV 1
#endif
#ifndef COCODC_WAVES_PER_EU
#define COCODC_WAVES_PER_EU 0
#endif
#ifndef COCODC_NT_STORE
#define COCODC_NT_STORE 1
#endif
#include "cocodc_device.h"
#include "cocodc_host.h"

// ====================================================================== C ABI
extern "C" {

size_t cocodc_workspace_bytes_segmented(int32_t S, int32_t K, uint64_t n_total) {
  if (K < 1 || K > COCODC_MAX_FRAGMENTS || S < 0 || S > COCODC_MAX_SEGMENTS) return 0;
  return workspace_bytes(S, K, n_total);
}

size_t cocodc_workspace_bytes(int32_t K, uint64_t n_total) {
  if (K < 1 || K > COCODC_MAX_FRAGMENTS) return 0;
  return workspace_bytes(K, K, n_total);
}

int cocodc_pseudograd(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total,
                      const float* theta_g_snap, const float* theta_m, float* delta_m_out,
                      float* theta_m_send_out, void* workspace, size_t workspace_bytes_, void* stream) {
  if (!theta_g_snap || !theta_m || !delta_m_out) return COCODC_ERR_NULL;
  if (!all_aligned4({theta_g_snap, theta_m, delta_m_out, theta_m_send_out})) return COCODC_ERR_ALIGN;
  Plan pl;
  if (int rc = plan_table(frags, K, n_total, nullptr, nullptr, &pl)) return rc;
  if (int rc = check_workspace(workspace, workspace_bytes_, pl.S, K, n_total)) return rc;
  const size_t nb = n_total * sizeof(float);
  const Span in1{theta_g_snap, nb}, in2{theta_m, nb}, o1{delta_m_out, nb}, o2{theta_m_send_out, nb};
  const Span ws{workspace, workspace_bytes_};
  if (overlap(o1, in1) || overlap(o1, in2) || overlap(o2, in1) || overlap(o2, in2) || overlap(o1, o2) ||
      overlap(ws, in1) || overlap(ws, in2) || overlap(ws, o1) || overlap(ws, o2))
    return COCODC_ERR_ALIAS;
  hipStream_t s = static_cast<hipStream_t>(stream);
  WorkspaceView v = view(workspace, pl.S, K);
  if (int rc = upload_table(pl, v, s)) return rc;
  const bool vec = all_aligned16({theta_g_snap, theta_m, delta_m_out, theta_m_send_out});
  if (theta_m_send_out) {
    PseudoGradOp<true> op{theta_g_snap, theta_m, delta_m_out, theta_m_send_out};
    return launch_walk(vec, walk_of(v, pl), op, v.partials, s);
  }
  PseudoGradOp<false> op{theta_g_snap, theta_m, delta_m_out, nullptr};
  return launch_walk(vec, walk_of(v, pl), op, v.partials, s);
}

int cocodc_outer_nesterov(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total, float* theta_g,
                          float* momentum, const float* delta_g, const cocodc_hparams_t* hp,
                          void* workspace, size_t workspace_bytes_, void* stream) {
  if (!theta_g || !momentum || !delta_g) return COCODC_ERR_NULL;
  if (!all_aligned4({theta_g, momentum, delta_g})) return COCODC_ERR_ALIGN;
  if (int rc = check_hparams(hp)) return rc;
  Plan pl;
  if (int rc = plan_table(frags, K, n_total, nullptr, nullptr, &pl)) return rc;
  if (int rc = check_workspace(workspace, workspace_bytes_, pl.S, K, n_total)) return rc;
  const size_t nb = n_total * sizeof(float);
  const Span a{theta_g, nb}, b{momentum, nb}, c{delta_g, nb}, ws{workspace, workspace_bytes_};
  if (overlap(a, b) || overlap(a, c) || overlap(b, c) || overlap(ws, a) || overlap(ws, b) || overlap(ws, c))
    return COCODC_ERR_ALIAS;
  hipStream_t s = static_cast<hipStream_t>(stream);
  WorkspaceView v = view(workspace, pl.S, K);
  if (int rc = upload_table(pl, v, s)) return rc;
  const bool vec = all_aligned16({theta_g, momentum, delta_g});
  const DevHP d = to_dev(*hp);
  if (hp->nesterov) {
    OuterOp<true> op{theta_g, momentum, delta_g, d};
    return launch_walk(vec, walk_of(v, pl), op, v.partials, s);
  }
  OuterOp<false> op{theta_g, momentum, delta_g, d};
  return launch_walk(vec, walk_of(v, pl), op, v.partials, s);
}

int cocodc_delay_compensate(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total, float* theta_m,
                            const float* theta_m_send, const float* theta_g, const cocodc_hparams_t* hp,
                            void* workspace, size_t workspace_bytes_, void* stream) {
  if (!theta_m || !theta_g) return COCODC_ERR_NULL;
  if (!all_aligned4({theta_m, theta_m_send, theta_g})) return COCODC_ERR_ALIGN;
  if (int rc = check_hparams(hp)) return rc;
  if (!theta_m_send && hp->merge_mode == 0) return COCODC_ERR_NULL;  // Algorithm 1 needs theta^m_{p,t_p}
  if (hp->delta_src == 1 && hp->merge_mode == 0) return COCODC_ERR_RANGE;  // needs theta^g_{p,t_p-H}: fused only
  Plan pl;
  if (int rc = plan_table(frags, K, n_total, nullptr, nullptr, &pl)) return rc;
  if (int rc = check_workspace(workspace, workspace_bytes_, pl.S, K, n_total)) return rc;
  const size_t nb = n_total * sizeof(float);
  const Span a{theta_m, nb}, b{theta_m_send, nb}, c{theta_g, nb}, ws{workspace, workspace_bytes_};
  if (overlap(a, b) || overlap(a, c) || overlap(ws, a) || overlap(ws, b) || overlap(ws, c))
    return COCODC_ERR_ALIAS;
  hipStream_t s = static_cast<hipStream_t>(stream);
  WorkspaceView v = view(workspace, pl.S, K);
  if (int rc = upload_table(pl, v, s)) return rc;
  const bool vec = all_aligned16({theta_m, theta_m_send, theta_g});
  const DevHP d = to_dev(*hp);
  switch (merge_variant(*hp)) {
    case 0: {
      MergeOp<0> op{theta_m, theta_m_send, theta_g, d};
      return launch_walk(vec, walk_of(v, pl), op, v.partials, s);
    }
    case 1: {
      MergeOp<1, false> op{theta_m, nullptr, theta_g, d};
      return launch_walk(vec, walk_of(v, pl), op, v.partials, s);
    }
    case 2: {
      MergeOp<2, false> op{theta_m, nullptr, theta_g, d};
      return launch_walk(vec, walk_of(v, pl), op, v.partials, s);
    }
    default: {
      MergeOp<3> op{theta_m, theta_m_send, theta_g, d};
      return launch_walk(vec, walk_of(v, pl), op, v.partials, s);
    }
  }
}

static int fragment_scores_impl(Plan& pl, int32_t K, uint64_t n_total, const float* x, int32_t norm_kind,
                                double* R_out, double* sum_out, void* workspace, size_t workspace_bytes_,
                                void* stream) {
  if (int rc = check_workspace(workspace, workspace_bytes_, pl.S, K, n_total)) return rc;
  const Span xs{x, n_total * sizeof(float)}, r{R_out, sizeof(double) * K}, so{sum_out, sizeof(double) * K};
  const Span ws{workspace, workspace_bytes_};
  if (overlap(r, xs) || overlap(so, xs) || overlap(r, so) || overlap(ws, xs) || overlap(ws, r) ||
      overlap(ws, so))
    return COCODC_ERR_ALIAS;
  hipStream_t s = static_cast<hipStream_t>(stream);
  WorkspaceView v = view(workspace, pl.S, K);
  if (int rc = upload_table(pl, v, s)) return rc;
  const bool vec = aligned(x, 16);
  int rc;
  if (norm_kind == 2) {
    ScoreOp<2> op{x};
    rc = launch_walk(vec, walk_of(v, pl), op, v.partials, s);
  } else {
    ScoreOp<1> op{x};
    rc = launch_walk(vec, walk_of(v, pl), op, v.partials, s);
  }
  if (rc) return rc;
  return launch_finalize(pl, v, 1, 0, norm_kind == 2 ? 1 : 0, R_out, sum_out, 1, s);
}

int cocodc_fragment_scores(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total, const float* x,
                           const int64_t* I_p, int32_t norm_kind, double* R_out, double* sum_out,
                           void* workspace, size_t workspace_bytes_, void* stream) {
  if (!x || !I_p || !R_out) return COCODC_ERR_NULL;
  if (!aligned(x, 4) || !aligned(R_out, 8) || !aligned(sum_out, 8)) return COCODC_ERR_ALIGN;
  if (norm_kind != 1 && norm_kind != 2) return COCODC_ERR_RANGE;
  Plan pl;
  if (int rc = plan_table(frags, K, n_total, I_p, nullptr, &pl)) return rc;
  return fragment_scores_impl(pl, K, n_total, x, norm_kind, R_out, sum_out, workspace, workspace_bytes_, stream);
}

int cocodc_fragment_scores_segmented(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total,
                                     const float* x, const int64_t* I_p, int32_t norm_kind, double* R_out,
                                     double* sum_out, void* workspace, size_t workspace_bytes_, void* stream) {
  if (!x || !I_p || !R_out) return COCODC_ERR_NULL;
  if (!aligned(x, 4) || !aligned(R_out, 8) || !aligned(sum_out, 8)) return COCODC_ERR_ALIGN;
  if (norm_kind != 1 && norm_kind != 2) return COCODC_ERR_RANGE;
  Plan pl;
  if (int rc = plan_segments(segs, S, K, n_total, I_p, nullptr, &pl)) return rc;
  return fragment_scores_impl(pl, K, n_total, x, norm_kind, R_out, sum_out, workspace, workspace_bytes_, stream);
}

int cocodc_select_fragments(int32_t K, const double* R, const int64_t* t_b, int64_t t_g, int32_t H,
                            int32_t budget, int32_t* sel_out, int32_t* n_sel_out, void* workspace,
                            size_t workspace_bytes_, void* stream) {
  if (!R || !t_b || !sel_out || !n_sel_out) return COCODC_ERR_NULL;
  if (K < 1 || K > COCODC_MAX_FRAGMENTS || H < 1 || budget < 0) return COCODC_ERR_RANGE;
  if (!aligned(R, 8) || !aligned(sel_out, 4) || !aligned(n_sel_out, 4)) return COCODC_ERR_ALIGN;
  if (int rc = check_workspace(workspace, workspace_bytes_, K, K, 0)) return rc;
  const int n = budget < K ? budget : K;
  const Span r{R, sizeof(double) * K}, so{sel_out, sizeof(int32_t) * n}, ns{n_sel_out, sizeof(int32_t)};
  const Span ws{workspace, workspace_bytes_};
  if (overlap(r, so) || overlap(r, ns) || overlap(so, ns) || overlap(ws, r) || overlap(ws, so) ||
      overlap(ws, ns))
    return COCODC_ERR_ALIAS;
  Plan pl;  // no segments: only the per-fragment records (t_b) are needed
  if (int rc = plan_segments(nullptr, 0, K, 0, nullptr, t_b, &pl)) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  WorkspaceView v = view(workspace, pl.S, K);
  if (int rc = upload_table(pl, v, s)) return rc;
  return launch_select(pl, v, R, t_g, static_cast<int64_t>(H), n, sel_out, n_sel_out, s);
}

// The buffers of the fused step may not overlap, except that the pseudo-gradient may be written
// over delta_g.  A NULL entry (an optional buffer, or no workspace to check yet) overlaps nothing.
static int sync_step_overlaps(int32_t K, uint64_t n_total, const float* theta_m, const float* theta_m_send,
                              const float* theta_g, const float* momentum, const float* delta_g,
                              const float* delta_m_out, int n_sel_max, const double* R_out, const int32_t* sel_out,
                              const int32_t* n_sel_out, const double* sums_out, const void* workspace,
                              size_t workspace_bytes_) {
  const size_t nb = n_total * sizeof(float);
  const Span sp[] = {{theta_m, nb},     {theta_m_send, nb},           {theta_g, nb},
                     {momentum, nb},    {delta_g, nb},                {delta_m_out, nb},
                     {R_out, sizeof(double) * K}, {sel_out, sizeof(int32_t) * n_sel_max}, {n_sel_out, sizeof(int32_t)},
                     {sums_out, sizeof(double) * 4 * K}, {workspace, workspace_bytes_}};
  const int ns = static_cast<int>(sizeof(sp) / sizeof(sp[0]));
  for (int i = 0; i < ns; ++i) {
    for (int j = i + 1; j < ns; ++j) {
      if (i == 4 && j == 5 && delta_m_out == delta_g) continue;  // in-place pseudo-gradient
      if (overlap(sp[i], sp[j])) return COCODC_ERR_ALIAS;
    }
  }
  return COCODC_OK;
}

static int sync_step_impl(Plan& pl, int32_t K, uint64_t n_total, float* theta_m, const float* theta_m_send,
                          float* theta_g, float* momentum, const float* delta_g, float* delta_m_out, int64_t t_g,
                          int32_t budget, const cocodc_hparams_t* hp, double* R_out, int32_t* sel_out,
                          int32_t* n_sel_out, double* sums_out, void* workspace, size_t workspace_bytes_,
                          void* stream) {
  if (int rc = check_workspace(workspace, workspace_bytes_, pl.S, K, n_total)) return rc;
  int candidates = 0, taking_part = 0;  // fragments Algorithm 2 may choose; fragments this call updates
  for (int32_t p = 0; p < K; ++p) {
    candidates += pl.groups[p].in_flight ? 0 : 1;
    taking_part += pl.groups[p].takes_part ? 1 : 0;
  }
  const int n = budget < candidates ? budget : candidates;
  if (int rc = sync_step_overlaps(K, n_total, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, n, R_out,
                                  sel_out, n_sel_out, sums_out, workspace, workspace_bytes_))
    return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  WorkspaceView v = view(workspace, pl.S, K);
  if (int rc = upload_table(pl, v, s)) return rc;
  if (taking_part > 0) {
    const bool vec = all_aligned16({theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out});
    const DevHP d = to_dev(*hp);
    int rc = hp->nesterov ? launch_fused_m<true>(merge_variant(*hp), vec, walk_of(v, pl), theta_m, theta_m_send,
                                                 theta_g, momentum, delta_g, delta_m_out, d, v.partials, s)
                          : launch_fused_m<false>(merge_variant(*hp), vec, walk_of(v, pl), theta_m, theta_m_send,
                                                  theta_g, momentum, delta_g, delta_m_out, d, v.partials, s);
    if (rc) return rc;
    const int which = (hp->score_src ? 2 : 0) + (hp->norm_kind == 2 ? 0 : 1);
    if (int rc2 = launch_finalize(pl, v, kSums, which, hp->norm_kind == 2 ? 1 : 0, R_out, sums_out, kSums, s)) return rc2;
  }
  return launch_select(pl, v, R_out, t_g, static_cast<int64_t>(hp->H), n, sel_out, n_sel_out, s);
}

static int sync_step_check(float* theta_m, const float* theta_m_send, float* theta_g, float* momentum,
                           const float* delta_g, float* delta_m_out, const int64_t* I_p, const int64_t* t_b,
                           int32_t budget, const cocodc_hparams_t* hp, double* R_out, int32_t* sel_out,
                           int32_t* n_sel_out, double* sums_out) {
  if (!theta_m || !theta_g || !momentum || !delta_g) return COCODC_ERR_NULL;
  if (!I_p || !t_b || !R_out || !sel_out || !n_sel_out) return COCODC_ERR_NULL;
  if (!all_aligned4({theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, sel_out, n_sel_out}))
    return COCODC_ERR_ALIGN;
  if (!aligned(R_out, 8) || !aligned(sums_out, 8)) return COCODC_ERR_ALIGN;
  if (int rc = check_hparams(hp)) return rc;
  if (!theta_m_send && (hp->merge_mode == 0 || hp->score_src == 1)) return COCODC_ERR_NULL;
  if (budget < 0) return COCODC_ERR_RANGE;
  return COCODC_OK;
}

int cocodc_sync_step(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total, float* theta_m,
                     const float* theta_m_send, float* theta_g, float* momentum, const float* delta_g,
                     float* delta_m_out, const int64_t* I_p, const int64_t* t_b, int64_t t_g,
                     int32_t budget, const cocodc_hparams_t* hp, double* R_out, int32_t* sel_out,
                     int32_t* n_sel_out, double* sums_out, void* workspace, size_t workspace_bytes_,
                     void* stream) {
  if (int rc = sync_step_check(theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p, t_b, budget, hp,
                               R_out, sel_out, n_sel_out, sums_out))
    return rc;
  Plan pl;
  if (int rc = plan_table(frags, K, n_total, I_p, t_b, &pl)) return rc;
  return sync_step_impl(pl, K, n_total, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, t_g, budget,
                        hp, R_out, sel_out, n_sel_out, sums_out, workspace, workspace_bytes_, stream);
}

// ---- the fused step for callers that cannot allocate device memory --------------------------
// The device-side table and the per-tile partial sums, which the other entry points keep in the
// caller's workspace, live in this file-scope array instead: one copy per GPU, held from the
// moment the library's code is loaded on that GPU until the process ends.  `scratch` is only the
// host-side name of the symbol; its device address on each GPU is looked up once, with that GPU
// current, and kept in g_scratch_ptr.  Host code uses that pointer, never the name.
static __device__ __align__(256) unsigned char scratch[COCODC_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

int scratch_of_current_device(void** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return COCODC_ERR_RANGE;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return hip_fail(hipErrorInvalidSymbol);
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return COCODC_OK;
}
}  // namespace

int cocodc_sync_step_noalloc(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total, float* theta_m,
                             const float* theta_m_send, float* theta_g, float* momentum, const float* delta_g,
                             float* delta_m_out, const int64_t* I_p, const int64_t* t_b, int64_t t_g,
                             int32_t budget, const cocodc_hparams_t* hp, double* R_out, int32_t* sel_out,
                             int32_t* n_sel_out, double* sums_out, void* stream) {
  if (int rc = sync_step_check(theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p, t_b, budget, hp,
                               R_out, sel_out, n_sel_out, sums_out))
    return rc;
  Plan pl;
  if (int rc = plan_table(frags, K, n_total, I_p, t_b, &pl)) return rc;
  // the fixed array must hold what cocodc_workspace_bytes(K, n_total) asks for
  if (workspace_bytes(pl.S, K, n_total) > static_cast<size_t>(COCODC_NOALLOC_SCRATCH_BYTES)) return COCODC_ERR_WORKSPACE;
  if (int rc = sync_step_overlaps(K, n_total, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out,
                                  budget < K ? budget : K, R_out, sel_out, n_sel_out, sums_out, nullptr, 0))
    return rc;
  void* ws = nullptr;  // every check that needs no device is done: only now is the GPU touched
  if (int rc = scratch_of_current_device(&ws)) return rc;
  // Nothing in the array has to start at zero: the table is rewritten by every call and every
  // partial-sum slot that the reduction reads was written by this call's streaming kernel.
  return sync_step_impl(pl, K, n_total, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, t_g, budget,
                        hp, R_out, sel_out, n_sel_out, sums_out, ws, COCODC_NOALLOC_SCRATCH_BYTES, stream);
}

int cocodc_sync_event(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total, const uint8_t* recv_mask,
                      float* theta_m, const float* theta_m_send, float* theta_g, float* momentum,
                      const float* delta_g, float* delta_m_out, const int64_t* I_p, const int64_t* t_b, int64_t t_g,
                      int32_t budget, const cocodc_hparams_t* hp, double* R, int32_t* sel_out, int32_t* n_sel_out,
                      double* sums_out, void* workspace, size_t workspace_bytes_, void* stream) {
  if (!recv_mask) return COCODC_ERR_NULL;
  if (int rc = sync_step_check(theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p, t_b, budget, hp,
                               R, sel_out, n_sel_out, sums_out))
    return rc;
  Plan pl;
  if (int rc = plan_table(frags, K, n_total, I_p, t_b, &pl, recv_mask)) return rc;
  return sync_step_impl(pl, K, n_total, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, t_g, budget,
                        hp, R, sel_out, n_sel_out, sums_out, workspace, workspace_bytes_, stream);
}

int cocodc_sync_step_segmented(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total,
                               float* theta_m, const float* theta_m_send, float* theta_g, float* momentum,
                               const float* delta_g, float* delta_m_out, const int64_t* I_p, const int64_t* t_b,
                               int64_t t_g, int32_t budget, const cocodc_hparams_t* hp, double* R_out,
                               int32_t* sel_out, int32_t* n_sel_out, double* sums_out, void* workspace,
                               size_t workspace_bytes_, void* stream) {
  if (int rc = sync_step_check(theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p, t_b, budget, hp,
                               R_out, sel_out, n_sel_out, sums_out))
    return rc;
  Plan pl;
  if (int rc = plan_segments(segs, S, K, n_total, I_p, t_b, &pl)) return rc;
  return sync_step_impl(pl, K, n_total, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, t_g, budget,
                        hp, R_out, sel_out, n_sel_out, sums_out, workspace, workspace_bytes_, stream);
}

int cocodc_sync_event_segmented(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total,
                                const uint8_t* recv_mask, float* theta_m, const float* theta_m_send, float* theta_g,
                                float* momentum, const float* delta_g, float* delta_m_out, const int64_t* I_p,
                                const int64_t* t_b, int64_t t_g, int32_t budget, const cocodc_hparams_t* hp, double* R,
                                int32_t* sel_out, int32_t* n_sel_out, double* sums_out, void* workspace,
                                size_t workspace_bytes_, void* stream) {
  if (!recv_mask) return COCODC_ERR_NULL;
  if (int rc = sync_step_check(theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p, t_b, budget, hp,
                               R, sel_out, n_sel_out, sums_out))
    return rc;
  Plan pl;
  if (int rc = plan_segments(segs, S, K, n_total, I_p, t_b, &pl, recv_mask)) return rc;
  return sync_step_impl(pl, K, n_total, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, t_g, budget,
                        hp, R, sel_out, n_sel_out, sums_out, workspace, workspace_bytes_, stream);
}

int cocodc_pseudograd_bf16(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total,
                           const float* theta_g_snap, const uint16_t* theta_m, uint16_t* delta_m_out,
                           uint16_t* theta_m_send_out, int32_t pg_format, void* workspace, size_t workspace_bytes_,
                           void* stream) {
  if (!theta_g_snap || !theta_m || !delta_m_out) return COCODC_ERR_NULL;
  if (pg_format != COCODC_PG_BF16 && pg_format != COCODC_PG_F16) return COCODC_ERR_RANGE;
  if (!aligned(theta_g_snap, 4) || !aligned(theta_m, 2) || !aligned(delta_m_out, 2) || !aligned(theta_m_send_out, 2))
    return COCODC_ERR_ALIGN;
  Plan pl;
  if (int rc = plan_table(frags, K, n_total, nullptr, nullptr, &pl)) return rc;
  if (int rc = check_workspace(workspace, workspace_bytes_, pl.S, K, n_total)) return rc;
  const Span in1{theta_g_snap, n_total * 4}, in2{theta_m, n_total * 2}, o1{delta_m_out, n_total * 2},
      o2{theta_m_send_out, n_total * 2}, ws{workspace, workspace_bytes_};
  if (overlap(o1, in1) || overlap(o1, in2) || overlap(o2, in1) || overlap(o2, in2) || overlap(o1, o2) ||
      overlap(ws, in1) || overlap(ws, in2) || overlap(ws, o1) || overlap(ws, o2))
    return COCODC_ERR_ALIAS;
  hipStream_t s = static_cast<hipStream_t>(stream);
  WorkspaceView v = view(workspace, pl.S, K);
  if (int rc = upload_table(pl, v, s)) return rc;
  const bool vec = all_aligned16({theta_g_snap, theta_m, delta_m_out, theta_m_send_out});
  const HostWalk wk = walk_of(v, pl);
  if (pg_format == COCODC_PG_F16) {
    if (theta_m_send_out) {
      PseudoGradBf16Op<true, true> op{theta_g_snap, theta_m, delta_m_out, theta_m_send_out};
      return launch_walk(vec, wk, op, v.partials, s);
    }
    PseudoGradBf16Op<false, true> op{theta_g_snap, theta_m, delta_m_out, nullptr};
    return launch_walk(vec, wk, op, v.partials, s);
  }
  if (theta_m_send_out) {
    PseudoGradBf16Op<true> op{theta_g_snap, theta_m, delta_m_out, theta_m_send_out};
    return launch_walk(vec, wk, op, v.partials, s);
  }
  PseudoGradBf16Op<false> op{theta_g_snap, theta_m, delta_m_out, nullptr};
  return launch_walk(vec, wk, op, v.partials, s);
}

// ---- the fused step on 16-bit local parameters --------------------------------------------------
static int sync_step_bf16_check(const uint16_t* theta_m, const uint16_t* theta_m_send, const float* theta_g,
                                const float* momentum, const float* delta_g, const uint16_t* delta_m_out,
                                const int64_t* I_p, const int64_t* t_b, int32_t budget, const cocodc_hparams_t* hp,
                                const double* R_out, const int32_t* sel_out, const int32_t* n_sel_out,
                                const double* sums_out) {
  if (!theta_m || !theta_g || !momentum || !delta_g) return COCODC_ERR_NULL;
  if (!I_p || !t_b || !R_out || !sel_out || !n_sel_out) return COCODC_ERR_NULL;
  if (!all_aligned4({theta_g, momentum, delta_g, sel_out, n_sel_out})) return COCODC_ERR_ALIGN;
  if (!aligned(theta_m, 2) || !aligned(theta_m_send, 2) || !aligned(delta_m_out, 2)) return COCODC_ERR_ALIGN;
  if (!aligned(R_out, 8) || !aligned(sums_out, 8)) return COCODC_ERR_ALIGN;
  if (int rc = check_hparams(hp)) return rc;
  if (!theta_m_send && (hp->merge_mode == 0 || hp->score_src == 1)) return COCODC_ERR_NULL;
  if (budget < 0) return COCODC_ERR_RANGE;
  return COCODC_OK;
}

// No two buffers of the 16-bit step may overlap (the incoming average is fp32 and the outgoing
// pseudo-gradient 16-bit, so there is no in-place exchange buffer here).
static int sync_step_bf16_overlaps(int32_t K, uint64_t n_total, const uint16_t* theta_m, const uint16_t* theta_m_send,
                                   const float* theta_g, const float* momentum, const float* delta_g,
                                   const uint16_t* delta_m_out, int n_sel_max, const double* R_out,
                                   const int32_t* sel_out, const int32_t* n_sel_out, const double* sums_out,
                                   const void* workspace, size_t workspace_bytes_) {
  const Span sp[] = {{theta_m, n_total * 2},      {theta_m_send, n_total * 2},    {theta_g, n_total * 4},
                     {momentum, n_total * 4},     {delta_g, n_total * 4},         {delta_m_out, n_total * 2},
                     {R_out, sizeof(double) * K}, {sel_out, sizeof(int32_t) * n_sel_max}, {n_sel_out, sizeof(int32_t)},
                     {sums_out, sizeof(double) * 4 * K}, {workspace, workspace_bytes_}};
  const int ns = static_cast<int>(sizeof(sp) / sizeof(sp[0]));
  for (int i = 0; i < ns; ++i) {
    for (int j = i + 1; j < ns; ++j) {
      if (overlap(sp[i], sp[j])) return COCODC_ERR_ALIAS;
    }
  }
  return COCODC_OK;
}

static int sync_step_bf16_impl(Plan& pl, int32_t K, uint64_t n_total, uint16_t* theta_m, const uint16_t* theta_m_send,
                               float* theta_g, float* momentum, const float* delta_g, uint16_t* delta_m_out,
                               int64_t t_g, int32_t budget, const cocodc_hparams_t* hp, double* R_out,
                               int32_t* sel_out, int32_t* n_sel_out, double* sums_out, void* workspace,
                               size_t workspace_bytes_, void* stream) {
  if (int rc = check_workspace(workspace, workspace_bytes_, pl.S, K, n_total)) return rc;
  int candidates = 0, taking_part = 0;  // fragments Algorithm 2 may choose; fragments this call updates
  for (int32_t p = 0; p < K; ++p) {
    candidates += pl.groups[p].in_flight ? 0 : 1;
    taking_part += pl.groups[p].takes_part ? 1 : 0;
  }
  const int n = budget < candidates ? budget : candidates;
  if (int rc = sync_step_bf16_overlaps(K, n_total, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, n,
                                       R_out, sel_out, n_sel_out, sums_out, workspace, workspace_bytes_))
    return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  WorkspaceView v = view(workspace, pl.S, K);
  if (int rc = upload_table(pl, v, s)) return rc;
  if (taking_part > 0) {
    const bool vec = all_aligned16({theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out});
    const DevHP d = to_dev(*hp);
    const bool pg_f16 = hp->pg_format == COCODC_PG_F16;
    int rc = hp->nesterov ? launch_fused_bf16_m<true>(merge_variant(*hp), vec, walk_of(v, pl), theta_m, theta_m_send,
                                                      theta_g, momentum, delta_g, delta_m_out, pg_f16, d, v.partials, s)
                          : launch_fused_bf16_m<false>(merge_variant(*hp), vec, walk_of(v, pl), theta_m, theta_m_send,
                                                       theta_g, momentum, delta_g, delta_m_out, pg_f16, d, v.partials, s);
    if (rc) return rc;
    const int which = (hp->score_src ? 2 : 0) + (hp->norm_kind == 2 ? 0 : 1);
    if (int rc2 = launch_finalize(pl, v, kSums, which, hp->norm_kind == 2 ? 1 : 0, R_out, sums_out, kSums, s)) return rc2;
  }
  return launch_select(pl, v, R_out, t_g, static_cast<int64_t>(hp->H), n, sel_out, n_sel_out, s);
}

int cocodc_sync_step_bf16(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total, uint16_t* theta_m,
                          const uint16_t* theta_m_send, float* theta_g, float* momentum, const float* delta_g,
                          uint16_t* delta_m_out, const int64_t* I_p, const int64_t* t_b, int64_t t_g,
                          int32_t budget, const cocodc_hparams_t* hp, double* R_out, int32_t* sel_out,
                          int32_t* n_sel_out, double* sums_out, void* workspace, size_t workspace_bytes_,
                          void* stream) {
  if (int rc = sync_step_bf16_check(theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p, t_b, budget,
                                    hp, R_out, sel_out, n_sel_out, sums_out))
    return rc;
  Plan pl;
  if (int rc = plan_table(frags, K, n_total, I_p, t_b, &pl)) return rc;
  return sync_step_bf16_impl(pl, K, n_total, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, t_g,
                             budget, hp, R_out, sel_out, n_sel_out, sums_out, workspace, workspace_bytes_, stream);
}

int cocodc_sync_step_bf16_segmented(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total,
                                    uint16_t* theta_m, const uint16_t* theta_m_send, float* theta_g, float* momentum,
                                    const float* delta_g, uint16_t* delta_m_out, const int64_t* I_p,
                                    const int64_t* t_b, int64_t t_g, int32_t budget, const cocodc_hparams_t* hp,
                                    double* R_out, int32_t* sel_out, int32_t* n_sel_out, double* sums_out,
                                    void* workspace, size_t workspace_bytes_, void* stream) {
  if (int rc = sync_step_bf16_check(theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p, t_b, budget,
                                    hp, R_out, sel_out, n_sel_out, sums_out))
    return rc;
  Plan pl;
  if (int rc = plan_segments(segs, S, K, n_total, I_p, t_b, &pl)) return rc;
  return sync_step_bf16_impl(pl, K, n_total, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, t_g,
                             budget, hp, R_out, sel_out, n_sel_out, sums_out, workspace, workspace_bytes_, stream);
}

int cocodc_sync_event_bf16(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total, const uint8_t* recv_mask,
                           uint16_t* theta_m, const uint16_t* theta_m_send, float* theta_g, float* momentum,
                           const float* delta_g, uint16_t* delta_m_out, const int64_t* I_p, const int64_t* t_b,
                           int64_t t_g, int32_t budget, const cocodc_hparams_t* hp, double* R, int32_t* sel_out,
                           int32_t* n_sel_out, double* sums_out, void* workspace, size_t workspace_bytes_,
                           void* stream) {
  if (!recv_mask) return COCODC_ERR_NULL;
  if (int rc = sync_step_bf16_check(theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p, t_b, budget,
                                    hp, R, sel_out, n_sel_out, sums_out))
    return rc;
  Plan pl;
  if (int rc = plan_table(frags, K, n_total, I_p, t_b, &pl, recv_mask)) return rc;
  return sync_step_bf16_impl(pl, K, n_total, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, t_g,
                             budget, hp, R, sel_out, n_sel_out, sums_out, workspace, workspace_bytes_, stream);
}

int cocodc_sync_event_bf16_segmented(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total,
                                     const uint8_t* recv_mask, uint16_t* theta_m, const uint16_t* theta_m_send,
                                     float* theta_g, float* momentum, const float* delta_g, uint16_t* delta_m_out,
                                     const int64_t* I_p, const int64_t* t_b, int64_t t_g, int32_t budget,
                                     const cocodc_hparams_t* hp, double* R, int32_t* sel_out, int32_t* n_sel_out,
                                     double* sums_out, void* workspace, size_t workspace_bytes_, void* stream) {
  if (!recv_mask) return COCODC_ERR_NULL;
  if (int rc = sync_step_bf16_check(theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, I_p, t_b, budget,
                                    hp, R, sel_out, n_sel_out, sums_out))
    return rc;
  Plan pl;
  if (int rc = plan_segments(segs, S, K, n_total, I_p, t_b, &pl, recv_mask)) return rc;
  return sync_step_bf16_impl(pl, K, n_total, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, t_g,
                             budget, hp, R, sel_out, n_sel_out, sums_out, workspace, workspace_bytes_, stream);
}

int cocodc_select_fragments_bytes(int32_t K, const double* R, const int64_t* t_b, int64_t t_g, int32_t H,
                                  const uint64_t* frag_bytes, uint64_t byte_budget, int32_t* sel_out,
                                  int32_t* n_sel_out, void* workspace, size_t workspace_bytes_, void* stream) {
  if (!R || !t_b || !frag_bytes || !sel_out || !n_sel_out) return COCODC_ERR_NULL;
  if (K < 1 || K > COCODC_MAX_FRAGMENTS || H < 1) return COCODC_ERR_RANGE;
  if (!aligned(R, 8) || !aligned(sel_out, 4) || !aligned(n_sel_out, 4)) return COCODC_ERR_ALIGN;
  if (int rc = check_workspace(workspace, workspace_bytes_, K, K, 0)) return rc;
  const Span r{R, sizeof(double) * K}, so{sel_out, sizeof(int32_t) * K}, ns{n_sel_out, sizeof(int32_t)};
  const Span ws{workspace, workspace_bytes_};
  if (overlap(r, so) || overlap(r, ns) || overlap(so, ns) || overlap(ws, r) || overlap(ws, so) ||
      overlap(ws, ns))
    return COCODC_ERR_ALIAS;
  Plan pl;
  if (int rc = plan_segments(nullptr, 0, K, 0, nullptr, t_b, &pl)) return rc;
  for (int32_t p = 0; p < K; ++p) pl.groups[p].bytes = frag_bytes[p];
  pl.in_args = false;  // this kernel reads the records from the workspace, whatever their number
  hipStream_t s = static_cast<hipStream_t>(stream);
  WorkspaceView v = view(workspace, pl.S, K);
  if (int rc = upload_table(pl, v, s)) return rc;
  hipLaunchKernelGGL(k_select_bytes<GroupTable>, dim3(1), dim3(kThreads), 0, s, GroupTable{v.groups}, K, R, t_g,
                     static_cast<int64_t>(H), static_cast<unsigned long long>(byte_budget), sel_out, n_sel_out);
  HIP_TRY(hipGetLastError());
  return COCODC_OK;
}

int cocodc_sync_plan(int32_t K, int32_t H, double gamma, double T_c, double T_s, int64_t* N_out,
                     int64_t* h_out) {
  if (!N_out || !h_out) return COCODC_ERR_NULL;
  if (K < 1 || H < 1) return COCODC_ERR_RANGE;
  if (std::isnan(gamma) || std::isnan(T_c) || std::isnan(T_s) || std::isinf(T_c) || std::isinf(T_s))
    return COCODC_ERR_NONFINITE;
  if (gamma <= 0.0 || gamma > 1.0 || T_c <= 0.0 || T_s <= 0.0) return COCODC_ERR_RANGE;
  // Eq. 9: how many fragment synchronisations fit into H compute steps at utilisation gamma.
  const double fit = std::floor(gamma * ((static_cast<double>(H) * T_c) / T_s));
  int64_t N = K;
  if (fit > static_cast<double>(K)) N = fit >= 9.0e18 ? std::numeric_limits<int64_t>::max() : static_cast<int64_t>(fit);
  *N_out = N;
  *h_out = static_cast<int64_t>(H) / N;  // Eq. 10
  return COCODC_OK;
}

}  // extern "C"

#include "cocodc_loop.h"

extern "C" {

uint64_t cocodc_layout_stride_bytes(uint64_t n_total) {
  constexpr uint64_t GiB = 1ull << 30;
  const uint64_t bytes = n_total * sizeof(float);
  uint64_t stride = std::max<uint64_t>(40 * GiB, (bytes + GiB - 1) / GiB * GiB);
  if (stride % (32 * GiB) == 0) stride += 2 * GiB;
  return stride;
}

int cocodc_debug_stream_mix(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total, float* a, const float* b,
                            float* c, float* d, const float* e, float* f, void* workspace,
                            size_t workspace_bytes_, void* stream) {
  if (!a || !b || !c || !d || !e || !f) return COCODC_ERR_NULL;
  if (!all_aligned4({a, b, c, d, e, f})) return COCODC_ERR_ALIGN;
  Plan pl;
  if (int rc = plan_table(frags, K, n_total, nullptr, nullptr, &pl)) return rc;
  if (int rc = check_workspace(workspace, workspace_bytes_, pl.S, K, n_total)) return rc;
  const size_t nb = n_total * sizeof(float);
  const Span sp[] = {{a, nb}, {b, nb}, {c, nb}, {d, nb}, {e, nb}, {f, nb}, {workspace, workspace_bytes_}};
  for (int i = 0; i < 7; ++i) {
    for (int j = i + 1; j < 7; ++j) {
      if (overlap(sp[i], sp[j])) return COCODC_ERR_ALIAS;
    }
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  WorkspaceView v = view(workspace, pl.S, K);
  if (int rc = upload_table(pl, v, s)) return rc;
  StreamMixOp op{a, b, c, d, e, f};
  return launch_walk(all_aligned16({a, b, c, d, e, f}), walk_of(v, pl), op, v.partials, s);
}

uint64_t cocodc_tile_elements(uint64_t n_total) { return uint64_t(1) << tile_shift_for(n_total); }

int cocodc_debug_tile_plan(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total,
                           uint64_t* seg_offset_out, uint64_t* seg_slot_begin_out, uint64_t* frag_slot_begin_out,
                           uint64_t* tile_capacity_out) {
  if (!seg_offset_out || !seg_slot_begin_out || !frag_slot_begin_out || !tile_capacity_out) return COCODC_ERR_NULL;
  Plan pl;
  if (int rc = plan_segments(segs, S, K, n_total, nullptr, nullptr, &pl)) return rc;
  for (int32_t j = 0; j <= S; ++j) {
    seg_offset_out[j] = pl.segs[j].offset;
    seg_slot_begin_out[j] = pl.segs[j].slot_begin;
  }
  for (int32_t p = 0; p <= K; ++p) frag_slot_begin_out[p] = pl.groups[p].slot_begin;
  *tile_capacity_out = max_tiles(S, n_total);
  return COCODC_OK;
}

int cocodc_last_hip_error(void) { return g_last_hip_error; }

const char* cocodc_status_string(int status) {
  switch (status) {
    case COCODC_OK: return "COCODC_OK";
    case COCODC_ERR_NULL: return "COCODC_ERR_NULL";
    case COCODC_ERR_ALIGN: return "COCODC_ERR_ALIGN";
    case COCODC_ERR_RANGE: return "COCODC_ERR_RANGE";
    case COCODC_ERR_NONFINITE: return "COCODC_ERR_NONFINITE";
    case COCODC_ERR_WORKSPACE: return "COCODC_ERR_WORKSPACE";
    case COCODC_ERR_HIP: return "COCODC_ERR_HIP";
    case COCODC_ERR_ALIAS: return "COCODC_ERR_ALIAS";
    default: return "COCODC_ERR_UNKNOWN";
  }
}

int cocodc_set_blocks_per_cu(int blocks_per_cu) {
  return g_blocks_per_cu.exchange(blocks_per_cu < 0 ? 0 : blocks_per_cu);
}

int cocodc_set_tables_in_args(int enabled) { return g_tables_in_args.exchange(enabled ? 1 : 0); }

int cocodc_profiler_enable(int32_t max_records) {
  if (max_records < 1 || max_records > 65536) return COCODC_ERR_RANGE;
  std::lock_guard<std::mutex> lock(g_prof.mu);
  if (g_prof.on.load()) return COCODC_ERR_RANGE;
  g_prof.start.resize(max_records);
  g_prof.stop.resize(max_records);
  for (int i = 0; i < max_records; ++i) {
    HIP_TRY(hipEventCreate(&g_prof.start[i]));
    HIP_TRY(hipEventCreate(&g_prof.stop[i]));
  }
  g_prof.used = 0;
  g_prof.on.store(true, std::memory_order_release);
  return COCODC_OK;
}

int cocodc_profiler_collect(float* ms_out, int32_t capacity) {
  if (!ms_out) return COCODC_ERR_NULL;
  std::lock_guard<std::mutex> lock(g_prof.mu);
  if (!g_prof.on.load()) return COCODC_ERR_RANGE;
  const int n = std::min<int>(g_prof.used, capacity);
  for (int i = 0; i < n; ++i) {
    HIP_TRY(hipEventSynchronize(g_prof.stop[i]));
    HIP_TRY(hipEventElapsedTime(&ms_out[i], g_prof.start[i], g_prof.stop[i]));
  }
  g_prof.used = 0;
  return n;
}

int cocodc_profiler_disable(void) {
  std::lock_guard<std::mutex> lock(g_prof.mu);
  if (!g_prof.on.load()) return COCODC_OK;
  g_prof.on.store(false, std::memory_order_release);
  for (size_t i = 0; i < g_prof.start.size(); ++i) {
    (void)hipEventDestroy(g_prof.start[i]);
    (void)hipEventDestroy(g_prof.stop[i]);
  }
  g_prof.start.clear();
  g_prof.stop.clear();
  g_prof.used = 0;
  return COCODC_OK;
}

}  // extern "C"
