// cocodc.hip -- gfx950 (MI355X) kernels and C ABI of the CoCoDC outer-synchronisation path.
//
// One streaming pass per call.  Every kernel walks the same list of TILES: a tile is the
// part of one fragment that falls into one aligned window of 2^tile_shift elements of the flat
// buffers, so a tile never straddles two fragments and, inside a tile, element indices that
// are multiples of 4 are 16-byte aligned whenever the buffer bases are.  A workgroup of
// 256 threads (4 wavefronts of 64) handles a tile with 128-bit loads and stores, several
// independent loads in flight per lane, fp64 arithmetic in registers and one rounding per
// stored fp32 value.  Per-fragment sums (paper Eq. 11) are produced as one fp64 partial per
// tile (lane -> wavefront shuffle -> LDS -> tile slot) and combined by a second kernel in a
// fixed order, so scores are bit-reproducible and independent of the launch shape.
//
// No MFMA: nothing on this path is a contraction; the bound is HBM bandwidth
// (20 B read + 16 B written per parameter in the fused step).
//
// Compile with -ffp-contract=off: the few fused multiply-adds used are written explicitly
// so that the fused kernel and the single-step kernels round identically.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <mutex>
#include <vector>

#include "cocodc.h"

#ifndef COCODC_TILE
#define COCODC_TILE 16384
#endif
#ifndef COCODC_DEPTH
#define COCODC_DEPTH 2
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

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
// Tile size: 2^14 elements for large buffers; 2^11 for small ones (below 2^24 elements), so
// that even a 1M-element call spreads over more workgroups than there are compute units.  It
// depends on n_total alone, so the workspace size and the summation order are functions of
// the arguments and not of the machine.
constexpr int kTileShiftLarge = 14, kTileShiftSmall = 11;
constexpr uint64_t kSmallBufferElements = 1ull << 24;
static_assert((1u << kTileShiftLarge) == COCODC_TILE, "COCODC_TILE must match the large tile");
inline int tile_shift_for(uint64_t n_total) {
  return n_total < kSmallBufferElements ? kTileShiftSmall : kTileShiftLarge;
}
constexpr int kDepth = COCODC_DEPTH;  // independent 128-bit loads per stream kept in flight per lane
constexpr int kTableChunk = 64;       // fragment records carried by one table-upload launch
constexpr int kSums = 4;              // doubles per partial-sum slot

static_assert((1u << kTileShiftSmall) % (4 * kThreads) == 0, "a tile must be a whole number of workgroup-wide vector rows");

// Device-side description of one fragment.
struct FragRec {
  uint64_t offset;      // first element
  uint64_t length;      // elements
  uint64_t slot_begin;  // index of this fragment's first tile in the global tile list
  uint64_t tile0;       // absolute window index (offset >> tile_shift) of that first tile
  int64_t I_p;          // steps between the fragment's last two completed syncs (Eq. 11)
  int64_t t_b;          // step of its last completed sync (Algorithm 2)
};
static_assert(sizeof(FragRec) == 48, "FragRec layout");

struct TableChunk {
  FragRec rec[kTableChunk];
};

// Hyper-parameters in the form the kernels consume.
struct DevHP {
  double mu, eta, sign;
  double lambda, tauH;  // tauH = tau*H as a double; lambda is forced to 0 when tau == 0
  double coef;          // lambda / (tau*H), 0 when tau == 0 (used when COCODC_EXACT_DIV == 0)
  double alpha, one_minus_alpha;
};

typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int V>
struct Vec;
template <>
struct Vec<1> {
  using type = float;
};
template <>
struct Vec<4> {
  using type = f32x4;
};

template <int V>
__device__ __forceinline__ typename Vec<V>::type load_stream(const float* p) {
  using T = typename Vec<V>::type;
#if COCODC_NT_LOAD
  return __builtin_nontemporal_load(reinterpret_cast<const T*>(p));
#else
  return *reinterpret_cast<const T*>(p);
#endif
}

template <int V>
__device__ __forceinline__ void store_stream(float* p, typename Vec<V>::type v) {
  using T = typename Vec<V>::type;
#if COCODC_NT_STORE
  __builtin_nontemporal_store(v, reinterpret_cast<T*>(p));
#else
  *reinterpret_cast<T*>(p) = v;
#endif
}

__device__ __forceinline__ float lane_get(float v, int) { return v; }
__device__ __forceinline__ float lane_get(const f32x4& v, int k) { return v[k]; }
__device__ __forceinline__ void lane_set(float& v, int, float x) { v = x; }
__device__ __forceinline__ void lane_set(f32x4& v, int k, float x) { v[k] = x; }

// ---- 16-bit streams of the bf16 variant: four bf16 = one 64-bit access per lane.
template <int V>
struct VecU16;
template <>
struct VecU16<1> {
  using type = unsigned short;
};
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));
template <>
struct VecU16<4> {
  using type = u16x4;
};

template <int V>
__device__ __forceinline__ typename VecU16<V>::type load_stream_u16(const unsigned short* p) {
  using T = typename VecU16<V>::type;
#if COCODC_NT_LOAD
  return __builtin_nontemporal_load(reinterpret_cast<const T*>(p));
#else
  return *reinterpret_cast<const T*>(p);
#endif
}
template <int V>
__device__ __forceinline__ void store_stream_u16(unsigned short* p, typename VecU16<V>::type v) {
  using T = typename VecU16<V>::type;
#if COCODC_NT_STORE
  __builtin_nontemporal_store(v, reinterpret_cast<T*>(p));
#else
  *reinterpret_cast<T*>(p) = v;
#endif
}
__device__ __forceinline__ unsigned short lane_get(unsigned short v, int) { return v; }
__device__ __forceinline__ unsigned short lane_get(const u16x4& v, int k) { return v[k]; }
__device__ __forceinline__ void lane_set(u16x4& v, int k, unsigned short x) { v[k] = x; }
__device__ __forceinline__ void lane_set(unsigned short& v, int, unsigned short x) { v = x; }

// bfloat16 = upper half of a binary32.  Widening is exact.
__device__ __forceinline__ float widen_bf16(unsigned short b) {
  return __uint_as_float(static_cast<unsigned>(b) << 16);
}

// Nearest bfloat16 to an fp64 value in ONE rounding, ties to even; subnormals (spacing
// 2^-133) kept, overflow to infinity, any NaN -> 0x7FC0.
// The value is first rounded to binary32 by the hardware conversion, then to bf16 on the bit
// pattern.  Rounding twice differs from rounding once only when the binary32 value sits
// exactly half way between two bf16 values although the fp64 value did not: in that (rare)
// case the pattern is nudged one step towards the fp64 value before the second rounding.
__device__ __forceinline__ unsigned short round_bf16(double x) {
  const float f = static_cast<float>(x);
  unsigned u = __float_as_uint(f);
  if ((u & 0xFFFFu) == 0x8000u) {
    const double back = static_cast<double>(f);
    if (back != x) u += (fabs(x) > fabs(back)) ? 1u : 0xFFFFFFFFu;
  }
  const unsigned r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
  return static_cast<unsigned short>(x != x ? 0x7FC0u : r);
}

// ------------------------------------------------------------------ per-element arithmetic
// Eq. 2 with OuterOptim = SGD with momentum: m' = mu*m + dg ; step = dg + mu*m' (Nesterov)
// or m' (heavy ball) ; G = theta_g - eta*step.  Returns G rounded to fp32 (the value that is
// stored and that the merge below starts from).
// Every product and sum is rounded separately (no fused multiply-add): with decimal
// constants such as 0.9 and 0.7 and fp32 inputs, about one result in 10^4 lies exactly half
// way between two fp32 values before the final rounding, and a fused operation would break
// those ties differently from the plain sequence.
template <bool NESTEROV>
__device__ __forceinline__ float outer_update(float theta_g, float m, float dg, const DevHP& hp,
                                              float* m_new) {
  const double dgd = static_cast<double>(dg);
  const double m1 = hp.mu * static_cast<double>(m) + dgd;
  const double step = NESTEROV ? (dgd + hp.mu * m1) : m1;
  *m_new = static_cast<float>(m1);
  return static_cast<float>(static_cast<double>(theta_g) - hp.eta * step);
}

// d = tau * g with g the change rate of Eq. 4 (send-time minus current local parameters).
__device__ __forceinline__ double drift(float theta_send, float theta_m, const DevHP& hp) {
  return hp.sign * (static_cast<double>(theta_send) - static_cast<double>(theta_m));
}

// MERGE 0: Algorithm 1.  Eq. 7 put into Eq. 8 and multiplied out by tau:
//   theta_m <- G + d + (lambda/(tau*H)) * d*d*Delta,  Delta = G - theta_send.
// MERGE 3: the same with tau == 0 (no overlap): the last term is an exact zero.
// MERGE 1: Eq. 3 blend.  MERGE 2: adopt G.
template <int MERGE>
__device__ __forceinline__ double merge_local_f64(float G, float theta_send, float theta_m, double d,
                                                  const DevHP& hp, float theta_g_prev = 0.0f) {
  const double Gd = static_cast<double>(G);
  if (MERGE == 1) return hp.one_minus_alpha * static_cast<double>(theta_m) + hp.alpha * Gd;
  if (MERGE == 2) return Gd;
  if (MERGE == 3) return Gd + d + 0.0;
  // MERGE 4: the divergence term is the change accumulated before the send,
  // theta^m_{p,t_p} - theta^g_{p,t_p-H} (text after Eq. 6), instead of G - theta^m_{p,t_p}.
  const double Delta = (MERGE == 4) ? static_cast<double>(theta_send) - static_cast<double>(theta_g_prev)
                                    : Gd - static_cast<double>(theta_send);
#if COCODC_EXACT_DIV
  const double corr = hp.lambda * d * d * Delta / hp.tauH;
#else
  const double corr = hp.coef * d * d * Delta;
#endif
  return Gd + d + corr;
}

template <int MERGE>
__device__ __forceinline__ float merge_local(float G, float theta_send, float theta_m, double d,
                                             const DevHP& hp) {
  return static_cast<float>(merge_local_f64<MERGE>(G, theta_send, theta_m, d, hp));
}

// ------------------------------------------------------------------ streaming operations
// Each operation provides, for V = 1 (scalar) and V = 4 (128-bit):
//   Regs<V>           the values loaded for V consecutive elements,
//   load<V>(i)        issues the loads of elements [i, i+V),
//   apply<V>(i, r, a) computes, stores, and accumulates into a[kAcc].

// HAS_SEND false: no send-time record (merge modes 1 and 2 only): the drift and its sums are 0.
template <bool NESTEROV, int MERGE, bool HAS_PG, bool HAS_SEND = true>
struct FusedOp {
  static constexpr int kAcc = 4;
  static constexpr int kVec = 4;       // elements per lane per access (128-bit fp32)
  static constexpr int kLoads = kDepth;  // accesses per stream in flight per lane
  float* theta_m;
  const float* theta_send;
  float* theta_g;
  float* momentum;
  const float* delta_g;
  float* pg;  // may alias delta_g
  DevHP hp;

  template <int V>
  struct Regs {
    typename Vec<V>::type tm, ts, tg, m, dg;
  };

  template <int V>
  __device__ __forceinline__ Regs<V> load(uint64_t i) const {
    Regs<V> r;
    r.tm = load_stream<V>(theta_m + i);
    if (HAS_SEND) r.ts = load_stream<V>(theta_send + i);
    r.tg = load_stream<V>(theta_g + i);
    r.m = load_stream<V>(momentum + i);
    r.dg = load_stream<V>(delta_g + i);
    return r;
  }

  template <int V>
  __device__ __forceinline__ void apply(uint64_t i, const Regs<V>& r, double* a) const {
    typename Vec<V>::type o_tm, o_tg, o_m, o_pg;
#pragma unroll
    for (int k = 0; k < V; ++k) {
      const float tm = lane_get(r.tm, k), tg = lane_get(r.tg, k);
      const float ts = HAS_SEND ? lane_get(r.ts, k) : tm;
      const float m = lane_get(r.m, k), dg = lane_get(r.dg, k);
      float m1;
      const float G = outer_update<NESTEROV>(tg, m, dg, hp, &m1);
      const double d = HAS_SEND ? drift(ts, tm, hp) : 0.0;
      const float tm1 = static_cast<float>(merge_local_f64<MERGE>(G, ts, tm, d, hp, tg));
      const double dgd = static_cast<double>(dg);
      a[0] = fma(dgd, dgd, a[0]);  // exact product: same as a plain multiply-then-add
      a[1] += fabs(dgd);
      if (HAS_SEND) {
        a[2] += d * d;
        a[3] += fabs(d);
      }
      lane_set(o_tm, k, tm1);
      lane_set(o_tg, k, G);
      lane_set(o_m, k, m1);
      if (HAS_PG) lane_set(o_pg, k, tg - tm);  // pseudo-gradient, global minus local
    }
    store_stream<V>(theta_m + i, o_tm);
    store_stream<V>(theta_g + i, o_tg);
    store_stream<V>(momentum + i, o_m);
    if (HAS_PG) store_stream<V>(pg + i, o_pg);
  }
};

template <bool HAS_SEND>
struct PseudoGradOp {
  static constexpr int kAcc = 0;
  static constexpr int kVec = 4;       // elements per lane per access (128-bit fp32)
  static constexpr int kLoads = kDepth;  // accesses per stream in flight per lane
  const float* theta_g;
  const float* theta_m;
  float* pg;
  float* send_out;

  template <int V>
  struct Regs {
    typename Vec<V>::type tg, tm;
  };
  template <int V>
  __device__ __forceinline__ Regs<V> load(uint64_t i) const {
    Regs<V> r;
    r.tg = load_stream<V>(theta_g + i);
    r.tm = load_stream<V>(theta_m + i);
    return r;
  }
  template <int V>
  __device__ __forceinline__ void apply(uint64_t i, const Regs<V>& r, double*) const {
    typename Vec<V>::type o;
#pragma unroll
    for (int k = 0; k < V; ++k) lane_set(o, k, lane_get(r.tg, k) - lane_get(r.tm, k));
    store_stream<V>(pg + i, o);
    if (HAS_SEND) store_stream<V>(send_out + i, r.tm);
  }
};

template <bool NESTEROV>
struct OuterOp {
  static constexpr int kAcc = 0;
  static constexpr int kVec = 4;       // elements per lane per access (128-bit fp32)
  static constexpr int kLoads = kDepth;  // accesses per stream in flight per lane
  float* theta_g;
  float* momentum;
  const float* delta_g;
  DevHP hp;

  template <int V>
  struct Regs {
    typename Vec<V>::type tg, m, dg;
  };
  template <int V>
  __device__ __forceinline__ Regs<V> load(uint64_t i) const {
    Regs<V> r;
    r.tg = load_stream<V>(theta_g + i);
    r.m = load_stream<V>(momentum + i);
    r.dg = load_stream<V>(delta_g + i);
    return r;
  }
  template <int V>
  __device__ __forceinline__ void apply(uint64_t i, const Regs<V>& r, double*) const {
    typename Vec<V>::type o_tg, o_m;
#pragma unroll
    for (int k = 0; k < V; ++k) {
      float m1;
      const float G =
          outer_update<NESTEROV>(lane_get(r.tg, k), lane_get(r.m, k), lane_get(r.dg, k), hp, &m1);
      lane_set(o_tg, k, G);
      lane_set(o_m, k, m1);
    }
    store_stream<V>(theta_g + i, o_tg);
    store_stream<V>(momentum + i, o_m);
  }
};

template <int MERGE, bool HAS_SEND = true>
struct MergeOp {
  static constexpr int kAcc = 0;
  static constexpr int kVec = 4;       // elements per lane per access (128-bit fp32)
  static constexpr int kLoads = kDepth;  // accesses per stream in flight per lane
  float* theta_m;
  const float* theta_send;
  const float* theta_g;
  DevHP hp;

  template <int V>
  struct Regs {
    typename Vec<V>::type tm, ts, tg;
  };
  template <int V>
  __device__ __forceinline__ Regs<V> load(uint64_t i) const {
    Regs<V> r;
    r.tm = load_stream<V>(theta_m + i);
    if (HAS_SEND) r.ts = load_stream<V>(theta_send + i);
    r.tg = load_stream<V>(theta_g + i);
    return r;
  }
  template <int V>
  __device__ __forceinline__ void apply(uint64_t i, const Regs<V>& r, double*) const {
    typename Vec<V>::type o;
#pragma unroll
    for (int k = 0; k < V; ++k) {
      const float tm = lane_get(r.tm, k);
      const float ts = HAS_SEND ? lane_get(r.ts, k) : tm;
      const double d = HAS_SEND ? drift(ts, tm, hp) : 0.0;
      lane_set(o, k, merge_local<MERGE>(lane_get(r.tg, k), ts, tm, d, hp));
    }
    store_stream<V>(theta_m + i, o);
  }
};

// The fused step with bfloat16 local parameters: theta_m, theta_send and the outgoing
// pseudo-gradient are bf16 (2 bytes), theta_g, momentum, delta_g stay fp32: 28 B/param.
template <bool NESTEROV, int MERGE, bool HAS_PG, bool HAS_SEND = true>
struct FusedBf16Op {
  static constexpr int kAcc = 4;
  static constexpr int kVec = 4;       // 128-bit fp32 accesses, 64-bit bf16 accesses (8-wide measured slower)
  static constexpr int kLoads = kDepth;
  unsigned short* theta_m;
  const unsigned short* theta_send;
  float* theta_g;
  float* momentum;
  const float* delta_g;
  unsigned short* pg;
  DevHP hp;

  template <int V>
  struct Regs {
    typename VecU16<V>::type tm, ts;
    typename Vec<V>::type tg, m, dg;
  };

  template <int V>
  __device__ __forceinline__ Regs<V> load(uint64_t i) const {
    Regs<V> r;
    r.tm = load_stream_u16<V>(theta_m + i);
    if (HAS_SEND) r.ts = load_stream_u16<V>(theta_send + i);
    r.tg = load_stream<V>(theta_g + i);
    r.m = load_stream<V>(momentum + i);
    r.dg = load_stream<V>(delta_g + i);
    return r;
  }

  template <int V>
  __device__ __forceinline__ void apply(uint64_t i, const Regs<V>& r, double* a) const {
    typename VecU16<V>::type o_tm, o_pg;
    typename Vec<V>::type o_tg, o_m;
#pragma unroll
    for (int k = 0; k < V; ++k) {
      const float tm = widen_bf16(lane_get(r.tm, k)), tg = lane_get(r.tg, k);
      const float ts = HAS_SEND ? widen_bf16(lane_get(r.ts, k)) : tm;
      const float m = lane_get(r.m, k), dg = lane_get(r.dg, k);
      float m1;
      const float G = outer_update<NESTEROV>(tg, m, dg, hp, &m1);
      const double d = HAS_SEND ? drift(ts, tm, hp) : 0.0;
      const double tm1 = merge_local_f64<MERGE>(G, ts, tm, d, hp, tg);
      const double dgd = static_cast<double>(dg);
      a[0] = fma(dgd, dgd, a[0]);
      a[1] += fabs(dgd);
      if (HAS_SEND) {
        a[2] += d * d;
        a[3] += fabs(d);
      }
      lane_set(o_tm, k, round_bf16(tm1));
      lane_set(o_tg, k, G);
      lane_set(o_m, k, m1);
      if (HAS_PG) lane_set(o_pg, k, round_bf16(static_cast<double>(tg) - static_cast<double>(tm)));
    }
    store_stream_u16<V>(theta_m + i, o_tm);
    store_stream<V>(theta_g + i, o_tg);
    store_stream<V>(momentum + i, o_m);
    if (HAS_PG) store_stream_u16<V>(pg + i, o_pg);
  }
};

template <bool HAS_SEND>
struct PseudoGradBf16Op {
  static constexpr int kAcc = 0;
  static constexpr int kVec = 4;
  static constexpr int kLoads = kDepth;
  const float* theta_g;
  const unsigned short* theta_m;
  unsigned short* pg;
  unsigned short* send_out;

  template <int V>
  struct Regs {
    typename Vec<V>::type tg;
    typename VecU16<V>::type tm;
  };
  template <int V>
  __device__ __forceinline__ Regs<V> load(uint64_t i) const {
    Regs<V> r;
    r.tg = load_stream<V>(theta_g + i);
    r.tm = load_stream_u16<V>(theta_m + i);
    return r;
  }
  template <int V>
  __device__ __forceinline__ void apply(uint64_t i, const Regs<V>& r, double*) const {
    typename VecU16<V>::type o;
#pragma unroll
    for (int k = 0; k < V; ++k) {
      lane_set(o, k, round_bf16(static_cast<double>(lane_get(r.tg, k)) -
                                static_cast<double>(widen_bf16(lane_get(r.tm, k)))));
    }
    store_stream_u16<V>(pg + i, o);
    if (HAS_SEND) store_stream_u16<V>(send_out + i, r.tm);
  }
};

// Sum of squares (NORM 2) or of magnitudes (NORM 1) of any buffer: numerator of Eq. 11.
template <int NORM>
struct ScoreOp {
  static constexpr int kAcc = 1;
  static constexpr int kVec = 4;       // elements per lane per access (128-bit fp32)
  static constexpr int kLoads = kDepth;  // accesses per stream in flight per lane
  const float* x;

  template <int V>
  struct Regs {
    typename Vec<V>::type x;
  };
  template <int V>
  __device__ __forceinline__ Regs<V> load(uint64_t i) const {
    Regs<V> r;
    r.x = load_stream<V>(x + i);
    return r;
  }
  template <int V>
  __device__ __forceinline__ void apply(uint64_t, const Regs<V>& r, double* a) const {
#pragma unroll
    for (int k = 0; k < V; ++k) {
      const double v = static_cast<double>(lane_get(r.x, k));
      if (NORM == 2) {
        a[0] = fma(v, v, a[0]);
      } else {
        a[0] += fabs(v);
      }
    }
  }
};

// ------------------------------------------------------------------ reductions
// Sum over the 64 lanes of a wavefront; the result is valid in lane 0.  Fixed tree.
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
  return v;
}

// Sum of NA values over the workgroup in a fixed order; thread 0 returns the totals in a[].
template <int NA>
__device__ __forceinline__ void block_sum(double* a, double (*lds)[kSums]) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int k = 0; k < NA; ++k) {
    const double s = wave_sum(a[k]);
    if (lane == 0) lds[wave][k] = s;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int k = 0; k < NA; ++k) {
      double s = lds[0][k];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) s += lds[w][k];
      a[k] = s;
    }
  }
  __syncthreads();
}

// ------------------------------------------------------------------ kernels
__global__ void k_write_table(TableChunk chunk, FragRec* dst, int base, int count) {
  const int i = threadIdx.x;
  if (i < count) dst[base + i] = chunk.rec[i];
}

// Walks the tile list with stride gridDim.x.  tbl has K+1 records; tbl[K].slot_begin == T.
#if COCODC_WAVES_PER_EU > 0
#define COCODC_OCCUPANCY __attribute__((amdgpu_waves_per_eu(COCODC_WAVES_PER_EU)))
#else
#define COCODC_OCCUPANCY
#endif
template <class Op, bool VEC>
__global__ __launch_bounds__(kThreads) COCODC_OCCUPANCY void k_walk(const FragRec* __restrict__ tbl, uint64_t T,
                                                    int tile_shift, Op op, double* __restrict__ partials) {
  __shared__ double lds[kWaves][kSums];
  const uint64_t tid = threadIdx.x;
  int p = 0;
  for (uint64_t w = blockIdx.x; w < T; w += gridDim.x) {
    while (w >= tbl[p + 1].slot_begin) ++p;  // uniform; skips empty fragments
    const uint64_t f_off = tbl[p].offset, f_end = f_off + tbl[p].length;
    const uint64_t win = (tbl[p].tile0 + (w - tbl[p].slot_begin)) << tile_shift;
    const uint64_t win_end = win + (uint64_t(1) << tile_shift);
    const uint64_t lo = f_off > win ? f_off : win;
    const uint64_t hi = f_end < win_end ? f_end : win_end;

    double acc[Op::kAcc > 0 ? Op::kAcc : 1];
#pragma unroll
    for (int k = 0; k < (Op::kAcc > 0 ? Op::kAcc : 1); ++k) acc[k] = 0.0;

    if (VEC) {
      constexpr int W = Op::kVec;      // elements per vector access
      constexpr int D = Op::kLoads;    // vector accesses per stream in flight
      uint64_t lo4 = (lo + (W - 1)) & ~uint64_t(W - 1);
      if (lo4 > hi) lo4 = hi;
      uint64_t hi4 = hi & ~uint64_t(W - 1);
      if (hi4 < lo4) hi4 = lo4;
      if (tid < lo4 - lo) {  // unaligned head of the fragment (at most W-1 elements)
        const auto r = op.template load<1>(lo + tid);
        op.template apply<1>(lo + tid, r, acc);
      }
      const uint64_t nvec = (hi4 - lo4) / W;
      for (uint64_t v = tid; v < nvec; v += uint64_t(kThreads) * D) {
        typename Op::template Regs<W> r[D];
#pragma unroll
        for (int k = 0; k < D; ++k) {
          const uint64_t vk = v + uint64_t(k) * kThreads;
          if (vk < nvec) r[k] = op.template load<W>(lo4 + vk * W);
        }
#pragma unroll
        for (int k = 0; k < D; ++k) {
          const uint64_t vk = v + uint64_t(k) * kThreads;
          if (vk < nvec) op.template apply<W>(lo4 + vk * W, r[k], acc);
        }
      }
      if (tid < hi - hi4) {  // unaligned tail (at most W-1 elements)
        const auto r = op.template load<1>(hi4 + tid);
        op.template apply<1>(hi4 + tid, r, acc);
      }
    } else {
      for (uint64_t i = lo + tid; i < hi; i += kThreads) {
        const auto r = op.template load<1>(i);
        op.template apply<1>(i, r, acc);
      }
    }

    if (Op::kAcc > 0) {
      block_sum<(Op::kAcc > 0 ? Op::kAcc : 1)>(acc, lds);
      if (tid == 0) {
#pragma unroll
        for (int k = 0; k < Op::kAcc; ++k) partials[w * kSums + k] = acc[k];
      }
    }
  }
}

// One workgroup per fragment: adds that fragment's tile partials (thread t takes slots
// t, t+256, ... in ascending order, then the fixed workgroup tree) and evaluates Eq. 11.
//   which: index (0..3) of the sum that feeds R;  l2: take the square root of it.
__global__ __launch_bounds__(kThreads) void k_finalize(const FragRec* __restrict__ tbl,
                                                        const double* __restrict__ partials, int n_acc,
                                                        int which, int l2, double* __restrict__ R_out,
                                                        double* __restrict__ sums_out, int sums_stride) {
  __shared__ double lds[kWaves][kSums];
  const int p = blockIdx.x;
  const uint64_t s0 = tbl[p].slot_begin, s1 = tbl[p + 1].slot_begin;
  double acc[kSums] = {0.0, 0.0, 0.0, 0.0};
  for (uint64_t s = s0 + threadIdx.x; s < s1; s += kThreads) {
#pragma unroll
    for (int k = 0; k < kSums; ++k) {
      if (k < n_acc) acc[k] += partials[s * kSums + k];
    }
  }
  block_sum<kSums>(acc, lds);
  if (threadIdx.x == 0) {
    const int64_t I_p = tbl[p].I_p;
    const double s = acc[which];
    const double norm = l2 ? sqrt(s) : s;
    R_out[p] = (I_p <= 0) ? __builtin_huge_val() : norm / static_cast<double>(I_p);
    if (sums_out) {
      for (int k = 0; k < sums_stride; ++k) sums_out[p * sums_stride + k] = acc[k];
    }
  }
}

// Algorithm 2 applied `n` times without replacement == the first n entries of the order
// (class, -R, p) with class 0 = not synchronised for >= H steps, 1 = has a number as
// score, 2 = NaN score.  Every fragment counts how many fragments precede it.
__global__ __launch_bounds__(kThreads) void k_select(const FragRec* __restrict__ tbl, int K,
                                                      const double* __restrict__ R, int64_t t_g,
                                                      int64_t H, int n, int* __restrict__ sel,
                                                      int* __restrict__ n_sel) {
  __shared__ double sR[COCODC_MAX_FRAGMENTS];
  __shared__ unsigned char sC[COCODC_MAX_FRAGMENTS];
  for (int p = threadIdx.x; p < K; p += kThreads) {
    const double r = R[p];
    const bool overdue = (t_g - tbl[p].t_b) >= H;
    sR[p] = r;
    sC[p] = overdue ? 0 : (r != r ? 2 : 1);
  }
  __syncthreads();
  for (int p = threadIdx.x; p < K; p += kThreads) {
    const int cp = sC[p];
    const double rp = sR[p];
    int rank = 0;
    for (int q = 0; q < K; ++q) {
      const int cq = sC[q];
      bool before;
      if (cq != cp) {
        before = cq < cp;
      } else if (cp == 1) {
        const double rq = sR[q];
        before = (rq > rp) || (rq == rp && q < p);
      } else {
        before = q < p;
      }
      rank += before ? 1 : 0;
    }
    if (rank < n) sel[rank] = p;
  }
  if (threadIdx.x == 0) *n_sel = n;
}

// Same priority order, cut by a byte budget: fragments are taken in rank order while their sizes
// (FragRec::length of the group records, in bytes) still fit; the first that does not fit ends
// the selection.
__global__ __launch_bounds__(kThreads) void k_select_bytes(const FragRec* __restrict__ tbl, int K,
                                                            const double* __restrict__ R, int64_t t_g,
                                                            int64_t H, unsigned long long byte_budget,
                                                            int* __restrict__ sel, int* __restrict__ n_sel) {
  __shared__ double sR[COCODC_MAX_FRAGMENTS];
  __shared__ unsigned char sC[COCODC_MAX_FRAGMENTS];
  __shared__ int sOrder[COCODC_MAX_FRAGMENTS];
  for (int p = threadIdx.x; p < K; p += kThreads) {
    const double r = R[p];
    const bool overdue = (t_g - tbl[p].t_b) >= H;
    sR[p] = r;
    sC[p] = overdue ? 0 : (r != r ? 2 : 1);
  }
  __syncthreads();
  for (int p = threadIdx.x; p < K; p += kThreads) {
    const int cp = sC[p];
    const double rp = sR[p];
    int rank = 0;
    for (int q = 0; q < K; ++q) {
      const int cq = sC[q];
      bool before;
      if (cq != cp) {
        before = cq < cp;
      } else if (cp == 1) {
        const double rq = sR[q];
        before = (rq > rp) || (rq == rp && q < p);
      } else {
        before = q < p;
      }
      rank += before ? 1 : 0;
    }
    sOrder[rank] = p;  // ranks are a permutation of 0..K-1
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned long long left = byte_budget;
    int n = 0;
    for (int r = 0; r < K; ++r) {
      const int p = sOrder[r];
      const unsigned long long need = tbl[p].length;
      if (need > left) break;
      left -= need;
      sel[n++] = p;
    }
    *n_sel = n;
  }
}

__global__ void k_fill_inf(double* R, int K) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p < K) R[p] = __builtin_huge_val();
}

// ------------------------------------------------------------------ host side
thread_local int g_last_hip_error = 0;
int g_blocks_per_cu = 0;

int hip_fail(hipError_t e) {
  g_last_hip_error = static_cast<int>(e);
  return COCODC_ERR_HIP;
}

#define HIP_TRY(expr)                          \
  do {                                         \
    hipError_t e_ = (expr);                    \
    if (e_ != hipSuccess) return hip_fail(e_); \
  } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

uint64_t max_tiles(int32_t S, uint64_t n_total) {
  // a segment of length L overlaps at most (L >> tile_shift) + 2 windows
  return (n_total >> tile_shift_for(n_total)) + 2 * static_cast<uint64_t>(S) + 1;
}

// Device workspace: S+1 segment records (the tile walk), K+1 group records (one per fragment:
// its range of tile slots, I_p, t_b), then one slot of kSums doubles per tile.
struct WorkspaceView {
  FragRec* table;    // S + 1 segment records; table[S].slot_begin == number of tiles
  FragRec* groups;   // K + 1 fragment records; only slot_begin, I_p, t_b are meaningful
  double* partials;  // max_tiles * kSums
};

size_t table_bytes(int32_t S, int32_t K) {
  return align_up(sizeof(FragRec) * (static_cast<size_t>(S) + 1 + static_cast<size_t>(K) + 1), 256);
}

size_t workspace_bytes(int32_t S, int32_t K, uint64_t n_total) {
  return table_bytes(S, K) + align_up(max_tiles(S, n_total) * kSums * sizeof(double), 256);
}

WorkspaceView view(void* ws, int32_t S, int32_t K) {
  char* b = static_cast<char*>(ws);
  FragRec* t = reinterpret_cast<FragRec*>(b);
  return WorkspaceView{t, t + S + 1, reinterpret_cast<double*>(b + table_bytes(S, K))};
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

struct Span {
  const void* p;
  size_t bytes;
};
bool overlap(const Span& a, const Span& b) {
  if (!a.p || !b.p || a.bytes == 0 || b.bytes == 0) return false;
  const uintptr_t a0 = reinterpret_cast<uintptr_t>(a.p), b0 = reinterpret_cast<uintptr_t>(b.p);
  return a0 < b0 + b.bytes && b0 < a0 + a.bytes;
}

// Host-side plan of one call: the records to upload and the number of tiles.
struct Plan {
  std::vector<FragRec> recs;  // S+1 segment records followed by K+1 group records
  int32_t S = 0, K = 0;
  int tile_shift = kTileShiftLarge;
  uint64_t T = 0;
};

// Validates a segment list (every segment inside n_total, no two overlapping, fragment ids in
// [0, K)) and lays out the tile list: the segments of fragment 0 in the order given, then those
// of fragment 1, ...  so that each fragment owns one contiguous range of tile slots.
int plan_segments(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total, const int64_t* I_p,
                  const int64_t* t_b, Plan* plan) {
  if (!segs && S > 0) return COCODC_ERR_NULL;
  if (K < 1 || K > COCODC_MAX_FRAGMENTS || S < 0 || S > COCODC_MAX_SEGMENTS) return COCODC_ERR_RANGE;
  if (n_total > COCODC_MAX_ELEMENTS) return COCODC_ERR_RANGE;  // keeps every byte count far from overflow
  std::vector<std::pair<uint64_t, uint64_t>> sorted;
  sorted.reserve(S);
  for (int32_t i = 0; i < S; ++i) {
    if (segs[i].fragment < 0 || segs[i].fragment >= K) return COCODC_ERR_RANGE;
    if (segs[i].offset > n_total || segs[i].length > n_total - segs[i].offset) return COCODC_ERR_RANGE;
    if (segs[i].length) sorted.emplace_back(segs[i].offset, segs[i].offset + segs[i].length);
  }
  std::sort(sorted.begin(), sorted.end());
  for (size_t i = 1; i < sorted.size(); ++i) {
    if (sorted[i].first < sorted[i - 1].second) return COCODC_ERR_RANGE;  // segments overlap
  }
  std::vector<int32_t> order(static_cast<size_t>(S));
  for (int32_t i = 0; i < S; ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(),
                   [&](int32_t a, int32_t b) { return segs[a].fragment < segs[b].fragment; });
  plan->S = S;
  plan->K = K;
  plan->tile_shift = tile_shift_for(n_total);
  const int sh = plan->tile_shift;
  plan->recs.assign(static_cast<size_t>(S) + 1 + static_cast<size_t>(K) + 1, FragRec{});
  FragRec* seg_rec = plan->recs.data();
  FragRec* grp_rec = plan->recs.data() + S + 1;
  uint64_t slot = 0;
  int32_t next_group = 0;
  for (int32_t j = 0; j < S; ++j) {
    const cocodc_segment_t& sg = segs[order[j]];
    while (next_group <= sg.fragment) grp_rec[next_group++].slot_begin = slot;
    FragRec& r = seg_rec[j];
    r.offset = sg.offset;
    r.length = sg.length;
    r.slot_begin = slot;
    r.tile0 = r.offset >> sh;
    if (r.length) slot += ((r.offset + r.length - 1) >> sh) - r.tile0 + 1;
  }
  while (next_group <= K) grp_rec[next_group++].slot_begin = slot;
  seg_rec[S].slot_begin = slot;
  for (int32_t p = 0; p < K; ++p) {
    grp_rec[p].I_p = I_p ? I_p[p] : 0;
    grp_rec[p].t_b = t_b ? t_b[p] : 0;
  }
  plan->T = slot;
  return COCODC_OK;
}

// Contiguous fragments: fragment p is the single segment frags[p].
int plan_table(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total, const int64_t* I_p,
               const int64_t* t_b, Plan* plan) {
  if (!frags) return COCODC_ERR_NULL;
  if (K < 1 || K > COCODC_MAX_FRAGMENTS) return COCODC_ERR_RANGE;
  std::vector<cocodc_segment_t> segs(static_cast<size_t>(K));
  for (int32_t p = 0; p < K; ++p) segs[p] = cocodc_segment_t{frags[p].offset, frags[p].length, p, 0};
  return plan_segments(segs.data(), K, K, n_total, I_p, t_b, plan);
}

int upload_table(const std::vector<FragRec>& recs, FragRec* dst, hipStream_t s) {
  const int n = static_cast<int>(recs.size());
  for (int base = 0; base < n; base += kTableChunk) {
    TableChunk c;
    const int count = std::min(kTableChunk, n - base);
    std::memset(&c, 0, sizeof(c));
    std::memcpy(c.rec, recs.data() + base, sizeof(FragRec) * count);
    hipLaunchKernelGGL(k_write_table, dim3(1), dim3(kTableChunk), 0, s, c, dst, base, count);
    HIP_TRY(hipGetLastError());
  }
  return COCODC_OK;
}

int check_workspace(void* ws, size_t bytes, int32_t S, int32_t K, uint64_t n_total) {
  if (!ws) return COCODC_ERR_NULL;
  if (!aligned(ws, 256)) return COCODC_ERR_ALIGN;
  if (bytes < workspace_bytes(S, K, n_total)) return COCODC_ERR_WORKSPACE;
  return COCODC_OK;
}

int check_hparams(const cocodc_hparams_t* hp) {
  if (!hp) return COCODC_ERR_NULL;
  if (hp->tau < 0 || hp->H < 1) return COCODC_ERR_RANGE;
  if (hp->nesterov != 0 && hp->nesterov != 1) return COCODC_ERR_RANGE;
  if (hp->drift_sign != 1 && hp->drift_sign != -1) return COCODC_ERR_RANGE;
  if (hp->score_src != 0 && hp->score_src != 1) return COCODC_ERR_RANGE;
  if (hp->norm_kind != 1 && hp->norm_kind != 2) return COCODC_ERR_RANGE;
  if (hp->merge_mode < 0 || hp->merge_mode > 2) return COCODC_ERR_RANGE;
  if (hp->delta_src != 0 && hp->delta_src != 1) return COCODC_ERR_RANGE;
  if (!std::isfinite(hp->lambda) || !std::isfinite(hp->eta) || !std::isfinite(hp->mu) ||
      !std::isfinite(hp->alpha))
    return COCODC_ERR_NONFINITE;
  return COCODC_OK;
}

// Kernel variant of the merge: 0/1/2 as merge_mode, 3 = delay compensation with tau == 0,
// 4 = delay compensation with the accumulated-change reading of the divergence term.
int merge_variant(const cocodc_hparams_t& hp) {
  if (hp.merge_mode != 0) return hp.merge_mode;
  if (hp.tau < 1) return 3;
  return hp.delta_src == 1 ? 4 : 0;
}

DevHP to_dev(const cocodc_hparams_t& hp) {
  DevHP d;
  d.mu = hp.mu;
  d.eta = hp.eta;
  d.sign = static_cast<double>(hp.drift_sign);
  d.tauH = hp.tau >= 1 ? static_cast<double>(hp.tau) * static_cast<double>(hp.H) : 1.0;
  d.lambda = hp.tau >= 1 ? hp.lambda : 0.0;
  d.coef = d.lambda / d.tauH;
  d.alpha = hp.alpha;
  d.one_minus_alpha = 1.0 - hp.alpha;
  return d;
}

int device_cus() {
  static std::mutex mu;
  static int cached[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  std::lock_guard<std::mutex> lock(mu);
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

unsigned grid_for(uint64_t T) {
  uint64_t g = T;
  if (g_blocks_per_cu > 0) g = std::min<uint64_t>(T, static_cast<uint64_t>(device_cus()) * g_blocks_per_cu);
  return static_cast<unsigned>(std::min<uint64_t>(g, 0x7fffffffu));
}

template <class Op>
int launch_walk(bool vec, const FragRec* tbl, uint64_t T, int tile_shift, const Op& op, double* partials,
                hipStream_t s) {
  if (T == 0) return COCODC_OK;
  const dim3 grid(grid_for(T)), block(kThreads);
  if (vec) {
    hipLaunchKernelGGL((k_walk<Op, true>), grid, block, 0, s, tbl, T, tile_shift, op, partials);
  } else {
    hipLaunchKernelGGL((k_walk<Op, false>), grid, block, 0, s, tbl, T, tile_shift, op, partials);
  }
  HIP_TRY(hipGetLastError());
  return COCODC_OK;
}

bool all_aligned16(std::initializer_list<const void*> ps) {
  for (const void* p : ps) {
    if (p && !aligned(p, 16)) return false;
  }
  return true;
}
bool all_aligned4(std::initializer_list<const void*> ps) {
  for (const void* p : ps) {
    if (p && !aligned(p, 4)) return false;
  }
  return true;
}

// ---- kernel timer (measurement aid) ----
struct Profiler {
  std::mutex mu;
  std::vector<hipEvent_t> start, stop;
  int used = 0;
  bool on = false;
} g_prof;

template <bool NESTEROV, int MERGE>
int launch_fused(bool vec, const FragRec* tbl, uint64_t T, int sh, float* tm, const float* ts, float* tg,
                 float* m, const float* dg, float* pg, const DevHP& hp, double* partials, hipStream_t s) {
  if (MERGE == 1 || MERGE == 2) {
    if (!ts) {  // the blend and the plain replacement never look at the send-time record
      if (pg) {
        FusedOp<NESTEROV, (MERGE == 1 || MERGE == 2) ? MERGE : 1, true, false> op{tm, nullptr, tg, m, dg, pg, hp};
        return launch_walk(vec, tbl, T, sh, op, partials, s);
      }
      FusedOp<NESTEROV, (MERGE == 1 || MERGE == 2) ? MERGE : 1, false, false> op{tm, nullptr, tg, m, dg, nullptr, hp};
      return launch_walk(vec, tbl, T, sh, op, partials, s);
    }
  }
  if (pg) {
    FusedOp<NESTEROV, MERGE, true> op{tm, ts, tg, m, dg, pg, hp};
    return launch_walk(vec, tbl, T, sh, op, partials, s);
  }
  FusedOp<NESTEROV, MERGE, false> op{tm, ts, tg, m, dg, nullptr, hp};
  return launch_walk(vec, tbl, T, sh, op, partials, s);
}

template <bool NESTEROV>
int launch_fused_m(int merge, bool vec, const FragRec* tbl, uint64_t T, int sh, float* tm, const float* ts,
                   float* tg, float* m, const float* dg, float* pg, const DevHP& hp, double* partials,
                   hipStream_t s) {
  switch (merge) {
    case 0: return launch_fused<NESTEROV, 0>(vec, tbl, T, sh, tm, ts, tg, m, dg, pg, hp, partials, s);
    case 1: return launch_fused<NESTEROV, 1>(vec, tbl, T, sh, tm, ts, tg, m, dg, pg, hp, partials, s);
    case 2: return launch_fused<NESTEROV, 2>(vec, tbl, T, sh, tm, ts, tg, m, dg, pg, hp, partials, s);
    case 4: return launch_fused<NESTEROV, 4>(vec, tbl, T, sh, tm, ts, tg, m, dg, pg, hp, partials, s);
    default: return launch_fused<NESTEROV, 3>(vec, tbl, T, sh, tm, ts, tg, m, dg, pg, hp, partials, s);
  }
}

template <bool NESTEROV, int MERGE>
int launch_fused_bf16(bool vec, const FragRec* tbl, uint64_t T, int sh, unsigned short* tm, const unsigned short* ts,
                      float* tg, float* m, const float* dg, unsigned short* pg, const DevHP& hp, double* partials,
                      hipStream_t s) {
  if (MERGE == 1 || MERGE == 2) {
    if (!ts) {
      if (pg) {
        FusedBf16Op<NESTEROV, (MERGE == 1 || MERGE == 2) ? MERGE : 1, true, false> op{tm, nullptr, tg, m, dg, pg, hp};
        return launch_walk(vec, tbl, T, sh, op, partials, s);
      }
      FusedBf16Op<NESTEROV, (MERGE == 1 || MERGE == 2) ? MERGE : 1, false, false> op{tm, nullptr, tg, m, dg, nullptr, hp};
      return launch_walk(vec, tbl, T, sh, op, partials, s);
    }
  }
  if (pg) {
    FusedBf16Op<NESTEROV, MERGE, true> op{tm, ts, tg, m, dg, pg, hp};
    return launch_walk(vec, tbl, T, sh, op, partials, s);
  }
  FusedBf16Op<NESTEROV, MERGE, false> op{tm, ts, tg, m, dg, nullptr, hp};
  return launch_walk(vec, tbl, T, sh, op, partials, s);
}

template <bool NESTEROV>
int launch_fused_bf16_m(int merge, bool vec, const FragRec* tbl, uint64_t T, int sh, unsigned short* tm,
                        const unsigned short* ts, float* tg, float* m, const float* dg, unsigned short* pg,
                        const DevHP& hp, double* partials, hipStream_t s) {
  switch (merge) {
    case 0: return launch_fused_bf16<NESTEROV, 0>(vec, tbl, T, sh, tm, ts, tg, m, dg, pg, hp, partials, s);
    case 1: return launch_fused_bf16<NESTEROV, 1>(vec, tbl, T, sh, tm, ts, tg, m, dg, pg, hp, partials, s);
    case 2: return launch_fused_bf16<NESTEROV, 2>(vec, tbl, T, sh, tm, ts, tg, m, dg, pg, hp, partials, s);
    case 4: return launch_fused_bf16<NESTEROV, 4>(vec, tbl, T, sh, tm, ts, tg, m, dg, pg, hp, partials, s);
    default: return launch_fused_bf16<NESTEROV, 3>(vec, tbl, T, sh, tm, ts, tg, m, dg, pg, hp, partials, s);
  }
}

}  // namespace

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
  if (int rc = upload_table(pl.recs, v.table, s)) return rc;
  const bool vec = all_aligned16({theta_g_snap, theta_m, delta_m_out, theta_m_send_out});
  if (theta_m_send_out) {
    PseudoGradOp<true> op{theta_g_snap, theta_m, delta_m_out, theta_m_send_out};
    return launch_walk(vec, v.table, pl.T, pl.tile_shift, op, v.partials, s);
  }
  PseudoGradOp<false> op{theta_g_snap, theta_m, delta_m_out, nullptr};
  return launch_walk(vec, v.table, pl.T, pl.tile_shift, op, v.partials, s);
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
  if (int rc = upload_table(pl.recs, v.table, s)) return rc;
  const bool vec = all_aligned16({theta_g, momentum, delta_g});
  const DevHP d = to_dev(*hp);
  if (hp->nesterov) {
    OuterOp<true> op{theta_g, momentum, delta_g, d};
    return launch_walk(vec, v.table, pl.T, pl.tile_shift, op, v.partials, s);
  }
  OuterOp<false> op{theta_g, momentum, delta_g, d};
  return launch_walk(vec, v.table, pl.T, pl.tile_shift, op, v.partials, s);
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
  if (int rc = upload_table(pl.recs, v.table, s)) return rc;
  const bool vec = all_aligned16({theta_m, theta_m_send, theta_g});
  const DevHP d = to_dev(*hp);
  switch (merge_variant(*hp)) {
    case 0: {
      MergeOp<0> op{theta_m, theta_m_send, theta_g, d};
      return launch_walk(vec, v.table, pl.T, pl.tile_shift, op, v.partials, s);
    }
    case 1: {
      MergeOp<1, false> op{theta_m, nullptr, theta_g, d};
      return launch_walk(vec, v.table, pl.T, pl.tile_shift, op, v.partials, s);
    }
    case 2: {
      MergeOp<2, false> op{theta_m, nullptr, theta_g, d};
      return launch_walk(vec, v.table, pl.T, pl.tile_shift, op, v.partials, s);
    }
    default: {
      MergeOp<3> op{theta_m, theta_m_send, theta_g, d};
      return launch_walk(vec, v.table, pl.T, pl.tile_shift, op, v.partials, s);
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
  if (int rc = upload_table(pl.recs, v.table, s)) return rc;
  const bool vec = aligned(x, 16);
  int rc;
  if (norm_kind == 2) {
    ScoreOp<2> op{x};
    rc = launch_walk(vec, v.table, pl.T, pl.tile_shift, op, v.partials, s);
  } else {
    ScoreOp<1> op{x};
    rc = launch_walk(vec, v.table, pl.T, pl.tile_shift, op, v.partials, s);
  }
  if (rc) return rc;
  hipLaunchKernelGGL(k_finalize, dim3(K), dim3(kThreads), 0, s, v.groups, v.partials, 1, 0,
                     norm_kind == 2 ? 1 : 0, R_out, sum_out, 1);
  HIP_TRY(hipGetLastError());
  return COCODC_OK;
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
  if (int rc = upload_table(pl.recs, v.table, s)) return rc;
  hipLaunchKernelGGL(k_select, dim3(1), dim3(kThreads), 0, s, v.groups, K, R, t_g, static_cast<int64_t>(H),
                     n, sel_out, n_sel_out);
  HIP_TRY(hipGetLastError());
  return COCODC_OK;
}

static int sync_step_impl(Plan& pl, int32_t K, uint64_t n_total, float* theta_m, const float* theta_m_send,
                          float* theta_g, float* momentum, const float* delta_g, float* delta_m_out, int64_t t_g,
                          int32_t budget, const cocodc_hparams_t* hp, double* R_out, int32_t* sel_out,
                          int32_t* n_sel_out, double* sums_out, void* workspace, size_t workspace_bytes_,
                          void* stream) {
  if (int rc = check_workspace(workspace, workspace_bytes_, pl.S, K, n_total)) return rc;
  const int n = budget < K ? budget : K;
  const size_t nb = n_total * sizeof(float);
  const Span sp[] = {{theta_m, nb},     {theta_m_send, nb},           {theta_g, nb},
                     {momentum, nb},    {delta_g, nb},                {delta_m_out, nb},
                     {R_out, sizeof(double) * K}, {sel_out, sizeof(int32_t) * n}, {n_sel_out, sizeof(int32_t)},
                     {sums_out, sizeof(double) * 4 * K}, {workspace, workspace_bytes_}};
  const int ns = static_cast<int>(sizeof(sp) / sizeof(sp[0]));
  for (int i = 0; i < ns; ++i) {
    for (int j = i + 1; j < ns; ++j) {
      if (i == 4 && j == 5 && delta_m_out == delta_g) continue;  // in-place pseudo-gradient
      if (overlap(sp[i], sp[j])) return COCODC_ERR_ALIAS;
    }
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  WorkspaceView v = view(workspace, pl.S, K);
  if (int rc = upload_table(pl.recs, v.table, s)) return rc;
  const bool vec = all_aligned16({theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out});
  const DevHP d = to_dev(*hp);

  int slot = -1;
  {
    std::lock_guard<std::mutex> lock(g_prof.mu);
    if (g_prof.on && g_prof.used < static_cast<int>(g_prof.start.size())) slot = g_prof.used++;
  }
  if (slot >= 0) HIP_TRY(hipEventRecord(g_prof.start[slot], s));
  int rc = hp->nesterov ? launch_fused_m<true>(merge_variant(*hp), vec, v.table, pl.T, pl.tile_shift, theta_m, theta_m_send, theta_g,
                                               momentum, delta_g, delta_m_out, d, v.partials, s)
                        : launch_fused_m<false>(merge_variant(*hp), vec, v.table, pl.T, pl.tile_shift, theta_m, theta_m_send,
                                                theta_g, momentum, delta_g, delta_m_out, d, v.partials, s);
  if (slot >= 0) HIP_TRY(hipEventRecord(g_prof.stop[slot], s));
  if (rc) return rc;

  const int which = (hp->score_src ? 2 : 0) + (hp->norm_kind == 2 ? 0 : 1);
  hipLaunchKernelGGL(k_finalize, dim3(K), dim3(kThreads), 0, s, v.groups, v.partials, kSums, which,
                     hp->norm_kind == 2 ? 1 : 0, R_out, sums_out, kSums);
  HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(k_select, dim3(1), dim3(kThreads), 0, s, v.groups, K, R_out, t_g,
                     static_cast<int64_t>(hp->H), n, sel_out, n_sel_out);
  HIP_TRY(hipGetLastError());
  return COCODC_OK;
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

int cocodc_pseudograd_bf16(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total,
                           const float* theta_g_snap, const uint16_t* theta_m, uint16_t* delta_m_out,
                           uint16_t* theta_m_send_out, void* workspace, size_t workspace_bytes_, void* stream) {
  if (!theta_g_snap || !theta_m || !delta_m_out) return COCODC_ERR_NULL;
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
  if (int rc = upload_table(pl.recs, v.table, s)) return rc;
  const bool vec = all_aligned16({theta_g_snap, theta_m, delta_m_out, theta_m_send_out});
  if (theta_m_send_out) {
    PseudoGradBf16Op<true> op{theta_g_snap, theta_m, delta_m_out, theta_m_send_out};
    return launch_walk(vec, v.table, pl.T, pl.tile_shift, op, v.partials, s);
  }
  PseudoGradBf16Op<false> op{theta_g_snap, theta_m, delta_m_out, nullptr};
  return launch_walk(vec, v.table, pl.T, pl.tile_shift, op, v.partials, s);
}

int cocodc_sync_step_bf16(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total, uint16_t* theta_m,
                          const uint16_t* theta_m_send, float* theta_g, float* momentum, const float* delta_g,
                          uint16_t* delta_m_out, const int64_t* I_p, const int64_t* t_b, int64_t t_g,
                          int32_t budget, const cocodc_hparams_t* hp, double* R_out, int32_t* sel_out,
                          int32_t* n_sel_out, double* sums_out, void* workspace, size_t workspace_bytes_,
                          void* stream) {
  if (!theta_m || !theta_g || !momentum || !delta_g) return COCODC_ERR_NULL;
  if (!I_p || !t_b || !R_out || !sel_out || !n_sel_out) return COCODC_ERR_NULL;
  if (!all_aligned4({theta_g, momentum, delta_g, sel_out, n_sel_out})) return COCODC_ERR_ALIGN;
  if (!aligned(theta_m, 2) || !aligned(theta_m_send, 2) || !aligned(delta_m_out, 2)) return COCODC_ERR_ALIGN;
  if (!aligned(R_out, 8) || !aligned(sums_out, 8)) return COCODC_ERR_ALIGN;
  if (int rc = check_hparams(hp)) return rc;
  if (!theta_m_send && (hp->merge_mode == 0 || hp->score_src == 1)) return COCODC_ERR_NULL;
  if (budget < 0) return COCODC_ERR_RANGE;
  Plan pl;
  if (int rc = plan_table(frags, K, n_total, I_p, t_b, &pl)) return rc;
  if (int rc = check_workspace(workspace, workspace_bytes_, pl.S, K, n_total)) return rc;
  const int n = budget < K ? budget : K;
  const Span sp[] = {{theta_m, n_total * 2},      {theta_m_send, n_total * 2},    {theta_g, n_total * 4},
                     {momentum, n_total * 4},     {delta_g, n_total * 4},         {delta_m_out, n_total * 2},
                     {R_out, sizeof(double) * K}, {sel_out, sizeof(int32_t) * n}, {n_sel_out, sizeof(int32_t)},
                     {sums_out, sizeof(double) * 4 * K}, {workspace, workspace_bytes_}};
  const int ns = static_cast<int>(sizeof(sp) / sizeof(sp[0]));
  for (int i = 0; i < ns; ++i) {
    for (int j = i + 1; j < ns; ++j) {
      if (overlap(sp[i], sp[j])) return COCODC_ERR_ALIAS;
    }
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  WorkspaceView v = view(workspace, pl.S, K);
  if (int rc = upload_table(pl.recs, v.table, s)) return rc;
  const bool vec = all_aligned16({theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out});
  const DevHP d = to_dev(*hp);
  int slot = -1;
  {
    std::lock_guard<std::mutex> lock(g_prof.mu);
    if (g_prof.on && g_prof.used < static_cast<int>(g_prof.start.size())) slot = g_prof.used++;
  }
  if (slot >= 0) HIP_TRY(hipEventRecord(g_prof.start[slot], s));
  int rc = hp->nesterov ? launch_fused_bf16_m<true>(merge_variant(*hp), vec, v.table, pl.T, pl.tile_shift, theta_m, theta_m_send,
                                                    theta_g, momentum, delta_g, delta_m_out, d, v.partials, s)
                        : launch_fused_bf16_m<false>(merge_variant(*hp), vec, v.table, pl.T, pl.tile_shift, theta_m, theta_m_send,
                                                     theta_g, momentum, delta_g, delta_m_out, d, v.partials, s);
  if (slot >= 0) HIP_TRY(hipEventRecord(g_prof.stop[slot], s));
  if (rc) return rc;
  const int which = (hp->score_src ? 2 : 0) + (hp->norm_kind == 2 ? 0 : 1);
  hipLaunchKernelGGL(k_finalize, dim3(K), dim3(kThreads), 0, s, v.groups, v.partials, kSums, which,
                     hp->norm_kind == 2 ? 1 : 0, R_out, sums_out, kSums);
  HIP_TRY(hipGetLastError());
  hipLaunchKernelGGL(k_select, dim3(1), dim3(kThreads), 0, s, v.groups, K, R_out, t_g,
                     static_cast<int64_t>(hp->H), n, sel_out, n_sel_out);
  HIP_TRY(hipGetLastError());
  return COCODC_OK;
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
  for (int32_t p = 0; p < K; ++p) pl.recs[static_cast<size_t>(pl.S) + 1 + p].length = frag_bytes[p];
  hipStream_t s = static_cast<hipStream_t>(stream);
  WorkspaceView v = view(workspace, pl.S, K);
  if (int rc = upload_table(pl.recs, v.table, s)) return rc;
  hipLaunchKernelGGL(k_select_bytes, dim3(1), dim3(kThreads), 0, s, v.groups, K, R, t_g, static_cast<int64_t>(H),
                     static_cast<unsigned long long>(byte_budget), sel_out, n_sel_out);
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

// ---------------------------------------------------------------- Sec. 3.2 loop
}  // extern "C"

struct cocodc_loop {
  std::vector<cocodc_fragment_t> frags;
  uint64_t n_total = 0;
  cocodc_hparams_t hp{};
  double gamma = 1.0, T_c = 1.0, T_s = 1.0;
  int64_t N = 1, h = 1;
  std::vector<int64_t> t_b, I_p, in_flight;
};

namespace {
int replan(cocodc_loop* L) {
  int64_t N = 0, h = 0;
  if (int rc = cocodc_sync_plan(static_cast<int32_t>(L->frags.size()), L->hp.H, L->gamma, L->T_c, L->T_s, &N, &h))
    return rc;
  L->N = N;
  L->h = h < 1 ? 1 : h;  // more syncs than steps: at most one send per step
  return COCODC_OK;
}
}  // namespace

extern "C" {

int cocodc_loop_create(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total,
                       const cocodc_hparams_t* hp, double gamma, double T_c, double T_s,
                       cocodc_loop_t** loop_out) {
  if (!loop_out) return COCODC_ERR_NULL;
  *loop_out = nullptr;
  if (int rc = check_hparams(hp)) return rc;
  Plan pl;
  if (int rc = plan_table(frags, K, n_total, nullptr, nullptr, &pl)) return rc;
  cocodc_loop* L = new cocodc_loop();
  L->frags.assign(frags, frags + K);
  L->n_total = n_total;
  L->hp = *hp;
  L->gamma = gamma;
  L->T_c = T_c;
  L->T_s = T_s;
  L->t_b.assign(K, 0);
  L->I_p.assign(K, 0);
  L->in_flight.assign(K, -1);
  if (int rc = replan(L)) {
    delete L;
    return rc;
  }
  *loop_out = L;
  return COCODC_OK;
}

void cocodc_loop_destroy(cocodc_loop_t* loop) { delete loop; }

int cocodc_loop_reset_scores(cocodc_loop_t* loop, double* R, void* stream) {
  if (!loop || !R) return COCODC_ERR_NULL;
  if (!aligned(R, 8)) return COCODC_ERR_ALIGN;
  const int K = static_cast<int>(loop->frags.size());
  hipLaunchKernelGGL(k_fill_inf, dim3((K + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream), R, K);
  HIP_TRY(hipGetLastError());
  return COCODC_OK;
}

int cocodc_loop_observe(cocodc_loop_t* loop, double T_c_sample, double T_s_sample, double beta) {
  if (!loop) return COCODC_ERR_NULL;
  if (std::isnan(T_c_sample) || std::isnan(T_s_sample) || std::isnan(beta)) return COCODC_ERR_NONFINITE;
  if (!(T_c_sample > 0.0) || !(T_s_sample > 0.0) || std::isinf(T_c_sample) || std::isinf(T_s_sample) ||
      beta < 0.0 || beta > 1.0)
    return COCODC_ERR_RANGE;
  loop->T_c = (1.0 - beta) * loop->T_c + beta * T_c_sample;
  loop->T_s = (1.0 - beta) * loop->T_s + beta * T_s_sample;
  return replan(loop);
}

int cocodc_loop_plan(const cocodc_loop_t* loop, int64_t* N_out, int64_t* h_out) {
  if (!loop || !N_out || !h_out) return COCODC_ERR_NULL;
  *N_out = loop->N;
  *h_out = loop->h;
  return COCODC_OK;
}

int cocodc_loop_due(const cocodc_loop_t* loop, int64_t t, int32_t* due_out, int32_t* n_due_out) {
  if (!loop || !due_out || !n_due_out) return COCODC_ERR_NULL;
  int32_t n = 0;
  for (size_t p = 0; p < loop->frags.size(); ++p) {
    if (loop->in_flight[p] >= 0 && loop->in_flight[p] + loop->hp.tau == t) due_out[n++] = static_cast<int32_t>(p);
  }
  *n_due_out = n;
  return COCODC_OK;
}

int cocodc_loop_state(const cocodc_loop_t* loop, int64_t* t_b_out, int64_t* I_p_out, int64_t* in_flight_out) {
  if (!loop || !t_b_out || !I_p_out || !in_flight_out) return COCODC_ERR_NULL;
  for (size_t p = 0; p < loop->frags.size(); ++p) {
    t_b_out[p] = loop->t_b[p];
    I_p_out[p] = loop->I_p[p];
    in_flight_out[p] = loop->in_flight[p];
  }
  return COCODC_OK;
}

int cocodc_loop_step(cocodc_loop_t* loop, int64_t t, const cocodc_loop_buffers_t* buf, void* stream,
                     int32_t* received_out, int32_t* n_received_out, int32_t* sent_out) {
  if (!loop || !buf || !received_out || !n_received_out || !sent_out) return COCODC_ERR_NULL;
  if (t < 1) return COCODC_ERR_RANGE;
  if (!buf->R || !buf->sel || !buf->n_sel || !buf->theta_m_send) return COCODC_ERR_NULL;
  const int32_t K = static_cast<int32_t>(loop->frags.size());
  *n_received_out = 0;
  *sent_out = -1;
  hipStream_t s = static_cast<hipStream_t>(stream);

  // 1. fragments whose all-reduce completes now
  for (int32_t p = 0; p < K; ++p) {
    if (loop->in_flight[p] < 0 || loop->in_flight[p] + loop->hp.tau != t) continue;
    const int64_t I = loop->in_flight[p] - loop->t_b[p];  // Eq. 11: I_p = t_p - t_{p,b}
    const int64_t tb = loop->t_b[p];
    if (int rc = cocodc_sync_step(&loop->frags[p], 1, loop->n_total, buf->theta_m, buf->theta_m_send,
                                  buf->theta_g, buf->momentum, buf->delta_g, nullptr, &I, &tb, t, 0, &loop->hp,
                                  buf->R + p, buf->sel, buf->n_sel, nullptr, buf->workspace,
                                  buf->workspace_bytes, stream))
      return rc;
    loop->I_p[p] = I;
    loop->t_b[p] = t;
    loop->in_flight[p] = -1;
    received_out[(*n_received_out)++] = p;
  }

  // 2. time to start the next fragment synchronisation?
  if (t % loop->h != 0) return COCODC_OK;
  int32_t n_flying = 0;
  for (int32_t p = 0; p < K; ++p) n_flying += loop->in_flight[p] >= 0 ? 1 : 0;
  if (n_flying >= K) return COCODC_OK;
  const int32_t want = n_flying + 1;  // the first fragment of the priority order that is not in flight
  if (int rc = cocodc_select_fragments(K, buf->R, loop->t_b.data(), t, loop->hp.H, want, buf->sel, buf->n_sel,
                                       buf->workspace, buf->workspace_bytes, stream))
    return rc;
  std::vector<int32_t> order(static_cast<size_t>(want));
  HIP_TRY(hipMemcpyAsync(order.data(), buf->sel, sizeof(int32_t) * want, hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  int32_t p_star = -1;
  for (int32_t q : order) {
    if (q >= 0 && q < K && loop->in_flight[q] < 0) {
      p_star = q;
      break;
    }
  }
  if (p_star < 0) return COCODC_OK;
  if (int rc = cocodc_pseudograd(&loop->frags[p_star], 1, loop->n_total, buf->theta_g, buf->theta_m,
                                 buf->delta_m_out, buf->theta_m_send, buf->workspace, buf->workspace_bytes, stream))
    return rc;
  loop->in_flight[p_star] = t;
  *sent_out = p_star;
  return COCODC_OK;
}

uint64_t cocodc_layout_stride_bytes(uint64_t n_total) {
  constexpr uint64_t GiB = 1ull << 30;
  const uint64_t bytes = n_total * sizeof(float);
  uint64_t stride = std::max<uint64_t>(40 * GiB, (bytes + GiB - 1) / GiB * GiB);
  if (stride % (32 * GiB) == 0) stride += 2 * GiB;
  return stride;
}

uint64_t cocodc_tile_elements(uint64_t n_total) { return uint64_t(1) << tile_shift_for(n_total); }

int cocodc_debug_tile_plan(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total,
                           uint64_t* seg_offset_out, uint64_t* seg_slot_begin_out, uint64_t* frag_slot_begin_out,
                           uint64_t* tile_capacity_out) {
  if (!seg_offset_out || !seg_slot_begin_out || !frag_slot_begin_out || !tile_capacity_out) return COCODC_ERR_NULL;
  Plan pl;
  if (int rc = plan_segments(segs, S, K, n_total, nullptr, nullptr, &pl)) return rc;
  for (int32_t j = 0; j <= S; ++j) {
    seg_offset_out[j] = pl.recs[j].offset;
    seg_slot_begin_out[j] = pl.recs[j].slot_begin;
  }
  for (int32_t p = 0; p <= K; ++p) frag_slot_begin_out[p] = pl.recs[static_cast<size_t>(S) + 1 + p].slot_begin;
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
  const int old = g_blocks_per_cu;
  g_blocks_per_cu = blocks_per_cu < 0 ? 0 : blocks_per_cu;
  return old;
}

int cocodc_profiler_enable(int32_t max_records) {
  if (max_records < 1 || max_records > 65536) return COCODC_ERR_RANGE;
  std::lock_guard<std::mutex> lock(g_prof.mu);
  if (g_prof.on) return COCODC_ERR_RANGE;
  g_prof.start.resize(max_records);
  g_prof.stop.resize(max_records);
  for (int i = 0; i < max_records; ++i) {
    HIP_TRY(hipEventCreate(&g_prof.start[i]));
    HIP_TRY(hipEventCreate(&g_prof.stop[i]));
  }
  g_prof.used = 0;
  g_prof.on = true;
  return COCODC_OK;
}

int cocodc_profiler_collect(float* ms_out, int32_t capacity) {
  if (!ms_out) return COCODC_ERR_NULL;
  std::lock_guard<std::mutex> lock(g_prof.mu);
  if (!g_prof.on) return COCODC_ERR_RANGE;
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
  if (!g_prof.on) return COCODC_OK;
  for (size_t i = 0; i < g_prof.start.size(); ++i) {
    (void)hipEventDestroy(g_prof.start[i]);
    (void)hipEventDestroy(g_prof.stop[i]);
  }
  g_prof.start.clear();
  g_prof.stop.clear();
  g_prof.used = 0;
  g_prof.on = false;
  return COCODC_OK;
}

}  // extern "C"
