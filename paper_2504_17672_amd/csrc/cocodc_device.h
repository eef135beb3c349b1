// cocodc_device.h -- device code of the CoCoDC outer-synchronisation library (gfx950):
// stream access helpers, the per-element arithmetic, the streaming operations, the workgroup
// reductions and the kernels.  Included by cocodc.hip only.
#pragma once

namespace {

constexpr int kThreads = COCODC_THREADS;
constexpr int kWaves = kThreads / 64;
// Tile size: 2^12 elements for large buffers -- kThreads lanes x one 128-bit access x kDepth, so
// a workgroup loads its whole tile, computes, stores and ends (measured faster than workgroups
// that loop over a larger tile) -- and 2^11 for small ones (below 2^24 elements), so that even a
// 1M-element call spreads over more workgroups than there are compute units.  It depends on
// n_total alone, so the workspace size and the summation order are functions of the
// arguments and not of the machine.
constexpr int ilog2(unsigned v) { return v <= 1 ? 0 : 1 + ilog2(v >> 1); }
constexpr int kTileShiftLarge = ilog2(COCODC_TILE), kTileShiftSmall = kTileShiftLarge < 11 ? kTileShiftLarge : 11;
constexpr uint64_t kSmallBufferElements = 1ull << 24;
static_assert((1u << kTileShiftLarge) == COCODC_TILE && kTileShiftLarge >= 10, "COCODC_TILE: a power of two >= 1024");
inline int tile_shift_for(uint64_t n_total) {
  return n_total < kSmallBufferElements ? kTileShiftSmall : kTileShiftLarge;
}
constexpr int kDepth = COCODC_DEPTH;  // independent 128-bit loads per stream kept in flight per lane
constexpr int kTableChunkWords = 240;  // 16-byte words of table carried by one upload launch
constexpr int kSums = 4;              // doubles per partial-sum slot

static_assert((1u << kTileShiftSmall) % (4 * kThreads) == 0 && kTileShiftSmall >= 10, "a tile must be a whole number of workgroup-wide vector rows");

// Device-side description of one segment (a contiguous piece of a fragment).
struct SegRec {
  uint64_t offset;      // first element
  uint64_t length;      // elements (0: the segment takes no part in this call)
  uint64_t slot_begin;  // index of this segment's first tile in the global tile list
  uint64_t tile0;       // absolute window index (offset >> tile_shift) of that first tile
};
static_assert(sizeof(SegRec) == 32, "SegRec layout");

// Device-side description of one fragment as a whole (one record per fragment, K + 1 of them;
// record K only closes the last fragment's range of tile slots).
struct GroupRec {
  uint64_t slot_begin;   // index of the fragment's first tile in the global tile list
  uint64_t bytes;        // its size, for the selection under a byte budget
  int64_t I_p;           // steps between the fragment's last two completed syncs (Eq. 11)
  int64_t t_b;           // step of its last completed sync (Algorithm 2)
  uint32_t takes_part;   // 1: this call updates the fragment and its score; 0: it leaves both alone
  uint32_t in_flight;    // 1: an all-reduce of the fragment is under way: Algorithm 2 passes it over
  uint64_t reserved;
};
static_assert(sizeof(GroupRec) == 48, "GroupRec layout");

// What a streaming kernel walks: S segment records (plus a closing one whose slot_begin is the
// number of tiles T) and the tile size.  The records themselves come either from the workspace
// (SegTable / GroupTable: a pointer) or, for tables of at most kInlineRecs segments and fragments,
// inside the kernel arguments (SegInline / GroupInline: no upload launch before the kernel).
struct Walk {
  uint64_t T;
  int32_t S;
  int32_t tile_shift;
};

constexpr int kInlineRecs = 32;
struct SegTable {
  const SegRec* p;
  __device__ __forceinline__ const SegRec& operator[](int i) const { return p[i]; }
};
struct SegInline {
  SegRec r[kInlineRecs + 1];
  __device__ __forceinline__ const SegRec& operator[](int i) const { return r[i]; }
};
struct GroupTable {
  const GroupRec* p;
  __device__ __forceinline__ const GroupRec& operator[](int i) const { return p[i]; }
};
struct GroupInline {
  GroupRec r[kInlineRecs + 1];
  __device__ __forceinline__ const GroupRec& operator[](int i) const { return r[i]; }
};

// The tables travel to the device as kernel arguments, kTableChunkWords 16-byte words per launch.
struct TableChunk {
  uint4 w[kTableChunkWords];
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

// A = true: the address is a multiple of the access size (128-bit accesses on 16-byte
// boundaries).  A = false: only the element alignment is known; the same access is then made
// through a type of that alignment, which the compiler may split into narrower accesses.
typedef f32x4 f32x4_unaligned __attribute__((aligned(4)));
template <int V, bool A>
struct VecAccess {
  using type = typename Vec<V>::type;
};
template <>
struct VecAccess<4, false> {
  using type = f32x4_unaligned;
};

template <int V, bool A = true>
__device__ __forceinline__ typename Vec<V>::type load_stream(const float* p) {
  using T = typename VecAccess<V, A>::type;
#if COCODC_NT_LOAD
  return __builtin_nontemporal_load(reinterpret_cast<const T*>(p));
#else
  return *reinterpret_cast<const T*>(p);
#endif
}

template <int V, bool A = true>
__device__ __forceinline__ void store_stream(float* p, typename Vec<V>::type v) {
  using T = typename VecAccess<V, A>::type;
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

typedef u16x4 u16x4_unaligned __attribute__((aligned(2)));
template <int V, bool A>
struct VecU16Access {
  using type = typename VecU16<V>::type;
};
template <>
struct VecU16Access<4, false> {
  using type = u16x4_unaligned;
};

template <int V, bool A = true>
__device__ __forceinline__ typename VecU16<V>::type load_stream_u16(const unsigned short* p) {
  using T = typename VecU16Access<V, A>::type;
#if COCODC_NT_LOAD
  return __builtin_nontemporal_load(reinterpret_cast<const T*>(p));
#else
  return *reinterpret_cast<const T*>(p);
#endif
}
template <int V, bool A = true>
__device__ __forceinline__ void store_stream_u16(unsigned short* p, typename VecU16<V>::type v) {
  using T = typename VecU16Access<V, A>::type;
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

// Nearest IEEE binary16 to an fp64 value in ONE rounding, ties to even; subnormals (spacing
// 2^-24) kept, 65520 and above to infinity, any NaN -> 0x7E00.
// binary32 carries 13 more significant bits than binary16 and reaches far below its subnormals,
// so the value is first brought to binary32 "rounded to odd" (the truncated magnitude, with the
// last bit set whenever anything was cut off), which no later rounding to fewer bits can be
// fooled by; the hardware conversion binary32 -> binary16 (to nearest even) then gives the same
// pattern as rounding the fp64 value directly.
__device__ __forceinline__ unsigned short round_f16(double x) {
  const float f = static_cast<float>(x);  // hardware conversion, to nearest
  unsigned u = __float_as_uint(f);
  const double back = static_cast<double>(f);
  if (back != x && (u & 0x7F800000u) != 0x7F800000u) {  // inexact (and neither overflowed nor NaN)
    if (fabs(back) > fabs(x)) u -= 1u;                  // back to the truncated magnitude
    u |= 1u;
  }
  const _Float16 h = static_cast<_Float16>(__uint_as_float(u));
  unsigned short r;
  __builtin_memcpy(&r, &h, sizeof(r));
  return static_cast<unsigned short>(x != x ? 0x7E00u : r);
}

// The 16-bit pattern of an outgoing pseudo-gradient: bfloat16 or IEEE binary16.
template <bool F16>
__device__ __forceinline__ unsigned short round_pg16(double x) {
  return F16 ? round_f16(x) : round_bf16(x);
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

  template <int V, bool A = true>
  __device__ __forceinline__ Regs<V> load(uint64_t i) const {
    Regs<V> r;
    r.tm = load_stream<V, A>(theta_m + i);
    if (HAS_SEND) r.ts = load_stream<V, A>(theta_send + i);
    r.tg = load_stream<V, A>(theta_g + i);
    r.m = load_stream<V, A>(momentum + i);
    r.dg = load_stream<V, A>(delta_g + i);
    return r;
  }

  template <int V, bool A = true>
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
    store_stream<V, A>(theta_m + i, o_tm);
    store_stream<V, A>(theta_g + i, o_tg);
    store_stream<V, A>(momentum + i, o_m);
    if (HAS_PG) store_stream<V, A>(pg + i, o_pg);
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
  template <int V, bool A = true>
  __device__ __forceinline__ Regs<V> load(uint64_t i) const {
    Regs<V> r;
    r.tg = load_stream<V, A>(theta_g + i);
    r.tm = load_stream<V, A>(theta_m + i);
    return r;
  }
  template <int V, bool A = true>
  __device__ __forceinline__ void apply(uint64_t i, const Regs<V>& r, double*) const {
    typename Vec<V>::type o;
#pragma unroll
    for (int k = 0; k < V; ++k) lane_set(o, k, lane_get(r.tg, k) - lane_get(r.tm, k));
    store_stream<V, A>(pg + i, o);
    if (HAS_SEND) store_stream<V, A>(send_out + i, r.tm);
  }
};

// Measurement aid: the nine streams of the fused step (five read, four written, three of them in
// place) with one fp32 addition per stored value and no sums -- what the memory system gives this
// access pattern when the arithmetic costs nothing.
struct StreamMixOp {
  static constexpr int kAcc = 0;
  static constexpr int kVec = 4;
  static constexpr int kLoads = kDepth;
  float* a;        // read and written
  const float* b;  // read
  float* c;        // read and written
  float* d;        // read and written
  const float* e;  // read
  float* f;        // written

  template <int V>
  struct Regs {
    typename Vec<V>::type a, b, c, d, e;
  };
  template <int V, bool A = true>
  __device__ __forceinline__ Regs<V> load(uint64_t i) const {
    Regs<V> r;
    r.a = load_stream<V, A>(a + i);
    r.b = load_stream<V, A>(b + i);
    r.c = load_stream<V, A>(c + i);
    r.d = load_stream<V, A>(d + i);
    r.e = load_stream<V, A>(e + i);
    return r;
  }
  template <int V, bool A = true>
  __device__ __forceinline__ void apply(uint64_t i, const Regs<V>& r, double*) const {
    typename Vec<V>::type oa, oc, od, of;
#pragma unroll
    for (int k = 0; k < V; ++k) {
      lane_set(oa, k, lane_get(r.a, k) + lane_get(r.b, k));
      lane_set(oc, k, lane_get(r.c, k) + lane_get(r.e, k));
      lane_set(od, k, lane_get(r.d, k) + lane_get(r.e, k));
      lane_set(of, k, lane_get(r.b, k) + lane_get(r.c, k));
    }
    store_stream<V, A>(a + i, oa);
    store_stream<V, A>(c + i, oc);
    store_stream<V, A>(d + i, od);
    store_stream<V, A>(f + i, of);
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
  template <int V, bool A = true>
  __device__ __forceinline__ Regs<V> load(uint64_t i) const {
    Regs<V> r;
    r.tg = load_stream<V, A>(theta_g + i);
    r.m = load_stream<V, A>(momentum + i);
    r.dg = load_stream<V, A>(delta_g + i);
    return r;
  }
  template <int V, bool A = true>
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
    store_stream<V, A>(theta_g + i, o_tg);
    store_stream<V, A>(momentum + i, o_m);
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
  template <int V, bool A = true>
  __device__ __forceinline__ Regs<V> load(uint64_t i) const {
    Regs<V> r;
    r.tm = load_stream<V, A>(theta_m + i);
    if (HAS_SEND) r.ts = load_stream<V, A>(theta_send + i);
    r.tg = load_stream<V, A>(theta_g + i);
    return r;
  }
  template <int V, bool A = true>
  __device__ __forceinline__ void apply(uint64_t i, const Regs<V>& r, double*) const {
    typename Vec<V>::type o;
#pragma unroll
    for (int k = 0; k < V; ++k) {
      const float tm = lane_get(r.tm, k);
      const float ts = HAS_SEND ? lane_get(r.ts, k) : tm;
      const double d = HAS_SEND ? drift(ts, tm, hp) : 0.0;
      lane_set(o, k, merge_local<MERGE>(lane_get(r.tg, k), ts, tm, d, hp));
    }
    store_stream<V, A>(theta_m + i, o);
  }
};

// The fused step with bfloat16 local parameters: theta_m, theta_send and the outgoing
// pseudo-gradient are bf16 (2 bytes), theta_g, momentum, delta_g stay fp32: 28 B/param.
template <bool NESTEROV, int MERGE, bool HAS_PG, bool HAS_SEND = true, bool PG_F16 = false>
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

  template <int V, bool A = true>
  __device__ __forceinline__ Regs<V> load(uint64_t i) const {
    Regs<V> r;
    r.tm = load_stream_u16<V, A>(theta_m + i);
    if (HAS_SEND) r.ts = load_stream_u16<V, A>(theta_send + i);
    r.tg = load_stream<V, A>(theta_g + i);
    r.m = load_stream<V, A>(momentum + i);
    r.dg = load_stream<V, A>(delta_g + i);
    return r;
  }

  template <int V, bool A = true>
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
      if (HAS_PG) lane_set(o_pg, k, round_pg16<PG_F16>(static_cast<double>(tg) - static_cast<double>(tm)));
    }
    store_stream_u16<V, A>(theta_m + i, o_tm);
    store_stream<V, A>(theta_g + i, o_tg);
    store_stream<V, A>(momentum + i, o_m);
    if (HAS_PG) store_stream_u16<V, A>(pg + i, o_pg);
  }
};

template <bool HAS_SEND, bool PG_F16 = false>
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
  template <int V, bool A = true>
  __device__ __forceinline__ Regs<V> load(uint64_t i) const {
    Regs<V> r;
    r.tg = load_stream<V, A>(theta_g + i);
    r.tm = load_stream_u16<V, A>(theta_m + i);
    return r;
  }
  template <int V, bool A = true>
  __device__ __forceinline__ void apply(uint64_t i, const Regs<V>& r, double*) const {
    typename VecU16<V>::type o;
#pragma unroll
    for (int k = 0; k < V; ++k) {
      lane_set(o, k, round_pg16<PG_F16>(static_cast<double>(lane_get(r.tg, k)) -
                                        static_cast<double>(widen_bf16(lane_get(r.tm, k)))));
    }
    store_stream_u16<V, A>(pg + i, o);
    if (HAS_SEND) store_stream_u16<V, A>(send_out + i, r.tm);
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
  template <int V, bool A = true>
  __device__ __forceinline__ Regs<V> load(uint64_t i) const {
    Regs<V> r;
    r.x = load_stream<V, A>(x + i);
    return r;
  }
  template <int V, bool A = true>
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

// Sum of NA values over a workgroup of NW wavefronts in a fixed order; thread 0 returns the
// totals in a[].
template <int NA, int NW = kWaves>
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
      for (int w = 1; w < NW; ++w) s += lds[w][k];
      a[k] = s;
    }
  }
  __syncthreads();
}

// ------------------------------------------------------------------ kernels
__global__ void k_write_table(TableChunk chunk, uint4* dst, int base, int count) {
  const int i = threadIdx.x;
  if (i < count) dst[base + i] = chunk.w[i];
}

// The elements [lo, hi) of one tile (hi - lo <= 2^tile_shift, the tile's window is aligned to
// that size): a head up to a multiple of the vector width, whole vector rows, a tail.
// VEC: every buffer base is 16-byte aligned, so are the element indices that are multiples of W,
// and the accesses below are single 128-bit ones.  Otherwise the same accesses are made through
// element-aligned types.  Either way lane t handles the same elements in the same order, so the
// sums do not depend on the alignment of the buffers.
template <class Op, bool VEC>
__device__ __forceinline__ void walk_tile(const Op& op, uint64_t lo, uint64_t hi, double* acc) {
  const uint64_t tid = threadIdx.x;
  constexpr int W = Op::kVec;      // elements per vector access
  constexpr int D = Op::kLoads;    // vector accesses per stream in flight
  uint64_t lo4 = (lo + (W - 1)) & ~uint64_t(W - 1);
  if (lo4 > hi) lo4 = hi;
  uint64_t hi4 = hi & ~uint64_t(W - 1);
  if (hi4 < lo4) hi4 = lo4;
  if (tid < lo4 - lo) {  // head of the fragment up to a multiple of W (at most W-1 elements)
    const auto r = op.template load<1>(lo + tid);
    op.template apply<1>(lo + tid, r, acc);
  }
  const uint64_t nvec = (hi4 - lo4) / W;
  for (uint64_t v = tid; v < nvec; v += uint64_t(kThreads) * D) {
    typename Op::template Regs<W> r[D];
#pragma unroll
    for (int k = 0; k < D; ++k) {
      const uint64_t vk = v + uint64_t(k) * kThreads;
      if (vk < nvec) r[k] = op.template load<W, VEC>(lo4 + vk * W);
    }
#pragma unroll
    for (int k = 0; k < D; ++k) {
      const uint64_t vk = v + uint64_t(k) * kThreads;
      if (vk < nvec) op.template apply<W, VEC>(lo4 + vk * W, r[k], acc);
    }
  }
  if (tid < hi - hi4) {  // tail (at most W-1 elements)
    const auto r = op.template load<1>(hi4 + tid);
    op.template apply<1>(hi4 + tid, r, acc);
  }
}

// One workgroup per tile (or, with a persistent grid, a walk over the tile list with stride
// gridDim.x).  wk.tbl has S+1 segment records; wk.tbl[S].slot_begin == wk.T, the number of tiles.
#if COCODC_WAVES_PER_EU > 0
#define COCODC_OCCUPANCY __attribute__((amdgpu_waves_per_eu(COCODC_WAVES_PER_EU)))
#else
#define COCODC_OCCUPANCY
#endif
// The segment that tile w belongs to: the last record whose slot_begin is <= w (records of empty
// segments share their successor's slot_begin, so they are never the last).  A workgroup lives for
// one tile of a few microseconds, so this is a bisection, not a scan.
template <class Segs>
__device__ __forceinline__ int segment_of_tile(const Segs& tbl, int S, uint64_t w) {
  int p = 0, hi = S;
  while (hi - p > 1) {
    const int mid = (p + hi) >> 1;
    if (tbl[mid].slot_begin <= w) p = mid; else hi = mid;
  }
  return p;
}

// The element range [lo, hi) of tile w of segment p.
template <class Segs>
__device__ __forceinline__ void tile_bounds(const Segs& tbl, int p, uint64_t w, int tile_shift, uint64_t* lo,
                                            uint64_t* hi) {
  const uint64_t f_off = tbl[p].offset, f_end = f_off + tbl[p].length;
  const uint64_t win = (tbl[p].tile0 + (w - tbl[p].slot_begin)) << tile_shift;
  const uint64_t win_end = win + (uint64_t(1) << tile_shift);
  *lo = f_off > win ? f_off : win;
  *hi = f_end < win_end ? f_end : win_end;
}

template <class Op, bool VEC, class Segs>
__global__ __launch_bounds__(kThreads) COCODC_OCCUPANCY void k_walk(Segs tbl, Walk wk, Op op, double* __restrict__ partials) {
  __shared__ double lds[kWaves][kSums];
  const uint64_t T = wk.T;
  const int tile_shift = wk.tile_shift;
  int p = blockIdx.x < T ? segment_of_tile(tbl, wk.S, blockIdx.x) : 0;
  for (uint64_t w = blockIdx.x; w < T; w += gridDim.x) {
    while (w >= tbl[p + 1].slot_begin) ++p;  // uniform; later tiles of a persistent grid
    uint64_t lo, hi;
    tile_bounds(tbl, p, w, tile_shift, &lo, &hi);

    double acc[Op::kAcc > 0 ? Op::kAcc : 1];
#pragma unroll
    for (int k = 0; k < (Op::kAcc > 0 ? Op::kAcc : 1); ++k) acc[k] = 0.0;

    walk_tile<Op, VEC>(op, lo, hi, acc);

    if (Op::kAcc > 0) {
      block_sum<(Op::kAcc > 0 ? Op::kAcc : 1)>(acc, lds);
      if (threadIdx.x == 0) {
#pragma unroll
        for (int k = 0; k < Op::kAcc; ++k) partials[w * kSums + k] = acc[k];
      }
    }
  }
}

// The same walk over ONE fragment that is named in device memory: *chosen is the index of a
// fragment picked by an earlier kernel on the same stream (Algorithm 2), so the host does not
// have to know it to launch the work.  tbl / groups are the tables of ALL fragments (nothing
// masked out); the chosen fragment owns the tile slots [groups[p].slot_begin,
// groups[p+1].slot_begin), whatever number of segments it consists of.  The grid is sized by the
// host for the largest fragment that could have been chosen; workgroups beyond the chosen
// fragment's tiles return at once, and all of them do when *chosen is out of range (nothing was
// eligible).  Element-wise operations only (no per-fragment sums).
template <class Op, bool VEC, class Segs, class Groups>
__global__ __launch_bounds__(kThreads) COCODC_OCCUPANCY void k_walk_chosen(Segs tbl, int S, Groups groups, int K,
                                                                          const int* __restrict__ chosen,
                                                                          int tile_shift, Op op) {
  static_assert(Op::kAcc == 0, "the walk over a chosen fragment keeps no sums");
  const int q = *chosen;
  if (q < 0 || q >= K) return;
  const uint64_t s0 = groups[q].slot_begin, s1 = groups[q + 1].slot_begin;
  if (s0 + blockIdx.x >= s1) return;
  int p = segment_of_tile(tbl, S, s0 + blockIdx.x);
  for (uint64_t w = s0 + blockIdx.x; w < s1; w += gridDim.x) {
    while (w >= tbl[p + 1].slot_begin) ++p;
    uint64_t lo, hi;
    tile_bounds(tbl, p, w, tile_shift, &lo, &hi);
    double acc[1] = {0.0};
    walk_tile<Op, VEC>(op, lo, hi, acc);
  }
}

// One workgroup of kFinalizeThreads per fragment: adds that fragment's tile partials (thread t
// takes slots t, t+kFinalizeThreads, ... in ascending order, four slots in flight, then the
// fixed workgroup tree) and evaluates Eq. 11.
//   which: index (0..3) of the sum that feeds R;  l2: take the square root of it.
constexpr int kFinalizeThreads = 1024;
template <class Groups>
__global__ __launch_bounds__(kFinalizeThreads) void k_finalize(Groups tbl,
                                                                const double* __restrict__ partials, int n_acc,
                                                                int which, int l2, double* __restrict__ R_out,
                                                                double* __restrict__ sums_out, int sums_stride) {
  typedef double f64x2 __attribute__((ext_vector_type(2)));
  static_assert(kSums == 4, "a slot is read as two 16-byte halves");
  constexpr int U = 4;
  __shared__ double lds[kFinalizeThreads / 64][kSums];
  const int p = blockIdx.x;
  if (tbl[p].takes_part == 0) return;  // the fragment takes no part in this call: its score stays
  const uint64_t s0 = tbl[p].slot_begin, s1 = tbl[p + 1].slot_begin;
  const f64x2* __restrict__ slots = reinterpret_cast<const f64x2*>(partials);
  double acc[kSums] = {0.0, 0.0, 0.0, 0.0};
  for (uint64_t s = s0 + threadIdx.x; s < s1; s += uint64_t(kFinalizeThreads) * U) {
    f64x2 a[U], b[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint64_t su = s + uint64_t(u) * kFinalizeThreads;
      a[u] = b[u] = f64x2{0.0, 0.0};
      if (su < s1) {
        a[u] = slots[su * 2];
        if (n_acc > 2) b[u] = slots[su * 2 + 1];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (s + uint64_t(u) * kFinalizeThreads < s1) {
        acc[0] += a[u].x;
        if (n_acc > 1) acc[1] += a[u].y;
        if (n_acc > 2) acc[2] += b[u].x;
        if (n_acc > 3) acc[3] += b[u].y;
      }
    }
  }
  block_sum<kSums, kFinalizeThreads / 64>(acc, lds);
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
// (class, -R, p) with class 0 = not synchronised for >= H steps, 1 = has a number as score,
// 2 = NaN score, 3 = in flight (never a candidate; the host keeps n within the number of
// candidates).  Every fragment counts how many fragments precede it.
template <class Groups>
__device__ __forceinline__ void load_priorities(const Groups& tbl, int K,
                                                const double* __restrict__ R, int64_t t_g, int64_t H,
                                                double* sR, unsigned char* sC) {
  for (int p = threadIdx.x; p < K; p += kThreads) {
    const double r = R[p];
    const bool overdue = (t_g - tbl[p].t_b) >= H;
    sR[p] = r;
    sC[p] = tbl[p].in_flight ? 3 : (overdue ? 0 : (r != r ? 2 : 1));
  }
  __syncthreads();
}

__device__ __forceinline__ int priority_rank(int p, int K, const double* sR, const unsigned char* sC) {
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
  return rank;
}

template <class Groups>
__global__ __launch_bounds__(kThreads) void k_select(Groups tbl, int K,
                                                      const double* __restrict__ R, int64_t t_g,
                                                      int64_t H, int n, int* __restrict__ sel,
                                                      int* __restrict__ n_sel) {
  __shared__ double sR[COCODC_MAX_FRAGMENTS];
  __shared__ unsigned char sC[COCODC_MAX_FRAGMENTS];
  load_priorities(tbl, K, R, t_g, H, sR, sC);
  for (int p = threadIdx.x; p < K; p += kThreads) {
    const int rank = priority_rank(p, K, sR, sC);
    if (rank < n) sel[rank] = p;
  }
  if (threadIdx.x == 0) *n_sel = n;
}

// Same priority order, cut by a byte budget: fragments are taken in rank order while their sizes
// (GroupRec::bytes) still fit; the first that does not fit ends the selection.
template <class Groups>
__global__ __launch_bounds__(kThreads) void k_select_bytes(Groups tbl, int K,
                                                            const double* __restrict__ R, int64_t t_g,
                                                            int64_t H, unsigned long long byte_budget,
                                                            int* __restrict__ sel, int* __restrict__ n_sel) {
  __shared__ double sR[COCODC_MAX_FRAGMENTS];
  __shared__ unsigned char sC[COCODC_MAX_FRAGMENTS];
  __shared__ int sOrder[COCODC_MAX_FRAGMENTS];
  load_priorities(tbl, K, R, t_g, H, sR, sC);
  for (int p = threadIdx.x; p < K; p += kThreads) sOrder[priority_rank(p, K, sR, sC)] = p;  // a permutation
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned long long left = byte_budget;
    int n = 0;
    for (int r = 0; r < K; ++r) {
      const int p = sOrder[r];
      if (sC[p] == 3) break;  // only fragments in flight are left
      const unsigned long long need = tbl[p].bytes;
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

}  // namespace
