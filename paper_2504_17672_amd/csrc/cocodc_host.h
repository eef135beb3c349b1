// cocodc_host.h -- host side of the library: error bookkeeping, workspace layout, validation of
// fragment / segment tables and their tile plan, launch helpers, kernel timer.
// Included by cocodc.hip only, after cocodc_device.h.
#pragma once

namespace {

// ------------------------------------------------------------------ host side
thread_local int g_last_hip_error = 0;
std::atomic<int> g_blocks_per_cu{0};
std::atomic<int> g_tables_in_args{1};  // small tables travel inside the kernel arguments (0: always upload)

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

// Device workspace: S+1 segment records (the tile walk), K+1 fragment records (one per fragment:
// its range of tile slots, I_p, t_b, flags), then one slot of kSums doubles per tile.
struct WorkspaceView {
  SegRec* table;     // S + 1 segment records; table[S].slot_begin == number of tiles
  GroupRec* groups;  // K + 1 fragment records
  double* partials;  // max_tiles * kSums
};

size_t table_bytes(int32_t S, int32_t K) {
  return align_up(sizeof(SegRec) * (static_cast<size_t>(S) + 1) + sizeof(GroupRec) * (static_cast<size_t>(K) + 1), 256);
}

size_t workspace_bytes(int32_t S, int32_t K, uint64_t n_total) {
  return table_bytes(S, K) + align_up(max_tiles(S, n_total) * kSums * sizeof(double), 256);
}

WorkspaceView view(void* ws, int32_t S, int32_t K) {
  char* b = static_cast<char*>(ws);
  SegRec* t = reinterpret_cast<SegRec*>(b);
  return WorkspaceView{t, reinterpret_cast<GroupRec*>(t + S + 1), reinterpret_cast<double*>(b + table_bytes(S, K))};
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

// Host-side plan of one call: the records the kernels read and the number of tiles.
struct Plan {
  std::vector<SegRec> segs;      // S + 1 segment records
  std::vector<GroupRec> groups;  // K + 1 fragment records
  int32_t S = 0, K = 0;
  int tile_shift = kTileShiftLarge;
  uint64_t T = 0;
  // Small tables are handed to every kernel inside its arguments, which saves the upload launch
  // in front of it (a quarter of the time of a step on a cache-resident fragment set).  Set when
  // the plan is made; a caller that needs the tables in the workspace clears it before launching.
  bool in_args = false;
};

// What launch_walk needs to launch a streaming kernel over a plan.
struct HostWalk {
  const Plan* plan;
  const SegRec* dev_table;
};
HostWalk walk_of(const WorkspaceView& v, const Plan& pl) { return HostWalk{&pl, v.table}; }

SegInline seg_args(const Plan& pl) {
  SegInline a;
  std::memset(&a, 0, sizeof(a));
  std::memcpy(a.r, pl.segs.data(), sizeof(SegRec) * pl.segs.size());
  return a;
}
GroupInline group_args(const Plan& pl) {
  GroupInline a;
  std::memset(&a, 0, sizeof(a));
  std::memcpy(a.r, pl.groups.data(), sizeof(GroupRec) * pl.groups.size());
  return a;
}

// What a caller's event mask says about fragment p (no mask: every fragment takes part).
constexpr uint8_t kMaskArrived = 1, kMaskInFlight = 2;

// Validates a segment list (every segment inside n_total, no two overlapping, fragment ids in
// [0, K)) and lays out the tile list: the segments of fragment 0 in the order given, then those
// of fragment 1, ...  so that each fragment owns one contiguous range of tile slots.
// mask (nullable, K entries, bits kMaskArrived | kMaskInFlight): fragments without the arrived
// bit take no part in the call -- their segments get no tiles and their fragment record says so,
// so that the reduction leaves their score alone; fragments with the in-flight bit are passed
// over by the selection.
int plan_segments(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total, const int64_t* I_p,
                  const int64_t* t_b, Plan* plan, const uint8_t* mask = nullptr) {
  if (!segs && S > 0) return COCODC_ERR_NULL;
  if (K < 1 || K > COCODC_MAX_FRAGMENTS || S < 0 || S > COCODC_MAX_SEGMENTS) return COCODC_ERR_RANGE;
  if (n_total > COCODC_MAX_ELEMENTS) return COCODC_ERR_RANGE;  // keeps every byte count far from overflow
  if (mask) {
    for (int32_t p = 0; p < K; ++p) {
      if (mask[p] & ~(kMaskArrived | kMaskInFlight)) return COCODC_ERR_RANGE;
    }
  }
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
  plan->segs.assign(static_cast<size_t>(S) + 1, SegRec{});
  plan->groups.assign(static_cast<size_t>(K) + 1, GroupRec{});
  SegRec* seg_rec = plan->segs.data();
  GroupRec* grp_rec = plan->groups.data();
  uint64_t slot = 0;
  int32_t next_group = 0;
  for (int32_t j = 0; j < S; ++j) {
    const cocodc_segment_t& sg = segs[order[j]];
    while (next_group <= sg.fragment) grp_rec[next_group++].slot_begin = slot;
    SegRec& r = seg_rec[j];
    r.offset = sg.offset;
    r.length = (!mask || (mask[sg.fragment] & kMaskArrived)) ? sg.length : 0;
    r.slot_begin = slot;
    r.tile0 = r.offset >> sh;
    if (r.length) slot += ((r.offset + r.length - 1) >> sh) - r.tile0 + 1;
  }
  while (next_group <= K) grp_rec[next_group++].slot_begin = slot;
  seg_rec[S].slot_begin = slot;
  for (int32_t p = 0; p < K; ++p) {
    grp_rec[p].I_p = I_p ? I_p[p] : 0;
    grp_rec[p].t_b = t_b ? t_b[p] : 0;
    grp_rec[p].takes_part = (!mask || (mask[p] & kMaskArrived)) ? 1 : 0;
    grp_rec[p].in_flight = (mask && (mask[p] & kMaskInFlight)) ? 1 : 0;
  }
  plan->T = slot;
  plan->in_args = S <= kInlineRecs && K <= kInlineRecs && g_tables_in_args.load(std::memory_order_relaxed) != 0;
  return COCODC_OK;
}

// Contiguous fragments: fragment p is the single segment frags[p].
int plan_table(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total, const int64_t* I_p,
               const int64_t* t_b, Plan* plan, const uint8_t* mask = nullptr) {
  if (!frags) return COCODC_ERR_NULL;
  if (K < 1 || K > COCODC_MAX_FRAGMENTS) return COCODC_ERR_RANGE;
  std::vector<cocodc_segment_t> segs(static_cast<size_t>(K));
  for (int32_t p = 0; p < K; ++p) segs[p] = cocodc_segment_t{frags[p].offset, frags[p].length, p, 0};
  return plan_segments(segs.data(), K, K, n_total, I_p, t_b, plan, mask);
}

// Both tables go to the head of the workspace (segment records, then fragment records) as kernel
// arguments of a few small launches: no memcpy node, so a call records into a HIP graph.
int upload_table(const Plan& pl, const WorkspaceView& v, hipStream_t s) {
  if (pl.in_args) return COCODC_OK;  // every kernel of this call gets the records with its arguments
  static_assert(sizeof(SegRec) % 16 == 0 && sizeof(GroupRec) % 16 == 0, "tables are moved in 16-byte words");
  const size_t seg_bytes = sizeof(SegRec) * pl.segs.size(), grp_bytes = sizeof(GroupRec) * pl.groups.size();
  std::vector<unsigned char> blob(seg_bytes + grp_bytes);
  std::memcpy(blob.data(), pl.segs.data(), seg_bytes);
  std::memcpy(blob.data() + seg_bytes, pl.groups.data(), grp_bytes);
  const int n = static_cast<int>(blob.size() / 16);
  for (int base = 0; base < n; base += kTableChunkWords) {
    TableChunk c;
    const int count = std::min(kTableChunkWords, n - base);
    std::memset(&c, 0, sizeof(c));
    std::memcpy(c.w, blob.data() + static_cast<size_t>(base) * 16, static_cast<size_t>(count) * 16);
    hipLaunchKernelGGL(k_write_table, dim3(1), dim3(kTableChunkWords), 0, s, c, reinterpret_cast<uint4*>(v.table), base,
                       count);
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
  if (hp->pg_format != COCODC_PG_BF16 && hp->pg_format != COCODC_PG_F16) return COCODC_ERR_RANGE;
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
  const int per_cu = g_blocks_per_cu.load(std::memory_order_relaxed);
  if (per_cu > 0) g = std::min<uint64_t>(T, static_cast<uint64_t>(device_cus()) * per_cu);
  // a launch may not exceed 2^32 - 1 threads per dimension; the kernels stride over what is left
  return static_cast<unsigned>(std::min<uint64_t>(g, 0xffffffffu / kThreads));
}

// ---- kernel timer (measurement aid) ----
struct Profiler {
  std::mutex mu;
  std::vector<hipEvent_t> start, stop;
  int used = 0;
  std::atomic<bool> on{false};  // read without the lock on every launch: the timer is normally off
} g_prof;

// A slot of the timer for the launch that follows, or -1 (timer off or full).
int prof_begin(hipStream_t s) {
  if (!g_prof.on.load(std::memory_order_acquire)) return -1;
  int slot = -1;
  {
    std::lock_guard<std::mutex> lock(g_prof.mu);
    if (g_prof.on.load(std::memory_order_relaxed) && g_prof.used < static_cast<int>(g_prof.start.size()))
      slot = g_prof.used++;
  }
  if (slot >= 0 && hipEventRecord(g_prof.start[slot], s) != hipSuccess) return -1;
  return slot;
}

int prof_end(int slot, hipStream_t s) {
  if (slot >= 0) HIP_TRY(hipEventRecord(g_prof.stop[slot], s));
  return COCODC_OK;
}

// Every streaming kernel is launched here; while the timer is on, each launch is bracketed by a
// pair of events on the launch stream.
template <class Op>
int launch_walk(bool vec, const HostWalk& hw, const Op& op, double* partials, hipStream_t s) {
  const Plan& pl = *hw.plan;
  if (pl.T == 0) return COCODC_OK;
  const int slot = prof_begin(s);
  const dim3 grid(grid_for(pl.T)), block(kThreads);
  const Walk wk{pl.T, pl.S, pl.tile_shift};
  if (pl.in_args) {
    const SegInline tbl = seg_args(pl);
    if (vec) {
      hipLaunchKernelGGL((k_walk<Op, true, SegInline>), grid, block, 0, s, tbl, wk, op, partials);
    } else {
      hipLaunchKernelGGL((k_walk<Op, false, SegInline>), grid, block, 0, s, tbl, wk, op, partials);
    }
  } else {
    const SegTable tbl{hw.dev_table};
    if (vec) {
      hipLaunchKernelGGL((k_walk<Op, true, SegTable>), grid, block, 0, s, tbl, wk, op, partials);
    } else {
      hipLaunchKernelGGL((k_walk<Op, false, SegTable>), grid, block, 0, s, tbl, wk, op, partials);
    }
  }
  HIP_TRY(hipGetLastError());
  return prof_end(slot, s);
}

// Per-fragment sums of the tile partials and Eq. 11.
int launch_finalize(const Plan& pl, const WorkspaceView& v, int n_acc, int which, int l2, double* R_out,
                    double* sums_out, int sums_stride, hipStream_t s) {
  if (pl.in_args) {
    hipLaunchKernelGGL(k_finalize<GroupInline>, dim3(pl.K), dim3(kFinalizeThreads), 0, s, group_args(pl), v.partials,
                       n_acc, which, l2, R_out, sums_out, sums_stride);
  } else {
    hipLaunchKernelGGL(k_finalize<GroupTable>, dim3(pl.K), dim3(kFinalizeThreads), 0, s, GroupTable{v.groups},
                       v.partials, n_acc, which, l2, R_out, sums_out, sums_stride);
  }
  HIP_TRY(hipGetLastError());
  return COCODC_OK;
}

// Algorithm 2, n times.
int launch_select(const Plan& pl, const WorkspaceView& v, const double* R, int64_t t_g, int64_t H, int n, int32_t* sel,
                  int32_t* n_sel, hipStream_t s) {
  if (pl.in_args) {
    hipLaunchKernelGGL(k_select<GroupInline>, dim3(1), dim3(kThreads), 0, s, group_args(pl), pl.K, R, t_g, H, n, sel,
                       n_sel);
  } else {
    hipLaunchKernelGGL(k_select<GroupTable>, dim3(1), dim3(kThreads), 0, s, GroupTable{v.groups}, pl.K, R, t_g, H, n,
                       sel, n_sel);
  }
  HIP_TRY(hipGetLastError());
  return COCODC_OK;
}

// The walk over the one fragment that *chosen (device memory) names.  `full` is the plan of ALL
// fragments (no mask): its tables are what the kernel walks (from its arguments when they are
// small, else from the workspace, where upload_table(full, ...) has put them); max_tiles_ = the
// number of tiles of the largest fragment that could be named.
template <class Op>
int launch_walk_chosen(bool vec, const Plan& full, const WorkspaceView& v, const int32_t* chosen,
                       uint64_t max_tiles_, const Op& op, hipStream_t s) {
  if (max_tiles_ == 0) return COCODC_OK;
  const int slot = prof_begin(s);
  const dim3 grid(grid_for(max_tiles_)), block(kThreads);
  if (full.in_args) {
    const SegInline tbl = seg_args(full);
    const GroupInline grp = group_args(full);
    if (vec) {
      hipLaunchKernelGGL((k_walk_chosen<Op, true, SegInline, GroupInline>), grid, block, 0, s, tbl, full.S, grp, full.K,
                         chosen, full.tile_shift, op);
    } else {
      hipLaunchKernelGGL((k_walk_chosen<Op, false, SegInline, GroupInline>), grid, block, 0, s, tbl, full.S, grp, full.K,
                         chosen, full.tile_shift, op);
    }
  } else {
    const SegTable tbl{v.table};
    const GroupTable grp{v.groups};
    if (vec) {
      hipLaunchKernelGGL((k_walk_chosen<Op, true, SegTable, GroupTable>), grid, block, 0, s, tbl, full.S, grp, full.K,
                         chosen, full.tile_shift, op);
    } else {
      hipLaunchKernelGGL((k_walk_chosen<Op, false, SegTable, GroupTable>), grid, block, 0, s, tbl, full.S, grp, full.K,
                         chosen, full.tile_shift, op);
    }
  }
  HIP_TRY(hipGetLastError());
  return prof_end(slot, s);
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

template <bool NESTEROV, int MERGE>
int launch_fused(bool vec, const HostWalk& wk, float* tm, const float* ts, float* tg,
                 float* m, const float* dg, float* pg, const DevHP& hp, double* partials, hipStream_t s) {
  if (MERGE == 1 || MERGE == 2) {
    if (!ts) {  // the blend and the plain replacement never look at the send-time record
      if (pg) {
        FusedOp<NESTEROV, (MERGE == 1 || MERGE == 2) ? MERGE : 1, true, false> op{tm, nullptr, tg, m, dg, pg, hp};
        return launch_walk(vec, wk, op, partials, s);
      }
      FusedOp<NESTEROV, (MERGE == 1 || MERGE == 2) ? MERGE : 1, false, false> op{tm, nullptr, tg, m, dg, nullptr, hp};
      return launch_walk(vec, wk, op, partials, s);
    }
  }
  if (pg) {
    FusedOp<NESTEROV, MERGE, true> op{tm, ts, tg, m, dg, pg, hp};
    return launch_walk(vec, wk, op, partials, s);
  }
  FusedOp<NESTEROV, MERGE, false> op{tm, ts, tg, m, dg, nullptr, hp};
  return launch_walk(vec, wk, op, partials, s);
}

template <bool NESTEROV>
int launch_fused_m(int merge, bool vec, const HostWalk& wk, float* tm, const float* ts,
                   float* tg, float* m, const float* dg, float* pg, const DevHP& hp, double* partials,
                   hipStream_t s) {
  switch (merge) {
    case 0: return launch_fused<NESTEROV, 0>(vec, wk, tm, ts, tg, m, dg, pg, hp, partials, s);
    case 1: return launch_fused<NESTEROV, 1>(vec, wk, tm, ts, tg, m, dg, pg, hp, partials, s);
    case 2: return launch_fused<NESTEROV, 2>(vec, wk, tm, ts, tg, m, dg, pg, hp, partials, s);
    case 4: return launch_fused<NESTEROV, 4>(vec, wk, tm, ts, tg, m, dg, pg, hp, partials, s);
    default: return launch_fused<NESTEROV, 3>(vec, wk, tm, ts, tg, m, dg, pg, hp, partials, s);
  }
}

// The binary16 pseudo-gradient is an output format: it only exists where a pseudo-gradient is written.
template <bool NESTEROV, int MERGE>
int launch_fused_bf16(bool vec, const HostWalk& wk, unsigned short* tm, const unsigned short* ts,
                      float* tg, float* m, const float* dg, unsigned short* pg, bool pg_f16, const DevHP& hp,
                      double* partials, hipStream_t s) {
  if (MERGE == 1 || MERGE == 2) {
    if (!ts) {
      constexpr int M = (MERGE == 1 || MERGE == 2) ? MERGE : 1;
      if (pg && pg_f16) {
        FusedBf16Op<NESTEROV, M, true, false, true> op{tm, nullptr, tg, m, dg, pg, hp};
        return launch_walk(vec, wk, op, partials, s);
      }
      if (pg) {
        FusedBf16Op<NESTEROV, M, true, false> op{tm, nullptr, tg, m, dg, pg, hp};
        return launch_walk(vec, wk, op, partials, s);
      }
      FusedBf16Op<NESTEROV, M, false, false> op{tm, nullptr, tg, m, dg, nullptr, hp};
      return launch_walk(vec, wk, op, partials, s);
    }
  }
  if (pg && pg_f16) {
    FusedBf16Op<NESTEROV, MERGE, true, true, true> op{tm, ts, tg, m, dg, pg, hp};
    return launch_walk(vec, wk, op, partials, s);
  }
  if (pg) {
    FusedBf16Op<NESTEROV, MERGE, true> op{tm, ts, tg, m, dg, pg, hp};
    return launch_walk(vec, wk, op, partials, s);
  }
  FusedBf16Op<NESTEROV, MERGE, false> op{tm, ts, tg, m, dg, nullptr, hp};
  return launch_walk(vec, wk, op, partials, s);
}

template <bool NESTEROV>
int launch_fused_bf16_m(int merge, bool vec, const HostWalk& wk, unsigned short* tm,
                        const unsigned short* ts, float* tg, float* m, const float* dg, unsigned short* pg,
                        bool pg_f16, const DevHP& hp, double* partials, hipStream_t s) {
  switch (merge) {
    case 0: return launch_fused_bf16<NESTEROV, 0>(vec, wk, tm, ts, tg, m, dg, pg, pg_f16, hp, partials, s);
    case 1: return launch_fused_bf16<NESTEROV, 1>(vec, wk, tm, ts, tg, m, dg, pg, pg_f16, hp, partials, s);
    case 2: return launch_fused_bf16<NESTEROV, 2>(vec, wk, tm, ts, tg, m, dg, pg, pg_f16, hp, partials, s);
    case 4: return launch_fused_bf16<NESTEROV, 4>(vec, wk, tm, ts, tg, m, dg, pg, pg_f16, hp, partials, s);
    default: return launch_fused_bf16<NESTEROV, 3>(vec, wk, tm, ts, tg, m, dg, pg, pg_f16, hp, partials, s);
  }
}

}  // namespace
