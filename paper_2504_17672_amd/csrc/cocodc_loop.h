// cocodc_loop.h -- the adaptive-transmission loop of the paper's Sec. 3.2 around the kernels:
// host-side schedule state and the cocodc_loop_* entry points.  Included by cocodc.hip only.
//
// A loop step never waits for the stream.  The send decision (Algorithm 2 among the fragments
// that are not in flight) is taken by the selection kernel, and the pseudo-gradient of the chosen
// fragment is produced by a kernel that reads the choice from device memory, so the host does not
// need to know p* to enqueue the work.  The choice is copied to a pinned host slot behind an
// event; the schedule reads it (waiting on that event only) when it next needs it: at the next
// send decision or when the fragment could be due, i.e. at least min(h, tau) steps later.
#pragma once

struct cocodc_loop {
  std::vector<cocodc_segment_t> segs;  // the fragments as lists of segments (a contiguous fragment is one)
  Plan full;                           // the tile plan of ALL fragments (the send step walks the chosen one in it)
  int32_t K = 0;
  uint64_t n_total = 0;
  cocodc_hparams_t hp{};
  double gamma = 1.0, T_c = 1.0, T_s = 1.0;
  int64_t N = 1, h = 1;
  std::vector<int64_t> t_b, I_p, in_flight;
  int64_t last_t = 0;  // the step of the previous cocodc_loop_step call; steps must increase
  // a send decision taken on the device whose outcome the host has not read yet
  bool pending = false;
  int64_t pending_t = 0;
  int32_t* chosen_host = nullptr;  // pinned host memory the chosen index is copied to
  hipEvent_t chosen_ready = nullptr;
  int64_t last_sent_t = -1;  // the most recent send decision that has been read back
  int32_t last_sent = -1;
};

namespace {
int replan(cocodc_loop* L) {
  int64_t N = 0, h = 0;
  if (int rc = cocodc_sync_plan(L->K, L->hp.H, L->gamma, L->T_c, L->T_s, &N, &h))
    return rc;
  L->N = N;
  L->h = h < 1 ? 1 : h;  // more syncs than steps: at most one send per step
  return COCODC_OK;
}

// Folds a pending send decision into the bookkeeping (waits for its read-back, nothing else).
int resolve_pending(cocodc_loop* L) {
  if (!L->pending) return COCODC_OK;
  HIP_TRY(hipEventSynchronize(L->chosen_ready));
  L->pending = false;
  const int32_t p = *L->chosen_host;
  L->last_sent_t = L->pending_t;
  L->last_sent = -1;
  if (p >= 0 && p < L->K && L->in_flight[p] < 0) {
    L->in_flight[p] = L->pending_t;
    L->last_sent = p;
  }
  return COCODC_OK;
}

bool due_at(const cocodc_loop* L, size_t p, int64_t t) {
  return L->in_flight[p] >= 0 && L->in_flight[p] + L->hp.tau <= t;
}
}  // namespace

extern "C" {

int cocodc_loop_create_segmented(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total,
                                 const cocodc_hparams_t* hp, double gamma, double T_c, double T_s,
                                 cocodc_loop_t** loop_out) {
  if (!loop_out) return COCODC_ERR_NULL;
  *loop_out = nullptr;
  if (int rc = check_hparams(hp)) return rc;
  Plan pl;
  if (int rc = plan_segments(segs, S, K, n_total, nullptr, nullptr, &pl)) return rc;
  cocodc_loop* L = new cocodc_loop();
  L->segs.assign(segs, segs + S);
  L->full = std::move(pl);
  L->K = K;
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

int cocodc_loop_create(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total,
                       const cocodc_hparams_t* hp, double gamma, double T_c, double T_s,
                       cocodc_loop_t** loop_out) {
  if (!loop_out) return COCODC_ERR_NULL;
  *loop_out = nullptr;
  if (!frags) return COCODC_ERR_NULL;
  if (K < 1 || K > COCODC_MAX_FRAGMENTS) return COCODC_ERR_RANGE;
  std::vector<cocodc_segment_t> segs(static_cast<size_t>(K));
  for (int32_t p = 0; p < K; ++p) segs[p] = cocodc_segment_t{frags[p].offset, frags[p].length, p, 0};
  return cocodc_loop_create_segmented(segs.data(), K, K, n_total, hp, gamma, T_c, T_s, loop_out);
}

void cocodc_loop_destroy(cocodc_loop_t* loop) {
  if (!loop) return;
  if (loop->pending) (void)hipEventSynchronize(loop->chosen_ready);
  if (loop->chosen_ready) (void)hipEventDestroy(loop->chosen_ready);
  if (loop->chosen_host) (void)hipHostFree(loop->chosen_host);
  delete loop;
}

int cocodc_loop_reset_scores(cocodc_loop_t* loop, double* R, void* stream) {
  if (!loop || !R) return COCODC_ERR_NULL;
  if (!aligned(R, 8)) return COCODC_ERR_ALIGN;
  const int K = loop->K;
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

int cocodc_loop_due(cocodc_loop_t* loop, int64_t t, int32_t* due_out, int32_t* n_due_out) {
  if (!loop || !due_out || !n_due_out) return COCODC_ERR_NULL;
  if (loop->pending && loop->pending_t + loop->hp.tau <= t) {
    if (int rc = resolve_pending(loop)) return rc;
  }
  int32_t n = 0;
  for (size_t p = 0; p < loop->t_b.size(); ++p) {
    if (due_at(loop, p, t)) due_out[n++] = static_cast<int32_t>(p);
  }
  *n_due_out = n;
  return COCODC_OK;
}

int cocodc_loop_state(cocodc_loop_t* loop, int64_t* t_b_out, int64_t* I_p_out, int64_t* in_flight_out) {
  if (!loop || !t_b_out || !I_p_out || !in_flight_out) return COCODC_ERR_NULL;
  if (int rc = resolve_pending(loop)) return rc;
  for (size_t p = 0; p < loop->t_b.size(); ++p) {
    t_b_out[p] = loop->t_b[p];
    I_p_out[p] = loop->I_p[p];
    in_flight_out[p] = loop->in_flight[p];
  }
  return COCODC_OK;
}

int cocodc_loop_last_sent(cocodc_loop_t* loop, int64_t* t_sent_out, int32_t* sent_out) {
  if (!loop || !t_sent_out || !sent_out) return COCODC_ERR_NULL;
  if (int rc = resolve_pending(loop)) return rc;
  *t_sent_out = loop->last_sent_t;
  *sent_out = loop->last_sent;
  return COCODC_OK;
}

}  // extern "C"

namespace {
// The buffers of a loop step in either precision: the local parameters, their send-time record
// and the send buffer are fp32 (half == false) or 16-bit patterns (half == true).
struct LoopIO {
  bool half;
  void* theta_m;
  void* theta_m_send;
  float* theta_g;
  float* momentum;
  float* delta_g;
  void* delta_m_out;
  double* R;
  int32_t* sel;
  int32_t* n_sel;
  void* workspace;
  size_t workspace_bytes;
};

// Everything either kind of event could need, checked without touching the device.
int loop_io_check(const cocodc_loop* L, const LoopIO& io) {
  static const int64_t kOne = 1;
  const int32_t K = L->K;
  const int32_t S = static_cast<int32_t>(L->segs.size());
  if (!io.delta_m_out || !io.theta_m_send) return COCODC_ERR_NULL;
  if (io.half) {
    const uint16_t* tm = static_cast<const uint16_t*>(io.theta_m);
    const uint16_t* ts = static_cast<const uint16_t*>(io.theta_m_send);
    const uint16_t* out = static_cast<const uint16_t*>(io.delta_m_out);
    if (int rc = sync_step_bf16_check(tm, ts, io.theta_g, io.momentum, io.delta_g, out, &kOne, &kOne, 1, &L->hp, io.R,
                                      io.sel, io.n_sel, nullptr))
      return rc;
    if (int rc = check_workspace(io.workspace, io.workspace_bytes, S, K, L->n_total)) return rc;
    return sync_step_bf16_overlaps(K, L->n_total, tm, ts, io.theta_g, io.momentum, io.delta_g, out, 1, io.R, io.sel,
                                   io.n_sel, nullptr, io.workspace, io.workspace_bytes);
  }
  float* tm = static_cast<float*>(io.theta_m);
  const float* ts = static_cast<const float*>(io.theta_m_send);
  float* out = static_cast<float*>(io.delta_m_out);
  if (int rc = sync_step_check(tm, ts, io.theta_g, io.momentum, io.delta_g, out, &kOne, &kOne, 1, &L->hp, io.R, io.sel,
                               io.n_sel, nullptr))
    return rc;
  if (int rc = check_workspace(io.workspace, io.workspace_bytes, S, K, L->n_total)) return rc;
  return sync_step_overlaps(K, L->n_total, tm, ts, io.theta_g, io.momentum, io.delta_g, out, 1, io.R, io.sel, io.n_sel,
                            nullptr, io.workspace, io.workspace_bytes);
}

// The fused step on the arrived fragments and Algorithm 2 among those not in flight.
int loop_event(const cocodc_loop* L, Plan& pl, const LoopIO& io, int64_t t, int32_t budget, void* stream) {
  if (io.half) {
    return sync_step_bf16_impl(pl, L->K, L->n_total, static_cast<uint16_t*>(io.theta_m),
                               static_cast<const uint16_t*>(io.theta_m_send), io.theta_g, io.momentum, io.delta_g,
                               nullptr, t, budget, &L->hp, io.R, io.sel, io.n_sel, nullptr, io.workspace,
                               io.workspace_bytes, stream);
  }
  return sync_step_impl(pl, L->K, L->n_total, static_cast<float*>(io.theta_m),
                        static_cast<const float*>(io.theta_m_send), io.theta_g, io.momentum, io.delta_g, nullptr, t,
                        budget, &L->hp, io.R, io.sel, io.n_sel, nullptr, io.workspace, io.workspace_bytes, stream);
}

// Pseudo-gradient and send-time record of the fragment that sel[0] names.
int loop_send(const cocodc_loop* L, const Plan& full, const WorkspaceView& v, const LoopIO& io, uint64_t widest,
              hipStream_t s) {
  const bool vec = all_aligned16({io.theta_g, io.theta_m, io.delta_m_out, io.theta_m_send});
  if (!io.half) {
    PseudoGradOp<true> op{io.theta_g, static_cast<const float*>(io.theta_m), static_cast<float*>(io.delta_m_out),
                          static_cast<float*>(io.theta_m_send)};
    return launch_walk_chosen(vec, full, v, io.sel, widest, op, s);
  }
  const unsigned short* tm = static_cast<const unsigned short*>(io.theta_m);
  unsigned short* out = static_cast<unsigned short*>(io.delta_m_out);
  unsigned short* rec = static_cast<unsigned short*>(io.theta_m_send);
  if (L->hp.pg_format == COCODC_PG_F16) {
    PseudoGradBf16Op<true, true> op{io.theta_g, tm, out, rec};
    return launch_walk_chosen(vec, full, v, io.sel, widest, op, s);
  }
  PseudoGradBf16Op<true, false> op{io.theta_g, tm, out, rec};
  return launch_walk_chosen(vec, full, v, io.sel, widest, op, s);
}

int loop_step_impl(cocodc_loop* loop, int64_t t, const LoopIO& io, void* stream, int32_t* received_out,
                   int32_t* n_received_out, int32_t* sent_out) {
  if (!received_out || !n_received_out || !sent_out) return COCODC_ERR_NULL;
  if (t < 1 || t <= loop->last_t) return COCODC_ERR_RANGE;  // steps are numbered 1, 2, ... and never go back
  const int32_t K = loop->K;
  const int32_t S = static_cast<int32_t>(loop->segs.size());
  // Checked before anything is enqueued, so that a rejected step leaves the buffers and the
  // schedule as they were.
  if (int rc = loop_io_check(loop, io)) return rc;
  *n_received_out = 0;
  *sent_out = -1;
  hipStream_t s = static_cast<hipStream_t>(stream);

  const bool decision_step = (t % loop->h == 0);
  if (loop->pending && (decision_step || loop->pending_t + loop->hp.tau <= t)) {
    if (int rc = resolve_pending(loop)) return rc;
  }

  // 1. fragments whose all-reduce completes now; 2. is it time to start the next one?  Both are
  //    one event: the arrived fragments are updated and all K are ranked for the decision.
  std::vector<uint8_t> mask(static_cast<size_t>(K), 0);
  std::vector<int64_t> I_new(loop->I_p), tb_new(loop->t_b), fly_new(loop->in_flight);
  int32_t n_rec = 0;
  for (int32_t p = 0; p < K; ++p) {
    if (!due_at(loop, static_cast<size_t>(p), t)) continue;
    // Eq. 11: I_p = t_p - t_{p,b}; a fragment sent again at the very step its previous
    // synchronisation completed has t_p = t_{p,b}: the interval is taken as one step, so that
    // R_p = +infinity stays what Sec. 3.2 reserves it for, fragments never synchronised.
    I_new[p] = std::max<int64_t>(1, loop->in_flight[p] - loop->t_b[p]);
    tb_new[p] = t;
    fly_new[p] = -1;
    mask[p] = kMaskArrived;
    received_out[n_rec++] = p;
  }
  int32_t n_flying = 0;
  for (int32_t p = 0; p < K; ++p) {
    if (fly_new[p] >= 0) {
      mask[p] |= kMaskInFlight;
      ++n_flying;
    }
  }
  const bool decide = decision_step && n_flying < K;  // (a pending decision was read back above)
  if (n_rec == 0 && !decide) {
    loop->last_t = t;
    return COCODC_OK;
  }

  Plan pl;
  if (int rc = plan_segments(loop->segs.data(), S, K, loop->n_total, I_new.data(), tb_new.data(), &pl, mask.data()))
    return rc;
  if (int rc = loop_event(loop, pl, io, t, decide ? 1 : 0, stream)) return rc;
  loop->I_p.swap(I_new);
  loop->t_b.swap(tb_new);
  loop->in_flight.swap(fly_new);
  loop->last_t = t;
  *n_received_out = n_rec;
  if (!decide) return COCODC_OK;

  // The chosen fragment's pseudo-gradient and send-time record, for whichever fragment sel[0]
  // names: a walk over that fragment's tiles in the table of ALL fragments (the event above
  // worked on the table of the arrived ones).  Stream order lets a large table reuse the head of
  // the workspace: the event's kernels are done with theirs when the upload runs.
  const Plan& full = loop->full;  // depends on the table alone: made once, when the loop was created
  uint64_t widest = 0;  // tiles of the largest fragment Algorithm 2 could choose
  for (int32_t p = 0; p < K; ++p) {
    if (loop->in_flight[p] < 0) widest = std::max<uint64_t>(widest, full.groups[p + 1].slot_begin - full.groups[p].slot_begin);
  }
  WorkspaceView v = view(io.workspace, full.S, K);
  if (int rc = upload_table(full, v, s)) return rc;
  if (int rc = loop_send(loop, full, v, io, widest, s)) return rc;
  if (!loop->chosen_host)
    HIP_TRY(hipHostMalloc(reinterpret_cast<void**>(&loop->chosen_host), sizeof(int32_t), hipHostMallocDefault));
  if (!loop->chosen_ready) HIP_TRY(hipEventCreateWithFlags(&loop->chosen_ready, hipEventDisableTiming));
  *loop->chosen_host = -1;
  HIP_TRY(hipMemcpyAsync(loop->chosen_host, io.sel, sizeof(int32_t), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipEventRecord(loop->chosen_ready, s));
  loop->pending = true;
  loop->pending_t = t;
  *sent_out = COCODC_LOOP_SENT_PENDING;
  return COCODC_OK;
}
}  // namespace

extern "C" {

int cocodc_loop_step(cocodc_loop_t* loop, int64_t t, const cocodc_loop_buffers_t* buf, void* stream,
                     int32_t* received_out, int32_t* n_received_out, int32_t* sent_out) {
  if (!loop || !buf) return COCODC_ERR_NULL;
  const LoopIO io{false,   buf->theta_m, buf->theta_m_send, buf->theta_g, buf->momentum,  buf->delta_g, buf->delta_m_out,
                  buf->R,  buf->sel,     buf->n_sel,        buf->workspace, buf->workspace_bytes};
  return loop_step_impl(loop, t, io, stream, received_out, n_received_out, sent_out);
}

int cocodc_loop_step_bf16(cocodc_loop_t* loop, int64_t t, const cocodc_loop_buffers_bf16_t* buf, void* stream,
                          int32_t* received_out, int32_t* n_received_out, int32_t* sent_out) {
  if (!loop || !buf) return COCODC_ERR_NULL;
  const LoopIO io{true,    buf->theta_m, buf->theta_m_send, buf->theta_g, buf->momentum,  buf->delta_g, buf->delta_m_out,
                  buf->R,  buf->sel,     buf->n_sel,        buf->workspace, buf->workspace_bytes};
  return loop_step_impl(loop, t, io, stream, received_out, n_received_out, sent_out);
}

}  // extern "C"
