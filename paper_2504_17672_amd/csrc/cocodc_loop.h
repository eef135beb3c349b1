// cocodc_loop.h -- the adaptive-transmission loop of the paper's Sec. 3.2 around the kernels:
// host-side schedule state and the cocodc_loop_* entry points.  Included by cocodc.hip only.
#pragma once

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

  // 1. fragments whose all-reduce completes now; 2. is it time to start the next one?  Both are
  //    one event: a single call updates the arrived fragments and ranks all K for the decision.
  std::vector<uint8_t> arrived(static_cast<size_t>(K), 0);
  std::vector<int64_t> I_new(loop->I_p), tb_new(loop->t_b), fly_new(loop->in_flight);
  int32_t n_rec = 0;
  for (int32_t p = 0; p < K; ++p) {
    if (loop->in_flight[p] < 0 || loop->in_flight[p] + loop->hp.tau != t) continue;
    I_new[p] = loop->in_flight[p] - loop->t_b[p];  // Eq. 11: I_p = t_p - t_{p,b}
    tb_new[p] = t;
    fly_new[p] = -1;
    arrived[p] = 1;
    received_out[n_rec++] = p;
  }
  int32_t n_flying = 0;
  for (int32_t p = 0; p < K; ++p) n_flying += fly_new[p] >= 0 ? 1 : 0;
  const bool decide = (t % loop->h == 0) && n_flying < K;
  // the first fragment of the priority order that is not in flight is among the first n_flying + 1
  const int32_t want = decide ? n_flying + 1 : 0;
  if (n_rec > 0) {
    if (int rc = cocodc_sync_event(loop->frags.data(), K, loop->n_total, arrived.data(), buf->theta_m,
                                   buf->theta_m_send, buf->theta_g, buf->momentum, buf->delta_g, nullptr,
                                   I_new.data(), tb_new.data(), t, want, &loop->hp, buf->R, buf->sel, buf->n_sel,
                                   nullptr, buf->workspace, buf->workspace_bytes, stream))
      return rc;
    loop->I_p.swap(I_new);
    loop->t_b.swap(tb_new);
    loop->in_flight.swap(fly_new);
    *n_received_out = n_rec;
  } else if (decide) {
    if (int rc = cocodc_select_fragments(K, buf->R, loop->t_b.data(), t, loop->hp.H, want, buf->sel, buf->n_sel,
                                         buf->workspace, buf->workspace_bytes, stream))
      return rc;
  }
  if (!decide) return COCODC_OK;
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

}  // extern "C"
