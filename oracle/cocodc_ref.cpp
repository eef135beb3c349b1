// cocodc_ref.cpp -- CPU oracle (fp64, index order) for the CoCoDC outer-sync path.
//
// TEST INFRASTRUCTURE ONLY; see cocodc_ref.h.  Shares nothing with the HIP sources.
// Build: g++ -O2 -ffp-contract=off -fopenmp -shared -fPIC (no fast-math: the order
// and rounding of every operation below is part of the definition).
//
// Notation (paper Sec. 2 and 3):
//   theta_g   : global state of a fragment; on entry theta^g_{p,t_p-H}, on exit theta^g_{p,t_p}
//   theta_m   : the worker's current local parameters theta^m_{p,t_l}
//   theta_send: the local parameters recorded when the fragment was sent, theta^m_{p,t_p}
//   delta_g   : the averaged global pseudo-gradient of Eq. 1, arriving tau steps late,
//               in the sign convention "global minus local" (descent direction)
//   m         : momentum buffer of the outer optimiser of Eq. 2

#include "cocodc_ref.h"

#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>

#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

constexpr int kOk = 0;
constexpr int kErrNull = -1;
constexpr int kErrRange = -3;

int check_table(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total) {
  if (frags == nullptr) return kErrNull;
  if (K < 1) return kErrRange;
  for (int32_t p = 0; p < K; ++p) {
    if (frags[p].offset > n_total || frags[p].length > n_total - frags[p].offset) return kErrRange;
  }
  for (int32_t p = 0; p < K; ++p) {
    for (int32_t q = p + 1; q < K; ++q) {
      if (frags[p].length == 0 || frags[q].length == 0) continue;
      const uint64_t a0 = frags[p].offset, a1 = a0 + frags[p].length;
      const uint64_t b0 = frags[q].offset, b1 = b0 + frags[q].length;
      if (a0 < b1 && b0 < a1) return kErrRange;  // fragments must be disjoint
    }
  }
  return kOk;
}

int check_hparams(const cocodc_ref_hparams_t* hp) {
  if (hp == nullptr) return kErrNull;
  if (hp->tau < 0 || hp->H < 1) return kErrRange;
  if (hp->drift_sign != 1 && hp->drift_sign != -1) return kErrRange;
  if (hp->score_src != 0 && hp->score_src != 1) return kErrRange;
  if (hp->norm_kind != 1 && hp->norm_kind != 2) return kErrRange;
  if (hp->merge_mode < 0 || hp->merge_mode > 2) return kErrRange;
  if (hp->delta_src != 0 && hp->delta_src != 1) return kErrRange;
  if (hp->pg_format != 0 && hp->pg_format != 1) return kErrRange;
  if (!std::isfinite(hp->lambda) || !std::isfinite(hp->eta) || !std::isfinite(hp->mu) ||
      !std::isfinite(hp->alpha))
    return kErrRange;
  return kOk;
}

// Eq. 2, OuterOptim = SGD with momentum mu and learning rate eta applied to the
// "gradient" delta_g:  m' = mu*m + delta_g ; step = delta_g + mu*m' (Nesterov) or m' ;
// theta^g_{p,t_p} = theta^g_{p,t_p-H} - eta*step.  Returns the unrounded new state.
inline double outer_update(double theta_g_old, double m_old, double dg,
                           const cocodc_ref_hparams_t& hp, double* m_new) {
  const double m1 = hp.mu * m_old + dg;
  const double step = hp.nesterov ? (dg + hp.mu * m1) : m1;
  *m_new = m1;
  return theta_g_old - hp.eta * step;
}

// d = tau * g, with g the change rate of Eq. 4: g = (theta^m_{p,t_p} - theta^m_{p,t_l}) / tau.
inline double drift_times_tau(double theta_send, double theta_m, const cocodc_ref_hparams_t& hp) {
  return static_cast<double>(hp.drift_sign) * (theta_send - theta_m);
}

// The merge of the new global state G (already rounded to fp32) into the local
// parameters.  merge_mode 0 is Algorithm 1:
//   Eq. 4:  g      = d / tau
//   Eq. 7:  g_corr = g + lambda * g*g * Delta / H,  Delta = G - theta_send (the difference
//           defined with Eq. 5), products taken element by element
//   Eq. 8:  theta^m_{p,t_l} <- G + g_corr * tau = G + d + lambda * d*d*Delta / (tau*H)
// Written in terms of d so that tau = 0 (no overlap, hence d = 0) needs no division.
// theta_g_prev is the global state before the outer step; only delta_src 1 looks at it.
inline double merge_local(double G, double theta_send, double theta_m, double d,
                          const cocodc_ref_hparams_t& hp, double theta_g_prev = 0.0) {
  if (hp.merge_mode == 1) return (1.0 - hp.alpha) * theta_m + hp.alpha * G;  // Eq. 3
  if (hp.merge_mode == 2) return G;  // blocking DiLoCo: adopt the global state
  const double Delta = hp.delta_src ? (theta_send - theta_g_prev) : (G - theta_send);
  double corr = 0.0;
  if (hp.tau >= 1) {
    const double tauH = static_cast<double>(hp.tau) * static_cast<double>(hp.H);
    corr = hp.lambda * d * d * Delta / tauH;
  }
  return G + d + corr;
}

struct Sums {
  double g2 = 0.0, g1 = 0.0, d2 = 0.0, d1 = 0.0;
};

// One element of the fused step.  Reads everything first (delta_m_out may alias delta_g).
inline void sync_element(uint64_t i, float* theta_m, const float* theta_send, float* theta_g,
                         float* momentum, const float* delta_g, float* delta_m_out,
                         const cocodc_ref_hparams_t& hp, Sums* s, const cocodc_ref_shadow_t* sh) {
  const double tg = theta_g[i], tm = theta_m[i];
  // Eq. 3 and the blocking merge have no send-time record: without one the drift is zero
  const double ts = theta_send ? theta_send[i] : tm;
  const double m0 = momentum[i], dg = delta_g[i];

  const float pg = static_cast<float>(tg - tm);  // pseudo-gradient, global minus local

  double m1;
  const double G64 = outer_update(tg, m0, dg, hp, &m1);
  const float G = static_cast<float>(G64);  // what an unfused caller would read back

  const double d = drift_times_tau(ts, tm, hp);
  const double tm_new = merge_local(static_cast<double>(G), ts, tm, d, hp, tg);

  s->g2 += dg * dg;  // Eq. 11 numerator, squared
  s->g1 += std::fabs(dg);
  s->d2 += d * d;
  s->d1 += std::fabs(d);

  if (delta_m_out) delta_m_out[i] = pg;
  momentum[i] = static_cast<float>(m1);
  theta_g[i] = G;
  theta_m[i] = static_cast<float>(tm_new);
  if (sh) {
    if (sh->theta_m) sh->theta_m[i] = tm_new;
    if (sh->theta_g) sh->theta_g[i] = G64;
    if (sh->momentum) sh->momentum[i] = m1;
  }
}

// Eq. 11 from the accumulated sums.
inline double score_from_sums(const Sums& s, int64_t I_p, const cocodc_ref_hparams_t& hp) {
  if (I_p <= 0) return std::numeric_limits<double>::infinity();
  const double s2 = hp.score_src ? s.d2 : s.g2;
  const double s1 = hp.score_src ? s.d1 : s.g1;
  const double norm = (hp.norm_kind == 2) ? std::sqrt(s2) : s1;
  return norm / static_cast<double>(I_p);
}

}  // namespace

extern "C" {

int cocodc_ref_pseudograd(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                          const float* theta_g_snap, const float* theta_m, float* delta_m_out,
                          float* theta_m_send_out) {
  if (!theta_g_snap || !theta_m || !delta_m_out) return kErrNull;
  if (int rc = check_table(frags, K, n_total)) return rc;
  for (int32_t p = 0; p < K; ++p) {
    for (uint64_t i = frags[p].offset; i < frags[p].offset + frags[p].length; ++i) {
      const double tg = theta_g_snap[i], tm = theta_m[i];
      delta_m_out[i] = static_cast<float>(tg - tm);
      if (theta_m_send_out) theta_m_send_out[i] = theta_m[i];
    }
  }
  return kOk;
}

int cocodc_ref_outer_nesterov(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                              float* theta_g, float* momentum, const float* delta_g,
                              const cocodc_ref_hparams_t* hp) {
  if (!theta_g || !momentum || !delta_g) return kErrNull;
  if (int rc = check_table(frags, K, n_total)) return rc;
  if (int rc = check_hparams(hp)) return rc;
  for (int32_t p = 0; p < K; ++p) {
    for (uint64_t i = frags[p].offset; i < frags[p].offset + frags[p].length; ++i) {
      double m1;
      const double G = outer_update(theta_g[i], momentum[i], delta_g[i], *hp, &m1);
      momentum[i] = static_cast<float>(m1);
      theta_g[i] = static_cast<float>(G);
    }
  }
  return kOk;
}

int cocodc_ref_delay_compensate(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                                float* theta_m, const float* theta_m_send, const float* theta_g,
                                const cocodc_ref_hparams_t* hp) {
  if (!theta_m || !theta_g) return kErrNull;
  if (int rc = check_table(frags, K, n_total)) return rc;
  if (int rc = check_hparams(hp)) return rc;
  if (!theta_m_send && hp->merge_mode == 0) return kErrNull;  // Algorithm 1 needs theta^m_{p,t_p}
  if (hp->delta_src == 1 && hp->merge_mode == 0) return kErrRange;  // needs theta^g_{p,t_p-H}: fused only
  for (int32_t p = 0; p < K; ++p) {
    for (uint64_t i = frags[p].offset; i < frags[p].offset + frags[p].length; ++i) {
      const double tm = theta_m[i], ts = theta_m_send ? theta_m_send[i] : tm, G = theta_g[i];
      const double d = drift_times_tau(ts, tm, *hp);
      theta_m[i] = static_cast<float>(merge_local(G, ts, tm, d, *hp));
    }
  }
  return kOk;
}

int cocodc_ref_fragment_scores(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                               const float* x, const int64_t* I_p, int32_t norm_kind,
                               double* R_out, double* sum_out) {
  if (!x || !I_p || !R_out) return kErrNull;
  if (int rc = check_table(frags, K, n_total)) return rc;
  if (norm_kind != 1 && norm_kind != 2) return kErrRange;
  for (int32_t p = 0; p < K; ++p) {
    double acc = 0.0;
    for (uint64_t i = frags[p].offset; i < frags[p].offset + frags[p].length; ++i) {
      const double v = x[i];
      acc += (norm_kind == 2) ? v * v : std::fabs(v);
    }
    if (sum_out) sum_out[p] = acc;
    const double norm = (norm_kind == 2) ? std::sqrt(acc) : acc;
    R_out[p] = (I_p[p] <= 0) ? std::numeric_limits<double>::infinity()
                             : norm / static_cast<double>(I_p[p]);
  }
  return kOk;
}

// Algorithm 2, run `budget` times; a fragment already chosen in this call is skipped, and so
// is one whose all-reduce is still in flight (in_flight, nullable: nobody is).
// Each run: the first fragment (lowest index) not synchronised for at least H steps
// wins; otherwise the fragment with the largest R_p, the first one on ties.  A NaN
// score never beats a number (it can only be chosen when nothing else is left).
namespace {
int select_among(int32_t K, const double* R, const int64_t* t_b, int64_t t_g, int32_t H,
                 int32_t budget, const uint8_t* in_flight, int32_t* sel_out, int32_t* n_sel_out) {
  std::vector<char> taken(static_cast<size_t>(K), 0);
  int32_t candidates = 0;
  for (int32_t p = 0; p < K; ++p) {
    if (in_flight && in_flight[p]) taken[p] = 1; else ++candidates;
  }
  const int32_t n_sel = budget < candidates ? budget : candidates;
  for (int32_t b = 0; b < n_sel; ++b) {
    int32_t p_star = -1;
    for (int32_t p = 0; p < K; ++p) {
      if (taken[p]) continue;
      if (t_g - t_b[p] >= static_cast<int64_t>(H)) {
        p_star = p;
        break;
      }
    }
    if (p_star < 0) {
      for (int32_t p = 0; p < K; ++p) {
        if (taken[p]) continue;
        if (p_star < 0) {
          p_star = p;
        } else if (std::isnan(R[p_star]) ? !std::isnan(R[p]) : (R[p] > R[p_star])) {
          p_star = p;
        }
      }
    }
    taken[p_star] = 1;
    sel_out[b] = p_star;
  }
  *n_sel_out = n_sel;
  return kOk;
}
}  // namespace

int cocodc_ref_select_fragments(int32_t K, const double* R, const int64_t* t_b, int64_t t_g,
                                int32_t H, int32_t budget, int32_t* sel_out, int32_t* n_sel_out) {
  if (!R || !t_b || !sel_out || !n_sel_out) return kErrNull;
  if (K < 1 || H < 1 || budget < 0) return kErrRange;
  return select_among(K, R, t_b, t_g, H, budget, nullptr, sel_out, n_sel_out);
}

int cocodc_ref_select_fragments_bytes(int32_t K, const double* R, const int64_t* t_b, int64_t t_g,
                                      int32_t H, const uint64_t* frag_bytes, uint64_t byte_budget,
                                      int32_t* sel_out, int32_t* n_sel_out) {
  if (!frag_bytes) return kErrNull;
  std::vector<int32_t> order(static_cast<size_t>(K > 0 ? K : 1));
  int32_t n_all = 0;
  if (int rc = cocodc_ref_select_fragments(K, R, t_b, t_g, H, K, order.data(), &n_all)) return rc;
  uint64_t left = byte_budget;
  int32_t n = 0;
  for (int32_t i = 0; i < n_all; ++i) {
    const uint64_t need = frag_bytes[order[i]];
    if (need > left) break;  // the next fragment in priority order does not fit: stop
    left -= need;
    sel_out[n++] = order[i];
  }
  *n_sel_out = n;
  return kOk;
}

int cocodc_ref_sync_step(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                         float* theta_m, const float* theta_m_send, float* theta_g,
                         float* momentum, const float* delta_g, float* delta_m_out,
                         const int64_t* I_p, const int64_t* t_b, int64_t t_g, int32_t budget,
                         const cocodc_ref_hparams_t* hp, double* R_out, int32_t* sel_out,
                         int32_t* n_sel_out, double* sums_out, const cocodc_ref_shadow_t* shadow) {
  if (!theta_m || !theta_g || !momentum || !delta_g) return kErrNull;
  if (!I_p || !t_b || !R_out || !sel_out || !n_sel_out) return kErrNull;
  if (int rc = check_table(frags, K, n_total)) return rc;
  if (int rc = check_hparams(hp)) return rc;
  if (!theta_m_send && (hp->merge_mode == 0 || hp->score_src == 1)) return kErrNull;
  if (budget < 0) return kErrRange;
  for (int32_t p = 0; p < K; ++p) {
    Sums s;
    for (uint64_t i = frags[p].offset; i < frags[p].offset + frags[p].length; ++i) {
      sync_element(i, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, *hp, &s,
                   shadow);
    }
    R_out[p] = score_from_sums(s, I_p[p], *hp);
    if (sums_out) {
      sums_out[4 * p + 0] = s.g2;
      sums_out[4 * p + 1] = s.g1;
      sums_out[4 * p + 2] = s.d2;
      sums_out[4 * p + 3] = s.d1;
    }
  }
  return cocodc_ref_select_fragments(K, R_out, t_b, t_g, hp->H, budget, sel_out, n_sel_out);
}

/* One event of the loop of Sec. 3.2.  recv_mask[q] bit 0: fragment q has just arrived (Alg. 1 and
 * Eq. 2 for it, its score R_q of Eq. 11 replaces the old one); the others keep their buffers and
 * their scores.  Bit 1: fragment q is in flight and cannot be chosen.  Then Alg. 2 looks at the
 * scores of all fragments that are not in flight. */
int cocodc_ref_sync_event(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                          const uint8_t* recv_mask, float* theta_m, const float* theta_m_send,
                          float* theta_g, float* momentum, const float* delta_g, float* delta_m_out,
                          const int64_t* I_p, const int64_t* t_b, int64_t t_g, int32_t budget,
                          const cocodc_ref_hparams_t* hp, double* R, int32_t* sel_out,
                          int32_t* n_sel_out, double* sums_out) {
  if (!recv_mask || !theta_m || !theta_g || !momentum || !delta_g) return kErrNull;
  if (!I_p || !t_b || !R || !sel_out || !n_sel_out) return kErrNull;
  if (int rc = check_table(frags, K, n_total)) return rc;
  if (int rc = check_hparams(hp)) return rc;
  if (!theta_m_send && (hp->merge_mode == 0 || hp->score_src == 1)) return kErrNull;
  if (budget < 0) return kErrRange;
  std::vector<uint8_t> in_flight(static_cast<size_t>(K), 0);
  for (int32_t q = 0; q < K; ++q) {
    if (recv_mask[q] > 3) return kErrRange;
    in_flight[q] = (recv_mask[q] & 2) ? 1 : 0;
  }
  for (int32_t q = 0; q < K; ++q) {
    if (!(recv_mask[q] & 1)) continue;
    Sums s;
    for (uint64_t i = frags[q].offset; i < frags[q].offset + frags[q].length; ++i) {
      sync_element(i, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, *hp, &s,
                   nullptr);
    }
    R[q] = score_from_sums(s, I_p[q], *hp);
    if (sums_out) {
      sums_out[4 * q + 0] = s.g2;
      sums_out[4 * q + 1] = s.g1;
      sums_out[4 * q + 2] = s.d2;
      sums_out[4 * q + 3] = s.d1;
    }
  }
  return select_among(K, R, t_b, t_g, hp->H, budget, in_flight.data(), sel_out, n_sel_out);
}

int cocodc_ref_sync_step_mt(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                            float* theta_m, const float* theta_m_send, float* theta_g,
                            float* momentum, const float* delta_g, float* delta_m_out,
                            const int64_t* I_p, const int64_t* t_b, int64_t t_g, int32_t budget,
                            const cocodc_ref_hparams_t* hp, double* R_out, int32_t* sel_out,
                            int32_t* n_sel_out, double* sums_out, int32_t n_threads) {
  if (!theta_m || !theta_g || !momentum || !delta_g) return kErrNull;
  if (!I_p || !t_b || !R_out || !sel_out || !n_sel_out) return kErrNull;
  if (int rc = check_table(frags, K, n_total)) return rc;
  if (int rc = check_hparams(hp)) return rc;
  if (!theta_m_send && (hp->merge_mode == 0 || hp->score_src == 1)) return kErrNull;
  if (budget < 0) return kErrRange;
  constexpr uint64_t kChunk = 65536;
  int used = 1;
#ifdef _OPENMP
  if (n_threads > 0) omp_set_num_threads(n_threads);
  used = omp_get_max_threads();
#else
  (void)n_threads;
#endif
  for (int32_t p = 0; p < K; ++p) {
    const uint64_t off = frags[p].offset, len = frags[p].length;
    const int64_t n_chunks = static_cast<int64_t>((len + kChunk - 1) / kChunk);
    std::vector<Sums> part(static_cast<size_t>(n_chunks));
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < n_chunks; ++c) {
      const uint64_t lo = off + static_cast<uint64_t>(c) * kChunk;
      const uint64_t hi = (lo + kChunk < off + len) ? lo + kChunk : off + len;
      Sums s;
      for (uint64_t i = lo; i < hi; ++i) {
        sync_element(i, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, *hp, &s,
                     nullptr);
      }
      part[static_cast<size_t>(c)] = s;
    }
    Sums s;
    for (int64_t c = 0; c < n_chunks; ++c) {
      s.g2 += part[c].g2;
      s.g1 += part[c].g1;
      s.d2 += part[c].d2;
      s.d1 += part[c].d1;
    }
    R_out[p] = score_from_sums(s, I_p[p], *hp);
    if (sums_out) {
      sums_out[4 * p + 0] = s.g2;
      sums_out[4 * p + 1] = s.g1;
      sums_out[4 * p + 2] = s.d2;
      sums_out[4 * p + 3] = s.d1;
    }
  }
  int rc = cocodc_ref_select_fragments(K, R_out, t_b, t_g, hp->H, budget, sel_out, n_sel_out);
  return rc < 0 ? rc : used;
}

namespace {
int check_segments(const cocodc_ref_segment_t* segs, int32_t S, int32_t K, uint64_t n_total) {
  if (segs == nullptr && S > 0) return kErrNull;
  if (K < 1 || S < 0) return kErrRange;
  for (int32_t i = 0; i < S; ++i) {
    if (segs[i].fragment < 0 || segs[i].fragment >= K) return kErrRange;
    if (segs[i].offset > n_total || segs[i].length > n_total - segs[i].offset) return kErrRange;
  }
  for (int32_t i = 0; i < S; ++i) {
    for (int32_t j = i + 1; j < S; ++j) {
      if (segs[i].length == 0 || segs[j].length == 0) continue;
      const uint64_t a0 = segs[i].offset, a1 = a0 + segs[i].length;
      const uint64_t b0 = segs[j].offset, b1 = b0 + segs[j].length;
      if (a0 < b1 && b0 < a1) return kErrRange;
    }
  }
  return kOk;
}
}  // namespace

int cocodc_ref_fragment_scores_segmented(const cocodc_ref_segment_t* segs, int32_t S, int32_t K,
                                         uint64_t n_total, const float* x, const int64_t* I_p,
                                         int32_t norm_kind, double* R_out, double* sum_out) {
  if (!x || !I_p || !R_out) return kErrNull;
  if (int rc = check_segments(segs, S, K, n_total)) return rc;
  if (norm_kind != 1 && norm_kind != 2) return kErrRange;
  for (int32_t p = 0; p < K; ++p) {
    double acc = 0.0;
    for (int32_t j = 0; j < S; ++j) {
      if (segs[j].fragment != p) continue;
      for (uint64_t i = segs[j].offset; i < segs[j].offset + segs[j].length; ++i) {
        const double v = x[i];
        acc += (norm_kind == 2) ? v * v : std::fabs(v);
      }
    }
    if (sum_out) sum_out[p] = acc;
    const double norm = (norm_kind == 2) ? std::sqrt(acc) : acc;
    R_out[p] = (I_p[p] <= 0) ? std::numeric_limits<double>::infinity()
                             : norm / static_cast<double>(I_p[p]);
  }
  return kOk;
}

int cocodc_ref_sync_step_segmented(const cocodc_ref_segment_t* segs, int32_t S, int32_t K,
                                   uint64_t n_total, float* theta_m, const float* theta_m_send,
                                   float* theta_g, float* momentum, const float* delta_g,
                                   float* delta_m_out, const int64_t* I_p, const int64_t* t_b,
                                   int64_t t_g, int32_t budget, const cocodc_ref_hparams_t* hp,
                                   double* R_out, int32_t* sel_out, int32_t* n_sel_out,
                                   double* sums_out, const cocodc_ref_shadow_t* shadow) {
  if (!theta_m || !theta_g || !momentum || !delta_g) return kErrNull;
  if (!I_p || !t_b || !R_out || !sel_out || !n_sel_out) return kErrNull;
  if (int rc = check_segments(segs, S, K, n_total)) return rc;
  if (int rc = check_hparams(hp)) return rc;
  if (!theta_m_send && (hp->merge_mode == 0 || hp->score_src == 1)) return kErrNull;
  if (budget < 0) return kErrRange;
  for (int32_t p = 0; p < K; ++p) {
    Sums s;
    for (int32_t j = 0; j < S; ++j) {
      if (segs[j].fragment != p) continue;
      for (uint64_t i = segs[j].offset; i < segs[j].offset + segs[j].length; ++i) {
        sync_element(i, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, *hp, &s,
                     shadow);
      }
    }
    R_out[p] = score_from_sums(s, I_p[p], *hp);
    if (sums_out) {
      sums_out[4 * p + 0] = s.g2;
      sums_out[4 * p + 1] = s.g1;
      sums_out[4 * p + 2] = s.d2;
      sums_out[4 * p + 3] = s.d1;
    }
  }
  return cocodc_ref_select_fragments(K, R_out, t_b, t_g, hp->H, budget, sel_out, n_sel_out);
}

/* One event of the loop of Sec. 3.2 for fragments made of segments (the strided shards of Sec. 4.1):
 * recv_mask per FRAGMENT as in cocodc_ref_sync_event; an arrived fragment's segments are walked in the
 * order listed. */
int cocodc_ref_sync_event_segmented(const cocodc_ref_segment_t* segs, int32_t S, int32_t K,
                                    uint64_t n_total, const uint8_t* recv_mask, float* theta_m,
                                    const float* theta_m_send, float* theta_g, float* momentum,
                                    const float* delta_g, float* delta_m_out, const int64_t* I_p,
                                    const int64_t* t_b, int64_t t_g, int32_t budget,
                                    const cocodc_ref_hparams_t* hp, double* R, int32_t* sel_out,
                                    int32_t* n_sel_out, double* sums_out) {
  if (!recv_mask || !theta_m || !theta_g || !momentum || !delta_g) return kErrNull;
  if (!I_p || !t_b || !R || !sel_out || !n_sel_out) return kErrNull;
  if (int rc = check_segments(segs, S, K, n_total)) return rc;
  if (int rc = check_hparams(hp)) return rc;
  if (!theta_m_send && (hp->merge_mode == 0 || hp->score_src == 1)) return kErrNull;
  if (budget < 0) return kErrRange;
  std::vector<uint8_t> in_flight(static_cast<size_t>(K), 0);
  for (int32_t q = 0; q < K; ++q) {
    if (recv_mask[q] > 3) return kErrRange;
    in_flight[q] = (recv_mask[q] & 2) ? 1 : 0;
  }
  for (int32_t q = 0; q < K; ++q) {
    if (!(recv_mask[q] & 1)) continue;
    Sums s;
    for (int32_t j = 0; j < S; ++j) {
      if (segs[j].fragment != q) continue;
      for (uint64_t i = segs[j].offset; i < segs[j].offset + segs[j].length; ++i) {
        sync_element(i, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, *hp, &s,
                     nullptr);
      }
    }
    R[q] = score_from_sums(s, I_p[q], *hp);
    if (sums_out) {
      sums_out[4 * q + 0] = s.g2;
      sums_out[4 * q + 1] = s.g1;
      sums_out[4 * q + 2] = s.d2;
      sums_out[4 * q + 3] = s.d1;
    }
  }
  return select_among(K, R, t_b, t_g, hp->H, budget, in_flight.data(), sel_out, n_sel_out);
}

// ---- bf16 local parameters ------------------------------------------------------------
// bfloat16 = the upper half of an IEEE binary32: 8 significant bits, exponents -126..127,
// subnormal spacing 2^-133.
double cocodc_ref_widen_bf16(uint16_t b) {
  const uint32_t u = static_cast<uint32_t>(b) << 16;
  float f;
  std::memcpy(&f, &u, sizeof(f));
  return static_cast<double>(f);
}

// Nearest bf16 to x, ties to even: scale so that one bf16 step becomes 1, round to the
// nearest integer (current rounding mode = to nearest even), scale back.  All three steps
// are exact except the rounding itself.
uint16_t cocodc_ref_round_bf16(double x) {
  if (std::isnan(x)) return 0x7FC0;
  double r = x;
  if (x != 0.0 && !std::isinf(x)) {
    int e = std::ilogb(x);       // x = f * 2^e, 1 <= |f| < 2
    if (e < -126) e = -126;      // subnormal range: fixed spacing
    const int q = e - 7;         // exponent of one unit in the last place
    r = std::ldexp(std::nearbyint(std::ldexp(x, -q)), q);
  }
  const float f = static_cast<float>(r);  // exact for every bf16 value; beyond the range -> inf
  uint32_t u;
  std::memcpy(&u, &f, sizeof(u));
  return static_cast<uint16_t>(u >> 16);
}

// IEEE binary16: 11 significant bits, exponents -14..15, subnormal spacing 2^-24, largest
// finite value 65504.
double cocodc_ref_widen_f16(uint16_t b) {
  const int sign = (b >> 15) & 1, e = (b >> 10) & 0x1F, m = b & 0x3FF;
  double v;
  if (e == 0x1F) {
    v = m ? std::numeric_limits<double>::quiet_NaN() : std::numeric_limits<double>::infinity();
  } else if (e == 0) {
    v = std::ldexp(static_cast<double>(m), -24);           // subnormal: m * 2^-24
  } else {
    v = std::ldexp(static_cast<double>(1024 + m), e - 25);  // (1 + m/1024) * 2^(e-15)
  }
  return sign ? -v : v;
}

// Nearest binary16 to x, ties to even: scale so that one binary16 step at x's magnitude becomes
// 1, round to the nearest integer (current rounding mode = to nearest even), and read the
// exponent and fraction fields off that integer.
uint16_t cocodc_ref_round_f16(double x) {
  if (std::isnan(x)) return 0x7E00;
  const uint16_t sign = std::signbit(x) ? 0x8000 : 0;
  const double a = std::fabs(x);
  if (a == 0.0) return sign;
  if (std::isinf(a)) return sign | 0x7C00;
  int e = std::ilogb(a);             // a = f * 2^e, 1 <= f < 2
  if (e < -14) e = -14;              // subnormal range: fixed spacing 2^-24
  if (e > 15) return sign | 0x7C00;  // beyond the largest exponent
  double q = std::nearbyint(std::ldexp(a, 10 - e));  // a in units of 2^(e-10): 1024 <= q <= 2048, or q < 1024 (subnormal)
  if (q >= 2048.0) {                 // rounded up to the next power of two
    q = 1024.0;
    e += 1;
    if (e > 15) return sign | 0x7C00;  // 65520 and above round to infinity
  }
  const int qi = static_cast<int>(q);
  if (qi < 1024) return sign | static_cast<uint16_t>(qi);  // subnormal (or zero): exponent field 0
  return sign | static_cast<uint16_t>(((e + 15) << 10) | (qi - 1024));
}

namespace {
inline uint16_t round_half(double x, int32_t pg_format) {
  return pg_format ? cocodc_ref_round_f16(x) : cocodc_ref_round_bf16(x);
}
}  // namespace

int cocodc_ref_pseudograd_bf16(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                               const float* theta_g_snap, const uint16_t* theta_m,
                               uint16_t* delta_m_out, uint16_t* theta_m_send_out, int32_t pg_format) {
  if (!theta_g_snap || !theta_m || !delta_m_out) return kErrNull;
  if (pg_format != 0 && pg_format != 1) return kErrRange;
  if (int rc = check_table(frags, K, n_total)) return rc;
  for (int32_t p = 0; p < K; ++p) {
    for (uint64_t i = frags[p].offset; i < frags[p].offset + frags[p].length; ++i) {
      const double tg = theta_g_snap[i], tm = cocodc_ref_widen_bf16(theta_m[i]);
      delta_m_out[i] = round_half(tg - tm, pg_format);
      if (theta_m_send_out) theta_m_send_out[i] = theta_m[i];
    }
  }
  return kOk;
}

namespace {
// One element of the fused step when the local parameters, their send-time record and the outgoing
// pseudo-gradient are 16-bit: widened exactly on load, the arithmetic of sync_element, one rounding
// on store (local parameters to bf16, pseudo-gradient to hp.pg_format).
inline void sync_element_bf16(uint64_t i, uint16_t* theta_m, const uint16_t* theta_send, float* theta_g,
                              float* momentum, const float* delta_g, uint16_t* delta_m_out,
                              const cocodc_ref_hparams_t& hp, Sums* s, const cocodc_ref_shadow_t* sh) {
  const double tg = theta_g[i], tm = cocodc_ref_widen_bf16(theta_m[i]);
  const double ts = theta_send ? cocodc_ref_widen_bf16(theta_send[i]) : tm;
  const double m0 = momentum[i], dg = delta_g[i];
  double m1;
  const double G64 = outer_update(tg, m0, dg, hp, &m1);   // Eq. 2
  const float G = static_cast<float>(G64);                 // the stored fp32 global state
  const double d = drift_times_tau(ts, tm, hp);            // Eq. 4 times tau
  const double tm_new = merge_local(static_cast<double>(G), ts, tm, d, hp, tg);  // Eq. 7, 8
  s->g2 += dg * dg;
  s->g1 += std::fabs(dg);
  s->d2 += d * d;
  s->d1 += std::fabs(d);
  if (delta_m_out) delta_m_out[i] = round_half(tg - tm, hp.pg_format);
  momentum[i] = static_cast<float>(m1);
  theta_g[i] = G;
  theta_m[i] = cocodc_ref_round_bf16(tm_new);
  if (sh) {
    if (sh->theta_m) sh->theta_m[i] = tm_new;
    if (sh->theta_g) sh->theta_g[i] = G64;
    if (sh->momentum) sh->momentum[i] = m1;
  }
}

inline void store_sums(const Sums& s, int32_t p, double* sums_out) {
  if (!sums_out) return;
  sums_out[4 * p + 0] = s.g2;
  sums_out[4 * p + 1] = s.g1;
  sums_out[4 * p + 2] = s.d2;
  sums_out[4 * p + 3] = s.d1;
}

int check_sync_bf16(const uint16_t* theta_m, const uint16_t* theta_m_send, const float* theta_g,
                    const float* momentum, const float* delta_g, const int64_t* I_p, const int64_t* t_b,
                    int32_t budget, const cocodc_ref_hparams_t* hp, const double* R, const int32_t* sel_out,
                    const int32_t* n_sel_out) {
  if (!theta_m || !theta_g || !momentum || !delta_g) return kErrNull;
  if (!I_p || !t_b || !R || !sel_out || !n_sel_out) return kErrNull;
  if (int rc = check_hparams(hp)) return rc;
  if (!theta_m_send && (hp->merge_mode == 0 || hp->score_src == 1)) return kErrNull;
  if (budget < 0) return kErrRange;
  return kOk;
}
}  // namespace

int cocodc_ref_sync_step_bf16(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                              uint16_t* theta_m, const uint16_t* theta_m_send, float* theta_g,
                              float* momentum, const float* delta_g, uint16_t* delta_m_out,
                              const int64_t* I_p, const int64_t* t_b, int64_t t_g, int32_t budget,
                              const cocodc_ref_hparams_t* hp, double* R_out, int32_t* sel_out,
                              int32_t* n_sel_out, double* sums_out,
                              const cocodc_ref_shadow_t* shadow) {
  if (int rc = check_sync_bf16(theta_m, theta_m_send, theta_g, momentum, delta_g, I_p, t_b, budget, hp, R_out,
                               sel_out, n_sel_out))
    return rc;
  if (int rc = check_table(frags, K, n_total)) return rc;
  for (int32_t p = 0; p < K; ++p) {
    Sums s;
    for (uint64_t i = frags[p].offset; i < frags[p].offset + frags[p].length; ++i) {
      sync_element_bf16(i, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, *hp, &s, shadow);
    }
    R_out[p] = score_from_sums(s, I_p[p], *hp);
    store_sums(s, p, sums_out);
  }
  return cocodc_ref_select_fragments(K, R_out, t_b, t_g, hp->H, budget, sel_out, n_sel_out);
}

/* The same step over fragments made of segments (the strided shards of Sec. 4.1 with the 16-bit
 * local parameters of its mixed-precision training): a fragment's segments are walked in the order
 * listed. */
int cocodc_ref_sync_step_bf16_segmented(const cocodc_ref_segment_t* segs, int32_t S, int32_t K,
                                        uint64_t n_total, uint16_t* theta_m, const uint16_t* theta_m_send,
                                        float* theta_g, float* momentum, const float* delta_g,
                                        uint16_t* delta_m_out, const int64_t* I_p, const int64_t* t_b,
                                        int64_t t_g, int32_t budget, const cocodc_ref_hparams_t* hp,
                                        double* R_out, int32_t* sel_out, int32_t* n_sel_out,
                                        double* sums_out) {
  if (int rc = check_sync_bf16(theta_m, theta_m_send, theta_g, momentum, delta_g, I_p, t_b, budget, hp, R_out,
                               sel_out, n_sel_out))
    return rc;
  if (int rc = check_segments(segs, S, K, n_total)) return rc;
  for (int32_t p = 0; p < K; ++p) {
    Sums s;
    for (int32_t j = 0; j < S; ++j) {
      if (segs[j].fragment != p) continue;
      for (uint64_t i = segs[j].offset; i < segs[j].offset + segs[j].length; ++i) {
        sync_element_bf16(i, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, *hp, &s, nullptr);
      }
    }
    R_out[p] = score_from_sums(s, I_p[p], *hp);
    store_sums(s, p, sums_out);
  }
  return cocodc_ref_select_fragments(K, R_out, t_b, t_g, hp->H, budget, sel_out, n_sel_out);
}

/* One event of the loop of Sec. 3.2 on 16-bit local parameters; recv_mask as for
 * cocodc_ref_sync_event (bit 0: has just arrived, bit 1: in flight). */
int cocodc_ref_sync_event_bf16(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                               const uint8_t* recv_mask, uint16_t* theta_m, const uint16_t* theta_m_send,
                               float* theta_g, float* momentum, const float* delta_g,
                               uint16_t* delta_m_out, const int64_t* I_p, const int64_t* t_b, int64_t t_g,
                               int32_t budget, const cocodc_ref_hparams_t* hp, double* R, int32_t* sel_out,
                               int32_t* n_sel_out, double* sums_out) {
  if (!recv_mask) return kErrNull;
  if (int rc = check_sync_bf16(theta_m, theta_m_send, theta_g, momentum, delta_g, I_p, t_b, budget, hp, R,
                               sel_out, n_sel_out))
    return rc;
  if (int rc = check_table(frags, K, n_total)) return rc;
  std::vector<uint8_t> in_flight(static_cast<size_t>(K), 0);
  for (int32_t q = 0; q < K; ++q) {
    if (recv_mask[q] > 3) return kErrRange;
    in_flight[q] = (recv_mask[q] & 2) ? 1 : 0;
  }
  for (int32_t q = 0; q < K; ++q) {
    if (!(recv_mask[q] & 1)) continue;
    Sums s;
    for (uint64_t i = frags[q].offset; i < frags[q].offset + frags[q].length; ++i) {
      sync_element_bf16(i, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, *hp, &s, nullptr);
    }
    R[q] = score_from_sums(s, I_p[q], *hp);
    store_sums(s, q, sums_out);
  }
  return select_among(K, R, t_b, t_g, hp->H, budget, in_flight.data(), sel_out, n_sel_out);
}

/* The 16-bit event for fragments made of segments: the paper's own configuration in one call per event
 * (strided shards, bf16 local parameters; Sec. 3.2, Sec. 4.1). */
int cocodc_ref_sync_event_bf16_segmented(const cocodc_ref_segment_t* segs, int32_t S, int32_t K,
                                         uint64_t n_total, const uint8_t* recv_mask, uint16_t* theta_m,
                                         const uint16_t* theta_m_send, float* theta_g, float* momentum,
                                         const float* delta_g, uint16_t* delta_m_out, const int64_t* I_p,
                                         const int64_t* t_b, int64_t t_g, int32_t budget,
                                         const cocodc_ref_hparams_t* hp, double* R, int32_t* sel_out,
                                         int32_t* n_sel_out, double* sums_out) {
  if (!recv_mask) return kErrNull;
  if (int rc = check_sync_bf16(theta_m, theta_m_send, theta_g, momentum, delta_g, I_p, t_b, budget, hp, R,
                               sel_out, n_sel_out))
    return rc;
  if (int rc = check_segments(segs, S, K, n_total)) return rc;
  std::vector<uint8_t> in_flight(static_cast<size_t>(K), 0);
  for (int32_t q = 0; q < K; ++q) {
    if (recv_mask[q] > 3) return kErrRange;
    in_flight[q] = (recv_mask[q] & 2) ? 1 : 0;
  }
  for (int32_t q = 0; q < K; ++q) {
    if (!(recv_mask[q] & 1)) continue;
    Sums s;
    for (int32_t j = 0; j < S; ++j) {
      if (segs[j].fragment != q) continue;
      for (uint64_t i = segs[j].offset; i < segs[j].offset + segs[j].length; ++i) {
        sync_element_bf16(i, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out, *hp, &s, nullptr);
      }
    }
    R[q] = score_from_sums(s, I_p[q], *hp);
    store_sums(s, q, sums_out);
  }
  return select_among(K, R, t_b, t_g, hp->H, budget, in_flight.data(), sel_out, n_sel_out);
}

// Eq. 9: N = max(K, floor(gamma * H * T_c / T_s)); Eq. 10: h = floor(H / N).
int cocodc_ref_sync_plan(int32_t K, int32_t H, double gamma, double T_c, double T_s,
                         int64_t* N_out, int64_t* h_out) {
  if (!N_out || !h_out) return kErrNull;
  if (K < 1 || H < 1) return kErrRange;
  if (!(gamma > 0.0) || !(gamma <= 1.0) || !(T_c > 0.0) || !(T_s > 0.0)) return kErrRange;
  if (!std::isfinite(T_c) || !std::isfinite(T_s)) return kErrRange;
  const double cap = std::floor(gamma * ((static_cast<double>(H) * T_c) / T_s));
  int64_t N = static_cast<int64_t>(K);
  if (cap > static_cast<double>(N)) N = (cap < 9.0e18) ? static_cast<int64_t>(cap) : INT64_MAX;
  *N_out = N;
  *h_out = static_cast<int64_t>(H) / N;
  return kOk;
}

}  // extern "C"
