/*
 * cocodc_ref.h -- CPU oracle for the CoCoDC per-fragment outer-synchronisation path.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, plain, fp64 definition that the GPU
 * library is checked against.  Nothing in the product path may include, link or call
 * it; it shares no header, helper, table or constant with the HIP sources and
 * therefore declares its own copies of the (layout-compatible) argument structs.
 *
 * Every pointer is a HOST pointer.  All parameter buffers are flat fp32 arrays of
 * n_total elements; a fragment is a contiguous range {offset, length} of elements
 * (paper Sec. 2.1: the model is split along depth into K disjoint fragments).
 *
 * Arithmetic: every fp32 input is widened to fp64, the step is evaluated in fp64 in
 * the order the paper states it, and each stored fp32 output is rounded exactly once.
 * The new global state is rounded to fp32 BEFORE it enters the delay-compensation
 * step, because in the unfused sequence that step reads it back from an fp32 buffer.
 *
 * Pinned by tests/test_oracle_*.py: hand-computed scalars (each step, and one element
 * through the whole fused step in exact binary fractions), closed forms, textbook /
 * library special cases (torch's SGD with Nesterov momentum, torch's vector norms),
 * brute force, exhaustive enumeration, the identity "fused step == the five steps in
 * sequence", and the one worked example the paper prints (the planner's N = 8, h = 12).
 * The paper prints no numerical example of the update itself.
 *
 * Return value of every function: 0 on success, negative on invalid arguments
 * (-1 null pointer, -3 out-of-range scalar or fragment table).
 */
#ifndef COCODC_REF_H
#define COCODC_REF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  uint64_t offset; /* first element of the fragment in every flat buffer */
  uint64_t length; /* number of elements (0 allowed: empty fragment)     */
} cocodc_ref_fragment_t;

typedef struct {
  int32_t tau;        /* overlap depth tau >= 0 (Sec. 2.1)                              */
  int32_t H;          /* local period H >= 1 (Sec. 2.1, Eq. 5-7)                        */
  double lambda;      /* compensation strength lambda (Eq. 7)                           */
  double eta;         /* outer learning rate (Eq. 2; value not given by the paper)      */
  double mu;          /* outer momentum (Eq. 2; value not given by the paper)           */
  int32_t nesterov;   /* 1: Nesterov look-ahead step, 0: heavy-ball                     */
  int32_t drift_sign; /* +1: Eq. 4 as printed (send-time minus current); -1: reversed   */
  int32_t score_src;  /* 0: score the global pseudo-gradient (Eq. 11); 1: score drift d */
  int32_t norm_kind;  /* 2: L2 norm (Eq. 11); 1: L1 norm                                */
  int32_t merge_mode; /* 0: delay compensation (Eq. 8); 1: blend (Eq. 3); 2: replace    */
  double alpha;       /* mixing factor of Eq. 3, used by merge_mode 1 only              */
  int32_t delta_src;  /* divergence term of Eq. 5-7: 0 = theta^g_{p,t_p} - theta^m_{p,t_p} (the
                         equation that introduces Eq. 5); 1 = theta^m_{p,t_p} - theta^g_{p,t_p-H}
                         (the change accumulated over H steps that the text after Eq. 6 describes);
                         1 needs the previous global state: fused step only              */
  int32_t pg_format;  /* bf16 calls only: the outgoing pseudo-gradient is 0: bfloat16, 1: IEEE binary16 */
} cocodc_ref_hparams_t;

/* Optional fp64 (unrounded) copies of the three stored outputs of the fused step. */
typedef struct {
  double* theta_m;  /* n_total, nullable */
  double* theta_g;  /* n_total, nullable */
  double* momentum; /* n_total, nullable */
} cocodc_ref_shadow_t;

/* Sec. 2.1 (text before Eq. 1): pseudo-gradient of each fragment, with the sign
 * "global snapshot minus local" (the negative of the summand of Eq. 1); optionally
 * records the send-time local parameters. */
int cocodc_ref_pseudograd(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                          const float* theta_g_snap, const float* theta_m, float* delta_m_out,
                          float* theta_m_send_out /* nullable */);

/* Eq. 2 with OuterOptim = SGD with (Nesterov) momentum, descent on delta_g. */
int cocodc_ref_outer_nesterov(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                              float* theta_g, float* momentum, const float* delta_g,
                              const cocodc_ref_hparams_t* hp);

/* Algorithm 1 (Eq. 4, 7, 8), or Eq. 3 / plain replacement for the other merge modes.
 * theta_m_send may be NULL for merge modes 1 and 2 (they do not use it). */
int cocodc_ref_delay_compensate(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                                float* theta_m, const float* theta_m_send, const float* theta_g,
                                const cocodc_ref_hparams_t* hp);

/* Eq. 11: R_p = ||x_p|| / I_p, +inf when I_p <= 0 (never synchronised).
 * sum_out (nullable, K): the raw sum (of squares for L2, of magnitudes for L1). */
int cocodc_ref_fragment_scores(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                               const float* x, const int64_t* I_p, int32_t norm_kind,
                               double* R_out, double* sum_out /* nullable */);

/* Algorithm 2 applied `budget` times without replacement. */
int cocodc_ref_select_fragments(int32_t K, const double* R, const int64_t* t_b, int64_t t_g,
                                int32_t H, int32_t budget, int32_t* sel_out, int32_t* n_sel_out);

/* Algorithm 2 under a byte budget (a reading of "bandwidth budget"; the paper has none): Algorithm
 * 2 is applied repeatedly; a chosen fragment is sent if its size still fits into what is left of
 * byte_budget, otherwise the selection ends there (a lower-priority fragment never overtakes). */
int cocodc_ref_select_fragments_bytes(int32_t K, const double* R, const int64_t* t_b, int64_t t_g,
                                      int32_t H, const uint64_t* frag_bytes, uint64_t byte_budget,
                                      int32_t* sel_out, int32_t* n_sel_out);

/* All of the above in one pass per element.  sums_out (nullable, 4*K):
 * per fragment {sum dg^2, sum |dg|, sum d^2, sum |d|}.  theta_m_send may be NULL for merge
 * modes 1 and 2 with score_src 0; the drift and its two sums are then zero. */
int cocodc_ref_sync_step(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                         float* theta_m, const float* theta_m_send, float* theta_g,
                         float* momentum, const float* delta_g,
                         float* delta_m_out /* nullable; may alias delta_g */,
                         const int64_t* I_p, const int64_t* t_b, int64_t t_g, int32_t budget,
                         const cocodc_ref_hparams_t* hp, double* R_out, int32_t* sel_out,
                         int32_t* n_sel_out, double* sums_out /* nullable */,
                         const cocodc_ref_shadow_t* shadow /* nullable */);

/* One event of the loop of Sec. 3.2 in one call.  Bit 0 of recv_mask[q] marks the fragments whose
 * averaged pseudo-gradient has just arrived: they get the fused step (Eq. 2, Alg. 1, next
 * pseudo-gradient) and a fresh score R[q] (Eq. 11, from I_p[q]); every other fragment keeps its
 * buffers, its R[p] and its row of sums_out.  R is therefore read and written: it holds the
 * scores of earlier events (+inf before a fragment's first synchronisation).  Bit 1 marks the
 * fragments whose all-reduce is still in flight.  Then Alg. 2 runs `budget` times over the scores
 * of the fragments that are not in flight, with t_b as passed (the caller has already set t_b of
 * the arrived fragments to the current step). */
int cocodc_ref_sync_event(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                          const uint8_t* recv_mask, float* theta_m, const float* theta_m_send,
                          float* theta_g, float* momentum, const float* delta_g, float* delta_m_out,
                          const int64_t* I_p, const int64_t* t_b, int64_t t_g, int32_t budget,
                          const cocodc_ref_hparams_t* hp, double* R, int32_t* sel_out,
                          int32_t* n_sel_out, double* sums_out);

/* Same per-element arithmetic as cocodc_ref_sync_step, spread over host threads in
 * fixed 65536-element chunks whose partial sums are added in chunk order (so the
 * result does not depend on n_threads).  Exists only so the CPU baseline can be timed
 * on all host cores; n_threads <= 0 uses the OpenMP default.  Returns the number of
 * threads used (> 0) or a negative error. */
int cocodc_ref_sync_step_mt(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                            float* theta_m, const float* theta_m_send, float* theta_g,
                            float* momentum, const float* delta_g, float* delta_m_out,
                            const int64_t* I_p, const int64_t* t_b, int64_t t_g, int32_t budget,
                            const cocodc_ref_hparams_t* hp, double* R_out, int32_t* sel_out,
                            int32_t* n_sel_out, double* sums_out, int32_t n_threads);

/* Fragments made of several contiguous segments (Sec. 4.1: strided shards).  A fragment's
 * elements are visited segment by segment in the order the segments are listed, index order
 * inside a segment.  Everything else as in the contiguous functions above. */
typedef struct {
  uint64_t offset, length;
  int32_t fragment; /* 0..K-1 */
  int32_t reserved;
} cocodc_ref_segment_t;

int cocodc_ref_fragment_scores_segmented(const cocodc_ref_segment_t* segs, int32_t S, int32_t K,
                                         uint64_t n_total, const float* x, const int64_t* I_p,
                                         int32_t norm_kind, double* R_out, double* sum_out);

int cocodc_ref_sync_step_segmented(const cocodc_ref_segment_t* segs, int32_t S, int32_t K,
                                   uint64_t n_total, float* theta_m, const float* theta_m_send,
                                   float* theta_g, float* momentum, const float* delta_g,
                                   float* delta_m_out, const int64_t* I_p, const int64_t* t_b,
                                   int64_t t_g, int32_t budget, const cocodc_ref_hparams_t* hp,
                                   double* R_out, int32_t* sel_out, int32_t* n_sel_out,
                                   double* sums_out, const cocodc_ref_shadow_t* shadow);

/* ---- bf16 local parameters (Sec. 4.1: the worker trains in bf16 mixed precision) ----
 * theta_m, theta_m_send and the outgoing pseudo-gradient are bfloat16 (raw 16-bit patterns:
 * 1 sign, 8 exponent, 7 fraction bits); the global state, the momentum and delta_g stay fp32.
 * Every bf16 input is widened exactly, the step is evaluated in fp64 as above, and each bf16
 * output is the fp64 value rounded ONCE to the nearest bf16 (ties to even; subnormals kept;
 * overflow to infinity; any NaN becomes 0x7FC0). */
uint16_t cocodc_ref_round_bf16(double x);
double cocodc_ref_widen_bf16(uint16_t b);

/* The outgoing pseudo-gradient alone may instead be IEEE binary16 (pg_format 1: 1 sign, 5 exponent,
 * 10 fraction bits; the usual 16-bit wire format of an all-reduce): the fp64 difference rounded
 * ONCE to the nearest binary16, ties to even, subnormals (spacing 2^-24) kept, magnitudes of
 * 65520 and more to infinity, any NaN to 0x7E00. */
uint16_t cocodc_ref_round_f16(double x);
double cocodc_ref_widen_f16(uint16_t b);

int cocodc_ref_pseudograd_bf16(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                               const float* theta_g_snap, const uint16_t* theta_m,
                               uint16_t* delta_m_out, uint16_t* theta_m_send_out /* nullable */,
                               int32_t pg_format);

/* shadow (nullable): unrounded fp64 theta_m / theta_g / momentum as in cocodc_ref_sync_step. */
int cocodc_ref_sync_step_bf16(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                              uint16_t* theta_m, const uint16_t* theta_m_send, float* theta_g,
                              float* momentum, const float* delta_g,
                              uint16_t* delta_m_out /* nullable */, const int64_t* I_p,
                              const int64_t* t_b, int64_t t_g, int32_t budget,
                              const cocodc_ref_hparams_t* hp, double* R_out, int32_t* sel_out,
                              int32_t* n_sel_out, double* sums_out /* nullable */,
                              const cocodc_ref_shadow_t* shadow /* nullable */);

/* cocodc_ref_sync_event for fragments made of segments (recv_mask, I_p, t_b, R, sums_out per fragment). */
int cocodc_ref_sync_event_segmented(const cocodc_ref_segment_t* segs, int32_t S, int32_t K,
                                    uint64_t n_total, const uint8_t* recv_mask, float* theta_m,
                                    const float* theta_m_send, float* theta_g, float* momentum,
                                    const float* delta_g, float* delta_m_out /* nullable */,
                                    const int64_t* I_p, const int64_t* t_b, int64_t t_g, int32_t budget,
                                    const cocodc_ref_hparams_t* hp, double* R, int32_t* sel_out,
                                    int32_t* n_sel_out, double* sums_out /* nullable */);

/* cocodc_ref_sync_step_bf16 over fragments made of segments (Sec. 4.1: strided shards, mixed-precision
 * local parameters); a fragment's segments are walked in the order listed. */
int cocodc_ref_sync_step_bf16_segmented(const cocodc_ref_segment_t* segs, int32_t S, int32_t K,
                                        uint64_t n_total, uint16_t* theta_m, const uint16_t* theta_m_send,
                                        float* theta_g, float* momentum, const float* delta_g,
                                        uint16_t* delta_m_out /* nullable */, const int64_t* I_p,
                                        const int64_t* t_b, int64_t t_g, int32_t budget,
                                        const cocodc_ref_hparams_t* hp, double* R_out, int32_t* sel_out,
                                        int32_t* n_sel_out, double* sums_out /* nullable */);

/* cocodc_ref_sync_event (one event of the loop of Sec. 3.2) on 16-bit local parameters. */
int cocodc_ref_sync_event_bf16(const cocodc_ref_fragment_t* frags, int32_t K, uint64_t n_total,
                               const uint8_t* recv_mask, uint16_t* theta_m, const uint16_t* theta_m_send,
                               float* theta_g, float* momentum, const float* delta_g,
                               uint16_t* delta_m_out /* nullable */, const int64_t* I_p, const int64_t* t_b,
                               int64_t t_g, int32_t budget, const cocodc_ref_hparams_t* hp, double* R,
                               int32_t* sel_out, int32_t* n_sel_out, double* sums_out /* nullable */);

/* cocodc_ref_sync_event_bf16 for fragments made of segments. */
int cocodc_ref_sync_event_bf16_segmented(const cocodc_ref_segment_t* segs, int32_t S, int32_t K,
                                         uint64_t n_total, const uint8_t* recv_mask, uint16_t* theta_m,
                                         const uint16_t* theta_m_send, float* theta_g, float* momentum,
                                         const float* delta_g, uint16_t* delta_m_out /* nullable */,
                                         const int64_t* I_p, const int64_t* t_b, int64_t t_g,
                                         int32_t budget, const cocodc_ref_hparams_t* hp, double* R,
                                         int32_t* sel_out, int32_t* n_sel_out,
                                         double* sums_out /* nullable */);

/* Eq. 9 and Eq. 10: N = max(K, floor(gamma*H*T_c/T_s)), h = floor(H/N). */
int cocodc_ref_sync_plan(int32_t K, int32_t H, double gamma, double T_c, double T_s,
                         int64_t* N_out, int64_t* h_out);

#ifdef __cplusplus
}
#endif
#endif /* COCODC_REF_H */
