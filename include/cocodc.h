/*
 * cocodc.h -- C ABI of the MI355X (gfx950) library for the CoCoDC per-fragment
 * outer-synchronisation path (Zhu et al., "Cross-region Model Training with
 * Communication-Computation Overlapping and Delay Compensation").
 *
 * What the path computes, once per fragment synchronisation (paper Sec. 2 and 3):
 *   - the local pseudo-gradient of a fragment (Sec. 2.1, text before Eq. 1),
 *   - the outer-optimiser update of the fragment's global state from the averaged,
 *     delayed global pseudo-gradient (Eq. 2; SGD with Nesterov momentum),
 *   - the Taylor delay-compensation merge into the local parameters (Algorithm 1,
 *     Eq. 4, 7, 8),
 *   - the adaptive-transmission change score of each fragment (Eq. 11) and the choice
 *     of the next fragments to send (Algorithm 2, Eq. 12).
 * The cross-worker average of Eq. 1 is an INPUT (delta_g); no collective is issued.
 *
 * ---------------------------------------------------------------------------------
 * Conventions that hold for every entry point
 * ---------------------------------------------------------------------------------
 * Buffers.  Parameter-like buffers (theta_m, theta_m_send, theta_g, momentum, delta_g,
 *   delta_m_out, x) are DEVICE pointers to flat fp32 arrays of n_total elements.  A
 *   fragment is the contiguous element range [offset, offset+length) of every such
 *   buffer (Sec. 2.1: K disjoint fragments along the depth of the model).  R_out,
 *   sums_out, sel_out and n_sel_out are DEVICE pointers.  The fragment table, I_p,
 *   t_b and the hyper-parameter struct are HOST pointers; they are consumed before the
 *   call returns and may be freed or changed right after it.
 * Ownership.  The caller owns every buffer, including the workspace.  The library
 *   allocates no device memory (its code carries one fixed 64 MiB device array per GPU,
 *   used by cocodc_sync_step_noalloc only).  A workspace of cocodc_workspace_bytes(K, n_total)
 *   bytes, 256-byte aligned, holds the device copy of the fragment table and the
 *   partial sums; it carries no state between calls, but two calls that are in flight
 *   at the same time (different streams) must use different workspaces.
 * Alignment.  fp32 buffers must be 4-byte aligned (bf16 buffers 2-byte).  The kernels
 *   make 128-bit accesses at element indices that are multiples of 4 (a fragment's head
 *   and tail up to such an index are handled element by element, so fragment offsets may
 *   be odd).  They are fastest when every buffer base is a multiple of 128 bytes, as
 *   hipMalloc's are: bases 16 bytes or 4 bytes off a 128-byte boundary cost about 11 %
 *   (every wavefront access then straddles cache lines).  Results, scores included, do
 *   not depend on the alignment of the buffers.
 * Aliasing.  Distinct arguments must not overlap, with one exception: delta_m_out may
 *   be exactly delta_g (the all-reduce buffer is reused in place).
 * Streams.  `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   All work is enqueued on it and the call returns without synchronising (the only waits
 *   in the library are on the loop's own 4-byte read-back of a send decision, see
 *   cocodc_loop_step, and in cocodc_profiler_collect).
 * Errors.  Every function returns COCODC_OK (0) or a negative cocodc_status_t.
 *   Arguments are validated on the host before anything is enqueued: on an error
 *   other than COCODC_ERR_HIP nothing has been launched and no buffer was touched.
 *   Device-side NaN/Inf values are not errors: they propagate as IEEE arithmetic
 *   dictates, and a NaN score ranks last in the selection.
 * Arithmetic.  Every fp32 input is widened to fp64, the update is evaluated in fp64
 *   registers and each stored fp32 value is rounded once.  Per-fragment sums are
 *   accumulated in fp64 in a fixed order that depends only on the fragment table and
 *   n_total (not on buffer addresses, launch shape or device), so
 *   repeated calls on the same bytes give bit-identical scores and selections (the
 *   property Sec. 3.2 relies on for coordination-free selection).
 * Limits.  1 <= K <= COCODC_MAX_FRAGMENTS, n_total <= COCODC_MAX_ELEMENTS.
 */
#ifndef COCODC_H
#define COCODC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define COCODC_MAX_FRAGMENTS 1024
#define COCODC_MAX_SEGMENTS 4096
#define COCODC_MAX_ELEMENTS (1ull << 44) /* n_total above this is rejected (COCODC_ERR_RANGE) */

typedef enum {
  COCODC_OK = 0,
  COCODC_ERR_NULL = -1,      /* a required pointer is NULL                                */
  COCODC_ERR_ALIGN = -2,     /* fp32 buffer not 4-byte, R/sums not 8-byte, workspace not  */
                             /* 256-byte aligned                                          */
  COCODC_ERR_RANGE = -3,     /* K, tau, H, budget, enum-like field, or fragment table     */
                             /* (out of n_total, overlapping) out of range                */
  COCODC_ERR_NONFINITE = -4, /* lambda, eta, mu or alpha is NaN or infinite               */
  COCODC_ERR_WORKSPACE = -5, /* workspace_bytes < cocodc_workspace_bytes(K, n_total)      */
  COCODC_ERR_HIP = -6,       /* a HIP runtime call failed; see cocodc_last_hip_error()    */
  COCODC_ERR_ALIAS = -7      /* two buffers overlap where the contract forbids it         */
} cocodc_status_t;

/* One fragment theta_p: a contiguous element range of every flat buffer (Sec. 2.1). */
typedef struct {
  uint64_t offset; /* first element                                    */
  uint64_t length; /* number of elements; 0 is allowed (empty fragment) */
} cocodc_fragment_t;

/* One contiguous piece of a fragment that is NOT contiguous in the flat buffers, e.g. the
 * strided shards of Sec. 4.1 (shard k = layers k, k+4, k+8 of a layer-ordered buffer). */
typedef struct {
  uint64_t offset;   /* first element                      */
  uint64_t length;   /* number of elements (0 allowed)     */
  int32_t fragment;  /* which fragment it belongs to, 0..K-1 */
  int32_t reserved;  /* set to 0                           */
} cocodc_segment_t;

/* Hyper-parameters, in the paper's notation. */
typedef struct {
  int32_t tau;        /* overlap depth tau >= 0: inner steps the all-reduce took (Sec. 2.1) */
  int32_t H;          /* local computation period H >= 1 (Sec. 2.1; divisor in Eq. 5-7)     */
  double lambda;      /* compensation strength lambda (Eq. 7)                               */
  double eta;         /* learning rate of the outer optimiser (Eq. 2)                       */
  double mu;          /* momentum of the outer optimiser (Eq. 2)                            */
  int32_t nesterov;   /* 1 = Nesterov look-ahead (the paper's example), 0 = heavy-ball      */
  int32_t drift_sign; /* +1: change rate exactly as Eq. 4 prints it (send-time minus        */
                      /*     current local); -1: current minus send-time                    */
  int32_t score_src;  /* 0: score ||delta_g||, Eq. 11; 1: score the local drift over the    */
                      /*    overlap (same kernel, other sum)                                */
  int32_t norm_kind;  /* 2: L2 norm (Eq. 11); 1: L1 norm                                    */
  int32_t merge_mode; /* 0: delay compensation (Eq. 8); 1: Streaming-DiLoCo blend (Eq. 3);  */
                      /* 2: adopt the new global state (blocking DiLoCo)                    */
  double alpha;       /* mixing factor of Eq. 3; read only when merge_mode == 1             */
  int32_t delta_src;  /* the divergence term Delta of Eq. 5-7.  0: theta^g_{p,t_p} - theta^m_{p,t_p}, */
                      /* the equation that introduces Eq. 5 (default).  1: theta^m_{p,t_p} -        */
                      /* theta^g_{p,t_p-H}, the change accumulated over the last H steps that the   */
                      /* text after Eq. 6 describes; it needs the previous global state, so only    */
                      /* the fused calls accept it (cocodc_delay_compensate: COCODC_ERR_RANGE)      */
  int32_t pg_format;  /* read by the bf16 calls only: 16-bit format of the outgoing                 */
                      /* pseudo-gradient, COCODC_PG_BF16 (0, default) or COCODC_PG_F16 (IEEE binary16)  */
} cocodc_hparams_t;

#define COCODC_PG_BF16 0
#define COCODC_PG_F16 1

/* Bytes of device workspace that any entry point below needs for (K, n_total).
 * Returns 0 if K is outside [1, COCODC_MAX_FRAGMENTS]. */
size_t cocodc_workspace_bytes(int32_t K, uint64_t n_total);

/* Local pseudo-gradient (Sec. 2.1, text before Eq. 1), in the descent sign convention
 * used throughout this library: delta_m_out[i] = theta_g_snap[i] - theta_m[i]
 * (the negative of the summand of Eq. 1), for every i of every listed fragment.
 * If theta_m_send_out is not NULL it also records theta_m_send_out[i] = theta_m[i],
 * the send-time copy theta^m_{p,t_p} that Algorithm 1 needs tau steps later.
 * Elements outside the listed fragments are not touched. */
int cocodc_pseudograd(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total,
                      const float* theta_g_snap, const float* theta_m, float* delta_m_out,
                      float* theta_m_send_out /* nullable */, void* workspace,
                      size_t workspace_bytes, void* stream);

/* Outer optimiser, Eq. 2, as SGD with momentum on the "gradient" delta_g:
 *   m' = mu*m + delta_g ;  step = nesterov ? delta_g + mu*m' : m' ;
 *   theta_g <- theta_g - eta*step.
 * In place: theta_g holds theta^g_{p,t_p-H} on entry and theta^g_{p,t_p} on exit;
 * momentum is updated to m'. */
int cocodc_outer_nesterov(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total,
                          float* theta_g, float* momentum, const float* delta_g,
                          const cocodc_hparams_t* hp, void* workspace, size_t workspace_bytes,
                          void* stream);

/* Delay-compensation merge, Algorithm 1.  With d = drift_sign*(theta_m_send - theta_m)
 * (= tau times the change rate g of Eq. 4) and Delta = theta_g - theta_m_send (the
 * difference introduced with Eq. 5), element by element:
 *   theta_m <- theta_g + d + lambda * d*d*Delta / (tau*H)      (Eq. 7 put into Eq. 8)
 * The last term is dropped when tau == 0.  merge_mode 1 computes Eq. 3 instead,
 * merge_mode 2 copies theta_g; neither reads theta_m_send, which may then be NULL.
 * theta_g must already be the NEW global state. */
int cocodc_delay_compensate(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total,
                            float* theta_m, const float* theta_m_send, const float* theta_g,
                            const cocodc_hparams_t* hp, void* workspace, size_t workspace_bytes,
                            void* stream);

/* Change score, Eq. 11: R_out[p] = norm(x over fragment p) / I_p[p], and +inf when
 * I_p[p] <= 0 (a fragment that never completed a synchronisation, Sec. 3.2).
 * x: any flat fp32 buffer (normally delta_g).  I_p: host, K entries.  R_out: device, K
 * doubles.  sum_out (device, K doubles, nullable): the raw fp64 sum (of squares for
 * norm_kind 2, of magnitudes for norm_kind 1). */
int cocodc_fragment_scores(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total,
                           const float* x, const int64_t* I_p, int32_t norm_kind, double* R_out,
                           double* sum_out /* nullable */, void* workspace,
                           size_t workspace_bytes, void* stream);

/* Fragment selection, Algorithm 2 / Eq. 12, applied `budget` times without replacement:
 * first every fragment with t_g - t_b[p] >= H in ascending p, then the remaining ones by
 * descending R[p] (ties: lower p; NaN last).  Writes n = min(budget, K) indices to
 * sel_out (device, >= n int32) and n to n_sel_out (device).  R: device, K doubles.
 * t_b: host, K entries (step at which fragment p last completed a synchronisation). */
int cocodc_select_fragments(int32_t K, const double* R, const int64_t* t_b, int64_t t_g, int32_t H,
                            int32_t budget, int32_t* sel_out, int32_t* n_sel_out, void* workspace,
                            size_t workspace_bytes, void* stream);

/* The same selection under a BYTE budget (a reading of "bandwidth budget"; the paper itself sends
 * one fragment per decision): the priority order above is walked and a fragment is taken while
 * its size frag_bytes[p] (host, K entries) still fits into what is left of byte_budget; the first
 * fragment that does not fit ends the selection, so a small low-priority fragment never overtakes
 * a large high-priority one.  sel_out: device, K int32; n_sel_out: device. */
int cocodc_select_fragments_bytes(int32_t K, const double* R, const int64_t* t_b, int64_t t_g, int32_t H,
                                  const uint64_t* frag_bytes, uint64_t byte_budget, int32_t* sel_out,
                                  int32_t* n_sel_out, void* workspace, size_t workspace_bytes, void* stream);

/* The whole path in one pass over memory: every element of every listed fragment is
 * read once from theta_m, theta_m_send, theta_g, momentum, delta_g and written once to
 * theta_m, theta_g, momentum (and delta_m_out if not NULL).  Equivalent, bit for bit,
 * to cocodc_pseudograd(theta_m_send_out = NULL) -> cocodc_outer_nesterov ->
 * cocodc_delay_compensate -> cocodc_fragment_scores(delta_g) ->
 * cocodc_select_fragments when score_src == 0.
 *   theta_m_send: may be NULL when merge_mode is 1 or 2 and score_src is 0 (Eq. 3 and the
 *                blocking merge keep no send-time record); the pass then moves 32 instead of
 *                36 bytes per parameter and the two drift sums are reported as 0.
 *   delta_m_out: nullable; may be exactly delta_g.
 *   I_p, t_b:    host, K entries each.      t_g: current global step.
 *   R_out:       device, K doubles.         sel_out / n_sel_out: as above.
 *   sums_out:    device, 4*K doubles, nullable: per fragment
 *                {sum delta_g^2, sum |delta_g|, sum d^2, sum |d|}.
 * It does not modify theta_m_send, I_p or t_b: recording a send belongs to the moment
 * the caller launches the next all-reduce (cocodc_pseudograd does it). */
int cocodc_sync_step(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total, float* theta_m,
                     const float* theta_m_send, float* theta_g, float* momentum,
                     const float* delta_g, float* delta_m_out /* nullable */, const int64_t* I_p,
                     const int64_t* t_b, int64_t t_g, int32_t budget, const cocodc_hparams_t* hp,
                     double* R_out, int32_t* sel_out, int32_t* n_sel_out,
                     double* sums_out /* nullable */, void* workspace, size_t workspace_bytes,
                     void* stream);

/* cocodc_sync_step for callers that cannot allocate device memory: code that runs under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, checks and
 * results (bit for bit) as cocodc_sync_step, without the workspace: the device-side fragment
 * table and the per-tile partial sums live in a fixed array of COCODC_NOALLOC_SCRATCH_BYTES inside
 * the library (one per GPU, held until the process ends).  The call itself allocates nothing on
 * the device and frees nothing.
 *   Limit: cocodc_workspace_bytes(K, n_total) <= COCODC_NOALLOC_SCRATCH_BYTES, i.e. about
 *   8.5e9 elements (the 7B fragment set needs 52 MB); larger calls return COCODC_ERR_WORKSPACE
 *   and launch nothing.
 *   The GPU that `stream` belongs to must be the current device.  The first call on a GPU looks up
 *   the array's address there (make it outside a graph capture).
 *   All calls on one GPU share the array: two of them must not be in flight at the same time
 *   (issue them on one stream, or order the streams); they would race on the partial sums.
 *   Nothing in the array needs clearing between calls. */
#define COCODC_NOALLOC_SCRATCH_BYTES (64u << 20)
int cocodc_sync_step_noalloc(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total, float* theta_m,
                             const float* theta_m_send, float* theta_g, float* momentum,
                             const float* delta_g, float* delta_m_out /* nullable */, const int64_t* I_p,
                             const int64_t* t_b, int64_t t_g, int32_t budget, const cocodc_hparams_t* hp,
                             double* R_out, int32_t* sel_out, int32_t* n_sel_out,
                             double* sums_out /* nullable */, void* stream);

/* One event of the loop of Sec. 3.2 in one call: "these fragments have just arrived, those are
 * still in flight; which fragment is sent next?".  recv_mask: host, K entries, each a combination
 * of COCODC_MASK_ARRIVED and COCODC_MASK_IN_FLIGHT (any other bit: COCODC_ERR_RANGE).
 * Fragments marked ARRIVED get exactly what cocodc_sync_step does for them (Eq. 2, Algorithm 1,
 * next pseudo-gradient) and a fresh score R[q] (Eq. 11, from I_p[q]); every other fragment keeps
 * its buffers, its R[p] and its row of sums_out, whatever I_p[p] says.  R (device, K) is
 * therefore read AND written: it must hold the scores of earlier events, +inf for fragments
 * that were never synchronised (cocodc_loop_reset_scores).  Algorithm 2 then runs over the
 * scores of the fragments NOT marked IN_FLIGHT (the send-time record of a fragment whose
 * all-reduce is still under way must not be overwritten), with t_b as passed: the caller has
 * already set t_b[q] of the arrived fragments to the current step.  It writes
 * min(budget, number of fragments not in flight) indices.  A mask without any mark reduces the
 * call to the selection.  Everything else (ownership, alignment, aliasing, errors) as for
 * cocodc_sync_step. */
#define COCODC_MASK_ARRIVED 1u
#define COCODC_MASK_IN_FLIGHT 2u
int cocodc_sync_event(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total,
                      const uint8_t* recv_mask, float* theta_m,
                      const float* theta_m_send /* nullable as in cocodc_sync_step */, float* theta_g,
                      float* momentum, const float* delta_g, float* delta_m_out /* nullable */,
                      const int64_t* I_p, const int64_t* t_b, int64_t t_g, int32_t budget,
                      const cocodc_hparams_t* hp, double* R /* in and out */, int32_t* sel_out,
                      int32_t* n_sel_out, double* sums_out /* nullable */, void* workspace,
                      size_t workspace_bytes, void* stream);

/* The same two calls for fragments made of several segments (Sec. 4.1: strided shards).
 * segs: host, S entries in any order; the segments of one fragment are summed in the order
 * listed.  Segments must not overlap; a fragment may have none.  I_p, t_b, R_out, sel_out,
 * sums_out are per FRAGMENT (K entries) exactly as above.  The element-wise single steps need no
 * segmented form: pass the segments to them as if each were a fragment.  Workspace size:
 * cocodc_workspace_bytes_segmented(S, K, n_total) (0 if S or K is out of range). */
size_t cocodc_workspace_bytes_segmented(int32_t S, int32_t K, uint64_t n_total);
int cocodc_fragment_scores_segmented(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total,
                                     const float* x, const int64_t* I_p, int32_t norm_kind, double* R_out,
                                     double* sum_out /* nullable */, void* workspace,
                                     size_t workspace_bytes, void* stream);
int cocodc_sync_step_segmented(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total,
                               float* theta_m, const float* theta_m_send, float* theta_g, float* momentum,
                               const float* delta_g, float* delta_m_out /* nullable */, const int64_t* I_p,
                               const int64_t* t_b, int64_t t_g, int32_t budget, const cocodc_hparams_t* hp,
                               double* R_out, int32_t* sel_out, int32_t* n_sel_out,
                               double* sums_out /* nullable */, void* workspace, size_t workspace_bytes,
                               void* stream);

/* cocodc_sync_event for fragments made of several segments (one event of the loop of Sec. 3.2 on
 * the strided shards of Sec. 4.1): recv_mask, I_p, t_b, R (read and written) and sums_out are per
 * FRAGMENT; segs and the workspace size as for cocodc_sync_step_segmented. */
int cocodc_sync_event_segmented(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total,
                                const uint8_t* recv_mask, float* theta_m,
                                const float* theta_m_send /* nullable as in cocodc_sync_step */,
                                float* theta_g, float* momentum, const float* delta_g,
                                float* delta_m_out /* nullable */, const int64_t* I_p, const int64_t* t_b,
                                int64_t t_g, int32_t budget, const cocodc_hparams_t* hp,
                                double* R /* in and out */, int32_t* sel_out, int32_t* n_sel_out,
                                double* sums_out /* nullable */, void* workspace, size_t workspace_bytes,
                                void* stream);

/* ---- bfloat16 local parameters ----
 * The paper's workers train in bf16 mixed precision (Sec. 4.1).  In these calls theta_m,
 * theta_m_send and the outgoing pseudo-gradient are bfloat16 (raw 16-bit patterns, 2-byte
 * aligned; 16-byte aligned for the fast path), while the global state, the outer momentum and
 * delta_g stay fp32 master copies.  Every bf16 input is widened exactly, the update is the
 * same fp64 arithmetic as above, and each bf16 output is the fp64 value rounded ONCE to the
 * nearest bf16 (ties to even, subnormals kept, overflow to infinity, NaN -> 0x7FC0).  The
 * fused pass then moves 28 instead of 36 bytes per parameter.  delta_m_out cannot alias
 * delta_g here (different element types).  Everything else as in the fp32 calls.
 *   The outgoing pseudo-gradient alone -- what goes on the wire -- may instead be IEEE binary16
 *   (pg_format = COCODC_PG_F16; the argument of cocodc_pseudograd_bf16, the field of the
 *   hyper-parameters for cocodc_sync_step_bf16): the same fp64 difference rounded ONCE to the
 *   nearest binary16, ties to even, subnormals (spacing 2^-24) kept, magnitudes of 65520 and
 *   more to infinity, NaN -> 0x7E00.  Same bytes, same speed; any other value of pg_format is
 *   COCODC_ERR_RANGE. */
int cocodc_pseudograd_bf16(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total,
                           const float* theta_g_snap, const uint16_t* theta_m, uint16_t* delta_m_out,
                           uint16_t* theta_m_send_out /* nullable */, int32_t pg_format, void* workspace,
                           size_t workspace_bytes, void* stream);
int cocodc_sync_step_bf16(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total, uint16_t* theta_m,
                          const uint16_t* theta_m_send, float* theta_g, float* momentum,
                          const float* delta_g, uint16_t* delta_m_out /* nullable */, const int64_t* I_p,
                          const int64_t* t_b, int64_t t_g, int32_t budget, const cocodc_hparams_t* hp,
                          double* R_out, int32_t* sel_out, int32_t* n_sel_out,
                          double* sums_out /* nullable */, void* workspace, size_t workspace_bytes,
                          void* stream);
/* cocodc_sync_step_bf16 for fragments made of several segments: Sec. 4.1 as the paper runs it,
 * strided shards of a model trained in bf16 mixed precision.  segs, the per-fragment arrays and
 * the workspace size as for cocodc_sync_step_segmented; buffers as for cocodc_sync_step_bf16. */
int cocodc_sync_step_bf16_segmented(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total,
                                    uint16_t* theta_m, const uint16_t* theta_m_send, float* theta_g,
                                    float* momentum, const float* delta_g,
                                    uint16_t* delta_m_out /* nullable */, const int64_t* I_p,
                                    const int64_t* t_b, int64_t t_g, int32_t budget,
                                    const cocodc_hparams_t* hp, double* R_out, int32_t* sel_out,
                                    int32_t* n_sel_out, double* sums_out /* nullable */, void* workspace,
                                    size_t workspace_bytes, void* stream);
/* cocodc_sync_event (one event of the loop of Sec. 3.2) on bf16 local parameters: recv_mask, R
 * (read and written), t_b and the selection among the fragments not in flight as there; buffers
 * and rounding as for cocodc_sync_step_bf16. */
int cocodc_sync_event_bf16(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total,
                           const uint8_t* recv_mask, uint16_t* theta_m,
                           const uint16_t* theta_m_send /* nullable as in cocodc_sync_step */,
                           float* theta_g, float* momentum, const float* delta_g,
                           uint16_t* delta_m_out /* nullable */, const int64_t* I_p, const int64_t* t_b,
                           int64_t t_g, int32_t budget, const cocodc_hparams_t* hp,
                           double* R /* in and out */, int32_t* sel_out, int32_t* n_sel_out,
                           double* sums_out /* nullable */, void* workspace, size_t workspace_bytes,
                           void* stream);

/* cocodc_sync_event_bf16 for fragments made of several segments: one event of the loop of Sec. 3.2
 * in the paper's own configuration (strided shards, bf16 local parameters).  Mask, scores and
 * bookkeeping per fragment; segs and workspace size as for cocodc_sync_step_segmented. */
int cocodc_sync_event_bf16_segmented(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total,
                                     const uint8_t* recv_mask, uint16_t* theta_m,
                                     const uint16_t* theta_m_send /* nullable as in cocodc_sync_step */,
                                     float* theta_g, float* momentum, const float* delta_g,
                                     uint16_t* delta_m_out /* nullable */, const int64_t* I_p,
                                     const int64_t* t_b, int64_t t_g, int32_t budget,
                                     const cocodc_hparams_t* hp, double* R /* in and out */,
                                     int32_t* sel_out, int32_t* n_sel_out, double* sums_out /* nullable */,
                                     void* workspace, size_t workspace_bytes, void* stream);

/* Host-only planner, Eq. 9 and Eq. 10: N = max(K, floor(gamma*H*T_c/T_s)) target
 * synchronisations per H steps and h = floor(H/N) steps between two sends.
 * gamma in (0,1]; T_c, T_s > 0 (any common unit).  No GPU work. */
int cocodc_sync_plan(int32_t K, int32_t H, double gamma, double T_c, double T_s, int64_t* N_out,
                     int64_t* h_out);

/* ---- the adaptive-transmission loop of Sec. 3.2 around the kernels ---- */

/* Host-side schedule state of one worker: which fragment was sent when, t_{p,b}, I_p, the
 * moving averages of T_c and T_s and the resulting N and h (Eq. 9, Eq. 10).  Opaque; lives in
 * host memory only (from the first send decision on it also owns four bytes of pinned host
 * memory and one HIP event).  One loop object is for one thread at a time. */
typedef struct cocodc_loop cocodc_loop_t;

/* Device buffers the loop works on (all caller-owned; see the conventions above). */
typedef struct {
  float* theta_m;        /* local parameters, advanced by the caller's inner optimiser          */
  float* theta_m_send;   /* send-time records theta^m_{p,t_p}                                   */
  float* theta_g;        /* global states of all fragments                                      */
  float* momentum;       /* outer-optimiser momentum                                            */
  float* delta_g;        /* where the averaged pseudo-gradient of a fragment has arrived        */
  float* delta_m_out;    /* where a sent fragment's pseudo-gradient is written; may be delta_g  */
                         /* (the in-place all-reduce buffer; with one worker the loop is closed) */
  double* R;             /* K scores R_p                                                        */
  int32_t* sel;          /* K int32 scratch for the selection                                   */
  int32_t* n_sel;        /* 1 int32 scratch                                                     */
  void* workspace;       /* cocodc_workspace_bytes(K, n_total), or ..._segmented(S, K, n_total) */
                         /* for a loop made with cocodc_loop_create_segmented                   */
  size_t workspace_bytes;
} cocodc_loop_buffers_t;

/* Creates the schedule for K fragments.  hp->H and hp->tau are the period and the overlap
 * depth; gamma, T_c, T_s feed Eq. 9 / Eq. 10 (N syncs per H steps, one send every
 * h = max(1, floor(H/N)) steps).  All t_{p,b} start at 0 and every R_p at +infinity (Sec. 3.2:
 * fragments that never completed a synchronisation go first). */
int cocodc_loop_create(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total,
                       const cocodc_hparams_t* hp, double gamma, double T_c, double T_s,
                       cocodc_loop_t** loop_out);
/* The same schedule for fragments made of several segments (the strided shards of Sec. 4.1:
 * K = 4 shards of a 12-layer model, shard k = layers k, k+4, k+8): segs as for
 * cocodc_sync_step_segmented.  The workspace of the loop's buffers must then hold
 * cocodc_workspace_bytes_segmented(S, K, n_total). */
int cocodc_loop_create_segmented(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total,
                                 const cocodc_hparams_t* hp, double gamma, double T_c, double T_s,
                                 cocodc_loop_t** loop_out);
void cocodc_loop_destroy(cocodc_loop_t* loop);

/* Writes +infinity to the K scores (enqueued on `stream`); call once before the first step. */
int cocodc_loop_reset_scores(cocodc_loop_t* loop, double* R, void* stream);

/* Online moving averages of the measured step time and fragment synchronisation time
 * (Sec. 3.2): T <- (1-beta)*T + beta*sample for each, then N and h are recomputed. */
int cocodc_loop_observe(cocodc_loop_t* loop, double T_c_sample, double T_s_sample, double beta);

/* Current plan: N (Eq. 9) and h (Eq. 10, at least 1). */
int cocodc_loop_plan(const cocodc_loop_t* loop, int64_t* N_out, int64_t* h_out);

/* Fragments whose all-reduce, launched at step t - tau or earlier, is complete at step t and has
 * not been received yet (ascending).  Lets the caller put their averaged pseudo-gradients into
 * delta_g before cocodc_loop_step.  Reads back a send decision that is still pending if that
 * fragment could be among them. */
int cocodc_loop_due(cocodc_loop_t* loop, int64_t t, int32_t* due_out, int32_t* n_due_out);

/* One inner step t of the worker, called after its local optimiser step; t >= 1 and larger than
 * the t of the previous call (COCODC_ERR_RANGE otherwise; steps without an event may be skipped):
 *  1. every fragment due at t is received, in ascending index: the fused step
 *     (cocodc_sync_step) on that fragment alone with I_p = max(1, t_p - t_{p,b}) (Eq. 11; the
 *     interval of a fragment sent again at the very step its previous synchronisation completed
 *     counts as one step, so that R_p = +infinity remains the mark of a fragment that was never
 *     synchronised), which updates R_p; then t_{p,b} <- t.
 *  2. if t is a multiple of h: Algorithm 2 picks p* among the fragments that are not in flight
 *     (t_g = t); its pseudo-gradient goes to delta_m_out and theta_m_send records the
 *     send-time parameters; it will be due at t + tau.
 * Both happen on the device and the call never waits for the stream: p* is chosen by the
 * selection kernel and the pseudo-gradient kernel reads it from device memory.
 * received_out (host, K int32), n_received_out.  sent_out (host): -1 if this step took no send
 * decision, COCODC_LOOP_SENT_PENDING if it took one; which fragment it was is copied to the host
 * asynchronously, and cocodc_loop_last_sent tells (it waits for that copy and for nothing else).
 * The schedule itself reads the copy back when it next needs it: at the next send decision or
 * when the fragment could be due, whichever comes first.
 * Every pointer of `buf` is checked before anything is enqueued (delta_m_out and theta_m_send are
 * required): a rejected step changes neither the buffers nor the schedule. */
#define COCODC_LOOP_SENT_PENDING (-2)
int cocodc_loop_step(cocodc_loop_t* loop, int64_t t, const cocodc_loop_buffers_t* buf, void* stream,
                     int32_t* received_out, int32_t* n_received_out, int32_t* sent_out);

/* The same step for a worker whose local parameters are bf16 (Sec. 4.1: bf16 mixed precision):
 * theta_m, theta_m_send and delta_m_out are 16-bit patterns as in cocodc_sync_step_bf16, the
 * outgoing pseudo-gradient in the format hp->pg_format of the hyper-parameters the loop was
 * created with; delta_g (the arriving average) stays fp32, so the send buffer cannot be delta_g.
 * A loop object is used with one of the two step functions throughout. */
typedef struct {
  uint16_t* theta_m;      /* bf16 local parameters                                         */
  uint16_t* theta_m_send; /* bf16 send-time records                                        */
  float* theta_g;
  float* momentum;
  float* delta_g;
  uint16_t* delta_m_out;  /* bf16 or binary16 pseudo-gradient of the fragment that is sent */
  double* R;
  int32_t* sel;
  int32_t* n_sel;
  void* workspace;
  size_t workspace_bytes;
} cocodc_loop_buffers_bf16_t;
int cocodc_loop_step_bf16(cocodc_loop_t* loop, int64_t t, const cocodc_loop_buffers_bf16_t* buf, void* stream,
                          int32_t* received_out, int32_t* n_received_out, int32_t* sent_out);

/* The most recent send decision: the step it was taken at and the fragment (-1, -1 before the
 * first; fragment -1 if nothing was eligible).  Waits until that decision has been copied to the
 * host.  A caller that launches the all-reduce from the host calls this right after the step. */
int cocodc_loop_last_sent(cocodc_loop_t* loop, int64_t* t_sent_out, int32_t* sent_out);

/* Copies the bookkeeping out (host arrays of K): t_{p,b}, the I_p used at the last receive
 * (0 = never), and the send step of a fragment in flight (-1 = not in flight).  Reads back a
 * pending send decision first. */
int cocodc_loop_state(cocodc_loop_t* loop, int64_t* t_b_out, int64_t* I_p_out, int64_t* in_flight_out);

/* ---- data layout in HBM (no paper counterpart) ---- */

/* Recommended distance in bytes between the base addresses of the flat buffers that one
 * call streams through together (theta_m, theta_m_send, theta_g, momentum, delta_g,
 * delta_m_out), for buffers of n_total fp32 elements carved out of ONE device allocation.
 * On MI355X the fused pass runs up to 18 % faster when the buffers it writes do not all lie
 * within the same third of the device memory (measured: 5.5-5.7 TB/s with all six buffers
 * inside one 96 GiB third, wherever; 6.2-6.5 TB/s as soon as a written one lies in another third,
 * also when the six lie back to back across the 96 GiB or the 192 GiB mark; 6.45-6.55 TB/s with
 * the bases 33-47 GiB apart, which spreads them over all three).  An allocation's place in the
 * device memory cannot be asked for, so a layout that matters is better probed than computed: see
 * tuned_spaced_buffers in the Python package's layout module.  The gaps can hold any other data.  Returns
 * max(40 GiB, buffer size rounded up to 1 GiB), moved off multiples of 32 GiB.  Purely
 * advisory: every entry point accepts any placement.  Host-only. */
uint64_t cocodc_layout_stride_bytes(uint64_t n_total);

/* ---- diagnostics and measurement aids (no paper counterpart) ---- */

/* Elements per tile (the aligned window of the flat buffers that one workgroup handles) for
 * buffers of n_total elements: 4096, or 2048 when n_total < 2^24 so that small calls still
 * spread over the whole chip. */
uint64_t cocodc_tile_elements(uint64_t n_total);

/* Host-only view of the tile list the kernels would walk for a segment table (for tests and
 * debugging; no GPU work).  Segments are walked grouped by fragment, in the order listed within a
 * fragment.  seg_offset_out / seg_slot_begin_out (S+1 entries): offset of the j-th walked segment
 * and the index of its first tile; entry S holds the total number of tiles.
 * frag_slot_begin_out (K+1 entries): fragment p owns tiles [p], [p+1]).  tile_capacity_out: the
 * number of tile slots that cocodc_workspace_bytes_segmented(S, K, n_total) provides. */
int cocodc_debug_tile_plan(const cocodc_segment_t* segs, int32_t S, int32_t K, uint64_t n_total,
                           uint64_t* seg_offset_out, uint64_t* seg_slot_begin_out,
                           uint64_t* frag_slot_begin_out, uint64_t* tile_capacity_out);

/* Measurement aid (no paper counterpart): streams the six device buffers exactly as the fused
 * step does -- a, c, d read and rewritten in place, b and e read, f written, 36 bytes per
 * element of every fragment -- with one fp32 addition per stored value (a += b, c += e, d += e,
 * f = b + c).  Its duration is what the memory system gives this access pattern when the
 * arithmetic is free; bench.py reports it beside the fused step.  Same table, workspace,
 * alignment and overlap rules as cocodc_sync_step (no two buffers may overlap). */
int cocodc_debug_stream_mix(const cocodc_fragment_t* frags, int32_t K, uint64_t n_total, float* a,
                            const float* b, float* c, float* d, const float* e, float* f,
                            void* workspace, size_t workspace_bytes, void* stream);

/* hipError_t of the most recent failing HIP call on this thread (0 if none). */
int cocodc_last_hip_error(void);

/* Static, human-readable name of a status code. */
const char* cocodc_status_string(int status);

/* Launch shape of the streaming kernels: blocks_per_cu > 0 launches a persistent grid
 * of (compute units x blocks_per_cu) workgroups that stride over the tiles; 0 launches
 * one workgroup per tile.  Results never depend on it.  Returns the previous value. */
int cocodc_set_blocks_per_cu(int blocks_per_cu);

/* Where the kernels read the fragment table from.  Tables of at most 32 segments and 32 fragments
 * normally travel inside the arguments of every kernel of a call, which saves the small upload
 * launch in front of them; larger tables are written to the head of the workspace first.
 * enabled = 0 makes every call upload (to compare the two paths; results never depend on it).
 * Returns the previous setting.  Process-wide; a loop object plans the table of its send step when
 * it is created and keeps the setting of that moment for it. */
int cocodc_set_tables_in_args(int enabled);

/* Kernel timer for benchmarks.  After cocodc_profiler_enable(n) every launch of a
 * streaming kernel (one per call of cocodc_sync_step*, cocodc_pseudograd*,
 * cocodc_outer_nesterov, cocodc_delay_compensate, cocodc_fragment_scores*) is bracketed
 * by a pair of HIP events on the caller's stream (up to n launches; not under graph
 * capture).  cocodc_profiler_collect synchronises those events, writes up to `capacity`
 * per-launch durations in milliseconds to ms_out (host), in launch order, and returns
 * how many it wrote; cocodc_profiler_disable releases the events.  Process-wide state:
 * not for concurrent use from several threads. */
int cocodc_profiler_enable(int32_t max_records);
int cocodc_profiler_collect(float* ms_out, int32_t capacity);
int cocodc_profiler_disable(void);

#ifdef __cplusplus
}
#endif
#endif /* COCODC_H */
