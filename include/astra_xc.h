/*
 * astra_xc.h -- C ABI of the MI355X (gfx950) classifier-layer hot path of ASTRA
 * (arXiv 2409.20156): hard-negative mining by exact top-k inner product, the
 * hard+uniform negative mixture, and the sampled BCE training step with a sparse
 * SGD update of the classifier rows.
 *
 * Conventions shared by every call
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     allocates nothing; temporary memory is a caller-provided workspace whose
 *     size is asked for first (xc_*_workspace).  Workspaces and all arrays must
 *     be 16-byte aligned.
 *   - Work is enqueued on the HIP stream passed as `stream` (a hipStream_t cast
 *     to void*, NULL = the default stream).  No call synchronises; results,
 *     including scalars, appear in device memory in stream order.
 *   - W is row-major L x d (one label per contiguous row), Z row-major B x d,
 *     both of type `t`.  Label ids are int32 in [0, L); any id outside that
 *     range (-1 by convention) is padding and is ignored.
 *   - Return value: XC_OK or a negative xc_status.  Shape and pointer errors are
 *     detected on the host before anything is launched; nothing is written then.
 *     After XC_EHIP, xc_last_hip_error() gives the hipError_t of this thread.
 */
#ifndef ASTRA_XC_H
#define ASTRA_XC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { XC_F32 = 0, XC_BF16 = 1 } xc_dtype;            /* storage of Z and W; sums are fp32 */
typedef enum { XC_LOSS_BCE = 0, XC_LOSS_SOFTMAX = 1 } xc_loss;

typedef enum {
    XC_OK = 0,
    XC_EINVAL = -1,      /* null or misaligned pointer, bad loss kind or margin   */
    XC_ESHAPE = -2,      /* unsupported or inconsistent sizes                     */
    XC_EWORKSPACE = -3,  /* workspace smaller than xc_*_workspace reports         */
    XC_EHIP = -4,        /* a HIP runtime call failed; see xc_last_hip_error()    */
    XC_EDTYPE = -5,      /* element type that is neither XC_F32 nor XC_BF16       */
    XC_ESCRATCH = -6     /* xc_step_static: the step's temporaries exceed
                            XC_STATIC_SCRATCH_BYTES                               */
} xc_status;

/* limits checked by the host side of every call */
#define XC_MAX_K_MINE 128      /* k_h accepted by xc_mine_negatives                */
#define XC_MAX_K_SAMPLE 1024   /* k_h accepted by xc_sample_negatives              */
#define XC_MAX_ROW_BYTES 4096  /* d * sizeof(element) accepted by xc_step          */
#define XC_MAX_CANDIDATES 16384 /* k_p + n_neg accepted by xc_step                 */
#define XC_MAX_KP 256          /* k_p accepted by xc_step                          */
#define XC_STATIC_SCRATCH_BYTES (32u << 20)  /* temporaries xc_step_static can hold    */

const char* xc_strerror(int status);
int xc_last_hip_error(void);
int xc_version(void);

/* ---------------------------------------------------------------------------
 * Mining (Alg. 1, the "ANNS refresh" step; Sec. 2.1 score f_l(x) = <w_l, z>).
 * Exact search stands in for the ANNS index, which the paper itself ran as a
 * control (Sec. 5.2.1 a).  For each of the Zq query rows of Z:
 *   shortlist[i*k_h + r] = id of the label with the r-th largest <z_i, w_l>,
 *   l in [0, L); equal scores are ordered by smaller id.
 *   scores[i*k_h + r]    = that inner product (fp32), if scores != NULL.
 * Products are accumulated in fp32.  The Zq x L score matrix is never stored.
 * Requires 1 <= k_h <= min(L, XC_MAX_K_MINE), d*sizeof(element) a multiple of 16.
 * A score that is NaN is never selected; a query with fewer than k_h finite
 * scores gets id -1 and score -inf in the remaining slots.
 * Two environment variables, read at every call, only choose between kernels
 * that return the same result (for A/B timing and tests): XC_MINE_GENERAL=1
 * sends every shape through the general tile kernel; XC_MINE_ROWS=narrow or
 * wide fixes the work-item width of the kernel for bf16 rows of 128..512 bytes.
 * ------------------------------------------------------------------------- */
int xc_mine_workspace(int64_t Zq, int64_t L, int d, int k_h, xc_dtype t, size_t* bytes);
int xc_mine_negatives(const void* Z, const void* W, int64_t Zq, int64_t L, int d, int k_h,
                      xc_dtype t, int32_t* shortlist /* [Zq*k_h] out */,
                      float* scores /* [Zq*k_h] out, or NULL */,
                      void* ws, size_t ws_bytes, void* stream);

/* The same search, with the same result in every case, started from the thresholds that the previous
 * search with this workspace left in it: Alg. 1 repeats the search every tau_r steps on a classifier that
 * has moved little, so the k_h-th score of a query, lowered by rel_margin * |score|, is a threshold
 * that its new k_h best labels almost always pass.  One sweep over the labels with these thresholds
 * and one selection replace the phased search.  If a query comes out of the sweep with fewer than
 * k_h candidates (the classifier moved further than the margin, or the workspace held nothing
 * useful), a flag is raised on the device for its tile of 256 queries and the call repeats the full
 * search for the flagged tiles; whatever the workspace holds, the result is exact and only the time
 * differs.  rel_margin >= 0.  The first 32-bit word of the workspace is 1 after the call if some tile
 * needed the full search, else 0 (device memory; read it after synchronising the stream). */
int xc_mine_negatives_warm(const void* Z, const void* W, int64_t Zq, int64_t L, int d, int k_h,
                           xc_dtype t, float rel_margin, int32_t* shortlist /* [Zq*k_h] out */,
                           float* scores /* [Zq*k_h] out, or NULL */,
                           void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * Negative sampling (Alg. 1, hard+random step; Sec. 3.1 Idea 2; p under Eq. 2).
 * For query i of the batch, neg[i*(k_h+k_r) + ...]:
 *   slots 0..k_h-1   the shortlist row of the query, copied verbatim, logq = 0
 *                    (taken with probability one, weight 1 in Eq. 2);
 *   slots k_h..      k_r independent uniform draws from [0,L) minus H_i, H_i the
 *                    distinct in-range ids of the row (u_i of them; u_i = k_h for
 *                    a mined shortlist), logq = log(k_r / (L - u_i)): the log of
 *                    the expected number of copies of a label, so exp(-logq) is
 *                    the 1/(p k_r) factor of Eq. 2.
 * shortlist == NULL selects the warm-up phase (Alg. 1, t < tau_s): all k_h+k_r
 * slots are uniform draws from [0,L) and logq = log((k_h+k_r)/L).
 * Draw j of query i is element r = floor(u*M / 2^64) of the complement, M its
 * size, u = fmix(fmix(seed ^ K1*(i+1)) + K2*(j+1)) with fmix the splitmix64
 * finaliser, K1 = 0x9E3779B97F4A7C15, K2 = 0xD1B54A32D192ED03 (64-bit wrapping).
 * Integer arithmetic only: the ids depend on (seed, i, j, shortlist row) and on
 * nothing else.  Requires 0 <= k_h <= XC_MAX_K_SAMPLE, k_h < L, k_h + k_r >= 1.
 * ------------------------------------------------------------------------- */
int xc_sample_negatives(const int32_t* shortlist /* [B*k_h] or NULL */, int64_t B, int k_h,
                        int k_r, int64_t L, uint64_t seed,
                        int32_t* neg /* [B*(k_h+k_r)] out */,
                        float* logq /* [B*(k_h+k_r)] out */, void* stream);

/* ---------------------------------------------------------------------------
 * Negative sampling from the mixture proposal itself (Sec. 3.1, Idea 2:
 * P = (1-r) P_imp + r P_unif with P_imp proportional to the sigmoid of the stale score,
 * r = k_r/(k_h+k_r)), in stratified form.  shortlist and scores are [B*M], M >= k_h wide
 * (for example the M best labels and their scores from xc_mine_negatives).  For query i:
 *   slots 0..k_h-1   independent draws of a shortlist slot m with probability w_m / T,
 *                    w_m an integer image of 2^32*sigmoid(score) (about 1e-4 relative; the
 *                    exact recipe is in the sampler's source), T the sum over the row;
 *                    slots whose id is outside [0,L) or whose score is NaN have weight 0;
 *   slots k_h..      independent uniform draws from all of [0,L);
 *   logq             for every slot, log(k_h*W_l/T + k_r/L), W_l the total weight of the
 *                    slots holding that label: the log of the expected number of copies,
 *                    so pairs weighted by exp(-logq) estimate the sum over all L labels
 *                    without bias.  A row without any weight: all slots uniform,
 *                    logq = log((k_h+k_r)/L).
 * Random words as in xc_sample_negatives (draw j of query i); the importance draw is
 * floor(u*T/2^64) located in the running sums of the weights in slot order.  Integer
 * arithmetic only for the ids.  Requires 1 <= M <= XC_MAX_K_SAMPLE, k_h + k_r >= 1.
 * ------------------------------------------------------------------------- */
int xc_sample_negatives_mixture(const int32_t* shortlist /* [B*M] */, const float* scores /* [B*M] */,
                                int64_t B, int M, int k_h, int k_r, int64_t L, uint64_t seed,
                                int32_t* neg /* [B*(k_h+k_r)] out */, float* logq /* [B*(k_h+k_r)] out */,
                                void* stream);

/* ---------------------------------------------------------------------------
 * Hard negatives SAMPLED WITHOUT REPLACEMENT from a wider stale shortlist, a slot with probability
 * proportional to the sigmoid of its stale score (Sec. 3.1: the importance distribution of
 * Observation 2 inside the mixture of Idea 2; the paper then retrieves the top scoring labels
 * instead, which xc_sample_negatives does).  shortlist and scores are [B*M] as above, weights w_m
 * as in xc_sample_negatives_mixture.  For query i, k = min(k_h, number of slots with weight) slots
 * are chosen with inclusion probability pi_m = min(1, k' w_m / T'):
 *   - slots with k' w_m >= T' (k' slots still to choose, T' the remaining total weight) are taken
 *     for certain, all at once, and the test is repeated with what remains;
 *   - the others by systematic sampling: on the axis of the running sums of the remaining weights,
 *     in slot order and scaled by k', the points U + j T' (j < k') are marked, U = floor(u T' / 2^64)
 *     with u the query's draw 0; a slot is taken when a point falls into its interval.  No slot is
 *     taken twice and exactly k' are taken.
 *   slots 0..k-1     the labels of the chosen slots, in slot order;
 *   slots k..        independent uniform draws from all of [0,L) (draw j for slot j);
 *   logq             log(sum of pi_m over the slots holding the label + (k_h + k_r - k) / L): the
 *                    log of the expected number of copies, so pairs weighted by exp(-logq) estimate
 *                    the sum over all L labels without bias.  A row without any weight: all slots
 *                    uniform.
 * Integer arithmetic only for the ids.  Requires 1 <= M <= XC_MAX_K_SAMPLE, 0 <= k_h <=
 * XC_MAX_K_SAMPLE, k_h + k_r >= 1.
 * ------------------------------------------------------------------------- */
int xc_sample_negatives_pps(const int32_t* shortlist /* [B*M] */, const float* scores /* [B*M] */,
                            int64_t B, int M, int k_h, int k_r, int64_t L, uint64_t seed,
                            int32_t* neg /* [B*(k_h+k_r)] out */, float* logq /* [B*(k_h+k_r)] out */,
                            void* stream);

/* ---------------------------------------------------------------------------
 * One training step of the classifier layer (Alg. 1: scores on positives and
 * sampled negatives, loss of Eq. 2, SGD on W; loss averaged over the batch).
 * Per query i with score s = <z_i, w_l> on the pre-update W:
 *   BCE      loss_i = sum_{l in pos_i} log(1+e^-s)
 *                   + sum_{j} m_ij e^{-logq_ij} (s + log(1+e^-s)),
 *            m_ij = 0 if neg_ij is padding or one of pos_i (the (1-y_l) factor);
 *   SOFTMAX  logits s - logq over pos_i and the unmasked negatives,
 *            loss_i = mean over pos_i of -log softmax (a query without a
 *            positive is skipped).
 *   loss[0] = (1/B) sum_i loss_i;  dZ = d loss / d Z (fp32, [B*d]);
 *   w_l <- w_l - lr * d loss / d w_l for every label in an unmasked pair;
 *   a label in several pairs gets the summed gradient, added in a fixed order
 *   (results are bitwise reproducible run to run), and is written once (rounded
 *   to nearest even for bf16).
 *   touched[0..n_touched[0]) = those labels, ascending; no other row changes.
 *   W_rows_out, if not NULL, receives the updated rows in that order.
 *   (How: the pairs are sorted by label first.  For the BCE loss a label with a single
 *   unmasked pair gets its row updated while that pair's score is computed, w - lr g z
 *   rounded once; the other labels are summed over their pairs in pair order afterwards.
 *   After the call the first 32-bit word of the workspace holds the number of rows of
 *   the first kind, for measurements.)
 * Z and dZ must not alias.  Requires B >= 1, 0 <= k_p <= XC_MAX_KP, n_neg >= 0,
 * 1 <= k_p + n_neg <= XC_MAX_CANDIDATES, B*(k_p+n_neg) < 2^31,
 * d*sizeof(element) a multiple of 16 and <= XC_MAX_ROW_BYTES.
 * The workspace size does not depend on L.
 * ------------------------------------------------------------------------- */
int xc_step_workspace(int64_t B, int d, int k_p, int n_neg, xc_dtype t, size_t* bytes);
int xc_step(const void* Z /* [B*d] */, void* W /* [L*d], updated in place */, int64_t B,
            int64_t L, int d, const int32_t* pos /* [B*k_p] */, int k_p,
            const int32_t* neg /* [B*n_neg] */, const float* logq /* [B*n_neg] */, int n_neg,
            float lr, xc_loss kind, xc_dtype t, float* loss /* [1] out */,
            float* dZ /* [B*d] out */, int32_t* touched /* [B*(k_p+n_neg)] out */,
            int32_t* n_touched /* [1] out */, void* W_rows_out /* [B*(k_p+n_neg)*d] or NULL */,
            void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * xc_step for callers that cannot allocate device memory and have no workspace to hand over:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and error behaviour as xc_step, without `ws`/`ws_bytes`: the step's
 * temporaries (sort pairs, coefficients, histograms, segment starts, partial sums) live in an
 * array of XC_STATIC_SCRATCH_BYTES that is part of the library's device image, one per GPU, held
 * until the process ends.  The call allocates and frees nothing; its first call on a device asks
 * the runtime once for the array's address there.  A shape for which xc_step_workspace reports
 * more than XC_STATIC_SCRATCH_BYTES is refused with XC_ESCRATCH before anything is launched
 * (the c2 and c3 benchmark shapes fit, c4 and c5 do not).  All calls on one GPU share that
 * GPU's array: calls that overlap in time on one GPU (two streams, two threads) race and give
 * wrong results; calls on one stream, or ordered by events, are safe.  Nothing needs clearing
 * between calls: every temporary is written before it is read.
 * ------------------------------------------------------------------------- */
int xc_step_static(const void* Z /* [B*d] */, void* W /* [L*d], updated in place */, int64_t B,
                   int64_t L, int d, const int32_t* pos /* [B*k_p] */, int k_p,
                   const int32_t* neg /* [B*n_neg] */, const float* logq /* [B*n_neg] */, int n_neg,
                   float lr, xc_loss kind, xc_dtype t, float* loss /* [1] out */,
                   float* dZ /* [B*d] out */, int32_t* touched /* [B*(k_p+n_neg)] out */,
                   int32_t* n_touched /* [1] out */, void* W_rows_out /* [B*(k_p+n_neg)*d] or NULL */,
                   void* stream);

/* ---------------------------------------------------------------------------
 * Measurement aid (no passage of the paper: used by the benchmark to time each
 * kernel with HIP events on the stream it is launched on).  While enabled, every
 * kernel launch of the three calls above is bracketed by a pair of events.
 * xc_profile_collect() waits for the recorded events (host-side wait), adds the
 * elapsed times to per-kernel totals and returns the number of kernel names;
 * xc_profile_get(i, ...) reads total milliseconds and launch count of name i;
 * xc_profile_reset() clears the totals.  Off by default; when off the calls
 * above record no events.  Not thread-safe against concurrent launches.
 * ------------------------------------------------------------------------- */
int xc_profile_enable(int on);
int xc_profile_collect(void);
int xc_profile_get(int i, const char** name, double* total_ms, int64_t* launches);
int xc_profile_reset(void);

/* Measurement aid: a plain device-to-device copy kernel (reads `bytes`, writes `bytes`;
 * both pointers device memory, 16-byte aligned, `bytes` a multiple of 16, buffers must not
 * overlap).  The benchmark launches it beside the library's kernels in hardware-counter runs
 * so that the traffic counters can be scaled by a kernel of known size.  Asynchronous on
 * `stream`.  XC_EINVAL on null or misaligned arguments. */
int xc_copy_probe(void* dst, const void* src, size_t bytes, void* stream);

/* Measurement aid: a register-resident loop of bf16 MFMA instructions (no memory traffic) on
 * 256 workgroups of 8 waves, `iters` (1 .. 2^20) rounds of 8 products per wave.  With
 * random_operands != 0 the operands are pseudo-random bf16 values, else zero: the rate the chip
 * sustains depends on the operand values through its power limit, and the benchmark reports it
 * beside the published peak.  `out` is device memory for 256*512 floats (a checksum, so that the
 * loop is not removed); `*flop` (host pointer, may be NULL) receives the floating-point
 * operations of one launch.  Asynchronous on `stream`. */
int xc_mfma_probe(float* out, int iters, int random_operands, double* flop, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ASTRA_XC_H */
