/* sdden.h -- C ABI of the target predictions D(y, k) used by the synthetic workloads.
 *
 * The method treats the target's drift as a black-box network (Sec. 3.1: the drift is given by a
 * trained network) that is evaluated on all drafted states of a window in one batched
 * call (Alg. "Speculative Sampling for DDM", the (Par.) line).  These are the stand-ins with a
 * plain definition; each maps rows X [R,d] with a per-row chain step krow [R] to out [R,d]:
 *
 *   gmm      E[x0 | x_t] of a diagonal-covariance Gaussian mixture (Bayes' rule over components)
 *   lowrank  E[x0 | x_t] of N(mu, U U^T + s2 I): two skinny fp32 MFMA GEMMs in the eigenbasis of
 *            U U^T with a per-row diagonal gain in between
 *   mlp      3-layer SiLU MLP on [x ; sinusoidal(k)], bf16 weights, fp32 accumulation (bf16 MFMA)
 *
 * Conventions as in sd.h: "dev" pointers are caller-owned device memory, "host" pointers are read
 * during the create call only.  Rows with krow < 0 or krow >= T are skipped: nothing is computed
 * for them and their output row is left untouched.  `alpha_bar_state` (host, length T+1) is the signal level of
 * chain state k: x = sqrt(ab) x0 + sqrt(1-ab) eps.  sdden_eval only enqueues kernels on `stream`.
 */
#ifndef SDDEN_H
#define SDDEN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sdden sdden;     /* opaque; owns device copies of its parameters and tables */

/* means, stds [M,d], logw [M] (log mixture weights), alpha_bar_state [T+1]: host. */
int sdden_gmm_create(int32_t M, int32_t d, const float* means, const float* stds,
                     const float* logw, int32_t T, const float* alpha_bar_state, sdden** out);

/* mu [d], U [d,r] row-major, alpha_bar_state [T+1]: host.  Builds the eigenbasis Q [d,r] of U U^T
 * and the per-step gain tables on the host in fp64. */
int sdden_lowrank_create(int32_t d, int32_t r, const float* mu, const float* U, float s2,
                         int32_t T, const float* alpha_bar_state, sdden** out);

/* W1 [(d+E),H], W2 [H,H], W3 [H,d]: bf16 bit patterns, row = input feature; b1,b2 [H], b3 [d]:
 * host.  Time embedding of width E: emb[i] = sin(k w_i), emb[E/2+i] = cos(k w_i),
 * w_i = 10000^(-2i/E); its product with the last E rows of W1 is folded into a per-step bias
 * table at create time.  Rmax: rows reserved right away (as by sdden_reserve).
 * d and H must be multiples of 256. */
int sdden_mlp_create(int32_t d, int32_t H, int32_t E, const uint16_t* W1, const float* b1,
                     const uint16_t* W2, const float* b2, const uint16_t* W3, const float* b3,
                     int32_t T, int32_t Rmax, sdden** out);

/* Setup call: allocate the per-call scratch (row lists, intermediate activations) that
 * evaluations of up to Rmax rows need.  The gmm denoiser needs none; lowrank and mlp return
 * SD_ERR_WORKSPACE from sdden_eval when R exceeds what was reserved.  May be called again with a
 * larger Rmax (not while evaluations are in flight). */
int sdden_reserve(sdden* den, int32_t Rmax);

/* out[r] = D(X[r], krow[r]) for every r < R with 0 <= krow[r] < T.
 * X [R,d], krow [R], out [R,d]: dev, 16-byte aligned; X and out must not overlap.
 * Enqueues kernels on `stream` only: no allocation, no synchronisation. */
int sdden_eval(sdden* den, int32_t R, const float* X, const int32_t* krow, float* out,
               void* stream);

/* sdden_eval for a caller that also holds the rows as bf16 (bit patterns, round-to-nearest-even of
 * the same fp32 values; sd_draft can write this image next to the fp32 drafts, see
 * sd_set_draft_mirror in sd.h).  The MLP reads its first layer's input from Xbf16 and skips its
 * own conversion pass; the other denoisers ignore it.  Rows with krow < 0 need no valid image. */
int sdden_eval_mirror(sdden* den, int32_t R, const float* X, const uint16_t* Xbf16,
                      const int32_t* krow, float* out, void* stream);

/* Optional device-resident row limit: when `count` (dev int32) is set, only rows
 * r < min(R, *count * rows_per_chain) are evaluated, which lets a fixed launch sequence follow
 * the batch as sd_advance shrinks it (see sd_set_active_count).  NULL removes the limit. */
int sdden_set_active_count(sdden* den, const int32_t* count /*dev*/, int32_t rows_per_chain);

/* Measurement aid: time the `which`-th kernel of every following sdden_eval with HIP events on
 * the evaluation's stream (gmm: 1 = posterior mean; lowrank: 1, 2 = the two GEMMs; mlp: 1..3 = the
 * three GEMMs; 0 = off, the default).  sdden_profile_collect waits for the recorded events, returns
 * the summed kernel time in ms and the number of timed launches, and starts a new collection.
 * Event objects are created on demand while profiling is on (never otherwise).
 * sdden_profile_min_rows restricts the timing to calls with R >= min_rows (default 0: every call),
 * e.g. to the batched evaluation of the drafted states rather than the window-start call. */
int sdden_profile(sdden* den, int32_t which);
int sdden_profile_min_rows(sdden* den, int32_t min_rows);
int sdden_profile_collect(sdden* den, double* total_ms, int64_t* launches);

/* Measurement aid (mlp only): which kernel serves the 256 x 256 GEMM tile of the batched call.
 * 0 = the default (alternating-phase kernel); 1 = the earlier hand-scheduled kernel, kept so that
 * the two can be timed side by side on the same data (results agree).  2, 3, 4 = the default
 * kernel with its fragment reads / its direct loads / both left out: TIMING ONLY, the results are
 * wrong -- they locate what bounds the kernel (4 = the MFMA and barrier schedule alone); 5 = the
 * default kernel without the fragment reads of the weight tile only (a third of its LDS reads),
 * TIMING ONLY as well. */
int sdden_mlp_select_gemm(sdden* den, int32_t variant);

int sdden_destroy(sdden* den);
const char* sdden_last_error(const sdden* den);

#ifdef __cplusplus
}
#endif
#endif /* SDDEN_H */
