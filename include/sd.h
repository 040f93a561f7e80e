/* sd.h -- C ABI of the speculative-sampling hot path for diffusion chains on MI355X (gfx950).
 *
 * One window of the method (paper: Alg. "Speculative Sampling for DDM" and its detailed form in
 * App. "Detailed implementation of speculative sampling for diffusion models"):
 *
 *     D0 = D(y_n, n)                         target prediction at the window start (caller, sdden.h)
 *     sd_draft   : y~_{n+1..n+Kt} from the frozen draft mean  a_k y~_k + c_k D0      (Sec. 3.1)
 *     Dq_j = D(y~_{n+j-1}, n+j-1)            one batched target call on the drafts  (caller)
 *     sd_verify  : accept test, first rejection, reflection-maximal-coupling resample (Sec. 3.3)
 *     sd_advance : n <- n + advance, finished chains leave the batch             (end of the loop body)
 *     sd_langevin_window : the whole window for unadjusted Langevin on a Gaussian-mixture energy,
 *                  fused in one launch (Sec. 5 and App. on Langevin diffusions)
 *
 * Notation: T = chain length (the paper's K), K = window length (the paper's L),
 * Kt = min(K, T - n) (the paper's L-tilde), B = chains in the batch, d = state dimension.
 * The chain is the Gaussian autoregression
 *     y_{k+1} ~ N( a[k] * y_k + c[k] * D(y_k, k),  sigma[k]^2 I ),   k = 0 .. T-1,
 * which covers the paper's Euler-Maruyama chain (a = 1, c = gamma, D = b^q), the DDPM ancestral
 * sampler with an x0-predicting network, and ULA (a = 1, c = -gamma, D = grad E, sigma = sqrt(2 gamma)).
 *
 * Conventions
 *  - Every pointer argument marked "dev" is DEVICE memory owned by the caller; "host" is host memory.
 *    Row-major everywhere; [B,K,d] keeps the K rows of one chain adjacent.  Buffers must not
 *    overlap unless a call says "in place".
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  The four window calls
 *    only enqueue kernels: no allocation, no host synchronisation, no use of another stream.
 *  - Return value: SD_OK or a negative sd_status.  Arguments are validated on the host before
 *    anything is enqueued; nothing is enqueued on error.  sd_last_error() gives the text.
 *  - Random numbers: Philox4x32-10 keyed by (seed; chain_id, state index k, stream, block), so a
 *    result depends on the chain's id and step only -- never on B, on the order of chains, or on
 *    how a run is split into calls.  Stream 0: noise that produces state k; stream 1: uniform
 *    that tests state k; stream 2: initial state.  32-bit word w -> u = ((w>>9)+1/2) 2^-23;
 *    normals by Box-Muller on word pairs (0,1) and (2,3) of a block (= 4 consecutive elements).
 *  - Accept iff  log u <= min(0, (-Z.Delta - |Delta|^2/2) / tau)  evaluated in fp64, where
 *    Delta = (m^p - m^q)/sigma and Z = (y~ - m^p)/sigma is recomputed from the stored draft.
 *    |Delta| = 0 accepts without reflection.
 */
#ifndef SD_H
#define SD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SD_OK = 0,
  SD_ERR_ARG = -1,        /* null pointer, non-positive size, K > SD_MAX_WINDOW, misuse            */
  SD_ERR_SCHEDULE = -2,   /* sigma <= 0 or a non-finite coefficient                               */
  SD_ERR_WORKSPACE = -3,  /* workspace missing or too small for this B                            */
  SD_ERR_HIP = -4,        /* a HIP runtime call failed (text in sd_last_error)                    */
  SD_ERR_UNSUPPORTED = -5 /* shape outside what the kernels were built for (text says which)      */
} sd_status;

#define SD_MAX_WINDOW 64          /* K <= 64: one wavefront ballot resolves the first rejection   */
#define SD_STATIC_MAX_CHAINS 65536 /* largest batch sd_advance_static serves                      */

#define SD_DRAFT_FROZEN 0         /* draft mean a y~ + c D0, D0 fixed over the window (Sec. 3.1)   */
#define SD_DRAFT_EXPLICIT 1       /* caller supplies the draft means mp[B,K,d] (any drafter)       */
#define SD_DRAFT_FROZEN_REUSED 2 /* frozen on a prediction carried over from the previous window:
                                    D(y~_n, n) at the DRAFT state of position n, which that window's
                                    verification already computed (the efficient frozen draft strategy
                                    of the App. on extending the draft models).  One batched target call per
                                    window; window arrays hold K+1 rows per chain, see below.      */

typedef struct sd_ctx sd_ctx;     /* opaque; owns only its device copy of the schedule            */

/* Host arrays of length T, copied at sd_create. */
typedef struct {
  int32_t T;
  const float* a;
  const float* c;
  const float* sigma;             /* > 0: Delta divides by it                                     */
} sd_schedule;

/* Create a context for chains of dimension d and window K on the current HIP device.
 * Allocates and fills the device schedule (the only allocation the library ever makes for the
 * window calls).  Errors: SD_ERR_ARG, SD_ERR_SCHEDULE, SD_ERR_HIP. */
int sd_create(const sd_schedule* schedule, int32_t d, int32_t K, sd_ctx** out);
int sd_destroy(sd_ctx* ctx);

int sd_set_seed(sd_ctx* ctx, uint64_t seed);            /* default 0                              */
int sd_set_draft_mode(sd_ctx* ctx, int mode);           /* SD_DRAFT_FROZEN (default) / _EXPLICIT / _FROZEN_REUSED */
/* FROZEN_REUSED layout and calls.  The window arrays have K+1 rows per chain:
 *   X_ext [B,K+1,d]   row 0 = y_n (copied by sd_draft), row j = y~_{n+j}
 *   krow_ext [B,K+1]  step index of each row the target must evaluate, else -1: row 0 (always), rows
 *                     1..Kt except a row whose index would be T (the chain's final state)
 *   Dq_ext [B,K+1,d]  the caller's ONE batched target call on (X_ext, krow_ext) as [B*(K+1), d]
 * sd_draft(ctx, B, y, n, chain_id, D_frozen, X_ext, krow_ext) freezes the draft mean on D_frozen [B,d];
 * sd_verify(ctx, B, y, n, chain_id, D_frozen, Dq_ext, X_ext, ...) tests every position including the
 * first (D_frozen is not the prediction at y_n, so Delta_1 != 0 in general);
 * sd_advance additionally writes, for every chain that stays in the batch, the next window's frozen
 * vector D_frozen[new position] = Dq_ext[b][adv[b]] when the two arrays have been registered with
 * sd_set_carry (both dev, D_frozen must not alias Dq_ext; NULL, NULL unregisters).  The caller
 * initialises D_frozen with the target's prediction at the initial states. */
int sd_set_carry(sd_ctx* ctx, const float* Dq_ext, float* D_frozen);
/* Which prediction sd_advance carries (App. on extending the draft models, last sentence of the
 * paragraph on the efficient frozen draft strategy): SD_CARRY_DRAFT (default) = Dq_ext[b][adv[b]], the
 * prediction at the draft state of the position the chain advanced to; SD_CARRY_LAST_ACCEPTED = after
 * a rejection Dq_ext[b][adv[b]-1] instead, the prediction at the last state the chain kept (row 0,
 * the window's own start state, when the first draft was rejected), at that state's step index;
 * chains without a rejection carry the same row under both rules.  With SD_CARRY_LAST_ACCEPTED
 * sd_advance needs its `rejected` argument (SD_ERR_ARG when it is NULL).  Errors: SD_ERR_ARG. */
#define SD_CARRY_DRAFT 0
#define SD_CARRY_LAST_ACCEPTED 1
int sd_set_carry_rule(sd_ctx* ctx, int32_t rule);
/* Temperature tau > 0 of the accept test (App. "Influence of the temperature"); 1 = exact.       */
int sd_set_temperature(sd_ctx* ctx, float tau);
/* Measurement aid: launch shape of the accept / reflect kernel for rows of more than 256 16-byte
 * columns, as (threads per chain, window positions per group): 1 = (256,4); 2 = (256,2);
 * 3 = (512,4); 4 = (512,2); 0 = the default for the row length (2 up to 1024 columns, 4 above).
 * Results are bit-identical among the shapes with the same number of threads. */
int sd_set_verify_shape(sd_ctx* ctx, int32_t shape);
/* Optional device-resident batch size.  When set (non-NULL, dev int32), every window call treats
 * only the first min(B, *count) chains as present, so a fixed launch sequence (for instance a
 * captured HIP graph) keeps working while sd_advance shrinks the batch.  NULL restores B.        */
int sd_set_active_count(sd_ctx* ctx, const int32_t* count);
/* Optional bf16 image of the drafts: when set (dev, same shape and layout as the Ytilde argument of
 * sd_draft, 16-byte aligned), sd_draft also writes every drafted value rounded to bf16
 * (round-to-nearest-even, bit patterns) there, so that a network with bf16 inputs needs no
 * conversion pass over the fp32 drafts (sdden_eval_mirror).  NULL (default) switches it off. */
int sd_set_draft_mirror(sd_ctx* ctx, uint16_t* Ytilde_bf16);
/* EXPLICIT mode only, optional: the target prediction at the window start, D(y_n, n), as its own
 * [B,d] array (dev).  When set, sd_verify reads it wherever it would read row 0 of Dq, so the
 * window-start call and the batched call on the drafts can write to separate dense outputs.
 * NULL (default) restores row 0 of Dq. */
int sd_set_start_prediction(sd_ctx* ctx, const float* D_start);

/* Scratch for sd_advance (parked ids and steps, ranks, per-workgroup survivor counts: 16 bytes per chain
 * plus 4 per 1024 chains): bytes needed for batches up to Bmax, and the buffer (8-byte aligned). */
size_t sd_workspace_bytes(const sd_ctx* ctx, int32_t Bmax);
int sd_set_workspace(sd_ctx* ctx, void* workspace /*dev*/, size_t bytes);

/* The chains' start: Y_0 ~ N(0, Id), n = 0 (first line of Alg. "Speculative Sampling for DDM").
 * chain_id [B] dev (in), y [B,d] dev (out), n [B] dev (out). */
int sd_init_state(sd_ctx* ctx, int32_t B, const int64_t* chain_id, float* y, int32_t* n,
                  void* stream);

/* Frozen draft rollout (eq. "frozen draft model"; detailed algorithm, first for-loop):
 *   y~_{k+1} = a[k] y~_k + c[k] D0 + sigma[k] z_{k+1},  k = n .. n+Kt-1,  y~_n = y.
 * in : y [B,d], n [B], chain_id [B], D0 [B,d] = D(y, n)                               (dev)
 * out: Ytilde [B,K,d], row j-1 = y~_{n+j} (zeros for j > Kt);
 *      krow [B,K] int32: the chain step at which the target must be evaluated on row j-1 of
 *      Ytilde, i.e. n+j for j <= Kt-1, and -1 otherwise.  The target is evaluated on states
 *      n .. n+Kt-1 only: state n is the window start (its prediction is D0) and the last draft is
 *      not evaluated.                                                                    (dev) */
int sd_draft(sd_ctx* ctx, int32_t B, const float* y, const int32_t* n, const int64_t* chain_id,
             const float* D0, float* Ytilde, int32_t* krow, void* stream);

/* One position of a drafter that calls a (cheaper) network at every position: the independent
 * draft model of Sec. 3.1, p(y_{k+1} | y_k) = N(a_k y_k + c_k D^p(y_k, k), sigma_k^2 I).
 * For window position j (1-based), k = n+j-1, and every chain with j <= Kt:
 *     mp[b][j-1] = a[k] prev[b] + c[k] Dp[b];   Ytilde[b][j-1] = mp[b][j-1] + sigma[k] z_{k+1}
 * with the same keyed noise as sd_draft; rows of chains with j > Kt are zero-filled.
 * in : prev [B,d] = y~_{n+j-1} (y for j = 1); Dp [B,d] = D^p(prev, n+j-1); n, chain_id       (dev)
 * out: mp, Ytilde [B,K,d] (row j-1 only); krow [B,K] (entry j-1, as in sd_draft);
 *      next [B,d] or NULL: the new state as a dense matrix (must not alias prev or Dp);
 *      knext [B] or NULL: its step index n+j, or -1 when j >= Kt (the row needs no further call):
 *      (next, knext) are the input of the drafter's call for position j+1.                  (dev)
 * The caller loops j = 1..K, calling its draft network between the steps, then the target on
 * (Ytilde, krow) and sd_verify in EXPLICIT mode with mp. */
int sd_draft_step(sd_ctx* ctx, int32_t B, int32_t j, const float* prev, const int32_t* n,
                  const int64_t* chain_id, const float* Dp, float* mp, float* Ytilde, int32_t* krow,
                  float* next, int32_t* knext, void* stream);

/* Accept test + first rejection + reflection (Alg. "REJECTION ... same covariance"; detailed
 * algorithm, second for-loop).  For j = 1 .. Kt, k = n+j-1, prev = y (j = 1) or Ytilde[j-2]:
 *   m^q = a[k] prev + c[k] Dq[j-1];  m^p = a[k] prev + c[k] D0 (FROZEN) or mp[j-1] (EXPLICIT)
 *   accept y~_{n+j} = Ytilde[j-1] as stated in the header comment; at the first rejection
 *   y_out = m^q + sigma[k] (I - 2 e e^T) Z,  e = Delta/|Delta|, adv = j, rejected = 1;
 *   with no rejection y_out = Ytilde[Kt-1], adv = Kt, rejected = 0.
 * FROZEN: row 0 of Dq is never read (the window-start prediction IS D0, so Delta_1 = 0 exactly).
 * in : y, n, chain_id as above; D0_or_mp = D0 [B,d] (FROZEN) or mp [B,K,d] (EXPLICIT);
 *      Dq [B,K,d], row j-1 = D(y~_{n+j-1}, n+j-1); Ytilde [B,K,d]                     (dev)
 * out: y_out [B,d]; adv [B] int32 in 1..Kt; rejected [B] uint8;
 *      logratio, logu [B,K] float or NULL: the log acceptance ratio (already divided by tau) and
 *      log u of every position j <= Kt (0 beyond), for diagnostics and parity checks.   (dev)
 *      With both NULL the rows of Ytilde and Dq that lie a whole group of 4 positions past the
 *      chain's first rejection are not read (they decide nothing). */
int sd_verify(sd_ctx* ctx, int32_t B, const float* y, const int32_t* n, const int64_t* chain_id,
              const float* D0_or_mp, const float* Dq, const float* Ytilde, float* y_out,
              int32_t* adv, uint8_t* rejected, float* logratio, float* logu, void* stream);

/* n += adv; a chain with n = T is finished: its state goes to out[chain_id] and it leaves the
 * batch; the others are packed to the front in their old order (last line of the while-loop body of
 * Alg. "Speculative Sampling for DDM" and the loop's condition).
 * in : y_out [B,d], adv [B], rejected [B] or NULL (only used for the counters)          (dev)
 * in place: y [B,d], n [B], chain_id [B] -- rewritten with the remaining chains        (dev)
 * out: out [*, d], row index = chain_id (caller sizes it); B_active: dev int32, number of
 *      remaining chains.  B_active may be the pointer given to sd_set_active_count.
 *      counters: dev int64[5] or NULL, accumulated: {sum adv, chains processed, rejections,
 *      windows, sum Kt (positions drafted)}.  Needs the workspace. */
int sd_advance(sd_ctx* ctx, int32_t B, const float* y_out, const int32_t* adv,
               const uint8_t* rejected, float* y, int32_t* n, int64_t* chain_id, float* out,
               int32_t* B_active, int64_t* counters, void* stream);

/* sd_advance for callers that cannot allocate device memory or hand over a workspace: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels and bit-identical results; the scratch that sd_advance keeps in the caller's
 * workspace lives in a device array inside the library instead (16 bytes per chain, 1 MiB + 256 B
 * per GPU, held from library load until the process ends; its address on the context's device is
 * resolved in sd_create).  No workspace needs to be set; nothing is allocated or freed.
 * B > SD_STATIC_MAX_CHAINS returns SD_ERR_WORKSPACE.  All contexts on one GPU share the one array
 * and every call overwrites what the previous call left there (nothing in it has to start at
 * zero): calls that overlap in time on one GPU -- two streams, two contexts, two host threads --
 * race and must be ordered by the caller. */
int sd_advance_static(sd_ctx* ctx, int32_t B, const float* y_out, const int32_t* adv,
                      const uint8_t* rejected, float* y, int32_t* n, int64_t* chain_id, float* out,
                      int32_t* B_active, int64_t* counters, void* stream);

/* One speculative window of unadjusted Langevin, fused (Alg. "Speculative Sampling for
 * Unadjusted Langevin Diffusion", frozen-gradient proxy):  E(x) = -log sum_m w_m N(x; mu_m, s^2 I),
 *   target  x - gamma grad E(x) + sqrt(2 gamma) w,   draft  x - gamma grad E(x_n) + sqrt(2 gamma) w,
 *   Delta_j = sqrt(gamma/2) (grad E(y~_{j-1}) - grad E(x_n)).
 * The context supplies T, K, d and the seed; its schedule arrays are not read.
 * in : x [B,d], n [B], chain_id [B]; means [M,d]; logw [M] (log weights); comp_std = s; gamma (dev)
 * out: x_out [B,d], adv [B], rejected [B] or NULL; logratio, logu [B,K] or NULL as in sd_verify.
 * Calls on one context must be ordered (one stream, or events between streams): for d <= 1024 the
 * kernel hands chains to its wavefronts through a counter that belongs to the context, zeroed by a
 * one-thread kernel ahead of every launch; two launches of one context in flight at once would
 * share it.  Different contexts are independent. */
int sd_langevin_window(sd_ctx* ctx, int32_t B, const float* x, const int32_t* n,
                       const int64_t* chain_id, const float* means, const float* logw,
                       float comp_std, int32_t M, float gamma, float* x_out, int32_t* adv,
                       uint8_t* rejected, float* logratio, float* logu, void* stream);

/* The same window for the phi^4 lattice energy of the Langevin appendix (table of sampling metrics)
 * on an L x L periodic grid, sites numbered row by row, d = L*L (3 <= L <= 16):
 *   E(x) = (beta/2) sum over ordered neighbour pairs (x_i - x_j)^2 + sum_i (x_i^2 - 1)^2
 *        = beta sum over bonds (x_i - x_j)^2 + sum_i (x_i^2 - 1)^2   (every bond counts twice),
 *   grad E_i = 2 beta (4 x_i - its four neighbours) + 4 x_i (x_i^2 - 1).
 * Arguments as in sd_langevin_window with (L, beta) in place of the mixture. */
int sd_langevin_window_phi4(sd_ctx* ctx, int32_t B, const float* x, const int32_t* n,
                            const int64_t* chain_id, int32_t L, float beta, float gamma,
                            float* x_out, int32_t* adv, uint8_t* rejected, float* logratio,
                            float* logu, void* stream);

/* The while-loop of the Langevin algorithm for each chain in one launch: up to max_windows (>= 2) windows
 * back to back per chain, each exactly what sd_langevin_window (or _phi4) computes, followed by what
 * sd_advance does to that chain (n += adv; stop at n = T) -- without the compaction, which only the
 * launch-per-window loop needs.  Chains do not interact in this algorithm (Sec. 5: each chain runs its
 * own draft-and-verify loop), so nothing forces them to step window by window together: a chain keeps its
 * state on chip from one window to the next, and no chain waits for the longest window of the batch.
 * Between two windows the state passes through fp32 as it does between two calls, so results equal the
 * window + advance loop bit for bit.
 * in : x [B,d], n [B] (start steps), chain_id [B]; the energy's parameters as in the window calls   (dev)
 * out: x_out [B,d] and n_out [B], row b = chain b of the input (x_out may be x, n_out may be n);
 *      counters: dev int64[5] or NULL, accumulated as in sd_advance: {sum adv, chain-windows, rejections,
 *      launches (+1), sum Kt}.
 * sd_langevin_run serves d <= 1024 (SD_ERR_UNSUPPORTED above: use the window loop); ordering of calls on one
 * context as for sd_langevin_window. */
int sd_langevin_run(sd_ctx* ctx, int32_t B, const float* x, const int32_t* n, const int64_t* chain_id,
                    const float* means, const float* logw, float comp_std, int32_t M, float gamma,
                    int32_t max_windows, float* x_out, int32_t* n_out, int64_t* counters, void* stream);
int sd_langevin_run_phi4(sd_ctx* ctx, int32_t B, const float* x, const int32_t* n,
                         const int64_t* chain_id, int32_t L, float beta, float gamma, int32_t max_windows,
                         float* x_out, int32_t* n_out, int64_t* counters, void* stream);

/* Text of the last error on this context (or of the last failed sd_create when ctx is NULL). */
const char* sd_last_error(const sd_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* SD_H */
