/*
 * psgd.h -- C ABI of the MI355X (gfx950) PowerSGD+ compressor library.
 *
 * The library implements the per-step, per-layer low-rank gradient compressor of
 * "From PowerSGD to PowerSGD+" (arXiv 2509.11254) for matrix variables X in R^{m x n}, m >= n
 * (Section 1, problem statement):
 *
 *   error feedback      M = (1/N) sum_i G^(i) + E                       Eq. (7a), averaged over workers
 *   SSP-Comp            P = M Q_{t-1};  P~ = QR(P);  Q_t = M^T P~       Algorithm 1, Eq. (9)
 *   SVD-Comp            P~ = U[:, :r] of SVD(M);     Q_t = M^T P~       Algorithm 1, Definition 3
 *   residual            E_{t+1} = M - P~ Q_t^T                          Algorithm 2 (error update)
 *   reconstruction      Delta_hat = P~ Q_t^T                            Algorithm 1 (return value)
 *
 * The N workers' gradients live on one GPU and are averaged there (this replaces the All-Reduce
 * Mean of Algorithm 1).  The library keeps a single error buffer E per layer, the mean of the
 * per-worker residuals e^(i); by linearity of the compressor (Appendix B, notations) P~, Q,
 * Delta_hat and mean_i e^(i) are the same as in the per-worker form.  Which of SSP-Comp and
 * SVD-Comp runs at step t (mod(t, tau) = 0 selects SVD-Comp, Algorithm 2) is the caller's decision:
 * call psgd_compress or psgd_compress_refresh.
 *
 * General conventions
 *   - Every matrix argument is caller-owned DEVICE memory; the library never frees or keeps it
 *     beyond the call.  Pointer tables (G, E, Q, P arrays of pointers) are HOST arrays of device
 *     pointers.  The library owns only the host-side psgd_ctx and works inside the device
 *     workspace the caller passes (psgd_workspace_bytes bytes, 256-byte aligned, device memory).
 *     The workspace carries state from call to call (pointer tables, per-layer iteration counts and diagnostics,
 *     operand copies of the factors): between calls with the same context the caller leaves its contents alone.  A
 *     context may be used with another workspace at any time (everything is uploaded again); a workspace that was
 *     freed, or written by someone else, must not come back under the same address without psgd_workspace_reset.
 *   - Storage: row-major, `rows x cols` with leading dimension `ld` (elements).  The logical
 *     matrix has m = max(rows, cols), n = min(rows, cols); when rows < cols the stored buffer is
 *     the transpose of the logical matrix and is used as is (no physical transpose).
 *     P~ is m x r and Q is n x r, both fp32, row-major, contiguous (leading dimension r).
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream) and
 *     the call returns without waiting for it.  No result is read back to the host; the one exception is a
 *     4-byte bookkeeping copy into pinned memory that psgd_compress_refresh enqueues behind its work (how many
 *     subspace iterations the next refresh can need at most), which a later call looks at only if it has arrived.
 *   - Return value: PSGD_OK or a negative PSGD_E_* code.  On an argument error nothing is
 *     enqueued.  No exceptions, no aborts.
 *   - Calls that share a workspace must be stream-ordered; two calls running at the same time on
 *     one workspace race.
 *   - HIP graphs: psgd_compress, psgd_compress_project / _finish, psgd_compress_refresh, psgd_flush_residual and the
 *     psgd_decompress* calls may be recorded by a capturing stream once the same call has been made eagerly with
 *     the same workspace and the same pointer tables (their contents, not the host arrays): the library then has
 *     nothing to upload and the recorded work is kernel launches only (no copy and no memset nodes).  A call that
 *     would have to upload returns PSGD_E_CAPTURE and records nothing; the next eager call uploads everything.  A
 *     captured psgd_compress_refresh launches the whole iteration budget and skips its bookkeeping copy; per-kernel
 *     profiling records nothing under capture.  psgd_refresh and psgd_status cannot be captured.  What a recorded call
 *     does is decided when it is recorded (which operand copies are in place, whether a residual is owed): replay it in
 *     the sequence it was recorded in, and make no eager call on the workspace between replays that changes that state.
 */
#ifndef PSGD_H_
#define PSGD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct psgd_ctx psgd_ctx;

enum { PSGD_F32 = 0, PSGD_BF16 = 1 };

enum {
    PSGD_OK = 0,
    PSGD_E_INVALID_ARG = -1, /* null pointer, bad enum, bad count                           */
    PSGD_E_SHAPE = -2,       /* rows/cols < 1, r < 1, r > min(rows, cols), r + oversampling too large */
    PSGD_E_ALIGN = -3,       /* ld < cols, ld not a multiple of 8, pointer not 16-byte aligned */
    PSGD_E_HIP = -4,         /* a HIP runtime call failed (psgd_last_hip_error gives its code) */
    PSGD_E_NOMEM = -5,       /* host allocation failed                                      */
    PSGD_E_CAPTURE = -6,     /* the stream is capturing and the call would have to upload pointer tables */
    PSGD_E_TOO_LARGE = -7    /* psgd_compress_static: the context needs more workspace than the built-in buffer has */
};

/* One matrix variable.  G^(i) and E of this layer all share rows, cols and ld. */
typedef struct {
    int64_t rows;       /* stored rows                                                       */
    int64_t cols;       /* stored columns                                                    */
    int64_t ld;         /* leading dimension in elements, >= cols, multiple of 8; 0 means round_up(cols, 8) == cols required */
    int32_t r;          /* compression rank, 1 <= r <= min(rows, cols)                       */
    int32_t grad_dtype; /* PSGD_F32 or PSGD_BF16: element type of the G^(i) buffers          */
} psgd_layer_desc;

typedef struct {
    int32_t refresh_iters;      /* maximum number of subspace iterations of the SVD refresh (at most 255); 0 = default
                                   (16).  A layer's first two refreshes on a workspace run all of them (the second
                                   is the first to meet the state error feedback builds up).  Later ones run the
                                   number that the convergence factor rho = (theta_b/theta_r)^2 seen at its
                                   last refresh needs for 1e-5, plus one, if that is within the maximum
                                   (rho <= 0.46 for 16); if it is not -- no gap after sigma_r to converge
                                   across in the budget -- they run what keeps the error of the step
                                   within 1e-5 ||M||^2 of the optimum of Eq. (6) by the same Ritz values, at
                                   least 2, at most the maximum                                         */
    int32_t refresh_oversample; /* extra block columns beyond r; negative = default max(8, r/4); the
                                   block width r + oversample is rounded up to a multiple of 8 and
                                   capped at n                                                       */
    int32_t refresh_warm_start; /* 1: psgd_compress_refresh starts from span(Q_{t-1}) plus random
                                   columns; 0: random start.  Default 1.                             */
    uint32_t seed;              /* seed of the counter-based generator for the random start      */
    float rank_tol;             /* a column of P whose part orthogonal to the earlier columns is
                                   at most rank_tol times its norm gives a zero column of P~;
                                   0 = default (1e-5)                                                */
    int32_t precision;          /* bf16 planes per fp32 operand of the matrix-core products: 2 = three
                                   products per term (16 mantissa bits), 3 = six products (24 bits,
                                   fp32-faithful); 0 = default: 3 if any layer has fp32 gradients,
                                   else 2                                                            */
    int32_t m_policy;           /* where M = mean G + E lives between the passes of an SSP step: 1 = stored
                                   over E by the first pass, 2 = formed again from G and E by every pass
                                   (E is only written by the residual; fewer bytes never, equal bytes for
                                   one bf16 worker, first pass read-only), 0 = default = 1                  */
    int32_t power_iters;        /* K of the power iteration inside psgd_compress (Eq. (8)): P~_k = QR(M Q_{k-1}),
                                   Q_k = M^T P~_k for k = 0..K-1, then the residual with (P~_{K-1}, Q_{K-1}).
                                   0 = default = 1, the single-step compressor of Algorithm 1; each further
                                   step costs two more passes over M                                      */
    int32_t lazy_residual;      /* 1: deferred residual.  psgd_compress does not run the pass E <- M - P~ Q^T for the
                                   layers stored with rows >= cols (for every layer if no rank exceeds 32); it
                                   leaves M_t in their E buffers, puts the
                                   operand copies of P~_t and Q_t aside in the workspace, and the forming pass of
                                   the next psgd_compress subtracts their product on the way (same arithmetic:
                                   E_{t+1} is rounded to fp32 before it enters M_{t+1}).  P~, Q and every later
                                   result are those of the immediate form; the E buffers hold E_{t+1} only after
                                   psgd_flush_residual (psgd_compress_refresh settles it by itself).  Saves the
                                   8 bytes per element of the residual pass.  Not with m_policy = 2; r <= 128.
                                   0 = default: immediate residual                                        */
    int32_t q_resident;         /* 1: the caller promises not to write the Q buffers between one compress-type call
                                   on a workspace and the next psgd_compress on it (a single-GPU loop; not a
                                   data-parallel one, which averages Q).  psgd_compress then takes Q_{t-1} from
                                   the operand copies the previous call left in the workspace instead of packing
                                   the Q buffers again (one launch less); the first call, and any call after
                                   one that re-packed the copies, packs as usual.  With lazy_residual = 1 the
                                   forming pass then also takes the Q of the owed residual from those copies
                                   instead of reading the ones put aside (same numbers; the sum over the rank
                                   runs in another order, so results agree with the default to fp32 rounding
                                   of that sum, not bit for bit).  0 = default: always pack                 */
} psgd_options;

/* Per-layer diagnostics written by the last call that touched the layer (read with psgd_status). */
typedef struct {
    int32_t rank_deficient; /* number of columns of P~ zeroed by the rank test                  */
    int32_t refresh_iters_next; /* iterations the layer's next refresh needs to converge, from the Ritz
                                   values of the last one (0: not known yet; above the maximum: it will
                                   run refresh_iters_no_gap of them, see refresh_iters)                 */
    float sigma_max;        /* refresh only: largest and r-th Ritz value (singular value estimates) */
    float sigma_r;
    int32_t refresh_iters_no_gap; /* iterations the next refresh runs when the count above is beyond the
                                   maximum: what keeps its error within 1e-5 ||M||^2 of the optimum of
                                   Eq. (6), at least 2 (the maximum caps it)                            */
} psgd_layer_status;

/* psgd_init -- plan the batched launches for a fixed set of layers (Algorithm 2, "Require"/"Initialize":
 * rank r per layer, number of workers N).  Host only; allocates the context with malloc.
 * Errors: INVALID_ARG (null out/layers, n_layers < 1, n_workers < 1, bad dtype), SHAPE, ALIGN, NOMEM. */
int psgd_init(psgd_ctx **out, int n_layers, const psgd_layer_desc *layers, int n_workers,
              const psgd_options *opt /* nullable: defaults */);

/* Bytes of device workspace every compute call needs (partials, packed operands, small factors). */
size_t psgd_workspace_bytes(const psgd_ctx *ctx);

/* Forget what the context knows about the contents of any workspace: the next call uploads its tables again, clears the
 * per-layer state (the next refresh of every layer runs its full iteration budget) and packs its operands.  For a
 * caller that recycles workspace memory.  Host only.  Not while a deferred residual is owed (flush first): INVALID_ARG. */
int psgd_workspace_reset(psgd_ctx *ctx);

/* psgd_compress -- one SSP-Comp step for every layer (Algorithm 1 SSP-Comp + Eq. (7a) + residual):
 *   M = mean_i G[l*N + i] + E[l];  P = M Q[l];  P~ = QR(P) (R_ii > 0);  Q[l] <- M^T P~;
 *   E[l] <- M - P~ Q[l]^T;  P[l] <- P~.
 * G: n_layers*n_workers read-only device pointers (layer-major), element type grad_dtype.
 * E: n_layers fp32 buffers rows x cols (ld), updated in place.  Q: n x r fp32, in Q_{t-1}, out Q_t.
 * P: m x r fp32, out.  Errors: INVALID_ARG (null table or entry), ALIGN (pointer alignment), HIP. */
int psgd_compress(psgd_ctx *ctx, void *workspace, void *stream, const void *const *G,
                  float *const *E, float *const *Q, float *const *P);

/* psgd_compress_static -- psgd_compress for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same step with the same kernels, but the
 * workspace is a buffer built into the library, a static device array of PSGD_STATIC_WORKSPACE_BYTES that every GPU
 * the library runs on holds from the first such call on it until the process ends.  The call allocates nothing
 * (no hipMalloc, hipHostMalloc or hipFree; tables travel as kernel arguments); G, E, Q, P are the caller's as in
 * psgd_compress.  All contexts and all calls on one GPU share that one buffer: calls that overlap on one GPU race, and
 * the buffer keeps what the last call left, so a context that finds another context's contents there uploads its
 * tables again and starts from cleared per-layer state (as after psgd_workspace_reset).  Mixing it with the
 * workspace-taking calls on the same context is allowed; the buffer then counts as one more workspace.
 * Errors: as psgd_compress; TOO_LARGE if psgd_workspace_bytes(ctx) exceeds the buffer (nothing is enqueued);
 * INVALID_ARG if a deferred residual of this context is owed in another workspace, or was owed in the buffer and
 * another context has used the buffer since; HIP if the buffer's address cannot be obtained. */
#define PSGD_STATIC_WORKSPACE_BYTES (64u * 1024u * 1024u)
int psgd_compress_static(psgd_ctx *ctx, void *stream, const void *const *G, float *const *E, float *const *Q,
                         float *const *P);

/* psgd_compress_project / psgd_compress_finish -- psgd_compress in the two halves between which a data-parallel job
 * exchanges P (Algorithm 1, SSP-Comp: "P = mean of P^(i)" between the projection and the QR; Algorithm 2 keeps one
 * error buffer e^(i) per node).  Each worker owns a context with n_workers = 1, its gradient and its e^(i):
 *   project: M^(i) = G^(i) + e^(i) is stored over E;  P[l] <- M^(i) Q[l]  (m x r, not orthonormalised).
 *   -- the caller averages P over the workers (an all-reduce) and hands every worker the mean --
 *   finish:  P[l] <- P~ = QR(P[l]);  Q[l] <- M^(i)T P~;  E[l] <- e^(i)_{t+1} = M^(i) - P~ Q[l]^T.
 *   -- the caller averages Q over the workers: Q_t --
 * With one worker, project followed by finish is psgd_compress.  Same buffers, layouts and errors as psgd_compress;
 * INVALID_ARG with lazy_residual, m_policy = 2 or power_iters > 1 (the halves assume M stored over E once). */
int psgd_compress_project(psgd_ctx *ctx, void *workspace, void *stream, const void *const *G,
                          float *const *E, float *const *Q, float *const *P);
int psgd_compress_finish(psgd_ctx *ctx, void *workspace, void *stream, float *const *E, float *const *Q,
                         float *const *P);

/* psgd_flush_residual -- with lazy_residual = 1: run the residual that the last psgd_compress left owed,
 * E[l] <- M_t - P~_t Q_t^T from the operand copies it put aside (Algorithm 2, error update), so that the E
 * buffers hold E_{t+1}.  Needed before the caller reads, replaces or checkpoints E, or drops the workspace.
 * A no-op when nothing is owed (and always with lazy_residual = 0).  E: the table given to psgd_compress.
 * Errors: INVALID_ARG (null, or a workspace other than the one the owed operands live in), ALIGN, HIP. */
int psgd_flush_residual(psgd_ctx *ctx, void *workspace, void *stream, float *const *E);

/* psgd_compress_refresh -- one SVD-Comp step for every layer (Algorithm 1 SVD-Comp + Eq. (7a) +
 * residual): as psgd_compress, but P~ spans the top-r left singular subspace of M (Definition 3)
 * and Q = M^T P~.  P~'s columns are the Ritz vectors in order of decreasing singular value.
 * Q on entry is only used as a starting guess (and not at all with refresh_warm_start = 0). */
int psgd_compress_refresh(psgd_ctx *ctx, void *workspace, void *stream, const void *const *G,
                          float *const *E, float *const *Q, float *const *P);

/* psgd_refresh -- the optimal rank-r compressor of Definition 3 on a given matrix, nothing else:
 * M (rows x cols, ld of layer `layer`, fp32, read-only) -> P (m x r), Q = M^T P~ (n x r),
 * sigma (r fp32 singular value estimates, device, nullable). */
int psgd_refresh(psgd_ctx *ctx, void *workspace, void *stream, int layer, const float *M, float *P,
                 float *Q, float *sigma);

/* psgd_decompress -- Delta_hat[l] = P~[l] Q[l]^T in the layer's storage orientation (Algorithm 1,
 * return value).  out[l]: rows x cols (ld), element type out_dtype (PSGD_F32 or PSGD_BF16).
 * P and Q both NULL: the factors of the last psgd_compress / psgd_compress_refresh / psgd_compress_finish call on
 * this workspace, taken from the operand copies that call left there (nothing is read from the P and Q buffers and
 * nothing is re-packed: one launch less); INVALID_ARG if no such call was the last to write them (any other call
 * with explicit P and Q, or psgd_refresh, comes in between).  The same holds for psgd_decompress_msgd and
 * psgd_decompress_adam.  After psgd_compress_finish the copies hold the worker's own Q, not the averaged one. */
int psgd_decompress(psgd_ctx *ctx, void *workspace, void *stream, const float *const *P,
                    const float *const *Q, void *const *out, int out_dtype);

/* psgd_decompress_msgd -- the step after the compressor, fused with the reconstruction (Eq. (7c), last lines
 * of Algorithm 2): m[l] <- mu m[l] + P~[l] Q[l]^T;  X[l] <- X[l] - eta m[l].  Delta_hat is never written.
 * mom, X: n_layers fp32 buffers rows x cols (ld) in the layer's storage orientation, updated in place.
 * Errors: INVALID_ARG (null table or entry, mu outside [0, 1), eta not a number), ALIGN, HIP. */
int psgd_decompress_msgd(psgd_ctx *ctx, void *workspace, void *stream, const float *const *P,
                         const float *const *Q, float *const *mom, float *const *X, float mu, float eta);

/* psgd_decompress_adam -- the same step with Adam as the base optimizer (the paper's pre-training and fine-tuning
 * runs, Section 5 and Appendix C, use Adam / AdamW on the compressed update; Claim 1 names it next to MSGD).  The
 * update is the published one with bias correction and decoupled weight decay, on D = P~[l] Q[l]^T:
 *   m1 <- beta1 m1 + (1 - beta1) D;   m2 <- beta2 m2 + (1 - beta2) D.D   (elementwise)
 *   X  <- X - eta ( (m1 / (1 - beta1^step)) / (sqrt(m2 / (1 - beta2^step)) + eps) + weight_decay X )
 * step counts from 1 (the caller increments it); weight_decay = 0 is plain Adam.  Delta_hat is never written.
 * m1, m2, X: n_layers fp32 buffers rows x cols (ld) in the layer's storage orientation, updated in place.
 * Errors: INVALID_ARG (null table or entry, step < 1, a beta outside [0, 1), eps < 0, a NaN), ALIGN, HIP. */
int psgd_decompress_adam(psgd_ctx *ctx, void *workspace, void *stream, const float *const *P,
                         const float *const *Q, float *const *m1, float *const *m2, float *const *X, int step,
                         float eta, float beta1, float beta2, float eps, float weight_decay);

/* Copy the per-layer diagnostics of the last call to the host.  Synchronises `stream`. */
int psgd_status(psgd_ctx *ctx, void *workspace, void *stream, int layer, psgd_layer_status *out);

/* Algorithmic HBM bytes of one psgd_compress over all layers: sum over layers of
 * rows*cols*min(N*sizeof(G) + 16, 2*N*sizeof(G) + 12) -- M stored between the two passes, or
 * formed twice -- plus 16*(rows + cols)*r for the thin matrices. */
double psgd_algorithmic_bytes(const psgd_ctx *ctx);

/* Algorithmic HBM bytes of one launch of a streaming kernel of psgd_compress over all layers, under the
 * context's m_policy (tag = PSGD_PROF_SWEEP1 / _SWEEP2 / _RESIDUAL): matrix bytes read and written + the
 * packed thin operands.  What a measured kernel duration is divided into for the roofline. */
double psgd_kernel_bytes(const psgd_ctx *ctx, int tag);

/* Plain device copy kernel (dst <- src, n_bytes multiple of 16) used to calibrate profiler counters
 * and to measure the attainable copy bandwidth with the same launch machinery. */
int psgd_copy_bytes(void *stream, void *dst, const void *src, size_t n_bytes);

/* Timing of the three streaming kernels of psgd_compress with HIP event pairs recorded on the
 * caller's stream around each launch: tag 0 = first pass (M formed, P = M Q), tag 1 = second pass
 * (Q = M^T P~), tag 2 = residual.  psgd_profile_enable allocates max_records event pairs (0 turns
 * timing off and frees them); once they are used up further launches are not timed.
 * psgd_profile_read waits for the recorded events, adds the elapsed milliseconds and the number of
 * records per tag into total_ms[0..n_tags) / count[0..n_tags) (host arrays), and resets the pool. */
enum { PSGD_PROF_SWEEP1 = 0, PSGD_PROF_SWEEP2 = 1, PSGD_PROF_RESIDUAL = 2, PSGD_PROF_TAGS = 3 };
int psgd_profile_enable(psgd_ctx *ctx, int max_records);
/* Which tags are timed (bit t = tag t; default all).  Every timed launch costs two event records on the stream,
 * about 6 microseconds of idle GPU each on this machine: time only what is needed inside a measured region. */
int psgd_profile_select(psgd_ctx *ctx, int tag_mask);
int psgd_profile_read(psgd_ctx *ctx, double *total_ms, int *count, int n_tags);

int psgd_last_hip_error(const psgd_ctx *ctx);
const char *psgd_strerror(int code);
void psgd_destroy(psgd_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* PSGD_H_ */
