/*
 * tsr.h - C ABI of the MI355X (gfx950) TSR-Adam per-matrix optimizer library.
 *
 * The calls follow the paper's statement of the update for one matrix block
 * W (m x n) with orthonormal bases U (m x r), V (n x r) and r x r core moments
 * (Algorithm 1, Sections 3.3-3.6):
 *
 *   refresh   (every K steps)  (U, V) <- randomized SVD of the gradient      tsr_refresh_rsvd
 *   project                    C = U^T G V                                    tsr_project_core
 *   average   (all-reduce stand-in on one GPU)  Cbar = mean_i C_i             tsr_core_average
 *   Adam on the core           m, v, D = mhat / (sqrt(vhat) + eps)            tsr_adam_core
 *   lift + apply               W <- W - lr (scale U D V^T + wd W)             tsr_backproject_apply
 *   all blocks of a model in grouped launches                                 tsr_plan_* / tsr_step_batched /
 *                                                                             tsr_refresh_batched
 *   refresh with N workers (averaged sketches, one GPU)                       tsr_refresh_rsvd_workers
 *   first moment re-expressed in refreshed bases (Appendix B)                 tsr_realign_moment
 *   comparison paths of the ablations (one-sided, exact SVD)                  tsr_project_one_sided,
 *                                                                             tsr_backproject_one_sided,
 *                                                                             tsr_refresh_exact_svd
 *
 * Conventions
 *   - Every matrix is dense row-major.  G and W take an explicit leading dimension
 *     (elements between consecutive rows); U, V, Omega, C, M, Vm, D are contiguous
 *     (leading dimension = number of columns).
 *   - Every data pointer is a DEVICE pointer unless the comment says "host".  The caller
 *     owns every buffer, including the workspace; the library allocates no device memory
 *     and keeps no hidden device state.  Workspaces must be 256-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work on that stream and return; results are ready once the stream has
 *     drained.  Calls on one stream are ordered.
 *   - Arguments are validated on the host before anything is launched; on error nothing
 *     is enqueued and a negative tsr_status is returned.  Non-finite inputs are not
 *     detected: they propagate into the outputs.
 *   - Fast paths need 16-byte aligned G / W base pointers and leading dimensions that
 *     are multiples of 8 elements; anything else is still computed correctly, slower.
 */
#ifndef TSR_H
#define TSR_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum tsr_status {
    TSR_OK = 0,
    TSR_INVALID_ARG = -1,         /* null pointer, misaligned workspace, t < 1 ...          */
    TSR_BAD_SHAPE = -2,           /* m, n, r <= 0, r > min(m, n), r + p > min(m, n), ld < n */
    TSR_BAD_DTYPE = -3,
    TSR_WORKSPACE_TOO_SMALL = -4,
    TSR_HIP_ERROR = -5,           /* a HIP runtime call failed (see tsr_last_hip_error)     */
    TSR_STATIC_SCRATCH_TOO_SMALL = -6   /* tsr_project_core_static: the problem needs more scratch than
                                           TSR_PROJECT_STATIC_SCRATCH_BYTES                          */
} tsr_status;

/* Storage type of the gradient G (everything else is fp32). */
typedef enum tsr_dtype { TSR_F32 = 0, TSR_BF16 = 1 } tsr_dtype;

/* Arithmetic of the dense contractions.  Both accumulate in fp32 on the matrix cores.
 *   TSR_PREC_SPLIT  fp32 operands are split into two bf16 pieces (hi + lo) and the three
 *                   leading cross products are summed: about 2^-17 relative per product,
 *                   for the "fp32 path" (cores / weights within 1e-4 of an fp64 result).
 *   TSR_PREC_BF16   operands that stream from the big matrices (G, V in G V; T, V in
 *                   T V^T) are rounded once to bf16: for bf16 gradients (within 1e-2).
 * The refresh always uses split arithmetic (three pieces where orthogonality depends on it). */
typedef enum tsr_precision { TSR_PREC_SPLIT = 0, TSR_PREC_BF16 = 1 } tsr_precision;

/* One matrix block of a model, for the batched calls.  All pointers are device pointers. */
typedef struct tsr_matrix_desc {
    const void* G;          /* gradients: n_workers consecutive m x n matrices             */
    int g_dtype;            /* tsr_dtype of G                                               */
    int m, n, r;
    long long ldg;          /* leading dimension of each G, elements                        */
    long long g_stride;     /* elements between consecutive workers' G (unused if 1 worker) */
    float* W;               /* m x n weights, updated in place                              */
    long long ldw;
    float* U;               /* m x r basis                                                  */
    float* V;               /* n x r basis                                                  */
    float* M;               /* r x r first moment, in place                                 */
    float* Vm;              /* r x r second moment, in place                                */
    float* C;               /* r x r averaged core (output)                                 */
    float* D;               /* r x r normalized core update (output)                        */
} tsr_matrix_desc;

typedef struct tsr_hyper {
    float lr, wd, beta1, beta2, eps;
    float scale;            /* multiplies U D V^T before lr (1 = Algorithm 1)               */
} tsr_hyper;

const char* tsr_status_string(int status);
/* hipError_t value of the last failing HIP call on this host thread (0 if none). */
int tsr_last_hip_error(void);
/* Number of GPUs HIP reports (0 without a GPU or driver); touches no device. */
int tsr_device_count(void);

/* ---------------------------------------------------------------- project (Section 3.3)
 * C <- alpha * U^T G V  (+ C if accumulate != 0).   Algorithm 1, projection line.
 * G m x n (dtype g, leading dimension ldg), U m x r, V n x r, C r x r.
 * alpha = 1/K with accumulate over K calls forms the K-worker average with no extra pass.
 * Workspace: tsr_project_workspace_bytes(m, n, r) bytes. */
size_t tsr_project_workspace_bytes(int m, int n, int r);
int tsr_project_core(const void* G, int g_dtype, int m, int n, long long ldg,
                     const float* U, const float* V, int r,
                     float alpha, int accumulate, float* C, int precision,
                     void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------- project, nothing allocated
 * tsr_project_core for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and kernels as tsr_project_core, minus the workspace: the scratch (P = G V
 * and the k-split partial cores) lives in a fixed array of TSR_PROJECT_STATIC_SCRATCH_BYTES inside
 * the library's code object, one copy per GPU, held until the process ends.  The call allocates
 * and frees no device memory.  A problem whose tsr_project_workspace_bytes(m, n, r) exceeds that
 * size is refused with TSR_STATIC_SCRATCH_TOO_SMALL before anything is launched (16 MiB covers
 * e.g. 2048 x 768 at r = 256; use tsr_project_core with a workspace beyond that).  The first
 * call on a device looks the array's address up once (make that call outside graph capture).
 * All calls on one GPU share that GPU's array: calls that may overlap in time (different
 * streams, or host threads) race on it and must be serialised by the caller; calls on one
 * stream are safe.  Nothing in the array has to be cleared between calls: every value read was
 * written earlier in the same call. */
#define TSR_PROJECT_STATIC_SCRATCH_BYTES (16u << 20)
int tsr_project_core_static(const void* G, int g_dtype, int m, int n, long long ldg,
                            const float* U, const float* V, int r,
                            float alpha, int accumulate, float* C, int precision, void* stream);

/* ---------------------------------------------------------------- average (all-reduce stand-in)
 * Cbar = (1/K) sum_i Cs[i], Cs = K consecutive r x r cores, summed in worker order.
 * Stands in, on one GPU, for the all-reduce-average of Algorithm 1.  Cbar may alias Cs. */
int tsr_core_average(const float* Cs, int K, int r, float* Cbar, void* stream);

/* ---------------------------------------------------------------- calibration
 * dst[i] = scale * src[i] for `count` floats (count % 4 == 0, 16-byte aligned, dst may equal
 * src): a plain streaming kernel of known traffic (4*count bytes read, 4*count written).  Not
 * part of the method: benchmarks use it to measure the HBM rate the machine actually reaches
 * and to calibrate the memory-traffic counters of the profiler. */
int tsr_stream_scale(float* dst, const float* src, long long count, float scale, void* stream);

/* ---------------------------------------------------------------- Adam on the core (Section 3.4)
 * m <- beta1 m + (1-beta1) C ; v <- beta2 v + (1-beta2) C.C ;
 * D = (m / (1-beta1^t)) / (sqrt(v / (1-beta2^t)) + eps).   t >= 1 is the global step count.
 * C, M, Vm, D hold `count` floats each (count = r*r for one block; any count works, so a
 * caller may pass all cores of a model laid out back to back).  D may alias C. */
int tsr_adam_core(const float* C, float* M, float* Vm, float* D, long long count, int t,
                  float beta1, float beta2, float eps, void* stream);

/* Momentum variant (Algorithm 2): m <- beta m + (1-beta) C ; D = m. */
int tsr_sgd_core(const float* C, float* M, float* D, long long count, float beta, void* stream);

/* ---------------------------------------------------------------- lift + apply (Section 3.4)
 * W <- W - lr * (scale * U D V^T + wd * W), in place.  Last two update lines of Algorithm 1.
 * Workspace: tsr_backproject_workspace_bytes(m, n, r). */
size_t tsr_backproject_workspace_bytes(int m, int n, int r);
int tsr_backproject_apply(float* W, int m, int n, long long ldw,
                          const float* U, const float* V, const float* D, int r,
                          float lr, float wd, float scale, int precision,
                          void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------- refresh (Section 3.5)
 * Randomized-SVD refresh of the bases for one worker (refresh branch of Algorithm 1):
 *   Y = G Omega ; Q = orth(Y) ; q times { Yrow = G^T Q ; Qrow = orth(Yrow) ; Y = G Qrow ;
 *   Q = orth(Y) } ; B = Q^T G ; B = Ut S Vt^T ; U = Q Ut[:, :r] ; V = Vt[:, :r].
 * Omega is n x (r+p), N(0,1), supplied by the caller (the paper shares it by RNG seed).
 * Requires r + p <= min(m, n).  Writes U (m x r), V (n x r) and, if sigma != NULL, the
 * r + p singular values of B in descending order.
 * orth is a Cholesky-based thin QR with fp64 factorization of the Gram matrix, repeated
 * twice for the final Q and for the factor of B^T and applied once to the sketches inside
 * the power iteration (same span, same Q factor of what follows; they only need to stay
 * well conditioned); a Gram matrix that is singular to working precision (a gradient of rank below
 * r + p, e.g. all zeros) gives zero columns in place of the undetermined directions.
 * Workspace: tsr_refresh_workspace_bytes(m, n, r, p). */
size_t tsr_refresh_workspace_bytes(int m, int n, int r, int p);
int tsr_refresh_rsvd(const void* G, int g_dtype, int m, int n, long long ldg,
                     const float* Omega, int r, int p, int q,
                     float* U, float* V, float* sigma,
                     void* ws, size_t ws_bytes, void* stream);

/* Refresh with N workers on one GPU (refresh branch of Algorithm 1, Section 3.5): every worker
 * runs the sketch chain above on its own gradient G_i with the shared Omega and forms
 * B_i = Q_i^T G_i; the sketches are averaged in device memory (the stand-in for the two
 * all-reduces), Bbar = mean B_i, Qbar = mean Q_i; Bbar = Ut S Vt^T; U = Qbar Ut[:, :r],
 * V = Vt[:, :r].  V is orthonormal; U is orthonormal only as far as the workers' Q_i agree.
 * G holds the n_workers gradients g_stride elements apart (g_stride >= (m-1) ldg + n).
 * The communicated sketch payload this stands in for is k (m + n) values per worker, k = r + p.
 * n_workers = 1 is tsr_refresh_rsvd.  Workspace: tsr_refresh_workers_workspace_bytes. */
size_t tsr_refresh_workers_workspace_bytes(int m, int n, int r, int p, int n_workers);
int tsr_refresh_rsvd_workers(const void* G, int g_dtype, int m, int n, long long ldg, long long g_stride,
                             int n_workers, const float* Omega, int r, int p, int q,
                             float* U, float* V, float* sigma,
                             void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------- comparison paths of the ablations
 * The two variants the paper's ablation compares TSR with (Section 4.3; the "One-sided" row of
 * the table of communication objects), on the same kernels, so that their cost and payload can be
 * measured beside the two-sided path.  They are not part of Algorithm 1.
 *
 * One-sided projection: the synchronized object is C1 = U^T G (r x n) instead of the r x r core.
 * It is held TRANSPOSED here, Ct = C1^T = G^T U (n x r, contiguous), which is also the layout
 * tsr_adam_core takes for the element-wise update (count = n * r) and the lift reads:
 *   Ct <- alpha G^T U (+ Ct if accumulate)                               tsr_project_one_sided
 *   W  <- W - lr (scale U Dt^T + wd W), Dt (n x r) = D1^T                tsr_backproject_one_sided
 * r <= m.  Workspace for either call: tsr_one_sided_workspace_bytes(m, n, r). */
size_t tsr_one_sided_workspace_bytes(int m, int n, int r);
int tsr_project_one_sided(const void* G, int g_dtype, int m, int n, long long ldg,
                          const float* U, int r, float alpha, int accumulate, float* Ct, int precision,
                          void* ws, size_t ws_bytes, void* stream);
int tsr_backproject_one_sided(float* W, int m, int n, long long ldw,
                              const float* U, const float* Dt, int r,
                              float lr, float wd, float scale, int precision,
                              void* ws, size_t ws_bytes, void* stream);

/* Exact-SVD refresh (what Section 3.5 replaces by the randomized sketch): U (m x r), V (n x r) =
 * the r leading singular vectors of G itself, sigma (optional) = all min(m, n) singular values,
 * descending.  No sketch and no Omega: the thin QR of the gradient held tall, then the SVD of its
 * triangular factor, on the kernels of tsr_refresh_rsvd's second half.  Requires
 * min(m, n) <= 1024 (the small-SVD kernels' limit), else TSR_BAD_SHAPE.  Singular values below
 * about 1e-3 of the largest lose relative accuracy (the Gram matrix squares the conditioning), and
 * directions at rounding level come out as zero columns; the leading r are what the comparison
 * needs.  Workspace: tsr_refresh_exact_workspace_bytes(m, n, r). */
size_t tsr_refresh_exact_workspace_bytes(int m, int n, int r);
int tsr_refresh_exact_svd(const void* G, int g_dtype, int m, int n, long long ldg, int r,
                          float* U, float* V, float* sigma,
                          void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------- moment re-alignment (Appendix B)
 * First moment re-expressed in refreshed bases, the refresh-alignment assumption of the
 * convergence analysis: the core whose lifted matrix is the old lifted moment projected onto
 * the new subspaces,  M <- (U_new^T U_old) M (V_old^T V_new)   (r x r, in place, fp32).
 * Algorithm 1 as printed does not do this (moments are kept as they are across a refresh);
 * a caller that wants it keeps copies of the old bases, refreshes, then calls this once per
 * block.  The second moment is not touched (the paper defines no re-expression of it).
 * Workspace: tsr_realign_workspace_bytes(m, n, r). */
size_t tsr_realign_workspace_bytes(int m, int n, int r);
int tsr_realign_moment(const float* U_old, const float* V_old, const float* U_new, const float* V_new,
                       int m, int n, int r, float* M, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------- batched all-layers calls
 * A plan holds, in caller-provided device workspace, the grouped-launch tables for a fixed
 * list of blocks, so that every phase of the step (and of the refresh) is a handful of
 * launches over all blocks.  `descs` is a HOST array; it is copied.  n_workers >= 1
 * gradients per block are projected and their cores averaged (the data-parallel stand-in).
 * p is the refresh oversampling (the plan reserves refresh scratch only if with_refresh).
 * tsr_plan_create synchronizes the stream once (table upload); of the other calls only
 * tsr_refresh_batched does (see there).  A plan with refresh of 8 blocks and more also owns
 * up to three HIP streams and four events (host objects, released by tsr_plan_destroy). */
typedef struct tsr_plan tsr_plan;
size_t tsr_plan_workspace_bytes(const tsr_matrix_desc* descs, int count, int n_workers,
                                int precision, int with_refresh, int p);
int tsr_plan_create(const tsr_matrix_desc* descs, int count, int n_workers, int precision,
                    int with_refresh, int p,
                    void* ws, size_t ws_bytes, void* stream, tsr_plan** plan_out);
void tsr_plan_destroy(tsr_plan* plan);

/* With TSR_PREC_BF16 the plan keeps bf16 copies of U, U^T, V, V^T in its workspace and
 * rebuilds them on the first step after creation and after every tsr_refresh_batched.  A
 * caller that writes U or V itself (a restored checkpoint, bases computed elsewhere) must
 * call this before the next step. */
int tsr_plan_bases_changed(tsr_plan* plan);

/* Which kernels the plan's per-step path runs: 1 = the k-contiguous bf16 family with the fused
 * lift (precision TSR_PREC_BF16, every gradient with a 16-byte aligned base, row pitch and worker
 * stride, a row pitch of at least n rounded up to 8 elements, every operand addressable with
 * 31-bit byte offsets), 0 = the
 * general grouped kernels (every other case; same results to the precision's tolerance).
 * A null plan gives -1. */
int tsr_plan_kernel_path(const tsr_plan* plan);

/* One TSR-Adam step (no refresh) for every block of the plan:
 * project all workers -> average -> Adam on the cores -> lift + apply.  t >= 1.
 * Once the plan has run a step since its bases last changed (the first such step also rebuilds the
 * bf16 copies of the bases), a step with stage timing off is kernel launches on `stream` only: no
 * allocation, no copy, no host synchronisation; it may be recorded into a HIP graph (t and *h are
 * then fixed in the recorded launches). */
int tsr_step_batched(tsr_plan* plan, int t, const tsr_hyper* h, void* stream);

/* Refresh (U, V) of every block from worker 0's gradient (randomized SVD, Algorithm 1's
 * refresh step).  Omegas is a HOST array of `count` device pointers (block i: n_i x (r_i + p)).
 * Plans of 8 blocks and more run the refresh as a few groups of blocks (three by default, at
 * most four) side by side: group
 * 0 on `stream`, the others on streams the plan owns (default priority), which start after the
 * work already queued on `stream` and which `stream` waits for before the call returns its
 * place in the queue to the caller; for the caller the call is ordered on `stream` like every
 * other.  The call waits on the host for its small table uploads before it enqueues the kernels.
 * While stage timing is on (tsr_plan_profile_begin) everything runs on `stream` alone. */
int tsr_refresh_batched(tsr_plan* plan, const float* const* Omegas, int q, void* stream);

/* Per-stage timing of the batched calls, for benchmarks.  Between begin and end every stage
 * the plan enqueues is bracketed by HIP events on the work stream.  tsr_plan_profile_end
 * synchronizes the stream and adds up, per stage kind, the elapsed milliseconds (ms[kind])
 * and the number of bracketed stages (launches[kind], may be NULL); both are HOST arrays of
 * TSR_PROF_KINDS entries.  Stage kinds of the step: G V, U^T P (with its split-k reduction),
 * Adam on the cores, U D, the fused T V^T weight update.  Of the refresh: the GEMMs that
 * read G (sketch and power iterations and B), the GEMMs of the thin QR, its Cholesky
 * kernels, the small SVD of the k x k factor (kind name "jacobi"), the two basis-update GEMMs. */
enum {
    TSR_PROF_GV = 0, TSR_PROF_UTP = 1, TSR_PROF_ADAM = 2, TSR_PROF_UD = 3, TSR_PROF_TVT = 4,
    TSR_PROF_SKETCH_GEMM = 5, TSR_PROF_ORTH_GEMM = 6, TSR_PROF_CHOL = 7, TSR_PROF_JACOBI = 8,
    TSR_PROF_BASIS_GEMM = 9, TSR_PROF_KINDS = 10
};
int tsr_plan_profile_begin(tsr_plan* plan);
int tsr_plan_profile_end(tsr_plan* plan, void* stream, float* ms, int* launches);

/* Bytes a worker would put on the wire per step for the plan's blocks: the r x r cores
 * (4 bytes each) and the dense gradients they replace (at bytes_per_dense_element). */
void tsr_plan_payload_bytes(const tsr_plan* plan, int bytes_per_dense_element,
                            long long* core_bytes, long long* dense_bytes);

#ifdef __cplusplus
}
#endif
#endif /* TSR_H */
