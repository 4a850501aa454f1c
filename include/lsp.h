/*
 * lsp.h -- C ABI of the MI355X (gfx950) library for the GPU hot path of LSP-Offload
 * (arXiv 2406.10181): compressing a weight gradient through two learned sparse projectors
 * and expanding the CPU-computed subspace update back onto the weight; beside the per-step
 * calls, the two GPU-side pieces of the projector refresh (MaybeUpdate, Alg. 1): the estimation
 * bias of Def. 2 and the re-projection of the optimiser state.
 *
 * Letters.  G and W are m x n, row-major, leading dimension n.  r is the subspace size
 * (number of columns of P and Q; S is r x r).  d is the number of stored entries per
 * projector row.  The paper names these the other way round: its "(d,r)-sparse projector"
 * (Def. 1) has subspace size d and r nonzeros per row.
 *
 * Projectors.  P (m x r) and Q (n x r) are (d,r)-sparse in the sense of Def. 1 and are passed
 * in ELL layout: idx[row][k] (int32, a column in [0, r)) and val[row][k] (fp32), k < d,
 * row-major.  The dense meaning is  Phat[i][a] = sum of val[i][k] over k with idx[i][k] == a:
 * duplicate columns within a row add up, and an entry with val == 0 is padding (its index
 * must still be in range).  Indices are NOT range-checked by the compute calls; an index
 * outside [0, r) is undefined behaviour.  lsp_validate_projector() checks them on request.
 *
 * Memory.  Every pointer named "device" is device memory of the current HIP device, owned by
 * the caller for the whole call and until the enqueued work has finished.  The library never
 * allocates, frees or copies device memory in the compute calls, never synchronises the
 * stream, and keeps no state between calls.  Buffers must not alias one another.
 * All base pointers must be aligned to 16 bytes.
 *
 * Execution.  Compute calls only enqueue kernels on `stream` (a hipStream_t passed as
 * void*; NULL = the default stream) and return; work on one stream runs in call order
 * (Alg. 3 issues these per layer, in backward order, asynchronously).
 *
 * Errors.  Every call returns LSP_OK (0) or a negative lsp_status.  All argument checks are
 * made before the first HIP call: on LSP_ERR_NULL / SHAPE / DTYPE / WORKSPACE / ALIGN nothing has
 * been enqueued and no output has been touched.  LSP_ERR_LAUNCH means the HIP runtime refused a
 * launch (or, in the set-up calls, a copy); a call that consists of several kernels, or a grouped
 * call that serves its problems one by one, may then have enqueued part of its work already, and
 * its outputs are undefined.
 */
#ifndef LSP_H
#define LSP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LSP_F32  = 0,   /* IEEE binary32 */
    LSP_F16  = 1,   /* IEEE binary16 */
    LSP_BF16 = 2    /* bfloat16 */
} lsp_dtype;

typedef enum {
    LSP_OK            =  0,
    LSP_ERR_NULL      = -1,  /* a required pointer is NULL */
    LSP_ERR_SHAPE     = -2,  /* m, n, r or d not positive, d > r, size overflow, r or d above the supported maximum */
    LSP_ERR_DTYPE     = -3,  /* dtype is not one of lsp_dtype */
    LSP_ERR_WORKSPACE = -4,  /* workspace / plan buffer missing, misaligned or too small */
    LSP_ERR_LAUNCH    = -5,  /* the HIP runtime refused a launch or a copy (see lsp_last_hip_error) */
    LSP_ERR_INDEX     = -6,  /* lsp_validate_projector found an index outside [0, r) */
    LSP_ERR_ALIGN     = -7,  /* a base pointer is not 16-byte aligned */
    LSP_ERR_SKEW      = -8,  /* lsp_plan_build: the columns of Q are used too unevenly for a plan; use lsp_compress */
    LSP_ERR_TOO_LARGE = -9   /* lsp_compress_planned_static: the problem needs more than LSP_STATIC_SCRATCH_BYTES of scratch */
} lsp_status;

#define LSP_MAX_R 2048       /* largest supported subspace size (the paper's largest setting) */
#define LSP_MAX_D 64         /* largest supported number of entries per projector row */
#define LSP_MAX_GROUP 16     /* most problems in one grouped call */
#define LSP_STATIC_SCRATCH_BYTES (24u << 20)   /* scratch held inside the library image, per GPU (lsp_compress_planned_static) */

/* ------------------------------------------------------------------------------------------
 * Compress:  S := P^T G Q.
 * The step "grad <- SendToCPU(P^T grad_W Q)" of Alg. 1 and the step that forms the projected
 * gradient of layer l in Alg. 3.  S is OVERWRITTEN (not accumulated); gradient accumulation
 * happens on G before the call.  G is widened exactly to fp32; all sums are fp32.
 *
 *   G          device, m*n elements of `dtype`, row-major
 *   P_idx/val  device, [m][d]
 *   Q_idx/val  device, [n][d]
 *   S          device, r*r fp32, row-major, written
 *   workspace  device scratch of at least lsp_compress_workspace_bytes(m,n,r,d) bytes,
 *              16-byte aligned; contents are clobbered; may be reused by later calls on
 *              the same stream
 *
 * This entry takes raw ELL projectors and needs no preparation: it builds the plan on the
 * device into the workspace and runs the planned kernels on it, all asynchronously; only
 * projectors too skewed for a plan are served by a scatter form (LDS and global fp32 atomics, far
 * slower, not bit-reproducible), chosen on the device.  An index outside [0, r) makes S NaN.
 * When the projectors stay fixed over many steps -- the paper refreshes them only every CheckFreq
 * steps in MaybeUpdate, Alg. 1 -- build a plan once with lsp_plan_build and call
 * lsp_compress_planned, which saves the build in every step.
 */
int lsp_compress(const void* G,
                 const int32_t* P_idx, const float* P_val,
                 const int32_t* Q_idx, const float* Q_val,
                 int64_t m, int64_t n, int32_t r, int32_t d,
                 float* S, lsp_dtype dtype,
                 void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of device scratch lsp_compress needs (0 on invalid shapes). */
size_t lsp_compress_workspace_bytes(int64_t m, int64_t n, int32_t r, int32_t d);

/* One size that serves every call of this header on an (m, n, r, d) problem: the largest of the
 * per-call workspace queries below (0 on invalid shapes or dtype).  The library holds no
 * workspace of its own: scratch is always an argument of the call that uses it. */
size_t lsp_workspace_bytes(int64_t m, int64_t n, int32_t r, int32_t d, lsp_dtype dtype);

/* ------------------------------------------------------------------------------------------
 * Projector plan: a device-resident, column-sorted copy of P and Q for one (m, n, r, d)
 * problem, valid until the projector arrays change (every CheckFreq steps at most, Alg. 1).
 * It lives entirely in a caller-owned device buffer of lsp_plan_bytes() bytes; there is no
 * host handle.  Building a plan only sorts and packs the projector entries (no arithmetic on
 * G, W or S) and happens on the device, where the projectors live: a radix sort of one key per
 * stored entry and a handful of small kernels (tens of microseconds; nothing is copied to the host).
 *
 * lsp_plan_build_async only enqueues that work on `stream`; it needs device scratch of
 * lsp_plan_build_workspace_bytes() and reports what only the data can show -- an index outside
 * [0, r) (LSP_ERR_INDEX) or columns too skewed for a plan (LSP_ERR_SKEW) -- in `status` (device,
 * one int32, may be NULL), written when the build has run; a failed build also leaves the buffer
 * marked as "no plan", so that compress calls with it fill S with NaN.
 * lsp_plan_build is the synchronous form: it allocates and frees the scratch itself (a set-up call,
 * NOT part of the per-step path), waits for `stream` and returns the build's status.
 * lsp_plan_build_host makes the same bytes with every pointer in HOST memory and no HIP call; the
 * result can be copied to the device by the caller.  lsp_plan_refresh_values (below) drops new
 * values into a plan whose positions are unchanged.
 */
size_t lsp_plan_bytes(int64_t m, int64_t n, int32_t r, int32_t d);

int lsp_plan_build(const int32_t* P_idx, const float* P_val,
                   const int32_t* Q_idx, const float* Q_val,
                   int64_t m, int64_t n, int32_t r, int32_t d,
                   void* plan, size_t plan_bytes, void* stream);

size_t lsp_plan_build_workspace_bytes(int64_t m, int64_t n, int32_t r, int32_t d);
int lsp_plan_build_async(const int32_t* P_idx, const float* P_val,
                         const int32_t* Q_idx, const float* Q_val,
                         int64_t m, int64_t n, int32_t r, int32_t d,
                         void* plan, size_t plan_bytes,
                         void* workspace, size_t workspace_bytes,
                         int32_t* status, void* stream);

int lsp_plan_build_host(const int32_t* P_idx, const float* P_val,
                        const int32_t* Q_idx, const float* Q_val,
                        int64_t m, int64_t n, int32_t r, int32_t d,
                        void* plan_host, size_t plan_bytes);

/* Same sums as lsp_compress, with the projectors given as a plan; gather form, no global
 * atomics unless a row of P^T has more than 256 entries (heavily skewed projectors), and
 * bit-reproducible from run to run whenever no row of P^T had to be cut for that reason
 * (columns of Q that are shared among several lanes are summed in a fixed order).
 * workspace: at least lsp_compress_planned_workspace_bytes(m,n,r,d) bytes.
 * The plan lives in device memory, so the host cannot check it: the kernels compare the (m, n, r,
 * d) recorded in the plan with those of the call, and when they differ (a plan built for another
 * problem, or a buffer that holds no plan) they follow none of its offsets, touch nothing but S
 * and fill S with NaN -- the call still returns LSP_OK, the mistake shows in S. */
int lsp_compress_planned(const void* G, const void* plan,
                         int64_t m, int64_t n, int32_t r, int32_t d,
                         float* S, lsp_dtype dtype,
                         void* workspace, size_t workspace_bytes, void* stream);

size_t lsp_compress_planned_workspace_bytes(int64_t m, int64_t n, int32_t r, int32_t d);

/* lsp_compress_planned for callers that cannot allocate device memory or hand in scratch: code
 * running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results (bit for bit) and errors as lsp_compress_planned, without the workspace: the
 * m x r fp32 intermediate lives in an array of LSP_STATIC_SCRATCH_BYTES (24 MiB) that is part of
 * the library image; every GPU the library runs on holds one copy of it until the process ends.
 * The call makes no allocation of any kind.  A problem whose intermediate does not fit (m * r * 4
 * bytes, rounded up to 256, above the limit; 11008 x 512 fits) is refused with LSP_ERR_TOO_LARGE
 * and nothing is enqueued.
 * All calls on one GPU share the array: calls on one stream are ordered and safe, calls whose
 * kernels can overlap in time (different streams, different host threads' streams) race on it and
 * give undefined S.  The array keeps the previous call's contents; nothing in it needs clearing. */
int lsp_compress_planned_static(const void* G, const void* plan,
                                int64_t m, int64_t n, int32_t r, int32_t d,
                                float* S, lsp_dtype dtype, void* stream);
size_t lsp_static_scratch_bytes(void);   /* LSP_STATIC_SCRATCH_BYTES */

/* ------------------------------------------------------------------------------------------
 * Decompress and apply:  W := rn( W - P S Q^T ), in place.
 * The step "W <- W - eta_t P Delta_W Q^T" of Alg. 1 and the last step of the layer loop of
 * Alg. 3.  The learning rate is already folded into S by the CPU optimiser (P (eta S) Q^T =
 * eta P S Q^T), so there is no scale argument.  Each W element is widened exactly to fp32,
 * the update is accumulated in fp32, and the result is rounded once (nearest, ties to even)
 * to `dtype`.  Needs no workspace and no plan (the ELL rows are read as they are).
 *
 *   W          device, m*n elements of `dtype`, row-major, read and written
 *   S          device, r*r fp32, row-major, read
 */
int lsp_decompress_apply(void* W, const float* S,
                         const int32_t* P_idx, const float* P_val,
                         const int32_t* Q_idx, const float* Q_val,
                         int64_t m, int64_t n, int32_t r, int32_t d,
                         lsp_dtype dtype, void* stream);

/* ------------------------------------------------------------------------------------------
 * Grouped calls: several independent matrices in one call.
 * Alg. 3 walks the model layer by layer, and the weight matrices of one layer (their gradients
 * are all there when the layer's backward pass ends) are independent problems with the same
 * subspace size: a grouped call serves them with one launch per kernel, so that workgroups of
 * different matrices fill the GPU together.  Results are those of the single calls, matrix by
 * matrix, bit for bit.
 *
 *   items      HOST array of `count` descriptors (1 <= count <= LSP_MAX_GROUP); read during the
 *              call only; every pointer inside is a device pointer with the meaning, layout and
 *              alignment of the same-named argument of the single call
 *   r, d, dtype  shared by all problems of the group; m and n are per problem
 * Problems of a group run concurrently: every item needs its own S and its own workspace
 * (LSP_ERR_WORKSPACE otherwise), and a W may appear only once (LSP_ERR_SHAPE).  Errors are
 * those of the single calls; on any error nothing is enqueued.  When the problems need different
 * kernel variants (e.g. some n divisible by 8 and some not) the call enqueues them one by one.
 */
typedef struct {
    const void* G;            /* device, m*n elements of `dtype` */
    const void* plan;         /* device, from lsp_plan_build for this problem's projectors */
    float*      S;            /* device, r*r fp32, written */
    void*       workspace;    /* device, >= lsp_compress_planned_workspace_bytes(m,n,r,d) */
    size_t      workspace_bytes;
    int64_t     m, n;
} lsp_compress_item;

typedef struct {
    void*          W;         /* device, m*n elements of `dtype`, read and written */
    const float*   S;         /* device, r*r fp32 */
    const int32_t* P_idx;     /* device, [m][d] */
    const float*   P_val;
    const int32_t* Q_idx;     /* device, [n][d] */
    const float*   Q_val;
    int64_t        m, n;
} lsp_apply_item;

int lsp_compress_planned_grouped(const lsp_compress_item* items, int32_t count,
                                 int32_t r, int32_t d, lsp_dtype dtype, void* stream);

int lsp_decompress_apply_grouped(const lsp_apply_item* items, int32_t count,
                                 int32_t r, int32_t d, lsp_dtype dtype, void* stream);

/* Optional preparation for the expand side (lsp_decompress_apply*, lsp_estimation_bias): a copy
 * of an ELL projector in which the d entries of every row are put in an order that makes the
 * kernels' LDS gathers collide less.  The projector is the same matrix (Def. 1 fixes which entries
 * a row has, not their order; they are summed), so the copy can be passed wherever Q is expected;
 * results differ only by the order of fp32 additions.  Meant for Q (the kernels gather by the
 * rows of Q); harmless for P.  Like the plan it is made once per change of projectors.
 *   idx, val           HOST, [rows][d]
 *   idx_out, val_out   HOST, [rows][d], distinct from the inputs
 * Returns LSP_OK, LSP_ERR_NULL, LSP_ERR_SHAPE or LSP_ERR_INDEX (an index outside [0, r)). */
int lsp_projector_reorder_host(const int32_t* idx, const float* val, int64_t rows, int32_t d, int32_t r,
                               int32_t* idx_out, float* val_out);
/* The same for DEVICE arrays: a set-up call like lsp_plan_build -- it waits for `stream`, copies the
 * arrays to the host (allocating host memory), reorders there and copies the result into the
 * device arrays idx_out / val_out; synchronous.  Adds LSP_ERR_LAUNCH to the errors above. */
int lsp_projector_reorder(const int32_t* idx, const float* val, int64_t rows, int32_t d, int32_t r,
                          int32_t* idx_out, float* val_out, void* stream);

/* ------------------------------------------------------------------------------------------
 * Dense-projector ablation of compress:  S := P^T G Q with DENSE projectors, on the matrix cores.
 * Def. 1 makes the projectors (d, r)-sparse, and the calls above never multiply by the zeros.  This call
 * is the yardstick for that choice: the same contraction with dense m x r and n x r projectors (what a
 * subspace method without the sparsity would run), as two matrix-core products in the storage type with
 * fp32 accumulation, T = G Q rounded to the storage type in between.  Its cost does not depend on d.
 *
 *   G          device, m*n elements of `dtype` (LSP_F16 or LSP_BF16; LSP_ERR_DTYPE otherwise), row-major
 *   Pt, Qt     device, the TRANSPOSED dense projectors P^T [r][m] and Q^T [r][n], row-major, in `dtype`
 *   S          device, r*r fp32, written
 *   workspace  device scratch of at least lsp_compress_dense_workspace_bytes(m, n, r) bytes, 16-byte aligned
 * Shapes: m a multiple of 128, n of 64, r of 128 (LSP_ERR_SHAPE otherwise; the size query then returns 0).
 * Asynchronous, three kernels, no atomics (bit-reproducible); all pointers 16-byte aligned.
 */
size_t lsp_compress_dense_workspace_bytes(int64_t m, int64_t n, int32_t r);
int lsp_compress_dense(const void* G, const void* Pt, const void* Qt,
                       int64_t m, int64_t n, int32_t r, float* S, lsp_dtype dtype,
                       void* workspace, size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Estimation bias of the projector pair on a gradient (Def. 2):
 *     b(P, Q; G) = || P P^T G Q Q^T - G ||_F / || G ||_F ,
 * the quantity MaybeUpdate in Alg. 1 compares with its threshold alpha to decide whether the
 * projectors are fitted again.  It composes the two steps above: the caller first compresses G
 * (lsp_compress or lsp_compress_planned: S = P^T G Q, which the training step computes anyway),
 * then this call rebuilds P S Q^T tile by tile in registers in one more streaming pass over G,
 * subtracts G and adds up the squares; no m x n temporary exists.  fp32 arithmetic; the
 * workgroups' sums are added in a fixed order in fp64, so the result is bit-reproducible.
 *
 *   G          device, m*n elements of `dtype`, row-major, read only
 *   S          device, r*r fp32: P^T G Q of the same G and projectors, read only
 *   out        device, 3 floats, overwritten: out[0] = || P S Q^T - G ||_F^2,
 *              out[1] = || G ||_F^2, out[2] = sqrt(out[0] / out[1]) (NaN by IEEE rules if G = 0)
 *   workspace  device scratch of at least lsp_estimation_bias_workspace_bytes(m,n,r,d) bytes,
 *              16-byte aligned; contents undefined afterwards
 * Errors as for lsp_decompress_apply, plus LSP_ERR_WORKSPACE.  Asynchronous on `stream`.
 */
int lsp_estimation_bias(const void* G, const float* S,
                        const int32_t* P_idx, const float* P_val,
                        const int32_t* Q_idx, const float* Q_val,
                        int64_t m, int64_t n, int32_t r, int32_t d, float* out,
                        void* workspace, size_t workspace_bytes,
                        lsp_dtype dtype, void* stream);
size_t lsp_estimation_bias_workspace_bytes(int64_t m, int64_t n, int32_t r, int32_t d);

/* ------------------------------------------------------------------------------------------
 * Optimiser-state re-projection: the last two assignments of MaybeUpdate in Alg. 1.  When the
 * projectors (P_prev, Q_prev) of a matrix are replaced by (P, Q), the first and second moments
 * kept in the subspace follow:
 *     M := (P^T P_prev) M (Q_prev^T Q)         V := (P^T P_prev)^2 V (Q_prev^T Q)^2
 * with the squares taken element by element (the reading under which V is the second moment of
 * the re-projected first-moment terms and stays non-negative).  Runs once per change of
 * projectors, on the device copy of the moments.
 *
 *   P_*, Pprev_*   device, [m][d] ELL pairs of the new and the previous left projector
 *   Q_*, Qprev_*   device, [n][d] ELL pairs of the new and the previous right projector
 *   M              device, r*r fp32, row-major, read and overwritten
 *   V              device, r*r fp32, read and overwritten; may be NULL (no second moment); not M
 *   workspace      device scratch of at least lsp_reproject_state_workspace_bytes(r) bytes,
 *                  16-byte aligned; contents undefined afterwards
 * The two r x r products of sparse matrices are accumulated with fp32 atomics: the result can
 * differ in the last bits from run to run.  The dense r x r products run in fp32 on the matrix
 * cores.  Errors as for the other calls; asynchronous on `stream`.
 */
int lsp_reproject_state(const int32_t* P_idx, const float* P_val,
                        const int32_t* Pprev_idx, const float* Pprev_val,
                        const int32_t* Q_idx, const float* Q_val,
                        const int32_t* Qprev_idx, const float* Qprev_val,
                        int64_t m, int64_t n, int32_t r, int32_t d,
                        float* M, float* V,
                        void* workspace, size_t workspace_bytes, void* stream);
size_t lsp_reproject_state_workspace_bytes(int32_t r);

/* ------------------------------------------------------------------------------------------
 * Projector fitting (the minimisation in MaybeUpdate, Alg. 1; Eq. 2): gradient of the data term
 *     F(P, Q) = 1/2 || P P^T G Q Q^T - G ||_F^2      (half the squared numerator of Def. 2's bias)
 * with respect to the stored projector values,
 *     gP[i][k] = dF / dP_val[i][k],      gQ[j][k] = dF / dQ_val[j][k]
 * (a stored value enters the dense projector linearly at its position, duplicates add; so two stored
 * entries of a row with the same column get the same derivative).  The paper's objective is
 * ||b||_F + beta * regulariser: its data term is sqrt(2 F), whose gradient is this one divided by ||b||_F
 * (lsp_estimation_bias gives the norm), and the regulariser -- written with different exponents in
 * Alg. 1 and in Eq. 2 -- is an element-wise function of the values; both are left to the caller's
 * optimiser.  fp32 arithmetic; G is streamed twice; no m x n temporary.
 *
 *   G            device, m*n elements of `dtype`, read only
 *   plan         device, the plan of these projectors WITH THEIR CURRENT VALUES (lsp_plan_build, or
 *                lsp_plan_refresh_values after the values changed); a plan of another problem makes
 *                every output NaN (see lsp_compress_planned)
 *   P_*, Q_*     device, the same projectors as ELL arrays
 *   gP, gQ       device, [m][d] and [n][d] fp32, overwritten
 *   workspace    device scratch of at least lsp_bias_gradient_workspace_bytes(m,n,r,d) bytes, 16-byte
 *                aligned; afterwards its first m*r floats hold T = G Q and the next r*r floats S = P^T G Q
 * The r x r products of sparse matrices inside use fp32 atomics (results can differ in the last bits from
 * run to run).  Errors as for lsp_estimation_bias.  Asynchronous on `stream`.
 */
int lsp_bias_gradient(const void* G, const void* plan,
                      const int32_t* P_idx, const float* P_val,
                      const int32_t* Q_idx, const float* Q_val,
                      int64_t m, int64_t n, int32_t r, int32_t d,
                      float* gP, float* gQ,
                      void* workspace, size_t workspace_bytes,
                      lsp_dtype dtype, void* stream);
size_t lsp_bias_gradient_workspace_bytes(int64_t m, int64_t n, int32_t r, int32_t d);

/* New values into an existing plan: for projectors whose positions (idx arrays) are unchanged since
 * the plan was built and whose values changed -- every iteration of projector fitting.  One small
 * kernel on `stream`; nothing is sorted again, the host is not involved, no synchronisation.
 *   plan         device, a plan built for (m, n, r, d) with the same P_idx / Q_idx; updated in place
 *                (a plan of another problem is left untouched)
 *   P_val/Q_val  device, [m][d] / [n][d], the new values
 */
int lsp_plan_refresh_values(void* plan, const float* P_val, const float* Q_val,
                            int64_t m, int64_t n, int32_t r, int32_t d, void* stream);

/* ------------------------------------------------------------------------------------------
 * Utilities.
 */

/* Checks every idx[row][k] against [0, r).  Enqueues a kernel on `stream`, then WAITS for it
 * (this call synchronises the stream).  Returns LSP_OK or LSP_ERR_INDEX.
 * flag: device, one int32 of scratch. */
int lsp_validate_projector(const int32_t* idx, int64_t rows, int32_t d, int32_t r,
                           int32_t* flag, void* stream);

/* Measurement aids (not part of the method): one plain streaming pass over `bytes` bytes of device
 * memory (a multiple of 16; fp32 data for the second call), to find out what a kernel with nothing
 * but the stream in it reaches on this GPU.  lsp_hbm_probe_read reads every byte once (compress reads G
 * once) and leaves one float per workgroup in `workspace` (>= lsp_hbm_probe_workspace_bytes(bytes));
 * lsp_hbm_probe_rmw does y[i] -= c on fp32 data (decompress-apply reads and writes W once).  Asynchronous
 * on `stream`; errors as above. */
size_t lsp_hbm_probe_workspace_bytes(size_t bytes);
int    lsp_hbm_probe_read(const void* buf, size_t bytes, void* workspace, size_t workspace_bytes, void* stream);
int    lsp_hbm_probe_rmw(void* buf, size_t bytes, float c, void* stream);

const char* lsp_strerror(int code);      /* static string for an lsp_status */
int         lsp_last_hip_error(void);    /* raw hipError_t of the last LSP_ERR_LAUNCH on this thread */
int         lsp_version(void);           /* major*10000 + minor*100 + patch */

#ifdef __cplusplus
}
#endif
#endif /* LSP_H */
