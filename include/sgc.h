/*
 * sgc.h - C ABI of the MI355X (gfx950) hot path of Sparse Gradient Compression (SGC).
 *
 * One optimizer step of SGC on C independent gradient chunks of length d (MESGC form,
 * paper Sec. 4.4, with one measurement matrix A shared by all chunks) is four calls:
 *
 *   sgc_sparsify_project   Alg. 2 line 1   idx,val = Sparsify_k(G);  p = A G~,  q = A G~^2
 *   sgc_adam_compressed    Alg. 2 lines 2-5 moments in R^r and their bias-corrected copies
 *   sgc_recover_omp        Alg. 2 line 6   x = OMP_A(mhat), z = OMP_A(vhat)  (eq. 9, App. B)
 *   sgc_apply              eq. 11 + eq. 3  W <- W - lr * alpha * x / (sqrt(z) + eps)
 * (sgc_recover_omp_shared is a variant of the third call that finds one support per chunk.)
 *
 * Conventions
 *   - Plain C. Every array pointer is a DEVICE pointer owned by the caller unless the
 *     parameter comment says "host". The library never allocates or frees device memory;
 *     scratch space is a caller-provided workspace whose size is queried first.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream). Every call only
 *     enqueues work on that stream and returns; results are ready after the stream is
 *     synchronised. Calls on one stream execute in order.
 *   - No call allocates device memory, synchronises, or enqueues a memset: calls may be recorded in a
 *     HIP graph (stream capture) and replayed. Scalars that depend on the step number are computed
 *     on the host, so a captured sgc_adam_compressed replays the step it was captured for.
 *   - Arguments are validated on the host before anything is launched. On error nothing is
 *     launched and a negative sgc_status is returned; the library never aborts or throws.
 *   - Work goes to the device that is current when a call is made; all pointers of a call must
 *     live there. The library keeps a little per-device host state (a second stream for large
 *     recoveries, the timing collection), so calls from several host threads must be serialised
 *     by the caller.
 *   - Chunk-local positions (`idx`, `sel`) are int32 in [0, d).
 *   - A is r x d with iid N(0, 1/r) entries (Sec. 4.3). It is handled transposed: "At" is
 *     d x r row-major, row i of At = column i of A (r contiguous floats).
 */
#ifndef SGC_H
#define SGC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t sgc_status;
enum {
    SGC_OK = 0,
    SGC_ERR_NULL = -1,      /* a required pointer is NULL */
    SGC_ERR_SHAPE = -2,     /* k == 0, k > d, k > r, n % d != 0, r % 4 != 0, size out of range */
    SGC_ERR_DTYPE = -3,     /* unknown gradient type or matrix mode */
    SGC_ERR_ALIGN = -4,     /* a pointer is not aligned to 16 bytes */
    SGC_ERR_WORKSPACE = -5, /* workspace smaller than the size query says (or than the static array) */
    SGC_ERR_STEP = -6,      /* step < 1, or a hyper-parameter outside its range */
    SGC_ERR_DEVICE = -7     /* a HIP call failed (launch error, no device) */
};

/* gradient element type of sgc_sparsify_project and sgc_outer_project */
enum { SGC_GRAD_F32 = 0, SGC_GRAD_BF16 = 1 };

/*
 * Option bit of sgc_matrix.flags, read by sgc_recover_omp* only. The correlation contraction only
 * has to find the candidates for the argmax: every position whose float score lies within 2^-10 of
 * the largest is re-scored in double before the selection is made. With this bit the contraction is
 * computed on the bfloat16 matrix cores from operands split in two bfloat16 terms (three products,
 * float accumulation, scores within ~1e-5 relative of the float ones) instead of on the float matrix
 * cores: the recovered support and values are unchanged, the contraction is several times faster.
 * Off by default: the default contraction is float throughout.
 */
enum { SGC_MATRIX_FLAG_SCREEN_BF16 = 1 };
/*
 * Option bit of sgc_matrix.flags for a generated (SGC_MATRIX_PHILOX) matrix, read by sgc_recover_omp* only.
 * By default a generated matrix of more than 64 MiB is never written to memory: its entries are regenerated
 * inside the contraction kernel and only the selected columns are kept. With this bit the call may instead
 * write the whole matrix once into its workspace (where the copies of the selected columns would be, so it
 * applies when d <= N k) and read it from there in every iteration: faster, at the price of d r 4 bytes of
 * HBM holding A for the duration of the call. Matrices of at most 64 MiB always go through a scratch panel
 * of that size, which stays in the memory-side cache.
 */
enum { SGC_MATRIX_FLAG_MATERIALIZE = 2 };
/*
 * Option bit of sgc_matrix.flags, read by sgc_recover_omp* only. A batch of at most 4 right-hand sides on
 * resident rows (a stored matrix, or a generated one of at most 64 MiB) of at most 6 MiB, with r <= 2048,
 * k <= 64 and k r <= 16384, is recovered in ONE launch: up to 68 workgroups stay resident for all k iterations,
 * keep their rows of At (or the least-squares state of a right-hand side) in LDS and exchange keys and
 * residuals through tagged words in the workspace, polling until they arrive. That needs all its workgroups on the device at once, which holds whenever the kernel gets the GPU to
 * itself; a caller that shares the GPU with other long-running kernels, or keeps more than three such
 * recoveries in flight at once on different streams (each wants up to 68 CUs for itself), sets this bit to keep
 * the three launches per iteration (same results). Should a word of the single launch not arrive within seconds, the
 * call gives up: for every right-hand side that was not finished sel is filled with -1 and x with 0, which
 * sgc_apply skips.
 */
enum { SGC_MATRIX_FLAG_MULTI_LAUNCH = 4 };

/* how the measurement matrix is provided */
enum {
    SGC_MATRIX_STORED = 0, /* At resident in device memory */
    SGC_MATRIX_PHILOX = 1  /* entries regenerated on the fly from `seed`; At is ignored */
};

/*
 * Measurement matrix A (Sec. 4.3: iid zero-mean normal entries, standard deviation 1/sqrt(r);
 * Sec. 4.4: the same A for every chunk).
 *
 * SGC_MATRIX_PHILOX defines A[j][i] (row j, column i) as follows: Philox4x32-10 with key
 * (seed & 0xffffffff, seed >> 32) and counter (i, j/4, 0, 0) gives words w0..w3; (w0,w1) and
 * (w2,w3) each feed one Box-Muller pair evaluated in float with fixed polynomials, giving rows
 * 4*(j/4)+0,1 and +2,3; the result is scaled by (float)(1/sqrt((double)r)). The transform uses
 * only exactly rounded operations, so sgc_matrix_fill reproduces the same bits everywhere.
 *
 * inv_colnorm[i] = 1/||A_:i||_2 (float), needed by sgc_recover_omp only; fill it with
 * sgc_matrix_colnorms.
 */
typedef struct sgc_matrix {
    int32_t mode; /* SGC_MATRIX_STORED | SGC_MATRIX_PHILOX */
    int32_t d;    /* columns of A = chunk length */
    int32_t r;    /* rows of A = measurements per chunk; multiple of 4 */
    int32_t flags; /* 0, or SGC_MATRIX_FLAG_* bits */
    uint64_t seed;            /* PHILOX mode */
    const float *At;          /* device [d][r], STORED mode; 16-byte aligned */
    const float *inv_colnorm; /* device [d]; may be NULL for sgc_sparsify_project */
    const double *gram;       /* device [d][d] or NULL: optional table for sgc_recover_omp* (see
                                 sgc_matrix_gram) */
} sgc_matrix;

/* AdamW-style hyper-parameters of Alg. 2 / eq. 11 (host values; no weight-decay term appears
 * in the paper's update, none is applied). */
typedef struct sgc_hyper {
    double beta1; /* in [0,1) */
    double beta2; /* in [0,1) */
    double eps;   /* > 0 */
    double lr;    /* eta of eq. 3 */
    double alpha; /* scaling factor of eq. 11 */
} sgc_hyper;

/* static string for a status code */
const char *sgc_status_string(sgc_status s);

/*
 * Materialise rows [row0, row0+rows) of At of the PHILOX matrix with the given seed and r into
 * At_out (device, [rows][r] floats, 16-byte aligned). Used to obtain a stored copy of a
 * generated matrix and to check the generator. Errors: NULL, SHAPE (r <= 0, r % 4, rows < 0).
 */
sgc_status sgc_matrix_fill(uint64_t seed, int32_t r, int64_t row0, int64_t rows, float *At_out,
                           void *stream);

/*
 * inv_colnorm_out[i] = 1/||A_:i||_2 for i in [0, A->d) (device, [d] floats). A->inv_colnorm is
 * not read. The norm is accumulated in double from the float entries (App. B selection rule
 * divides the correlation by this norm). A zero column yields 0.
 */
sgc_status sgc_matrix_colnorms(const sgc_matrix *A /* host */, float *inv_colnorm_out,
                               void *stream);

/*
 * gram_out[i][j] = <A_:i, A_:j> for all pairs of columns (device, [d][d] doubles = 8 d^2 bytes,
 * row-major, 16-byte aligned), accumulated in double from the float entries on the double matrix
 * cores. This is the Gram matrix A^H A that App. B precomputes. It is optional: with A->gram set,
 * sgc_recover_omp* take the inner products between the new column and the earlier selections from
 * this table instead of a pass over the selected columns (same values up to double rounding). A
 * per-matrix table like inv_colnorm: build it once for as long as A is in use, where 8 d^2 bytes
 * are affordable (2 GiB at d = 16384, 32 GiB at d = 65536). A->gram and A->inv_colnorm are not read.
 * Errors: NULL, SHAPE (d > 65536), DTYPE, ALIGN.
 */
sgc_status sgc_matrix_gram(const sgc_matrix *A /* host */, double *gram_out, void *stream);

/*
 * Alg. 2 line 1 for n/d chunks: per chunk keep the k entries of largest magnitude
 * (Sparsify_k, Sec. 4.2 / Def. 1) and project the kept values and their squares with A
 * (eq. 5-6).
 *   grad       [n] elements of grad_type (float, or bfloat16 as 16-bit patterns), chunk c is
 *              grad[c*d .. c*d+d)
 *   idx        out [n/d][k] chunk-local positions, ascending within a chunk
 *   val        out [n/d][k] the kept (signed) values widened to float
 *   p, q       out [n/d][r]; q may be NULL. Until the projection writes them, the call may use both as
 *              scratch (the top-k of float chunks longer than 16384 keeps its candidates there)
 * Magnitudes are ordered by the bit pattern with the sign cleared; among equal magnitudes
 * the lower position is kept. Squares are formed in float; sums are accumulated in float in
 * the order of ascending position.
 * Errors: NULL, SHAPE (d<=0, k<=0, k>d, k>r, n%d, r%4, k>4096), DTYPE, ALIGN.
 */
sgc_status sgc_sparsify_project(const void *grad, int32_t grad_type, int64_t n, int32_t d,
                                int32_t k, const sgc_matrix *A /* host */, int32_t *idx,
                                float *val, float *p, float *q, void *stream);

/*
 * Alg. 2 lines 2-5 on `count` state elements (count = chunks * r):
 *   m <- beta1 m + (1-beta1) p,  v <- beta2 v + (1-beta2) q          (in place, persistent)
 *   mhat = m / (1 - beta1^step), vhat = v / (1 - beta2^step)         (outputs for the recovery)
 * The stored state is the uncorrected moment, as in Adam; `step` counts from 1.
 * Errors: NULL, SHAPE (count < 0), STEP (step < 1 or betas outside [0,1)), ALIGN.
 */
sgc_status sgc_adam_compressed(const float *p, const float *q, float *m, float *v, float *mhat,
                               float *vhat, int64_t count, int32_t step,
                               const sgc_hyper *h /* host */, void *stream);

/* bytes of workspace sgc_recover_omp / sgc_recover_omp_shared need for N right-hand sides; 0 on invalid
 * sizes. sgc_omp_workspace_bytes covers any matrix (stored or generated) without the screening flag;
 * sgc_omp_workspace_bytes_for gives the exact need of one matrix (A->mode, A->d, A->r, A->flags are read): a
 * stored matrix is read in place and needs neither the copies of the selected columns nor a panel of
 * generated rows, and only a matrix with SGC_MATRIX_FLAG_SCREEN_BF16 needs the bfloat16 planes (4 d r bytes
 * more, at most 2 GiB), so callers who set that flag must size the workspace with this query. */
size_t sgc_omp_workspace_bytes(int32_t N, int32_t d, int32_t r, int32_t k);
size_t sgc_omp_workspace_bytes_for(int32_t N, int32_t k, const sgc_matrix *A /* host */);

/*
 * Batched orthogonal matching pursuit (eq. 9; selection rule and output of App. B): for each
 * of the N right-hand sides y_n in R^r, k iterations of
 *     lambda = argmax over unselected i of |<A_:i, res>| / ||A_:i||   (lowest i on exact ties)
 *     x      = argmin || y_n - A_Lambda x ||_2 ,   res = y_n - A_Lambda x
 *   y    [N][r]
 *   sel  out [N][k] selected positions in selection order
 *   x    out [N][k] least-squares values aligned with sel
 *   ws   workspace of at least sgc_omp_workspace_bytes_for(N, k, A) bytes (sgc_omp_workspace_bytes(N, d, r, k)
 *        is enough for any A without the screening flag), 256-byte aligned; contents are scratch
 * All N correlations of one iteration are one dense contraction At * R on the float matrix
 * cores; the near-maximal candidates are then re-scored in double, and the least-squares
 * update (inverse-Cholesky form of App. B) and the residual are computed in double.
 * Requires A->inv_colnorm. Errors: NULL, SHAPE (k<=0, k>d, k>r, k>1024, r%4, 4r+16k > 60 KiB, N<=0), DTYPE,
 * ALIGN, WORKSPACE.
 */
sgc_status sgc_recover_omp(const float *y, int32_t N, const sgc_matrix *A /* host */, int32_t k,
                           int32_t *sel, float *x, void *ws, size_t ws_bytes, void *stream);

/*
 * sgc_recover_omp for callers that cannot allocate device memory or hand over a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels, with the
 * workspace in a static device array of SGC_OMP_STATIC_WORKSPACE_BYTES that each GPU the library runs on
 * holds until the process ends. The call allocates and frees nothing and keeps all work on `stream`
 * (no library-owned second stream). Arguments and results as sgc_recover_omp.
 * Limit: sgc_omp_workspace_bytes_for(N, k, A) must not exceed sgc_omp_static_workspace_bytes(), else
 * SGC_ERR_WORKSPACE is returned and nothing is launched (32 MiB hold e.g. 2048 right-hand sides of
 * d = 2048, r = 220, k = 31 with a stored matrix, or 16 of d = 16384, r = 1024, k = 64).
 * All calls on one GPU share that GPU's array: two such calls whose kernels may overlap (different streams,
 * different host threads) race; calls on one stream are safe. The array keeps the previous call's contents;
 * every region read is written earlier in the same call.
 * Errors: as sgc_recover_omp; WORKSPACE as above; DEVICE if the array's address cannot be resolved.
 */
enum { SGC_OMP_STATIC_WORKSPACE_BYTES = 32 << 20 };
size_t sgc_omp_static_workspace_bytes(void);
sgc_status sgc_recover_omp_static(const float *y, int32_t N, const sgc_matrix *A /* host */, int32_t k,
                                  int32_t *sel, float *x, void *stream);

/*
 * Shared-support recovery for C chunks. Sec. 4.3 (the remark after eq. 11) rests the element-wise
 * division of eq. 11 on both recovered moments having their non-zeros at the same positions; this
 * call makes that hold by construction and halves the contraction work: the support and x come
 * from OMP on y_m alone (exactly sgc_recover_omp with N = C), and the second moment is fitted on
 * the same support, z = argmin || y_v - A_Lambda z ||_2 (in double, from the inverse Cholesky
 * factor the recovery has built).
 *   y_m, y_v  [C][r]  the bias-corrected first / second moments
 *   sel       out [C][k] selection order;  x, z  out [C][k] aligned with sel
 *   ws        at least sgc_omp_workspace_bytes(C, d, r, k) bytes, 256-byte aligned
 * Feed sgc_apply with (sel, x, sel, z). Errors: as sgc_recover_omp.
 */
sgc_status sgc_recover_omp_shared(const float *y_m, const float *y_v, int32_t C,
                                  const sgc_matrix *A /* host */, int32_t k, int32_t *sel, float *x,
                                  float *z, void *ws, size_t ws_bytes, void *stream);

/*
 * The same recovery with the correlation recurrence of App. B (Alg. 3) in place of the contraction:
 * with the table G = A^H A (A->gram, see sgc_matrix_gram) the correlation vector p = A^H res is formed
 * once, p0 = A^H y, and then updated in every iteration, p <- p - b_j a_j, where b_j = A^H q_j is the
 * image of the new orthonormal direction and follows from the earlier ones,
 * b_j = gamma_j (G_:lambda_j - sum_t c_t b_t). The b_t of every right-hand side are kept (the d x k
 * matrix B of App. B, floats): an iteration streams them, one row of G, and p. Selection and
 * least-squares update are those of sgc_recover_omp - the candidates near the maximum of p are re-scored
 * in double against the residual, so the support is the same whenever the float recurrence keeps the true
 * maximum within 2^-10 of its own (it does while the residual stays well above float rounding of y, i.e. not
 * after an exact recovery with iterations to spare).
 *   head  the recurrence serves the selections of iterations 0 .. head-1; from iteration `head` on the
 *         correlations come from the contraction of sgc_recover_omp, which needs no state of its own.
 *         head = k is App. B throughout. Iteration j of the recurrence moves 4 d (j + 5) bytes per right-hand
 *         side where the contraction spends 2 d r flop, so on this machine the recurrence is the cheaper of the
 *         two while j + 5 < r / 50 or so, and a head of that size the fastest choice for a caller that
 *         holds the table anyway
 *   other arguments as sgc_recover_omp; A->gram must be set; d % 4 == 0; a generated matrix must fit the
 *   workspace's panel whole (at most 64 MiB, or d <= N k)
 *   ws    at least sgc_omp_recurrence_workspace_bytes(N, d, r, k, head) bytes (0 for invalid sizes): the
 *         workspace of sgc_recover_omp plus N (head + 1) d floats
 * Errors: as sgc_recover_omp; SHAPE also for head < 1 or head > k; NULL also when A->gram is not set.
 */
size_t sgc_omp_recurrence_workspace_bytes(int32_t N, int32_t d, int32_t r, int32_t k, int32_t head);
sgc_status sgc_recover_omp_recurrence(const float *y, int32_t N, const sgc_matrix *A /* host */, int32_t k,
                                      int32_t head, int32_t *sel, float *x, void *ws, size_t ws_bytes,
                                      void *stream);

/*
 * SGCA re-alignment of compressed moments with a new measurement matrix (App. C, Alg. 4 lines
 * 9-12: every T steps A' is drawn and M <- A' OMP_A(M), V <- A' OMP_A(V), A <- A'):
 *   out[n] = scale * A' x_n   for N sparse vectors given as (sel[n], x[n]), k entries each,
 * as returned by sgc_recover_omp / sgc_recover_omp_shared; positions must be in [0, d).
 * OMP commutes with a positive scaling of its input, so the vectors the step has already recovered
 * from the bias-corrected moments serve: scale = 1 - beta1^step gives the re-aligned (uncorrected)
 * first-moment state from OMP(mhat), scale = 1 - beta2^step the second from OMP(vhat); vectors
 * recovered from the state itself take scale = 1. `out` ([N][r], 16-byte aligned) may be the state
 * array itself. Sums are accumulated in float in list order, then scaled.
 * Errors: NULL, SHAPE (N < 0, k <= 0, k > d, k > 4096, r % 4), DTYPE, ALIGN.
 */
sgc_status sgc_reproject(const int32_t *sel, const float *x, int64_t N, int32_t k,
                         const sgc_matrix *A_new /* host */, double scale, float *out, void *stream);
/* The same with scale = 1 - beta^step formed on the host exactly as sgc_adam_compressed forms its bias
 * correction (Alg. 4 lines 10-11 applied to the vectors recovered from mhat / vhat at step `step`).
 * Errors: as sgc_reproject; STEP (step < 1, beta outside [0,1)). */
sgc_status sgc_reproject_moment(const int32_t *sel, const float *x, int64_t N, int32_t k,
                                const sgc_matrix *A_new /* host */, double beta, int32_t step, float *out,
                                void *stream);

/*
 * eq. 11 and eq. 3 on the recovered supports of C chunks:
 *   for each position i in sel_m[c]: z = value of i in (sel_v[c], x_v[c]) or 0 if absent,
 *   W[c*d+i] -= lr * alpha * x_i / (sqrt(max(z,0)) + eps)
 * Positions outside sel_m[c] are not touched.
 *   W [C*d] in/out; sel_m,x_m / sel_v,x_v [C][k] as returned by sgc_recover_omp for mhat / vhat.
 * Errors: NULL, SHAPE (k<=0, k>d, k>4096, C<0).
 */
sgc_status sgc_apply(float *W, int64_t C, int32_t d, int32_t k, const int32_t *sel_m,
                     const float *x_m, const int32_t *sel_v, const float *x_v,
                     const sgc_hyper *h /* host */, void *stream);

/*
 * CESGC (Sec. 4.4): SGC on a gradient that a projection B has compressed first. For a weight matrix
 * W (m x n, row-major) with gradient G (m x n) and B (rho x m, row-major; the paper takes the leading
 * left singular vectors of a gradient and refreshes them every fixed number of steps: sgc_outer_refresh
 * below; to the two calls here B is an input) one step is
 *   sgc_outer_project       Gc = B G  (rho x n, row-major)
 *   the four calls of the plain step on Gc read as rho*n/d chunks of d entries (sgc_apply left out)
 *   sgc_outer_apply         W <- W - lr * B^T N,  N (rho x n) the update of eq. 11 in the compressed
 *                           space: on the support of x, N = alpha x / (sqrt(max(z, 0)) + eps)
 * Both calls take a batch of `count` equal-sized matrices stored one after the other (one launch for
 * all of them: a single matrix of a few tens of MB is too little work to fill the memory system):
 *   B    [count][rho][m], G and W [count][m][n], Gc out [count][rho][n]; n % 4 == 0; G, W, Gc
 *        16-byte aligned. G is float or bfloat16 bit patterns (grad_type: SGC_GRAD_F32 / SGC_GRAD_BF16,
 *        widened exactly); everything else is float
 *   sel_m, x_m, sel_v, x_v  [count*rho*n/d][k]: the chunks of the whole batch in order, as returned by
 *        sgc_recover_omp on [mhat; vhat] of all of them
 *   ws   at least sgc_outer_workspace_bytes(count, rho, m, n) bytes (0 for invalid sizes), 256-byte
 *        aligned; holds partial products (project) or N written out densely (apply), and may be
 *        the same memory for both calls
 * Products are accumulated in float on the matrix cores; the rows of G are summed in slices whose
 * partial results are added in a fixed order, so results are reproducible run to run.
 * Errors: NULL, SHAPE (count, rho, m, n <= 0, rho above 2^20, m or n above 2^22, count * ceil(rho/32)
 * above 65535, n % 4, rho*n % d, k <= 0, k > d, k > 4096), DTYPE, ALIGN, WORKSPACE, DEVICE.
 */
size_t sgc_outer_workspace_bytes(int32_t count, int32_t rho, int32_t m, int32_t n);
sgc_status sgc_outer_project(const float *B, const void *G, int32_t grad_type, int32_t count, int32_t rho,
                             int32_t m, int32_t n, float *Gc, void *ws, size_t ws_bytes, void *stream);
sgc_status sgc_outer_apply(float *W, const float *B, int32_t count, int32_t rho, int32_t m, int32_t n, int32_t d,
                           int32_t k, const int32_t *sel_m, const float *x_m, const int32_t *sel_v,
                           const float *x_v, const sgc_hyper *h /* host */, void *ws, size_t ws_bytes,
                           void *stream);

/*
 * CESGC (Sec. 4.4), the renewal of B every fixed number of steps: the rows of B become the rho leading
 * left singular vectors of the gradient matrix G (m x n), in the order of decreasing singular value,
 * each with its largest-magnitude entry positive (the sign of a singular vector is free).
 * Method: `iters` rounds of orthogonal iteration on G G^T started from the B handed in (the previous
 * matrix, or any rho x m matrix of full row rank, e.g. random), then a Rayleigh-Ritz step. Row i
 * converges at the rate (sigma_{i+1}/sigma_i)^2 per round, the subspace as a whole at
 * (sigma_{rho+1}/sigma_rho)^2; iters = 0 only rotates an orthonormal B inside its own subspace.
 * Like the two calls above it takes a batch of `count` equal-sized matrices (every kernel covers the
 * whole batch; the rho x rho factorisations of different matrices run in different workgroups):
 *   B      [count][rho][m] in/out, 16-byte aligned
 *   G      [count][m][n], float or bfloat16 bit patterns, 16-byte aligned
 *   sigma  [count][rho] out or NULL: the singular values, decreasing
 *   ws     at least sgc_outer_refresh_workspace_bytes(count, rho, m, n, grad_type) bytes (0 for invalid
 *          sizes), 256-byte aligned: a transposed copy of G, count rho x n matrices and small factors
 * The passes over G run on the matrix cores in float; Gram matrices, their Cholesky and Jacobi
 * factorisations and the rho x rho transforms are in double. Rows that depend on earlier rows to float
 * accuracy (G of rank below rho) come out as zero rows, with sigma 0; zero rows of a start matrix are
 * given generic entries first, so a later renewal on a gradient of full rank fills them again (except
 * with iters = 0, which only rotates what it is given).
 * Errors: NULL, SHAPE (count, rho, m, n <= 0, rho > 64, rho > m, rho > n, m or n above 2^22, m % 4, n % 4,
 * count * ceil(rho/32) above 65535, iters < 0 or > 1000), DTYPE, ALIGN, WORKSPACE, DEVICE.
 */
size_t sgc_outer_refresh_workspace_bytes(int32_t count, int32_t rho, int32_t m, int32_t n, int32_t grad_type);
sgc_status sgc_outer_refresh(float *B, const void *G, int32_t grad_type, int32_t count, int32_t rho, int32_t m,
                             int32_t n, int32_t iters, float *sigma, void *ws, size_t ws_bytes, void *stream);

/*
 * Instrumentation (not a step of the method): per-kernel timing with HIP events recorded on the
 * caller's stream around every kernel the library launches while enabled.
 *   sgc_profile_enable(1) starts collecting (and discards what was collected), (0) stops.
 *   sgc_profile_read waits for the recorded events, then fills `out` (host) with the summed
 *   duration in milliseconds and the launch count per kernel class, and clears the collection.
 * Kernel classes: 0 top-k, 1 projection, 2 Adam, 3 OMP correlation contraction, 4 OMP
 * select+update, 5 apply, 6 other (init, matrix helpers), 7 refill of the generated-matrix panel
 * inside the OMP iterations, 8 sgc_outer_project, 9 sgc_outer_apply (its scatter of N counts as 5), 10 sgc_outer_refresh (its
 * passes over G count as 8).
 * Not thread-safe; meant for a single measuring thread. Errors: NULL, DEVICE.
 * Independently of this, sgc_sparsify_project, sgc_adam_compressed, sgc_recover_omp, sgc_recover_omp_shared and
 * sgc_apply put a named range (the function's name) around their launches through the ROCTx marker library
 * when that library can be found at run time, so that `rocprofv3 --marker-trace` shows the four calls of a step.
 */
enum { SGC_PROFILE_CLASSES = 11 };
typedef struct sgc_profile {
    double ms[SGC_PROFILE_CLASSES];
    int64_t launches[SGC_PROFILE_CLASSES];
} sgc_profile;
sgc_status sgc_profile_enable(int32_t on);
sgc_status sgc_profile_read(sgc_profile *out /* host */);

/*
 * Machine probes (instrumentation, not a step of the method): one launch of a small kernel that exercises
 * a single resource, for the caller to time, so that fractions quoted against published peaks can be read
 * next to what the same machine delivers.
 *   SGC_PROBE_VALU  blocks x 256 threads, each `iters` x 64 dependent-chain v_fma_f32 (16 chains, plain
 *                   non-packed form, registers only): lane-instructions = blocks * 256 * iters * 64
 *   SGC_PROBE_MFMA  blocks x 4 wavefronts, each `iters` x 16 v_mfma_f32_32x32x2f32 (4096 flop each)
 *   SGC_PROBE_MFMA_VALU4, _VALU8  the MFMA probe with 4 (8) independent v_fma_f32 behind every MFMA: whether
 *                   vector-ALU work rides in the shadow of float matrix instructions or adds to their time
 *   SGC_PROBE_SPLIT_BOTH, _SPLIT_MFMA, _SPLIT_VALU  blocks x 8 wavefronts (two per SIMD): wavefronts 0-3 issue only
 *                   `iters` x 16 MFMAs, wavefronts 4-7 only `iters` x 256 plain v_fma_f32; both groups, or one of
 *                   them alone (the other leaves at once): whether vector-ALU work of other wavefronts on the same
 *                   SIMD runs beside float matrix instructions
 *   SGC_PROBE_READ  reads `bytes` of a with non-temporal 16-byte loads
 *   SGC_PROBE_RW44  reads four arrays of bytes/8 from a and writes four of bytes/8 to b (the Adam kernel's
 *                   traffic pattern: `bytes` moved in total); a and b must each hold bytes/2
 *   SGC_PROBE_COPY  copies bytes/2 from a to b
 * a (may be NULL for the VALU / MFMA / SPLIT kinds) and b (at least 4 bytes) are device pointers, 16-byte aligned; a
 * multiple of 128 bytes keeps every access whole. Errors: NULL, SHAPE, DTYPE (unknown kind), ALIGN, DEVICE.
 */
enum { SGC_PROBE_VALU = 0, SGC_PROBE_MFMA = 1, SGC_PROBE_READ = 2, SGC_PROBE_RW44 = 3, SGC_PROBE_COPY = 4,
       SGC_PROBE_MFMA_VALU4 = 5, SGC_PROBE_MFMA_VALU8 = 6, SGC_PROBE_SPLIT_BOTH = 7, SGC_PROBE_SPLIT_MFMA = 8,
       SGC_PROBE_SPLIT_VALU = 9 };
sgc_status sgc_probe(int32_t kind, const void *a, void *b, int64_t bytes, int32_t blocks, int32_t iters,
                     void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SGC_H */
