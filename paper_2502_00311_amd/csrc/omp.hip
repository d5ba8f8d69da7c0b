// Batched orthogonal matching pursuit (paper Sec. 4.3 eq. 9; selection rule, inverse-Cholesky
// update and output of App. B) for N right-hand sides that share the measurement matrix A.
//
// Per iteration:
//   contraction    P = At * R for all right-hand sides at once: a dense float contraction on the
//                  matrix cores (32x32x2 MFMA, LDS-staged tiles; corr_pipelined_kernel for full
//                  position tiles of resident rows, corr_kernel for everything else). P is never
//                  written: the epilogue scales by 1/||A_:i||, leaves out selected positions and keeps
//                  the two best (score, position) pairs of every position tile per right-hand side.
//                  Optionally (a flag of the matrix) the same contraction on the bfloat16 matrix cores
//                  from operands split in two bfloat16 terms: corr_split_kernel, or the bfloat16 form
//                  of corr_pipelined_kernel on full tiles. (The contraction kernels are in omp_corr.hip.)
//   pick / factor / residual   re-score the near-maximal candidates in double (so the argmax does
//                  not depend on float rounding), append the winning column, extend F = L^-H
//                  (App. B) by mat-vecs only, and recompute the residual y - A_Lambda x in double.
// After the last iteration refit_kernel can fit a second right-hand side on the support found.
// App. B precomputes the Gram matrix A^H A (d x d) to avoid the contraction; here the contraction
// is kept (it is what the matrix cores are for) and only inner products with selected columns are
// formed, so memory stays O(N k r).
#include <mutex>
#include <type_traits>

#include "omp_internal.h"
#include "philox_normal.h"

namespace sgc {

constexpr float RESCORE_TOL = 0x1.0p-10f; // candidates within this relative distance of the float maximum

OmpWorkspace carve_workspace(void *base, int32_t N, int32_t d, int32_t r, int32_t k, uint32_t need)
{
    OmpWorkspace w{};
    size_t off = 0;
    auto take = [&](size_t bytes) {
        void *p = base ? (void *)((char *)base + off) : nullptr;
        off += (bytes + 255) & ~(size_t)255;
        return p;
    };
    w.tiles_m = corr_tiles_m(d);
    w.words = (d + 31) / 32;
    w.res64 = (double *)take(sizeof(double) * (size_t)N * r);
    w.f_stride = (int64_t)k * k + 288;
    w.F = (double *)take(sizeof(double) * (size_t)N * w.f_stride);
    w.avec = (double *)take(sizeof(double) * (size_t)N * k);
    w.xs = (double *)take(sizeof(double) * (size_t)N * k * 2);
    w.xs_half = (int64_t)N * k;
    w.res32 = (float *)take(sizeof(float) * (size_t)N * r);
    w.res16 = reinterpret_cast<uint16_t *>(w.res32);
    // the per-right-hand-side copies of the selected columns and the panel serve generated matrices only:
    // a stored matrix is read in place
    const bool generated = (need & WS_NEED_GENERATED) != 0;
    w.cols = generated ? (float *)take(sizeof(float) * (size_t)N * k * r) : nullptr;
    // two keys per tile of positions; a small batch may be served by the single-launch recovery, whose
    // workgroups (up to SMALL_MAX_GROUPS) each leave two keys per right-hand side
    {
        const int32_t slots = N <= SMALL_MAX_RHS && w.tiles_m < SMALL_MAX_GROUPS ? SMALL_MAX_GROUPS : w.tiles_m;
        w.partial = (uint64_t *)take(sizeof(uint64_t) * (size_t)N * slots * 2);
    }
    w.sync = (uint32_t *)take(sizeof(uint32_t) * 64);
    // the single-launch recovery's exchange area: per right-hand side r tagged residual words and the selected position
    w.xchg = N <= SMALL_MAX_RHS ? (uint64_t *)take(sizeof(uint64_t) * (size_t)N * (r + SMALL_XCHG_PAD)) : nullptr;
    w.bitmap = (uint32_t *)take(sizeof(uint32_t) * (size_t)N * w.words);
    // Rows of a generated matrix, in whole tiles. A matrix of at most 64 MiB gets a panel of its own (it
    // then stays in the 256 MiB memory-side cache). A larger one is regenerated inside the contraction, or
    // goes through a 64 MiB panel that is refilled in every iteration; only if the matrix asks for it
    // (SGC_MATRIX_FLAG_MATERIALIZE) is it written out whole where the column copies would be, when it is
    // no larger than they are (d <= N k; the copies are not needed once the rows are resident).
    int64_t small_rows = ((int64_t)64 << 20) / ((int64_t)r * 4);
    small_rows = small_rows / 256 * 256;
    if (small_rows < 256)
        small_rows = 256;
    {
        const int64_t dpad = ((int64_t)d + 255) / 256 * 256;
        if (small_rows > dpad)
            small_rows = dpad;
        if (generated && (need & WS_NEED_WHOLE_MATRIX) && dpad > small_rows && dpad <= (int64_t)N * k) {
            w.panel_rows = (int32_t)dpad;
            w.panel = w.cols;
        } else {
            w.panel_rows = (int32_t)small_rows;
            w.panel = generated ? (float *)take(sizeof(float) * (size_t)small_rows * r) : nullptr;
        }
    }
    // bfloat16 planes of the matrix rows for the screening contraction (only when the matrix asks for it): the
    // whole matrix if that is at most 2 GiB, else a 64 MiB panel's worth (larger resident matrices then keep
    // the float contraction)
    w.a16_rows = 0;
    w.a16 = nullptr;
    if (need & WS_NEED_SCREEN) {
        const int64_t dpad = ((int64_t)d + 127) / 128 * 128;
        w.a16_rows = dpad * r * 4 <= ((int64_t)2 << 30) ? (int32_t)dpad : (int32_t)small_rows;
        w.a16 = (uint16_t *)take(sizeof(float) * (size_t)w.a16_rows * r);
    }
    w.wv = (double *)take(sizeof(double) * (size_t)N * k);
    w.gb = (double *)take(sizeof(double) * (size_t)N * 2);
    w.bytes = off;
    return w;
}

OmpWorkspace carve_recurrence(void *base, int32_t N, int32_t d, int32_t r, int32_t k, int32_t head, uint32_t need)
{
    OmpWorkspace w = carve_workspace(base, N, d, r, k, need);
    size_t off = w.bytes;
    auto take = [&](size_t bytes) {
        void *p = base ? (void *)((char *)base + off) : nullptr;
        off += (bytes + 255) & ~(size_t)255;
        return p;
    };
    w.rc_p = (float *)take(sizeof(float) * (size_t)N * d);
    w.rc_head = head;
    w.rc_d = d;
    w.rc_B = (float *)take(sizeof(float) * (size_t)N * head * d);
    w.cvec = (double *)take(sizeof(double) * (size_t)N * k);
    w.bytes = off;
    return w;
}

// res_split != 0: the float copy of the residual is written in split32 format instead (see corr_split_kernel)
__global__ __launch_bounds__(256) void omp_init_kernel(const float *__restrict__ y, int32_t r, int32_t words,
                                                       double *__restrict__ res64, float *__restrict__ res32,
                                                       uint32_t *__restrict__ bitmap, int32_t res_split,
                                                       uint32_t *__restrict__ sync, uint64_t *__restrict__ keys,
                                                       int32_t keys_per_rhs, uint64_t *__restrict__ xchg,
                                                       int32_t xchg_per_rhs)
{
    const int64_t n = blockIdx.x;
    // fills by a kernel, not memset nodes: the call may be captured in a graph
    if (n == 0 && threadIdx.x < 64)
        sync[threadIdx.x] = 0u;
    // a small batch may go to the single-launch recovery, whose tagged words must not carry tags of an earlier call
    for (int32_t i = threadIdx.x; i < keys_per_rhs; i += 256)
        keys[n * keys_per_rhs + i] = 0ull;
    for (int32_t i = threadIdx.x; i < xchg_per_rhs; i += 256)
        xchg[n * xchg_per_rhs + i] = 0ull;
    uint16_t *res16 = reinterpret_cast<uint16_t *>(res32);
    for (int32_t j = threadIdx.x; j < r; j += 256) {
        const float v = y[n * r + j];
        res64[n * r + j] = (double)v;
        if (res_split) { // split32 row: the same 4 r bytes as the float row
            uint16_t hi, lo;
            split_bf16_1(v, hi, lo);
            uint16_t *o = res16 + n * 2 * r + (j >> 5) * 64 + (j & 31);
            o[0] = hi;
            o[32] = lo;
        } else {
            res32[n * r + j] = v;
        }
    }
    for (int32_t w = threadIdx.x; w < words; w += 256)
        bitmap[n * words + w] = 0u;
}

// ----------------------------------------------------------------------------------------------
// Selection and least-squares update, two kernels per iteration:
//   pick_kernel      re-scores the near-maximal candidates in double and fixes lambda; then
//                    w_t = <A_:lambda_t, A_:lambda> for the earlier selections (a row-major mat-vec over
//                    the selected columns, one wavefront per row, spread over several workgroups)
//   update_kernel    the small dense part of App. B: c = F^H w, gamma, the new coefficient, the new
//                    column of F and x = F a, all in double; then res = y - A_Lambda x in double (a
//                    column-major mat-vec over the selected columns), plus the float copy for the
//                    next contraction
constexpr int PICK_THREADS_WIDE = 512, PICK_THREADS_NARROW = 128; // narrow: short columns (r <= 512) and k <= 128
constexpr int PICK_CAND_CAP = 64;
constexpr int FACTOR_MAX_THREADS = 1024;

struct IterArgs {
    const float *y; // [N][r]
    int32_t k, it;  // sparsity, current iteration (0-based)
    int32_t *sel;   // [N][k]
    float *x;       // [N][k]
    OmpWorkspace ws;
    // rows of At resident in memory (a stored matrix, or a generated one produced whole into the
    // panel): the least-squares passes then fetch the selected columns from here through `sel`,
    // where a matrix shared by many right-hand sides stays in cache, and ws.cols is not used.
    // NULL: the selected columns are kept per right-hand side in ws.cols.
    const float *At_rows;
    int32_t share_table; // update_kernel: its dynamic LDS also holds the [wavefront][k] table of shares
    int32_t res_split;   // update_kernel: != 0: the residual's float copy goes out in split32 format
};

template <bool GENERATED>
__device__ __forceinline__ float4 column_quad(const MatrixView &A, int32_t i, int32_t jb)
{
    if (GENERATED)
        return matrix_quad((uint32_t)i, (uint32_t)jb, A.key0, A.key1, A.scale);
    return reinterpret_cast<const float4 *>(A.At + (int64_t)i * A.r)[jb];
}

// The selection of one right-hand side from its np tile keys (App. B's rule, decided in double): the float maximum,
// the candidates within RESCORE_TOL of it, their re-scoring against the double residual res64[r], lowest
// position on equal scores. Called by a whole workgroup; every thread returns the selected position.
template <bool GENERATED, int PICK_THREADS>
__device__ __forceinline__ int32_t select_lambda(const MatrixView &A, const uint64_t *part, const int32_t np,
                                                 const double *res64)
{
    constexpr int PICK_WAVES = PICK_THREADS / 64;
    __shared__ uint64_t s_u64[PICK_WAVES];
    __shared__ double s_cscore[PICK_WAVES];
    __shared__ int32_t s_cidx[PICK_WAVES];
    __shared__ int32_t s_cand[PICK_CAND_CAP];
    __shared__ int32_t s_lambda, s_ncand;
    const int32_t r4 = A.r >> 2;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // known to be the same in all lanes: loops over wavefronts stay scalar

    // (1) float maximum over the tile partials
    uint64_t best = 0;
    for (int32_t e = tid; e < np; e += PICK_THREADS) {
        const uint64_t v = part[e];
        best = v > best ? v : best;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint64_t o = shfl_xor_u64(best, off);
        best = o > best ? o : best;
    }
    if (lane == 0)
        s_u64[wave] = best;
    if (tid == 0)
        s_ncand = 0;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < PICK_WAVES; ++u)
        best = s_u64[u] > best ? s_u64[u] : best;
    const float smax = __uint_as_float((uint32_t)(best >> 32));
    const float thr = smax * (1.0f - RESCORE_TOL);

    // (2) candidates: every kept pair whose float score is within the tolerance of the maximum
    for (int32_t e = tid; e < np; e += PICK_THREADS) {
        const uint64_t v = part[e];
        if (v != 0 && __uint_as_float((uint32_t)(v >> 32)) >= thr) {
            const int32_t slot = atomicAdd(&s_ncand, 1);
            if (slot < PICK_CAND_CAP)
                s_cand[slot] = (int32_t)(0xffffffffu - (uint32_t)v);
        }
    }
    __syncthreads();
    const int32_t ncand = s_ncand;

    // (3) a single candidate is the argmax; several are re-scored in double, one wavefront per
    //     candidate, winner = (score desc, position asc). More candidates than the list holds (an
    //     all-zero residual) are walked straight from the partials.
    double wbest = -1.0;
    int32_t widx = 0x7fffffff;
    if (ncand == 1) {
        wbest = 0.0;
        widx = s_cand[0];
    } else {
        const bool listed = ncand <= PICK_CAND_CAP;
        const int32_t count = listed ? ncand : np;
        for (int32_t e = wave; e < count; e += PICK_WAVES) {
            int32_t i;
            if (listed) {
                i = s_cand[e];
            } else {
                const uint64_t v = part[e];
                if (v == 0 || !(__uint_as_float((uint32_t)(v >> 32)) >= thr))
                    continue;
                i = (int32_t)(0xffffffffu - (uint32_t)v);
            }
            double dot = 0.0, nrm = 0.0;
            for (int32_t jb = lane; jb < r4; jb += 64) {
                const float4 a = column_quad<GENERATED>(A, i, jb);
                const double *rr = res64 + 4 * jb;
                dot += (double)a.x * rr[0] + (double)a.y * rr[1] + (double)a.z * rr[2] + (double)a.w * rr[3];
                nrm += (double)a.x * a.x + (double)a.y * a.y + (double)a.z * a.z + (double)a.w * a.w;
            }
            dot = __shfl(wave_sum(dot), 0, 64);
            nrm = __shfl(wave_sum(nrm), 0, 64);
            const double score = nrm > 0.0 ? fabs(dot) / sqrt(nrm) : 0.0;
            if (score > wbest || (score == wbest && i < widx)) {
                wbest = score;
                widx = i;
            }
        }
    }
    if (lane == 0) {
        s_cscore[wave] = wbest;
        s_cidx[wave] = widx;
    }
    __syncthreads();
    if (tid == 0) {
        double bs = s_cscore[0];
        int32_t bi = s_cidx[0];
        for (int u = 1; u < PICK_WAVES; ++u)
            if (s_cscore[u] > bs || (s_cscore[u] == bs && s_cidx[u] < bi)) {
                bs = s_cscore[u];
                bi = s_cidx[u];
            }
        // no candidate survives only when the scores are not numbers: fall back to the float
        // maximum so that every later access stays inside the matrix
        if (bi < 0 || bi >= A.d)
            bi = (int32_t)(0xffffffffu - (uint32_t)best);
        if (bi < 0 || bi >= A.d)
            bi = 0;
        s_lambda = bi;
    }
    __syncthreads();
    return s_lambda;
}

// grid (N, slices). Every slice of a right-hand side repeats the (cheap) selection so that no
// grid-wide synchronisation is needed; slice 0 also stores the column and the scalars.
// dynamic LDS: float a_col[r]
template <bool GENERATED, int PICK_THREADS>
__device__ __forceinline__ void pick_body(const MatrixView &A, const IterArgs &P, const int64_t n, const int slice,
                                          const int nslices, unsigned char *smem)
{
    constexpr int PICK_WAVES = PICK_THREADS / 64;
    float *a_col = reinterpret_cast<float *>(smem);
    __shared__ double s_red[2][PICK_WAVES];
    const int32_t r = A.r, r4 = A.r >> 2, k = P.k, it = P.it;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // known to be the same in all lanes: loops over wavefronts stay scalar
    if (slice != 0 && slice * PICK_WAVES >= it)
        return; // no earlier selection falls to this slice
    const OmpWorkspace &W = P.ws;
    const int32_t lam = select_lambda<GENERATED, PICK_THREADS>(A, W.partial + n * (int64_t)(W.tiles_m * 2), W.tiles_m * 2,
                                                               W.res64 + n * r);
    // with a table of column inner products, w_t = <A_:lambda_t, a> is a gather from its row lambda:
    // requested here, before the column itself is fetched, so that both travel at the same time
    constexpr int GQ = (1024 + PICK_THREADS - 1) / PICK_THREADS; // k <= 1024
    double gram_w[GQ];
    if (A.gram && slice == 0) {
        const double *grow = A.gram + (int64_t)lam * A.d;
        const int32_t *selq = P.sel + n * k;
#pragma unroll
        for (int q = 0; q < GQ; ++q) {
            const int32_t t = tid + q * PICK_THREADS;
            gram_w[q] = t < it ? grow[selq[t]] : 0.0;
        }
    }

    // (3) the new column to LDS; slice 0 stores it and g = ||a||^2, b = <a, y>
    float *cols = W.cols + (n * k) * (int64_t)r;
    {
        double g = 0.0, b = 0.0;
        const float *yy = P.y + n * r;
        for (int32_t jb = tid; jb < r4; jb += PICK_THREADS) {
            const float4 a = column_quad<GENERATED>(A, lam, jb);
            reinterpret_cast<float4 *>(a_col)[jb] = a;
            if (slice == 0) {
                if (!P.At_rows)
                    reinterpret_cast<float4 *>(cols + (int64_t)it * r)[jb] = a;
                const float4 yv = reinterpret_cast<const float4 *>(yy)[jb];
                g += (double)a.x * a.x + (double)a.y * a.y + (double)a.z * a.z + (double)a.w * a.w;
                b += (double)a.x * yv.x + (double)a.y * yv.y + (double)a.z * yv.z + (double)a.w * yv.w;
            }
        }
        if (slice == 0) {
            g = wave_sum(g);
            b = wave_sum(b);
            if (lane == 0) {
                s_red[0][wave] = g;
                s_red[1][wave] = b;
            }
        }
    }
    __syncthreads();
    if (slice == 0 && tid == 0) {
        double g = 0.0, b = 0.0;
        for (int u = 0; u < PICK_WAVES; ++u) {
            g += s_red[0][u];
            b += s_red[1][u];
        }
        W.gb[n * 2] = g;
        W.gb[n * 2 + 1] = b;
        P.sel[n * k + it] = lam;
        W.bitmap[n * W.words + (lam >> 5)] |= 1u << (lam & 31);
    }

    // (4) w_t = <A_:lambda_t, a>: from the table of column inner products if there is one, ...
    double *wv = W.wv + n * k;
    const int32_t *selp = P.sel + n * k;
    if (A.gram) {
        if (slice == 0) {
#pragma unroll
            for (int q = 0; q < GQ; ++q) {
                const int32_t t = tid + q * PICK_THREADS;
                if (t < it)
                    wv[t] = gram_w[q];
            }
        }
        return;
    }
    // ... else one wavefront per earlier selection, two rows in flight
    const int32_t gw = slice * PICK_WAVES + wave, GW = nslices * PICK_WAVES;
    for (int32_t t = gw; t < it; t += 2 * GW) {
        const int32_t t2 = t + GW;
        const bool two = t2 < it;
        const int32_t tb = two ? t2 : t;
        const float4 *c0 = reinterpret_cast<const float4 *>(
            P.At_rows ? P.At_rows + (int64_t)selp[t] * r : cols + (int64_t)t * r);
        const float4 *c1 = reinterpret_cast<const float4 *>(
            P.At_rows ? P.At_rows + (int64_t)selp[tb] * r : cols + (int64_t)tb * r);
        double s0 = 0.0, s1 = 0.0;
        for (int32_t jb = lane; jb < r4; jb += 64) {
            const float4 u0 = c0[jb];
            const float4 u1 = c1[jb];
            const float4 a = reinterpret_cast<const float4 *>(a_col)[jb];
            s0 += (double)u0.x * a.x + (double)u0.y * a.y + (double)u0.z * a.z + (double)u0.w * a.w;
            s1 += (double)u1.x * a.x + (double)u1.y * a.y + (double)u1.z * a.z + (double)u1.w * a.w;
        }
        s0 = wave_sum(s0);
        s1 = wave_sum(s1);
        if (lane == 0) {
            wv[t] = s0;
            if (two)
                wv[t2] = s1;
        }
    }
}

template <bool GENERATED, int PICK_THREADS>
__global__ __launch_bounds__(PICK_THREADS) void pick_kernel(MatrixView A, IterArgs P)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    pick_body<GENERATED, PICK_THREADS>(A, P, blockIdx.x, blockIdx.y, gridDim.y, smem);
}

// grid (N, slices); 256 threads (k <= 128) or 1024. dynamic LDS: double w[k]; double fsum[k]; double a[k];
// scratch (the table of shares [wavefronts][k] if it fits, later the partial residuals)
// First the small dense part of App. B in one pass over F: a wavefront takes column t of F (entries
// 0..t, contiguous), forms c_t = <F_:t, w> (coordinate t of the new column in the orthonormal basis
// Q = A_Lambda F) and at once adds c_t F_:t to its share of F c; the shares are then summed in
// wavefront order. Then, in the same workgroup (the dependency is per right-hand side only),
// res = y - A_Lambda x as a column mat-vec in double: a thread owns four measurements; when there are
// fewer such quads than threads, several threads share one and take every G-th column, and their
// parts are added in a fixed order.
// ROWS = rows of F per lane (k <= 64 * ROWS); FLIGHT = columns in flight per wavefront
template <int FACTOR_ROWS, int FLIGHT>
__device__ __forceinline__ void update_body(const IterArgs &P, const int32_t r, const int64_t n, const int slice,
                                            const int nslices, unsigned char *smem)
{
    const int32_t k = P.k, it = P.it;
    double *w_s = reinterpret_cast<double *>(smem);
    double *fsum = w_s + k;
    __shared__ double s_red[2][FACTOR_MAX_THREADS / 64];
    __shared__ double s_gamma, s_coef;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // known to be the same in all lanes: loops over wavefronts stay scalar
    const int nthreads = blockDim.x, nwaves = blockDim.x >> 6;
    const OmpWorkspace &W = P.ws;
    double *F = W.F + n * W.f_stride;
    double *avec = W.avec + n * k;
    // several workgroups (slices) may serve one right-hand side: each repeats the factor pass and takes
    // its share of the residual; slice 0 stores the factor and the solution. The solution is
    // double-buffered so that a late slice still reads the previous iteration's values.
    const bool writer = slice == 0;
    const double *xs = W.xs + (int64_t)((it + 1) & 1) * W.xs_half + n * k;
    double *xs_new = W.xs + (int64_t)(it & 1) * W.xs_half + n * k;

    // everything the update needs from memory besides F is fetched up front (one latency, not four)
    double *a_s = fsum + k;    // coefficients a_0 .. a_{it-1}
    double *scratch = a_s + k; // shares of F c, later partial residuals
    const double gb_g = W.gb[n * 2], gb_b = W.gb[n * 2 + 1];
    const double x_mine = tid < it ? xs[tid] : 0.0; // row tid of the solution (rows >= nthreads: read late)
    for (int32_t t = tid; t < it; t += nthreads) {
        w_s[t] = W.wv[n * k + t];
        a_s[t] = avec[t];
        fsum[t] = 0.0;
    }
    __syncthreads();
    const int nq = (it + 63) >> 6; // 64-row slabs in use
    double facc[FACTOR_ROWS];
#pragma unroll
    for (int q = 0; q < FACTOR_ROWS; ++q)
        facc[q] = 0.0;
    double cc = 0.0, ca = 0.0; // c.c and c.avec over this wavefront's columns
    for (int32_t t0 = wave; t0 < it; t0 += FLIGHT * nwaves) {
        // FLIGHT columns t0, t0 + nwaves, ... in flight: all loads are issued before any is used
        double v[FLIGHT][FACTOR_ROWS], dt[FLIGHT];
#pragma unroll
        for (int c = 0; c < FLIGHT; ++c) {
            const int32_t t = t0 + c * nwaves;
            const double *f = F + (int64_t)(t < it ? t : t0) * k;
#pragma unroll
            for (int q = 0; q < FACTOR_ROWS; ++q) {
                const int32_t u = q * 64 + lane;
                v[c][q] = (q < nq && t < it && u <= t) ? f[u] : 0.0;
            }
        }
#pragma unroll
        for (int c = 0; c < FLIGHT; ++c) {
            double acc = 0.0;
#pragma unroll
            for (int q = 0; q < FACTOR_ROWS; ++q) {
                const int32_t u = q * 64 + lane;
                acc += v[c][q] * ((q < nq && u < it) ? w_s[u] : 0.0);
            }
            dt[c] = __shfl(wave_sum(acc), 0, 64);
        }
#pragma unroll
        for (int c = 0; c < FLIGHT; ++c) {
            const int32_t t = t0 + c * nwaves;
#pragma unroll
            for (int q = 0; q < FACTOR_ROWS; ++q)
                facc[q] += v[c][q] * dt[c];
            cc += dt[c] * dt[c];
            ca += t < it ? dt[c] * a_s[t] : 0.0;
            if (W.cvec && writer && lane == 0 && t < it)
                W.cvec[n * k + t] = dt[c]; // the correlation recurrence combines the earlier image vectors with these
        }
    }
    if (lane == 0) {
        s_red[0][wave] = cc;
        s_red[1][wave] = ca;
    }
    // F c = sum of the wavefronts' shares, added in wavefront order (deterministic): through a
    // [wavefront][k] table when it fits (one barrier), else one wavefront after the other
    if (P.share_table) {
        double *share = scratch;
#pragma unroll
        for (int q = 0; q < FACTOR_ROWS; ++q) {
            const int32_t u = q * 64 + lane;
            if (q < nq && u < it)
                share[wave * k + u] = facc[q];
        }
        __syncthreads();
        for (int32_t u = tid; u < it; u += nthreads) {
            double a = 0.0;
            for (int wv = 0; wv < nwaves; ++wv)
                a += share[wv * k + u];
            fsum[u] = a;
        }
        __syncthreads();
    } else {
        for (int wv = 0; wv < nwaves; ++wv) {
            if (wave == wv) {
#pragma unroll
                for (int q = 0; q < FACTOR_ROWS; ++q) {
                    const int32_t u = q * 64 + lane;
                    if (q < nq && u < it)
                        fsum[u] += facc[q];
                }
            }
            __syncthreads();
        }
    }
    // gamma = 1/sqrt(g - c.c); new coefficient a_it = gamma (b - c.avec)
    if (tid == 0) {
        double tcc = 0.0, tca = 0.0;
        for (int u = 0; u < nwaves; ++u) {
            tcc += s_red[0][u];
            tca += s_red[1][u];
        }
        const double g = gb_g, b = gb_b;
        const double rem = g - tcc;
        const double gamma = rem > 0.0 ? 1.0 / sqrt(rem) : 0.0;
        const double coef = gamma * (b - tca);
        s_gamma = gamma;
        s_coef = coef;
        if (writer) {
            avec[it] = coef;
            F[(int64_t)it * k + it] = gamma;
        }
    }
    __syncthreads();
    const double gamma = s_gamma, coef = s_coef;
    // new column of F: -gamma F c on rows < it, and x <- [x; 0] + coef * F_:it
    // (w and fsum are dead from here: they become x and the float4 offsets of the selected columns)
    double *x_s = w_s;
    int64_t *row_s = reinterpret_cast<int64_t *>(fsum);
    const int32_t r4 = r >> 2;
    for (int32_t u = tid; u <= it; u += nthreads) {
        double xn;
        if (u < it) {
            const double f = -gamma * fsum[u];
            if (writer)
                F[(int64_t)it * k + u] = f;
            xn = (u == tid ? x_mine : xs[u]) + coef * f;
        } else {
            xn = coef * gamma;
        }
        if (writer) {
            xs_new[u] = xn;
            if (it == k - 1)
                P.x[n * k + u] = (float)xn;
        }
        x_s[u] = xn;
        row_s[u] = (P.At_rows ? (int64_t)P.sel[n * k + u] : (int64_t)u) * r4;
    }
    __syncthreads();

    // ---- residual ----
    const float4 *cbase = P.At_rows ? reinterpret_cast<const float4 *>(P.At_rows)
                                    : reinterpret_cast<const float4 *>(W.cols + (n * k) * (int64_t)r);
    // this slice's quads of measurements: [q0, q0 + nq4)
    const int32_t per = (r4 + nslices - 1) / nslices;
    const int32_t q0 = slice * per;
    const int32_t nq4 = q0 >= r4 ? 0 : (r4 - q0 < per ? r4 - q0 : per);
    const int32_t G = (nq4 > 0 && nq4 < nthreads) ? nthreads / nq4 : 1; // threads sharing one quad
    double *parts = scratch;                                              // [G-1][nq4][4]
    for (int32_t jb0 = 0; jb0 < nq4; jb0 += nthreads) {
        const int32_t jl = G > 1 ? tid % nq4 : jb0 + tid; // quad within the slice
        const int32_t jb = q0 + jl;
        const int32_t g = G > 1 ? tid / nq4 : 0;
        const bool active = jl < nq4 && g < G;
        double e0 = 0.0, e1 = 0.0, e2 = 0.0, e3 = 0.0;
        if (active) {
            if (g == 0) {
                const float4 yv = reinterpret_cast<const float4 *>(P.y + n * r)[jb];
                e0 = yv.x;
                e1 = yv.y;
                e2 = yv.z;
                e3 = yv.w;
            }
            const float4 *cj = cbase + jb;
            int32_t t = g;
            for (; t + 7 * G <= it; t += 8 * G) {
                float4 u[8];
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    u[q] = cj[row_s[t + q * G]];
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const double xt = x_s[t + q * G];
                    e0 -= xt * u[q].x;
                    e1 -= xt * u[q].y;
                    e2 -= xt * u[q].z;
                    e3 -= xt * u[q].w;
                }
            }
            for (; t <= it; t += G) {
                const float4 u = cj[row_s[t]];
                const double xt = x_s[t];
                e0 -= xt * u.x;
                e1 -= xt * u.y;
                e2 -= xt * u.z;
                e3 -= xt * u.w;
            }
        }
        if (G > 1) {
            if (active && g > 0) {
                double *o = parts + ((int64_t)(g - 1) * nq4 + jl) * 4;
                o[0] = e0;
                o[1] = e1;
                o[2] = e2;
                o[3] = e3;
            }
            __syncthreads();
            if (active && g == 0) {
                for (int32_t gg = 1; gg < G; ++gg) {
                    const double *o = parts + ((int64_t)(gg - 1) * nq4 + jl) * 4;
                    e0 += o[0];
                    e1 += o[1];
                    e2 += o[2];
                    e3 += o[3];
                }
            }
        }
        if (active && g == 0) {
            double *ro = W.res64 + n * r + 4 * jb;
            ro[0] = e0;
            ro[1] = e1;
            ro[2] = e2;
            ro[3] = e3;
            if (P.res_split) {
                uint16_t h[4], l[4];
                split_bf16_1((float)e0, h[0], l[0]);
                split_bf16_1((float)e1, h[1], l[1]);
                split_bf16_1((float)e2, h[2], l[2]);
                split_bf16_1((float)e3, h[3], l[3]);
                unsigned char *o = reinterpret_cast<unsigned char *>(W.res16) + n * ((int64_t)r * 4) + split32_quad_offset(jb);
                *reinterpret_cast<uint2 *>(o) = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
                *reinterpret_cast<uint2 *>(o + 64) = make_uint2(l[0] | ((uint32_t)l[1] << 16), l[2] | ((uint32_t)l[3] << 16));
            } else {
                reinterpret_cast<float4 *>(W.res32 + n * r)[jb] =
                    make_float4((float)e0, (float)e1, (float)e2, (float)e3);
            }
        }
    }
}

template <int FACTOR_ROWS, int FLIGHT>
__global__ __launch_bounds__(FACTOR_MAX_THREADS) void update_kernel(IterArgs P, int32_t r)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    update_body<FACTOR_ROWS, FLIGHT>(P, r, blockIdx.x, blockIdx.y, gridDim.y, smem);
}

// Least-squares fit of a second right-hand side on the support already found (shared-support
// recovery): z = (A_L^T A_L)^-1 A_L^T y_fit = F (F^T (A_L^T y_fit)) with the finished inverse
// Cholesky factor F of the support (App. B), all in double. grid N; dynamic LDS: double b[k], u[k]
constexpr int REFIT_THREADS = 1024;
__global__ __launch_bounds__(REFIT_THREADS) void refit_kernel(IterArgs P, const float *__restrict__ y_fit,
                                                              float *__restrict__ z, int32_t r)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    double *b_s = reinterpret_cast<double *>(smem);
    double *u_s = b_s + P.k;
    const int32_t k = P.k, r4 = r >> 2;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // known to be the same in all lanes: loops over wavefronts stay scalar
    constexpr int NW = REFIT_THREADS / 64;
    const int64_t n = blockIdx.x;
    const OmpWorkspace &W = P.ws;
    const int32_t *selp = P.sel + n * k;
    const float *cols = W.cols + (n * k) * (int64_t)r;
    const float4 *yy = reinterpret_cast<const float4 *>(y_fit + n * r);
    // b_t = <A_:lambda_t, y_fit>, one wavefront per selected column
    for (int32_t t = wave; t < k; t += NW) {
        const float4 *c = reinterpret_cast<const float4 *>(
            P.At_rows ? P.At_rows + (int64_t)selp[t] * r : cols + (int64_t)t * r);
        double acc = 0.0;
        for (int32_t jb = lane; jb < r4; jb += 64) {
            const float4 a = c[jb];
            const float4 yv = yy[jb];
            acc += (double)a.x * yv.x + (double)a.y * yv.y + (double)a.z * yv.z + (double)a.w * yv.w;
        }
        acc = wave_sum(acc);
        if (lane == 0)
            b_s[t] = acc;
    }
    __syncthreads();
    // u = F^T b: column t of F (rows 0..t, contiguous) against b
    const double *F = W.F + n * W.f_stride;
    for (int32_t t = wave; t < k; t += NW) {
        const double *f = F + (int64_t)t * k;
        double acc = 0.0;
        for (int32_t v = lane; v <= t; v += 64)
            acc += f[v] * b_s[v];
        acc = wave_sum(acc);
        if (lane == 0)
            u_s[t] = acc;
    }
    __syncthreads();
    // z = F u: row v of F holds the entries of columns t >= v
    for (int32_t v = tid; v < k; v += REFIT_THREADS) {
        double acc = 0.0;
        for (int32_t t = v; t < k; ++t)
            acc += F[(int64_t)t * k + v] * u_s[t];
        z[n * k + v] = (float)acc;
    }
}

// ---------------------------------------------------------------------------------------------
// The whole recovery of a small batch in ONE launch (at most SMALL_MAX_RHS right-hand sides, k <= 64,
// k r <= 16384, resident rows of At that fit the workgroups' LDS together). With so few right-hand sides every
// kernel of the iteration is a few microseconds of work behind a launch, and three dependent launches per
// iteration are the cost (27 us per iteration for one chunk of d = 4096, r = 256). Here G + N workgroups stay
// resident for all k iterations and nothing but a few words per iteration travels through memory:
//   workers (G workgroups)   each keeps a slice of rows of At in LDS for the whole call (the matrix is read from
//                            memory once, not once per iteration); per iteration the correlations of its rows
//                            with the N residuals on the vector ALUs (four lanes per row, float accumulation;
//                            with so few right-hand sides there is nothing for the matrix cores), scaled and
//                            masked; the two best keys per right-hand side go out, tagged with the iteration
//   owners (N workgroups)    each keeps the whole least-squares state of one right-hand side in LDS: the selected
//                            columns, the inverse Cholesky factor, coefficients, solution and the double
//                            residual. Per iteration: collect the keys of all workers, select (float maximum,
//                            double re-scoring of the near-maximal candidates: the same routine as pick_kernel),
//                            fetch the new column, App. B's factor update and the residual in double (the
//                            formulas of update_kernel); the float residual and the selected position go out
//                            as tagged words
//   workers                  collect the new residuals and selected positions, and go on.
// There is no barrier: every word that crosses between workgroups is 64 bits wide, carries the number of the
// iteration it belongs to, and is stored and loaded with device-scope atomics (which pass by the caches that
// are not coherent between XCDs), so a reader polls the data itself until every word shows the tag it waits
// for - one trip to the memory side per exchange, two per iteration. A writer cannot overwrite a word that a
// slower workgroup still needs: the keys of iteration it + 1 are written after the residual of iteration it has
// been read, and that residual is replaced only after all keys of iteration it + 1 have arrived.
// All workgroups must be resident at once: there are at most SMALL_MAX_GROUPS + SMALL_MAX_RHS and each fits a CU,
// so they are whenever the kernel gets the device; if some word does not arrive within SMALL_SPIN_LIMIT polls
// (seconds: some other work holds the CUs), the poller raises the give-up flag in the workspace, every workgroup
// leaves at its next poll, and the selected positions of the unfinished right-hand sides are set to -1 (values
// 0, which sgc_apply skips) - the grid always drains.
constexpr uint32_t SMALL_SPIN_LIMIT = 1u << 22;
constexpr int SMALL_THREADS = 256;
constexpr int SMALL_ROW_PAD = 4; // floats between rows in LDS: rows read side by side by a wavefront fall in different banks
constexpr int SMALL_MAX_K = 64;
constexpr int SMALL_MAX_KR = 16384;

// key as the selection reads it (score bits, ~position) <-> the same with the iteration's tag in bits 24..31 of
// the low word (positions are below 2^24 here, so those bits of ~position are all ones); 0 = no candidate
__device__ __forceinline__ uint64_t small_tag_key(uint64_t key, uint32_t tag)
{
    return (key & 0xffffffff00ffffffull) | ((uint64_t)tag << 24);
}
__device__ __forceinline__ uint64_t small_untag_key(uint64_t word)
{
    const uint64_t body = word & 0xffffffff00ffffffull;
    return body == 0ull ? 0ull : (body | 0xff000000ull);
}

// polls until `fetch` (which loads this thread's words and says whether all of them carry the tag) holds in
// every thread of the workgroup; false if the launch gives up
template <typename Fetch>
__device__ __forceinline__ bool small_wait(uint32_t *giveup, Fetch &&fetch)
{
    for (uint32_t spins = 0;; ++spins) {
        const bool ok = fetch();
        if (__syncthreads_and(ok ? 1 : 0))
            return true;
        if ((spins & 15u) == 15u) { // now and then: has the launch given up, or is it time to
            const bool stop = spins > SMALL_SPIN_LIMIT ||
                              __hip_atomic_load(giveup, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
            if (__syncthreads_or(stop ? 1 : 0)) {
                if (threadIdx.x == 0)
                    __hip_atomic_store(giveup, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                return false;
            }
        }
    }
}

// grid G + N: workgroups 0 .. G-1 are workers, G .. G+N-1 owners. dynamic LDS, workers: float rows[rows_per_group]
// [r + SMALL_ROW_PAD]; float inv[rows_per_group rounded up to 4]; float res[N][r]; unsigned char taken[N][rows_per_group].
// owners: double F[k][k]; double res[r]; double w[k], c[k], fc[k], x[k], a[k]; float y[r]; float cols[k][r]
__global__ __launch_bounds__(SMALL_THREADS) void omp_small_kernel(MatrixView A, IterArgs P, int32_t N, int32_t G,
                                                                  int32_t rows_per_group)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int32_t r = A.r, r4 = r >> 2, k = P.k, d = A.d;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6); // known to be the same in all lanes: loops over wavefronts stay scalar
    const int g = blockIdx.x;
    const OmpWorkspace &W = P.ws;
    uint32_t *giveup = W.sync;
    const int32_t xw = r + SMALL_XCHG_PAD; // exchange words per right-hand side

    if (g >= G) {
        // =============================== owner of right-hand side n ===============================
        const int64_t n = g - G;
        __shared__ uint64_t s_part[2 * SMALL_MAX_GROUPS]; // the keys of this right-hand side, all workers
        __shared__ double s_red[2][SMALL_THREADS / 64];
        __shared__ double s_gamma, s_coef;
        double *F_s = reinterpret_cast<double *>(smem); // column t at F_s[t * k + u], u <= t
        double *res_s = F_s + (size_t)k * k;
        double *w_s = res_s + r;
        double *c_s = w_s + k;
        double *fc_s = c_s + k;
        double *x_s = fc_s + k;
        double *av_s = x_s + k;
        float *y_s = reinterpret_cast<float *>(av_s + k);
        float *cols_s = y_s + r;
        const uint64_t *mine = W.partial + n * (int64_t)G * 2;
        uint64_t *out = W.xchg + n * xw;
        for (int32_t j = tid; j < r; j += SMALL_THREADS) {
            const float v = P.y[n * r + j];
            y_s[j] = v;
            res_s[j] = (double)v;
        }
        __syncthreads();
        bool aborted = false;
        for (int32_t it = 0; it < k; ++it) {
            const uint32_t tag = (uint32_t)(it + 1);
            if (!small_wait(giveup, [&]() {
                    bool ok = true;
                    for (int32_t e = tid; e < 2 * G; e += SMALL_THREADS) {
                        const uint64_t word = __hip_atomic_load(mine + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        ok = ok && (uint32_t)((word >> 24) & 0xffu) == tag;
                        s_part[e] = small_untag_key(word);
                    }
                    return ok;
                })) {
                aborted = true;
                break;
            }
            const int32_t lam = select_lambda<false, SMALL_THREADS>(A, s_part, 2 * G, res_s);
            // the new column: to LDS, with g = ||a||^2 and b = <a, y> in double
            {
                double gg = 0.0, bb = 0.0;
                float *dst = cols_s + (size_t)it * r;
                for (int32_t jb = tid; jb < r4; jb += SMALL_THREADS) {
                    const float4 a = reinterpret_cast<const float4 *>(P.At_rows + (int64_t)lam * r)[jb];
                    reinterpret_cast<float4 *>(dst)[jb] = a;
                    const float4 yv = reinterpret_cast<const float4 *>(y_s)[jb];
                    gg += (double)a.x * a.x + (double)a.y * a.y + (double)a.z * a.z + (double)a.w * a.w;
                    bb += (double)a.x * yv.x + (double)a.y * yv.y + (double)a.z * yv.z + (double)a.w * yv.w;
                }
                gg = wave_sum(gg);
                bb = wave_sum(bb);
                if (lane == 0) {
                    s_red[0][wave] = gg;
                    s_red[1][wave] = bb;
                }
            }
            __syncthreads();
            // w_t = <A_:lambda_t, a> for the earlier selections, one wavefront per column
            {
                const float4 *an = reinterpret_cast<const float4 *>(cols_s + (size_t)it * r);
                for (int32_t t = wave; t < it; t += SMALL_THREADS / 64) {
                    const float4 *ct = reinterpret_cast<const float4 *>(cols_s + (size_t)t * r);
                    double acc = 0.0;
                    for (int32_t jb = lane; jb < r4; jb += 64) {
                        const float4 u = ct[jb], a = an[jb];
                        acc += (double)u.x * a.x + (double)u.y * a.y + (double)u.z * a.z + (double)u.w * a.w;
                    }
                    acc = wave_sum(acc);
                    if (lane == 0)
                        w_s[t] = acc;
                }
            }
            __syncthreads();
            // App. B: c = F^H w (coordinates of the new column in the orthonormal basis), F c, gamma, the new
            // coefficient, the new column of F and x = F a
            if (tid < it) {
                double acc = 0.0;
                for (int32_t u = 0; u <= tid; ++u)
                    acc += F_s[(size_t)tid * k + u] * w_s[u];
                c_s[tid] = acc;
            }
            __syncthreads();
            if (tid < it) {
                double acc = 0.0;
                for (int32_t t = tid; t < it; ++t)
                    acc += F_s[(size_t)t * k + tid] * c_s[t];
                fc_s[tid] = acc;
            }
            if (tid == 0) {
                double gg = 0.0, bb = 0.0, cc = 0.0, ca = 0.0;
                for (int u = 0; u < SMALL_THREADS / 64; ++u) {
                    gg += s_red[0][u];
                    bb += s_red[1][u];
                }
                for (int32_t t = 0; t < it; ++t) {
                    cc += c_s[t] * c_s[t];
                    ca += c_s[t] * av_s[t];
                }
                const double rem = gg - cc;
                const double gamma = rem > 0.0 ? 1.0 / sqrt(rem) : 0.0;
                const double coef = gamma * (bb - ca);
                av_s[it] = coef;
                F_s[(size_t)it * k + it] = gamma;
                s_gamma = gamma;
                s_coef = coef;
            }
            __syncthreads();
            {
                const double gamma = s_gamma, coef = s_coef;
                if (tid < it) {
                    const double f = -gamma * fc_s[tid];
                    F_s[(size_t)it * k + tid] = f;
                    x_s[tid] += coef * f;
                } else if (tid == it) {
                    x_s[it] = coef * gamma;
                }
            }
            __syncthreads();
            // residual y - A_Lambda x in double; its float copy goes out in tagged words
            {
                const uint64_t tagw = (uint64_t)tag << 32;
                for (int32_t j = tid; j < r; j += SMALL_THREADS) {
                    double e = (double)y_s[j];
                    for (int32_t t = 0; t <= it; ++t)
                        e -= x_s[t] * (double)cols_s[(size_t)t * r + j];
                    res_s[j] = e;
                    __hip_atomic_store(out + j, tagw | __float_as_uint((float)e), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                if (tid == 0) {
                    P.sel[n * k + it] = lam;
                    __hip_atomic_store(out + r, tagw | (uint32_t)lam, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            __syncthreads();
        }
        if (aborted) { // this right-hand side was not finished
            for (int32_t e = tid; e < k; e += SMALL_THREADS) {
                P.sel[n * k + e] = -1;
                P.x[n * k + e] = 0.f;
            }
            return;
        }
        // results: x, and the factor and coefficients where the batched kernels keep them (the shared-support
        // fit of a second right-hand side reads the factor from there)
        for (int32_t u = tid; u < k; u += SMALL_THREADS) {
            P.x[n * k + u] = (float)x_s[u];
            W.avec[n * k + u] = av_s[u];
        }
        double *Fg = W.F + n * W.f_stride;
        for (int32_t e = tid; e < k * k; e += SMALL_THREADS) {
            const int32_t t = e / k, u = e - t * k;
            if (u <= t)
                Fg[e] = F_s[e];
        }
        return;
    }

    // ======================================== worker ========================================
    __shared__ uint64_t s_keys[SMALL_THREADS / 64][SMALL_MAX_RHS][2];
    const int32_t ld = r + SMALL_ROW_PAD;
    const int32_t row0 = g * rows_per_group;
    const int32_t rows = row0 >= d ? 0 : (d - row0 < rows_per_group ? d - row0 : rows_per_group);
    float *a_rows = reinterpret_cast<float *>(smem);
    float *inv = a_rows + (size_t)rows_per_group * ld;
    float *res = inv + ((rows_per_group + 3) & ~3); // keeps the residuals 16-byte aligned
    unsigned char *taken = reinterpret_cast<unsigned char *>(res + (size_t)N * r);

    // the workgroup's rows of At and their reciprocal norms, once for the whole call; the residuals = y
    for (int32_t e = tid; e < rows * r4; e += SMALL_THREADS) {
        const int32_t i = e / r4, jb = e - i * r4;
        *reinterpret_cast<float4 *>(a_rows + (size_t)i * ld + 4 * jb) =
            reinterpret_cast<const float4 *>(P.At_rows + (int64_t)(row0 + i) * r)[jb];
    }
    for (int32_t i = tid; i < rows; i += SMALL_THREADS)
        inv[i] = A.inv_colnorm[row0 + i];
    for (int32_t e = tid; e < N * r4; e += SMALL_THREADS)
        reinterpret_cast<float4 *>(res)[e] = reinterpret_cast<const float4 *>(P.y)[e];
    for (int32_t e = tid; e < N * rows_per_group; e += SMALL_THREADS)
        taken[e] = 0;
    __syncthreads();

    // a wavefront takes 16 rows at a time, four lanes per row, each lane a quarter of the depth
    const int sub = lane >> 2, part = lane & 3;
    for (int32_t it = 0; it < k; ++it) {
        const uint32_t tag = (uint32_t)(it + 1);
        uint64_t best[SMALL_MAX_RHS], second[SMALL_MAX_RHS];
#pragma unroll
        for (int u = 0; u < SMALL_MAX_RHS; ++u)
            best[u] = second[u] = 0;
        for (int32_t i0 = wave * 16; i0 < rows; i0 += (SMALL_THREADS / 64) * 16) {
            const int32_t i = i0 + sub;
            const bool live = i < rows;
            const float4 *ar = reinterpret_cast<const float4 *>(a_rows + (size_t)(live ? i : i0) * ld);
            float acc[SMALL_MAX_RHS];
#pragma unroll
            for (int u = 0; u < SMALL_MAX_RHS; ++u)
                acc[u] = 0.f;
            for (int32_t jb = part; jb < r4; jb += 4) {
                const float4 a = ar[jb];
#pragma unroll
                for (int u = 0; u < SMALL_MAX_RHS; ++u) {
                    if (u < N) {
                        const float4 b = reinterpret_cast<const float4 *>(res + (size_t)u * r)[jb];
                        acc[u] = __builtin_fmaf(a.x, b.x, acc[u]);
                        acc[u] = __builtin_fmaf(a.y, b.y, acc[u]);
                        acc[u] = __builtin_fmaf(a.z, b.z, acc[u]);
                        acc[u] = __builtin_fmaf(a.w, b.w, acc[u]);
                    }
                }
            }
            const float in = live ? inv[i] : 0.f;
#pragma unroll
            for (int u = 0; u < SMALL_MAX_RHS; ++u) {
                if (u < N) {
                    float v = acc[u];
                    v += __shfl_xor(v, 1, 64);
                    v += __shfl_xor(v, 2, 64);
                    const float score = fabsf(v) * in;
                    const bool ok = live && part == 0 && !taken[u * rows_per_group + (live ? i : 0)];
                    const uint64_t key = ok ? (((uint64_t)__float_as_uint(score) << 32) | (uint64_t)(0xffffffffu - (uint32_t)(row0 + i))) : 0ull;
                    const uint64_t lo = key < best[u] ? key : best[u];
                    best[u] = key < best[u] ? best[u] : key;
                    second[u] = lo < second[u] ? second[u] : lo;
                }
            }
        }
        // the two best of the wavefront's lanes, then of the workgroup's wavefronts
#pragma unroll
        for (int u = 0; u < SMALL_MAX_RHS; ++u) {
            if (u < N) {
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) {
                    const uint64_t ob = shfl_xor_u64(best[u], off), os = shfl_xor_u64(second[u], off);
                    const uint64_t hi = ob > best[u] ? ob : best[u];
                    const uint64_t mid = ob > best[u] ? best[u] : ob;
                    const uint64_t s2 = os > second[u] ? os : second[u];
                    best[u] = hi;
                    second[u] = mid > s2 ? mid : s2;
                }
                if (lane == 0) {
                    s_keys[wave][u][0] = best[u];
                    s_keys[wave][u][1] = second[u];
                }
            }
        }
        __syncthreads();
        if (tid < N) {
            uint64_t b = 0, sc = 0;
            for (int wv = 0; wv < SMALL_THREADS / 64; ++wv) {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const uint64_t key = s_keys[wv][tid][h];
                    const uint64_t lo = key < b ? key : b;
                    b = key < b ? b : key;
                    sc = lo < sc ? sc : lo;
                }
            }
            uint64_t *o = W.partial + ((int64_t)tid * G + g) * 2;
            __hip_atomic_store(o, small_tag_key(b, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(o + 1, small_tag_key(sc, tag), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (it + 1 == k)
            break; // nobody needs the last residual
        // the new residuals and selected positions
        if (!small_wait(giveup, [&]() {
                bool ok = true;
                for (int32_t e = tid; e < N * (r + 1); e += SMALL_THREADS) {
                    const int32_t u = e / (r + 1), j = e - u * (r + 1);
                    const uint64_t word = __hip_atomic_load(W.xchg + (int64_t)u * xw + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const bool mine_ok = (uint32_t)(word >> 32) == tag;
                    ok = ok && mine_ok;
                    if (mine_ok) {
                        if (j < r) {
                            res[(size_t)u * r + j] = __uint_as_float((uint32_t)word);
                        } else {
                            const int32_t lam = (int32_t)(uint32_t)word - row0;
                            if (lam >= 0 && lam < rows)
                                taken[u * rows_per_group + lam] = 1;
                        }
                    }
                }
                return ok;
            }))
            break;
    }
}

// ---------------------------------------------------------------------------------------------
// Host side of the recovery.
struct OmpPlan {
    bool panels;     // generated A produced into ws.panel and consumed from there
    bool pipelined;  // full tiles of stored rows: corr_pipelined_kernel
    bool screen;     // resident rows that fit ws.a16 and the matrix asks for it: corr_split_kernel, or
    bool screen_pipelined; // on full tiles the bfloat16 form of corr_pipelined_kernel
    int32_t tiles_m; // position tiles of the contraction in use (stride of ws.partial)
    MatrixView Apick; // the view pick_kernel fetches columns from
    size_t pick_smem, factor_smem;
    bool factor_share_table; // update_kernel sums its wavefronts' shares through an LDS table
    bool narrow;     // r <= 16 on resident rows: corr_narrow_kernel
    bool recurrence; // the correlation vector is updated by App. B's recurrence instead of contracted anew
    bool one_stream; // everything on the caller's stream (no library-owned stream or events are touched)
};

// the workspace as seen by the right-hand sides [n0, ...): every per-right-hand-side array shifted
static OmpWorkspace shift_workspace(const OmpWorkspace &ws, int32_t n0, int32_t r, int32_t k, int32_t tiles_m)
{
    OmpWorkspace w = ws;
    w.tiles_m = tiles_m;
    w.res64 += (int64_t)n0 * r;
    w.F += (int64_t)n0 * ws.f_stride;
    w.avec += (int64_t)n0 * k;
    w.xs += (int64_t)n0 * k;
    w.res32 += (int64_t)n0 * r;
    w.res16 += (int64_t)n0 * 2 * r;
    w.cols += (int64_t)n0 * k * r;
    // ws.tiles_m is the capacity the workspace was carved for: a half's keys start at the same place whatever
    // tiling its current producer uses (the two producers of the hybrid recovery tile differently)
    w.partial += (int64_t)n0 * ws.tiles_m * 2;
    w.bitmap += (int64_t)n0 * ws.words;
    w.wv += (int64_t)n0 * k;
    w.gb += (int64_t)n0 * 2;
    if (w.xchg)
        w.xchg += (int64_t)n0 * (r + SMALL_XCHG_PAD);
    if (w.rc_p) { // the recurrence's arrays
        w.rc_p += (int64_t)n0 * ws.rc_d;
        w.rc_B += (int64_t)n0 * ws.rc_head * ws.rc_d;
        w.cvec += (int64_t)n0 * k;
    }
    return w;
}

// One iteration for Ng right-hand sides whose arrays start at y / sel / x / w, enqueued on s:
// the contraction ...
static hipError_t omp_contraction(const OmpPlan &pl, const MatrixView &A, int32_t Ng, const OmpWorkspace &w,
                                  hipStream_t s)
{
    ProfileScope prof(KC_CORR, s);
    hipError_t e = hipSuccess;
    if (pl.panels) {
        for (int32_t p0 = 0; p0 < A.d && e == hipSuccess; p0 += w.panel_rows) {
            const int32_t rows = A.d - p0 < w.panel_rows ? A.d - p0 : w.panel_rows;
            if (w.panel_rows < A.d) { // a matrix larger than the panel is refilled panel by panel
                e = launch_matrix_fill(A.key0, A.key1, A.scale, A.r, p0, rows, w.panel, s, KC_FILL);
                if (e != hipSuccess)
                    break;
            }
            MatrixView Ap = A;
            Ap.generated = 0;
            Ap.At = w.panel;
            Ap.row0 = p0;
            if (pl.screen) {
                // a whole-matrix panel was split once per call; a refilled panel is split after each fill
                const bool whole = w.panel_rows >= A.d;
                if (!whole)
                    launch_split_rows(w.panel, rows, A.r, w.a16, s);
                e = corr_screen_launch(pl.screen_pipelined, Ap, w.a16, rows, Ng, w, pl.tiles_m, s);
            } else {
                e = pl.narrow      ? corr_narrow_launch(Ap, rows, w.res32, Ng, w, pl.tiles_m, s)
                    : pl.pipelined ? corr_pipelined_launch(Ap, rows, w.res32, Ng, w, pl.tiles_m, s)
                                   : corr_general_launch(false, Ap, rows, w.res32, Ng, w, pl.tiles_m, s);
            }
        }
    } else if (A.generated) {
        e = corr_general_launch(true, A, A.d, w.res32, Ng, w, pl.tiles_m, s);
    } else {
        e = pl.narrow      ? corr_narrow_launch(A, A.d, w.res32, Ng, w, pl.tiles_m, s)
            : pl.screen    ? corr_screen_launch(pl.screen_pipelined, A, w.a16, A.d, Ng, w, pl.tiles_m, s)
            : pl.pipelined ? corr_pipelined_launch(A, A.d, w.res32, Ng, w, pl.tiles_m, s)
                           : corr_general_launch(false, A, A.d, w.res32, Ng, w, pl.tiles_m, s);
    }
    return e;
}

// ... then the selection and the least-squares update
static void omp_select_update(const OmpPlan &pl, const MatrixView &A, const float *y, int32_t Ng, int32_t k,
                              int32_t it, int32_t *sel, float *x, const OmpWorkspace &w, hipStream_t s)
{
    ProfileScope prof(KC_SELECT, s);
    // short columns: two wavefronts per right-hand side keep their lanes busy and let sixteen workgroups
    // share a CU, which hides the chain of dependent loads this kernel consists of
    const bool narrow = A.r <= 512 && k <= 128;
    int slices = 2048 / Ng;
    slices = slices < 1 ? 1 : (slices > 8 ? 8 : slices);
    if (pl.Apick.gram)
        slices = 1; // no pass over the selected columns to spread
    const dim3 pgrid((unsigned)Ng, (unsigned)slices);
    IterArgs P{y, k, it, sel, x, w, pl.Apick.generated ? nullptr : pl.Apick.At, pl.factor_share_table ? 1 : 0,
               pl.screen ? 1 : 0};
    if (narrow) {
        if (pl.Apick.generated)
            pick_kernel<true, PICK_THREADS_NARROW><<<pgrid, PICK_THREADS_NARROW, pl.pick_smem, s>>>(pl.Apick, P);
        else
            pick_kernel<false, PICK_THREADS_NARROW><<<pgrid, PICK_THREADS_NARROW, pl.pick_smem, s>>>(pl.Apick, P);
    } else {
        if (pl.Apick.generated)
            pick_kernel<true, PICK_THREADS_WIDE><<<pgrid, PICK_THREADS_WIDE, pl.pick_smem, s>>>(pl.Apick, P);
        else
            pick_kernel<false, PICK_THREADS_WIDE><<<pgrid, PICK_THREADS_WIDE, pl.pick_smem, s>>>(pl.Apick, P);
    }
    // One workgroup per right-hand side, two when there are so few that half the chip would idle
    // (each repeats the factor pass and takes half of the residual). More slices were measured
    // slower: the repeated passes over F cost more than the wider residual pass saves.
    const dim3 ugrid((unsigned)Ng, Ng <= 128 ? 2u : 1u);
    if (k <= 128)
        update_kernel<2, 4><<<ugrid, 256, pl.factor_smem, s>>>(P, A.r);
    else if (k <= 256)
        update_kernel<4, 6><<<ugrid, FACTOR_MAX_THREADS, pl.factor_smem, s>>>(P, A.r);
    else
        update_kernel<16, 1><<<ugrid, FACTOR_MAX_THREADS, pl.factor_smem, s>>>(P, A.r);
}

// Whether a recovery is served by the single-launch kernel, and its shape: at most SMALL_MAX_RHS right-hand sides,
// resident rows without any option, and a matrix whose rows fit the LDS of at most SMALL_MAX_GROUPS workgroups
// (96 KiB of rows each at most; 64 KiB slices are preferred), k and k r small enough for an owner's LDS. The
// limits are where it was measured to win: an exchange between workgroups on different XCDs costs about 3.5 us,
// two per iteration, the correlation phase 1.5 us, the owner's work about 5 us: 14 us against 27 us per
// iteration for three dependent launches. With 8 right-hand sides or 256 workers the launches are no slower.
struct SmallPlan {
    int32_t groups, rows_per_group; // workers and their rows of At
    size_t smem;
};
static int device_cu_count()
{
    static int count[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
        return 0;
    if (count[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = -1;
        count[dev] = n;
    }
    return count[dev] > 0 ? count[dev] : 0;
}
static bool small_plan(const OmpPlan &pl, int32_t N, int32_t k, SmallPlan &sp)
{
    const MatrixView &A = pl.Apick;
    if (N > SMALL_MAX_RHS || A.generated || A.gram || pl.screen || pl.recurrence || pl.narrow || k > SMALL_MAX_K ||
        A.r > 2048 || (int64_t)k * A.r > SMALL_MAX_KR || (int64_t)N * A.r > 8192 || A.d >= (1 << 24) ||
        (A.flags & SGC_MATRIX_FLAG_MULTI_LAUNCH))
        return false;
    int cus = device_cu_count() - N; // the owners take a CU each
    if (cus > SMALL_MAX_GROUPS)
        cus = SMALL_MAX_GROUPS;
    if (cus < 8)
        return false;
    const int64_t row_bytes = (int64_t)(A.r + SMALL_ROW_PAD) * 4; // as laid out in LDS
    int64_t rows_per_group = (64 * 1024) / row_bytes;
    if (rows_per_group < 1)
        rows_per_group = 1;
    int64_t groups = ((int64_t)A.d + rows_per_group - 1) / rows_per_group;
    if (groups > cus) { // larger slices, up to 96 KiB
        groups = cus;
        rows_per_group = ((int64_t)A.d + groups - 1) / groups;
        if (rows_per_group * row_bytes > 96 * 1024)
            return false;
    }
    if (groups < 8 && A.d >= 8) { // a short matrix: a few workers still, so that the rows are scored side by side
        groups = 8;
        rows_per_group = ((int64_t)A.d + groups - 1) / groups;
    }
    groups = ((int64_t)A.d + rows_per_group - 1) / rows_per_group; // no worker without rows
    const size_t worker = (size_t)rows_per_group * row_bytes + (size_t)((rows_per_group + 3) & ~(int64_t)3) * 4 +
                          (size_t)N * A.r * 4 + (size_t)N * rows_per_group;
    const size_t owner = sizeof(double) * ((size_t)k * k + A.r + 5 * (size_t)k) + sizeof(float) * ((size_t)A.r + (size_t)k * A.r);
    sp.groups = (int32_t)groups;
    sp.rows_per_group = (int32_t)rows_per_group;
    sp.smem = ((worker > owner ? worker : owner) + 15) & ~(size_t)15;
    return sp.smem <= 150 * 1024;
}

// A second stream (default priority) and two events per device, created on first use, so that the
// two halves of a large batch can run their iterations side by side: while one half is in its
// memory-bound selection / update kernels the other half's contraction keeps the matrix cores busy.
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    bool ok = false, tried = false;
};
static SideStream *side_stream()
{
    static SideStream per_device[64];
    static std::mutex mu; // creation is guarded; the stream itself is still shared by all callers on the device
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
        return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    SideStream &ss = per_device[dev];
    if (!ss.tried) {
        ss.tried = true;
        ss.ok = hipStreamCreateWithFlags(&ss.stream, hipStreamNonBlocking) == hipSuccess &&
                hipEventCreateWithFlags(&ss.fork, hipEventDisableTiming) == hipSuccess &&
                hipEventCreateWithFlags(&ss.join, hipEventDisableTiming) == hipSuccess;
    }
    return ss.ok ? &ss : nullptr;
}

static hipError_t omp_iterations(const OmpPlan &pl, bool whole_matrix_panel, const float *y, int32_t N,
                                 const MatrixView &A, int32_t k, int32_t *sel, float *x, const OmpWorkspace &ws,
                                 hipStream_t s);

hipError_t launch_omp(const float *y, int32_t N, const MatrixView &A, int32_t k, int32_t *sel, float *x,
                      const OmpWorkspace &ws, hipStream_t s, const float *y_fit, float *z, bool recurrence,
                      bool one_stream)
{
    // A generated matrix is written out once per call when the workspace holds a panel for all of it (at
    // most 64 MiB, or the whole-matrix option). Otherwise it is regenerated inside the contraction when few
    // right-hand-side tiles share it (fewer than 1024 right-hand sides: every tile of 256 regenerates all
    // of A); with many tiles it is produced panel by panel into a cache-sized scratch in every iteration,
    // and consumed from there.
    // Stored rows in full tiles take the pipelined kernel (256-row tiles), everything else the
    // general one (128-row tiles).
    OmpPlan pl{};
    pl.panels = A.generated && (ws.panel_rows >= A.d || (N + CORR_BN - 1) / CORR_BN >= 8);
    pl.pipelined = (!A.generated || pl.panels) && corr_pipelined_ok(A, N, ws.panel_rows);
    // the bfloat16 screening contraction needs resident rows; a matrix regenerated inside the
    // contraction keeps the float kernel (its time is the generator's anyway)
    pl.screen = (A.flags & SGC_MATRIX_FLAG_SCREEN_BF16) && A.r % 32 == 0 &&
                (A.generated ? pl.panels && ws.a16_rows >= (ws.panel_rows < A.d ? ws.panel_rows : A.d)
                             : ws.a16_rows >= A.d);
    pl.screen_pipelined = pl.screen && N > 64 && corr_pipelined_ok(A, N, ws.panel_rows);
    if (pl.screen)
        pl.pipelined = false;
    pl.tiles_m = pl.pipelined || pl.screen_pipelined ? A.d / CORRP_BM : corr_tiles_m(A.d);
    // very few measurements: neither the matrix cores nor the bfloat16 copy have anything to offer
    pl.narrow = (!A.generated || pl.panels) && corr_narrow_ok(A.r, N);
    if (pl.narrow) {
        pl.pipelined = pl.screen = pl.screen_pipelined = false;
        pl.tiles_m = (A.d + 255) / 256;
    }
    pl.recurrence = recurrence;
    pl.one_stream = one_stream;
    if (recurrence && (!A.gram || !ws.rc_p || ws.rc_head < 1 || ws.rc_head > k || A.d % 4 != 0 ||
                       (A.generated && ws.panel_rows < A.d)))
        return hipErrorInvalidValue;
    pl.pick_smem = ((size_t)A.r * 4 + 15) & ~(size_t)15;
    pl.factor_smem = 3 * sizeof(double) * (size_t)k;
    {
        const size_t threads = k <= 128 ? 256 : FACTOR_MAX_THREADS;
        const size_t table = sizeof(double) * (size_t)k * (threads / 64); // one row per wavefront
        const size_t parts = threads * 4 * sizeof(double); // partial residuals of threads sharing a quad
        pl.factor_share_table = pl.factor_smem + table <= 48 * 1024;
        const size_t scratch = pl.factor_share_table && table > parts ? table : parts;
        pl.factor_smem += scratch;
    }
    {
        ProfileScope prof(KC_OTHER, s);
        const bool small = N <= SMALL_MAX_RHS;
        omp_init_kernel<<<dim3((unsigned)N), 256, 0, s>>>(y, A.r, ws.words, ws.res64, ws.res32, ws.bitmap,
                                                          pl.screen ? 1 : 0, ws.sync, ws.partial,
                                                          small ? 2 * SMALL_MAX_GROUPS : 0, ws.xchg,
                                                          small ? A.r + SMALL_XCHG_PAD : 0);
    }
    pl.Apick = A;
    const bool whole_matrix_panel = pl.panels && ws.panel_rows >= A.d;
    if (whole_matrix_panel) {
        hipError_t e = launch_matrix_fill(A.key0, A.key1, A.scale, A.r, 0, A.d, ws.panel, s, KC_FILL);
        if (e != hipSuccess)
            return e;
        pl.Apick.generated = 0;
        pl.Apick.At = ws.panel;
    }
    // screening contraction: the rows of At as bfloat16 planes, once per call where they fit
    if (pl.screen && (!A.generated || whole_matrix_panel)) {
        ProfileScope prof(KC_FILL, s);
        launch_split_rows(whole_matrix_panel ? ws.panel : A.At, A.d, A.r, ws.a16, s);
    }
    hipError_t e;
    SmallPlan sp{};
    if (small_plan(pl, N, k, sp)) {
        // a small batch: the whole iteration loop is one launch
        ProfileScope prof(KC_CORR, s);
        e = raise_dynamic_lds(reinterpret_cast<const void *>(omp_small_kernel), sp.smem);
        if (e != hipSuccess)
            return e;
        const OmpWorkspace w = shift_workspace(ws, 0, A.r, k, sp.groups);
        IterArgs P{y, k, 0, sel, x, w, pl.Apick.At, 0, 0};
        omp_small_kernel<<<dim3((unsigned)(sp.groups + N)), SMALL_THREADS, sp.smem, s>>>(pl.Apick, P, N, sp.groups,
                                                                                      sp.rows_per_group);
        e = hipGetLastError();
    } else {
        e = omp_iterations(pl, whole_matrix_panel, y, N, A, k, sel, x, ws, s);
    }
    if (e != hipSuccess || !y_fit)
        return e;
    {
        ProfileScope prof(KC_SELECT, s);
        const OmpWorkspace w = shift_workspace(ws, 0, A.r, k, pl.tiles_m);
        IterArgs P{y, k, k, sel, x, w, pl.Apick.generated ? nullptr : pl.Apick.At, 0, 0};
        refit_kernel<<<dim3((unsigned)N), REFIT_THREADS, 2 * sizeof(double) * (size_t)k, s>>>(P, y_fit, z, A.r);
    }
    return hipGetLastError();
}

static hipError_t omp_iterations(const OmpPlan &pl, bool whole_matrix_panel, const float *y, int32_t N,
                                 const MatrixView &A, int32_t k, int32_t *sel, float *x, const OmpWorkspace &ws,
                                 hipStream_t s)
{
    // A group of right-hand sides [n0, n0 + Ng) advancing on one stream. What produces the keys of
    // iteration `it`: the contraction, or - for the first rc_head iterations of the recurrence engine - p0
    // and then the update of p after the selection before. The two tile the positions differently, so the
    // selection kernel is handed the matching view of the workspace.
    struct Group {
        int32_t n0, Ng;
        OmpWorkspace wc, wr;
        hipStream_t st;
    };
    const int32_t head = pl.recurrence ? ws.rc_head : 0;
    auto make_group = [&](int32_t n0, int32_t Ng, hipStream_t st) {
        Group g{n0, Ng, shift_workspace(ws, n0, A.r, k, pl.tiles_m), shift_workspace(ws, n0, A.r, k, (A.d + 255) / 256), st};
        g.wc.cvec = nullptr; // nothing reads the coordinates once the contraction has taken over
        return g;
    };
    auto iterate = [&](const Group &g, int32_t it) -> hipError_t {
        hipError_t e;
        if (it < head) {
            ProfileScope prof(KC_CORR, g.st);
            if (it == 0) {
                e = recur_init_launch(pl.Apick, y + (int64_t)g.n0 * A.r, g.Ng, g.wr, g.st);
                if (e == hipSuccess)
                    e = recur_step_launch(true, A, g.Ng, k, 0, sel + (int64_t)g.n0 * k, g.wr, g.wr.tiles_m, g.st);
            } else {
                e = recur_step_launch(false, A, g.Ng, k, it - 1, sel + (int64_t)g.n0 * k, g.wr, g.wr.tiles_m, g.st);
            }
        } else {
            e = omp_contraction(pl, A, g.Ng, g.wc, g.st);
        }
        if (e != hipSuccess)
            return e;
        omp_select_update(pl, A, y + (int64_t)g.n0 * A.r, g.Ng, k, it, sel + (int64_t)g.n0 * k, x + (int64_t)g.n0 * k,
                          it < head ? g.wr : g.wc, g.st);
        return hipSuccess;
    };
    // two halves side by side when the batch is large (not while kernels are being timed one by one,
    // and not when both halves would have to share a panel that is refilled inside the iterations)
    const int32_t N0 = (N / 2 + CORR_BN - 1) / CORR_BN * CORR_BN;
    SideStream *ss = nullptr;
    if (N >= 4 * CORR_BN && N0 < N && !g_profile_on && !pl.one_stream && !(pl.panels && !whole_matrix_panel))
        ss = side_stream();
    if (!ss) {
        const Group g = make_group(0, N, s);
        for (int32_t it = 0; it < k; ++it) {
            const hipError_t e = iterate(g, it);
            if (e != hipSuccess)
                return e;
        }
        return hipGetLastError();
    }
    const Group g0 = make_group(0, N0, s), g1 = make_group(N0, N - N0, ss->stream);
    if (hipEventRecord(ss->fork, s) != hipSuccess || hipStreamWaitEvent(ss->stream, ss->fork, 0) != hipSuccess)
        return hipErrorUnknown;
    hipError_t e = hipSuccess;
    for (int32_t it = 0; it < k && e == hipSuccess; ++it) {
        e = iterate(g0, it);
        if (e == hipSuccess)
            e = iterate(g1, it);
    }
    // join even after a failed launch so that the caller's stream never runs ahead of the side stream
    if (hipEventRecord(ss->join, ss->stream) != hipSuccess || hipStreamWaitEvent(s, ss->join, 0) != hipSuccess)
        return hipErrorUnknown;
    return e != hipSuccess ? e : hipGetLastError();
}

} // namespace sgc
