// Batched orthogonal matching pursuit (paper Sec. 4.3 eq. 9; selection rule, inverse-Cholesky
// update and output of App. B) for N right-hand sides that share the measurement matrix A.
//
// Per iteration two kernels run:
//   corr_kernel    P = At * R for all right-hand sides at once: a dense float contraction on the
//                  matrix cores (32x32x2 MFMA, LDS-staged 128x128 tiles). P is never written: the
//                  epilogue scales by 1/||A_:i||, masks selected positions and keeps the two best
//                  (score, position) pairs of every 128-row tile per right-hand side.
//   select_update  one workgroup per right-hand side: re-scores the near-maximal candidates in
//                  double (so the argmax does not depend on float rounding), appends the winning
//                  column, extends F = L^-H (App. B) by mat-vecs only, and recomputes the residual
//                  y - A_Lambda x in double.
// App. B precomputes the Gram matrix A^H A (d x d) to avoid the contraction; here the contraction
// is kept (it is what the matrix cores are for) and only inner products with selected columns are
// formed, so memory stays O(N k r).
#include "philox_normal.h"
#include "sgc_internal.h"

namespace sgc {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int CORR_BK = 32;       // contraction depth staged per step
constexpr int CORR_LD = CORR_BK + 4; // LDS row stride in floats (16-byte aligned, conflict-free b128 reads)
constexpr int CORR_THREADS = 256;
constexpr float RESCORE_TOL = 0x1.0p-10f; // candidates within this relative distance of the float maximum

OmpWorkspace carve_workspace(void *base, int32_t N, int32_t d, int32_t r, int32_t k)
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
    w.F = (double *)take(sizeof(double) * (size_t)N * k * k);
    w.avec = (double *)take(sizeof(double) * (size_t)N * k);
    w.xs = (double *)take(sizeof(double) * (size_t)N * k);
    w.res32 = (float *)take(sizeof(float) * (size_t)N * r);
    w.cols = (float *)take(sizeof(float) * (size_t)N * k * r);
    w.partial = (uint64_t *)take(sizeof(uint64_t) * (size_t)N * w.tiles_m * 2);
    w.bitmap = (uint32_t *)take(sizeof(uint32_t) * (size_t)N * w.words);
    w.cand = (int32_t *)take(sizeof(int32_t) * (size_t)N * w.tiles_m * 2);
    w.bytes = off;
    return w;
}

// ----------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void omp_init_kernel(const float *__restrict__ y, int32_t r, int32_t words,
                                                       double *__restrict__ res64, float *__restrict__ res32,
                                                       uint32_t *__restrict__ bitmap)
{
    const int64_t n = blockIdx.x;
    for (int32_t j = threadIdx.x; j < r; j += 256) {
        const float v = y[n * r + j];
        res64[n * r + j] = (double)v;
        res32[n * r + j] = v;
    }
    for (int32_t w = threadIdx.x; w < words; w += 256)
        bitmap[n * words + w] = 0u;
}

// ----------------------------------------------------------------------------------------------
// keep the two largest keys seen
__device__ __forceinline__ void top2_insert(uint64_t key, uint64_t &best, uint64_t &second)
{
    const uint64_t lo = key < best ? key : best;
    best = key < best ? best : key;
    second = lo < second ? second : lo;
}

// Correlation contraction + fused selection epilogue.
//   grid.x = tiles over positions i (128 each), grid.y = tiles over right-hand sides (128 each)
//   wave (wm, wn) of the 2x2 wave grid owns a 64x64 sub-tile = 2x2 MFMA blocks of 32x32.
// MFMA 32x32x2 operands: lane l supplies At[row l%32][depth l/32] and R[rhs l%32][depth l/32]. Each
// lane reads four consecutive depths with one 16-byte LDS read; lanes 32..63 read depths +4..+7, so
// four MFMAs cover eight depths (the sum over depth does not depend on their order).
// Accumulator register v of lane l holds position 8*(v/4) + 4*(l/32) + v%4 of right-hand side l%32.
template <bool GENERATED>
__global__ __launch_bounds__(CORR_THREADS, 2) void corr_kernel(MatrixView A, const float *__restrict__ R,
                                                               int32_t N, const uint32_t *__restrict__ bitmap,
                                                               int32_t words, uint64_t *__restrict__ partial,
                                                               int32_t tiles_m)
{
    __shared__ __attribute__((aligned(16))) float lds_a[2][CORR_BM * CORR_LD];
    __shared__ __attribute__((aligned(16))) float lds_b[2][CORR_BN * CORR_LD];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int32_t d = A.d, r = A.r;
    const int32_t m0 = blockIdx.x * CORR_BM;
    const int32_t n0 = blockIdx.y * CORR_BN;

    // global -> register staging: 4 float4 of the At tile and 4 of the R tile per thread
    float4 ga[4], gb[4];
    int lrow[4], lcol[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int f = tid + CORR_THREADS * u;
        lrow[u] = f >> 3;
        lcol[u] = (f & 7) << 2;
    }
    auto load_global = [&](int32_t k0) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int32_t i = m0 + lrow[u];
            const int32_t kk = k0 + lcol[u];
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i < d && kk < r) {
                if (GENERATED)
                    a = matrix_quad((uint32_t)i, (uint32_t)(kk >> 2), A.key0, A.key1, A.scale);
                else
                    a = *reinterpret_cast<const float4 *>(A.At + (int64_t)i * r + kk);
            }
            ga[u] = a;
            const int32_t n = n0 + lrow[u];
            float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
            if (n < N && kk < r)
                b = *reinterpret_cast<const float4 *>(R + (int64_t)n * r + kk);
            gb[u] = b;
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            *reinterpret_cast<float4 *>(&lds_a[buf][lrow[u] * CORR_LD + lcol[u]]) = ga[u];
            *reinterpret_cast<float4 *>(&lds_b[buf][lrow[u] * CORR_LD + lcol[u]]) = gb[u];
        }
    };

    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[a][b][v] = 0.f;

    const int nkb = (r + CORR_BK - 1) / CORR_BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    const int l32 = lane & 31, lhalf = lane >> 5;
    for (int kb = 0; kb < nkb; ++kb) {
        const int buf = kb & 1;
        if (kb + 1 < nkb)
            load_global((kb + 1) * CORR_BK);
        const float *pa = &lds_a[buf][(wm * 64 + l32) * CORR_LD + lhalf * 4];
        const float *pb = &lds_b[buf][(wn * 64 + l32) * CORR_LD + lhalf * 4];
#pragma unroll
        for (int ks = 0; ks < CORR_BK; ks += 8) {
            const float4 a0 = *reinterpret_cast<const float4 *>(pa + ks);
            const float4 a1 = *reinterpret_cast<const float4 *>(pa + 32 * CORR_LD + ks);
            const float4 b0 = *reinterpret_cast<const float4 *>(pb + ks);
            const float4 b1 = *reinterpret_cast<const float4 *>(pb + 32 * CORR_LD + ks);
            const float av[2][4] = {{a0.x, a0.y, a0.z, a0.w}, {a1.x, a1.y, a1.z, a1.w}};
            const float bv[2][4] = {{b0.x, b0.y, b0.z, b0.w}, {b1.x, b1.y, b1.z, b1.w}};
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[a][t], bv[b][t], acc[a][b], 0, 0, 0);
        }
        if (kb + 1 < nkb)
            store_lds(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: normalise, mask, keep the two best per right-hand side ----
    uint64_t *red = reinterpret_cast<uint64_t *>(&lds_a[0][0]); // [2 wm][128 rhs][2]
    __syncthreads();
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int nl = wn * 64 + b * 32 + l32; // right-hand side within the tile
        const int32_t n = n0 + nl;
        uint64_t best = 0, second = 0;
#pragma unroll
        for (int a = 0; a < 2; ++a) {
            const int32_t ibase = m0 + wm * 64 + a * 32;
            uint32_t mask = 0xffffffffu;
            if (n < N && ibase < d)
                mask = bitmap[(int64_t)n * words + (ibase >> 5)];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int off = 8 * (v >> 2) + 4 * lhalf + (v & 3);
                const int32_t i = ibase + off;
                if (i < d && !((mask >> off) & 1u)) {
                    const float score = fabsf(acc[a][b][v]) * A.inv_colnorm[i];
                    const uint64_t key = ((uint64_t)__float_as_uint(score) << 32) | (uint64_t)(0xffffffffu - (uint32_t)i);
                    top2_insert(key, best, second);
                }
            }
        }
        // the other half-wave holds the remaining positions of the same right-hand side
        const uint64_t ob = shfl_xor_u64(best, 32), os = shfl_xor_u64(second, 32);
        top2_insert(ob, best, second);
        top2_insert(os, best, second);
        if (lhalf == 0) {
            red[(wm * CORR_BN + nl) * 2 + 0] = best;
            red[(wm * CORR_BN + nl) * 2 + 1] = second;
        }
    }
    __syncthreads();
    if (tid < CORR_BN) {
        const int32_t n = n0 + tid;
        if (n < N) {
            uint64_t best = red[tid * 2], second = red[tid * 2 + 1];
            top2_insert(red[(CORR_BN + tid) * 2], best, second);
            top2_insert(red[(CORR_BN + tid) * 2 + 1], best, second);
            uint64_t *o = partial + ((int64_t)n * tiles_m + blockIdx.x) * 2;
            o[0] = best;
            o[1] = second;
        }
    }
}

// ----------------------------------------------------------------------------------------------
constexpr int SEL_THREADS = 256;
constexpr int SEL_WAVES = SEL_THREADS / 64;

struct SelectArgs {
    const float *y;   // [N][r]
    int32_t k, it;    // sparsity, current iteration (0-based)
    int32_t *sel;     // [N][k]
    float *x;         // [N][k]
    OmpWorkspace ws;
};

template <bool GENERATED>
__device__ __forceinline__ float4 column_quad(const MatrixView &A, int32_t i, int32_t jb)
{
    if (GENERATED)
        return matrix_quad((uint32_t)i, (uint32_t)jb, A.key0, A.key1, A.scale);
    return reinterpret_cast<const float4 *>(A.At + (int64_t)i * A.r)[jb];
}

// dynamic LDS: float a_col[r]; double w[k]; double c[k]
template <bool GENERATED>
__global__ __launch_bounds__(SEL_THREADS) void select_update_kernel(MatrixView A, SelectArgs P)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int32_t r = A.r, r4 = A.r >> 2, k = P.k, it = P.it;
    float *a_col = reinterpret_cast<float *>(smem);
    double *w_s = reinterpret_cast<double *>(smem + (((size_t)r * 4 + 15) & ~(size_t)15));
    double *c_s = w_s + k;

    __shared__ uint64_t s_u64[SEL_WAVES];
    __shared__ double s_red[3][SEL_WAVES];
    __shared__ double s_cscore[SEL_WAVES];
    __shared__ int32_t s_cidx[SEL_WAVES];
    __shared__ int32_t s_ncand, s_lambda;
    __shared__ double s_gamma, s_coef;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t n = blockIdx.x;
    const OmpWorkspace &W = P.ws;
    const int32_t np = W.tiles_m * 2;
    const uint64_t *part = W.partial + n * np;
    const double *res64 = W.res64 + n * r;
    int32_t *cand = W.cand + n * np;

    // (1) float maximum over the tile partials
    uint64_t best = 0;
    for (int32_t e = tid; e < np; e += SEL_THREADS) {
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
    for (int u = 0; u < SEL_WAVES; ++u)
        best = s_u64[u] > best ? s_u64[u] : best;
    const float smax = __uint_as_float((uint32_t)(best >> 32));
    const float thr = smax * (1.0f - RESCORE_TOL);

    // (2) candidates: every kept pair whose float score is within the tolerance of the maximum
    for (int32_t e = tid; e < np; e += SEL_THREADS) {
        const uint64_t v = part[e];
        if (v != 0 && __uint_as_float((uint32_t)(v >> 32)) >= thr) {
            const int32_t slot = atomicAdd(&s_ncand, 1);
            cand[slot] = (int32_t)(0xffffffffu - (uint32_t)v);
        }
    }
    __syncthreads();
    const int32_t ncand = s_ncand;

    // (3) re-score in double, one wavefront per candidate; best = (score desc, position asc)
    double wbest = -1.0;
    int32_t widx = 0x7fffffff;
    for (int32_t cdx = wave; cdx < ncand; cdx += SEL_WAVES) {
        const int32_t i = cand[cdx];
        double dot = 0.0, nrm = 0.0;
        for (int32_t jb = lane; jb < r4; jb += 64) {
            const float4 a = column_quad<GENERATED>(A, i, jb);
            const double *rr = res64 + 4 * jb;
            dot += (double)a.x * rr[0] + (double)a.y * rr[1] + (double)a.z * rr[2] + (double)a.w * rr[3];
            nrm += (double)a.x * a.x + (double)a.y * a.y + (double)a.z * a.z + (double)a.w * a.w;
        }
        dot = wave_sum(dot);
        nrm = wave_sum(nrm);
        dot = __shfl(dot, 0, 64);
        nrm = __shfl(nrm, 0, 64);
        const double score = nrm > 0.0 ? fabs(dot) / sqrt(nrm) : 0.0;
        if (score > wbest || (score == wbest && i < widx)) {
            wbest = score;
            widx = i;
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
        for (int u = 1; u < SEL_WAVES; ++u)
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
    const int32_t lam = s_lambda;

    // (4) the new column: to LDS and to the column store; g = ||a||^2, b = <a, y>
    float *cols = W.cols + (n * k) * (int64_t)r;
    {
        double g = 0.0, b = 0.0;
        const float *yy = P.y + n * r;
        for (int32_t jb = tid; jb < r4; jb += SEL_THREADS) {
            const float4 a = column_quad<GENERATED>(A, lam, jb);
            reinterpret_cast<float4 *>(a_col)[jb] = a;
            reinterpret_cast<float4 *>(cols + (int64_t)it * r)[jb] = a;
            const float4 yv = reinterpret_cast<const float4 *>(yy)[jb];
            g += (double)a.x * a.x + (double)a.y * a.y + (double)a.z * a.z + (double)a.w * a.w;
            b += (double)a.x * yv.x + (double)a.y * yv.y + (double)a.z * yv.z + (double)a.w * yv.w;
        }
        g = wave_sum(g);
        b = wave_sum(b);
        if (lane == 0) {
            s_red[0][wave] = g;
            s_red[1][wave] = b;
        }
    }
    __syncthreads();
    double g = 0.0, b = 0.0;
#pragma unroll
    for (int u = 0; u < SEL_WAVES; ++u) {
        g += s_red[0][u];
        b += s_red[1][u];
    }

    // (5) w_t = <A_:lambda_t, a> for the earlier selections, one wavefront per t
    for (int32_t t = wave; t < it; t += SEL_WAVES) {
        const float4 *ct = reinterpret_cast<const float4 *>(cols + (int64_t)t * r);
        double s = 0.0;
        for (int32_t jb = lane; jb < r4; jb += 64) {
            const float4 u = ct[jb];
            const float4 a = reinterpret_cast<const float4 *>(a_col)[jb];
            s += (double)u.x * a.x + (double)u.y * a.y + (double)u.z * a.z + (double)u.w * a.w;
        }
        s = wave_sum(s);
        if (lane == 0)
            w_s[t] = s;
    }
    __syncthreads();

    // (6) c = F^H w (coordinates of a in the orthonormal basis Q = A_Lambda F); column t of F is
    //     stored contiguously with entries 0..t
    double *F = W.F + (n * k) * (int64_t)k;
    for (int32_t t = wave; t < it; t += SEL_WAVES) {
        const double *ft = F + (int64_t)t * k;
        double s = 0.0;
        for (int32_t u = lane; u <= t; u += 64)
            s += ft[u] * w_s[u];
        s = wave_sum(s);
        if (lane == 0)
            c_s[t] = s;
    }
    __syncthreads();

    // (7) gamma = 1/sqrt(g - c.c); new coefficient a_it = gamma (b - c.avec)
    double *avec = W.avec + n * k;
    {
        double cc = 0.0, ca = 0.0;
        for (int32_t t = tid; t < it; t += SEL_THREADS) {
            cc += c_s[t] * c_s[t];
            ca += c_s[t] * avec[t];
        }
        cc = wave_sum(cc);
        ca = wave_sum(ca);
        if (lane == 0) {
            s_red[0][wave] = cc;
            s_red[1][wave] = ca;
        }
        __syncthreads();
        if (tid == 0) {
            cc = 0.0;
            ca = 0.0;
            for (int u = 0; u < SEL_WAVES; ++u) {
                cc += s_red[0][u];
                ca += s_red[1][u];
            }
            const double rem = g - cc;
            const double gamma = rem > 0.0 ? 1.0 / sqrt(rem) : 0.0;
            const double coef = gamma * (b - ca);
            s_gamma = gamma;
            s_coef = coef;
            avec[it] = coef;
            F[(int64_t)it * k + it] = gamma;
        }
        __syncthreads();
    }
    const double gamma = s_gamma, coef = s_coef;

    // (8) new column of F: -gamma F c on rows < it; x <- [x; 0] + coef * F_:it. x goes to w_s.
    double *xs = W.xs + n * k;
    for (int32_t u = tid; u <= it; u += SEL_THREADS) {
        double xn;
        if (u < it) {
            double s = 0.0;
            for (int32_t t = u; t < it; ++t)
                s += F[(int64_t)t * k + u] * c_s[t];
            const double f = -gamma * s;
            F[(int64_t)it * k + u] = f;
            xn = xs[u] + coef * f;
        } else {
            xn = coef * gamma;
        }
        xs[u] = xn;
        if (it == k - 1)
            P.x[n * k + u] = (float)xn;
    }
    __syncthreads(); // all reads of w_s (step 6) are done
    for (int32_t u = tid; u <= it; u += SEL_THREADS)
        w_s[u] = xs[u];
    __syncthreads();

    // (9) residual = y - A_Lambda x, in double; float copy for the next contraction
    {
        const float *yy = P.y + n * r;
        for (int32_t jb = tid; jb < r4; jb += SEL_THREADS) {
            const float4 yv = reinterpret_cast<const float4 *>(yy)[jb];
            double e0 = yv.x, e1 = yv.y, e2 = yv.z, e3 = yv.w;
            for (int32_t t = 0; t < it; ++t) {
                const float4 u = reinterpret_cast<const float4 *>(cols + (int64_t)t * r)[jb];
                const double xt = w_s[t];
                e0 -= xt * u.x;
                e1 -= xt * u.y;
                e2 -= xt * u.z;
                e3 -= xt * u.w;
            }
            {
                const float4 u = reinterpret_cast<const float4 *>(a_col)[jb];
                const double xt = w_s[it];
                e0 -= xt * u.x;
                e1 -= xt * u.y;
                e2 -= xt * u.z;
                e3 -= xt * u.w;
            }
            double *ro = W.res64 + n * r + 4 * jb;
            ro[0] = e0;
            ro[1] = e1;
            ro[2] = e2;
            ro[3] = e3;
            reinterpret_cast<float4 *>(W.res32 + n * r)[jb] = make_float4((float)e0, (float)e1, (float)e2, (float)e3);
        }
    }
    if (tid == 0) {
        P.sel[n * k + it] = lam;
        W.bitmap[n * W.words + (lam >> 5)] |= 1u << (lam & 31);
    }
}

hipError_t launch_omp(const float *y, int32_t N, const MatrixView &A, int32_t k, int32_t *sel, float *x,
                      const OmpWorkspace &ws, hipStream_t s)
{
    {
        ProfileScope prof(KC_OTHER, s);
        omp_init_kernel<<<dim3((unsigned)N), 256, 0, s>>>(y, A.r, ws.words, ws.res64, ws.res32, ws.bitmap);
    }
    const dim3 cgrid((unsigned)ws.tiles_m, (unsigned)((N + CORR_BN - 1) / CORR_BN));
    const size_t smem = (((size_t)A.r * 4 + 15) & ~(size_t)15) + 2 * sizeof(double) * (size_t)k;
    SelectArgs P{y, k, 0, sel, x, ws};
    for (int32_t it = 0; it < k; ++it) {
        P.it = it;
        {
            ProfileScope prof(KC_CORR, s);
            if (A.generated)
                corr_kernel<true><<<cgrid, CORR_THREADS, 0, s>>>(A, ws.res32, N, ws.bitmap, ws.words, ws.partial, ws.tiles_m);
            else
                corr_kernel<false><<<cgrid, CORR_THREADS, 0, s>>>(A, ws.res32, N, ws.bitmap, ws.words, ws.partial, ws.tiles_m);
        }
        {
            ProfileScope prof(KC_SELECT, s);
            if (A.generated)
                select_update_kernel<true><<<dim3((unsigned)N), SEL_THREADS, smem, s>>>(A, P);
            else
                select_update_kernel<false><<<dim3((unsigned)N), SEL_THREADS, smem, s>>>(A, P);
        }
    }
    return hipGetLastError();
}

} // namespace sgc
