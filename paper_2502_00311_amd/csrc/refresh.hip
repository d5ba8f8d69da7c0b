// CESGC (Sec. 4.4): the projection matrix B is renewed every fixed number of steps from the singular
// value decomposition of the gradient matrix G (m x n): its rows are the rho leading left singular
// vectors. Only those rho vectors are wanted and rho << m, n, so the decomposition is computed by
// orthogonal (subspace) iteration on G G^T with the passes over G done by the streaming kernel of the
// outer projection, and every dense factorisation done on rho x rho matrices in double:
//
//   Gt = G^T                                        (once; lets both passes use the same kernel)
//   repeat `iters` times
//       Z = Q G        (rho x n)   orthonormalise the rows of Z:  Z Z^T = L L^T,  Z <- L^-1 Z
//       Y = Z Gt^T     (rho x m)   orthonormalise the rows of Y,  Q <- L^-1 Y
//   Z = Q G,  Z Z^T = V diag(lambda) V^T (Jacobi),  B = V^T Q,  sigma = sqrt(lambda)   (Rayleigh-Ritz)
//
// The triangular orthonormalisation makes row i converge to the i-th singular vector at the rate
// (sigma_{i+1} / sigma_i)^2 per iteration; the last step removes what mixing is left inside the subspace.
// A caller that refreshes periodically starts from the previous B and needs few iterations.
// Each half step is orthonormalised separately so that no Gram matrix is worse conditioned than
// (sigma_1 / sigma_rho)^2, which double precision carries for every spectrum float data can express.
#include "sgc_internal.h"

namespace sgc {

constexpr int GRAM_SLICES = 64; // partial Gram matrices (fixed: the summation order never depends on timing)
constexpr int GRAM_COLS = 128;  // columns per block of the Gram kernel
constexpr int REFRESH_LD = REFRESH_MAX_RHO + 1;

// dst[n][m] = src[m][n]^T, elements of 2 or 4 bytes moved as they are; grid.x: 32 x 32 tiles, grid.y: batch
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T *__restrict__ src, T *__restrict__ dst, int32_t m,
                                                        int32_t n, int32_t tiles_x)
{
    __shared__ T tile[32][33];
    src += (int64_t)blockIdx.y * m * n; // matrix of the batch
    dst += (int64_t)blockIdx.y * m * n;
    const int64_t bx = blockIdx.x % (uint32_t)tiles_x, by = blockIdx.x / (uint32_t)tiles_x;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
    for (int k = 0; k < 32; k += 8) {
        const int64_t row = by * 32 + ty + k, col = bx * 32 + tx;
        if (row < m && col < n)
            tile[ty + k][tx] = src[row * n + col];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 32; k += 8) {
        const int64_t row = bx * 32 + ty + k, col = by * 32 + tx;
        if (row < n && col < m)
            dst[row * m + col] = tile[tx][ty + k];
    }
}

// part[slice] = X_slice X_slice^T in double for the blocks of 128 columns the slice owns; X is rho x L;
// grid.y: matrix of the batch (GRAM_SLICES partial matrices are reserved for each).
// Thread (ti, tj) of 16 x 16 accumulates the entries (ti + 16 a, tj + 16 b).
__global__ __launch_bounds__(256) void gram_partial_kernel(const float *__restrict__ X, int32_t rho, int64_t L,
                                                           double *__restrict__ part)
{
    __shared__ float xs[REFRESH_MAX_RHO][GRAM_COLS + 1];
    X += (int64_t)blockIdx.y * rho * L;
    part += (int64_t)blockIdx.y * GRAM_SLICES * rho * rho;
    const int ti = threadIdx.x >> 4, tj = threadIdx.x & 15;
    double acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
            acc[a][b] = 0.0;
    const int64_t blocks = (L + GRAM_COLS - 1) / GRAM_COLS;
    for (int64_t blk = blockIdx.x; blk < blocks; blk += gridDim.x) {
        const int64_t c0 = blk * GRAM_COLS;
        for (int e = threadIdx.x; e < REFRESH_MAX_RHO * GRAM_COLS; e += 256) {
            const int i = e / GRAM_COLS, c = e % GRAM_COLS;
            xs[i][c] = (i < rho && c0 + c < L) ? X[(int64_t)i * L + c0 + c] : 0.f;
        }
        __syncthreads();
        for (int c = 0; c < GRAM_COLS; ++c) {
            double xi[4], xj[4];
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                xi[a] = (double)xs[ti + 16 * a][c];
                xj[a] = (double)xs[tj + 16 * a][c];
            }
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    acc[a][b] = __builtin_fma(xi[a], xj[b], acc[a][b]);
        }
        __syncthreads();
    }
    double *out = part + (int64_t)blockIdx.x * rho * rho;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int i = ti + 16 * a, j = tj + 16 * b;
            if (i < rho && j < rho)
                out[i * rho + j] = acc[a][b];
        }
}

// S = sum of the partial Gram matrices (LDS, leading dimension REFRESH_LD)
__device__ __forceinline__ void sum_partials(const double *__restrict__ part, int32_t slices, int32_t rho, double *S)
{
    for (int e = threadIdx.x; e < rho * rho; e += blockDim.x) {
        double s = 0.0;
        for (int sl = 0; sl < slices; ++sl)
            s += part[(int64_t)sl * rho * rho + e];
        S[(e / rho) * REFRESH_LD + e % rho] = s;
    }
}

// One workgroup: M = L^-1 for S = L L^T (Cholesky), so that M X has orthonormal rows. Computed in double
// by elimination on the augmented matrix [S | I]: pivot j subtracts multiples of row j from the rows
// below it, one barrier per pivot; what is left is [D L1^T | L1^-1] with S = L1 D L1^T, and
// L^-1 = D^-1/2 L1^-1.
// A pivot that is not above 1e-13 of the row's own squared norm (or not a number) marks a row that
// depends on the rows before it to the accuracy float data has: its row of M is zero, the row of M X too.
// dynamic LDS: double S[rho][REFRESH_LD], E[rho][REFRESH_LD], diag0[REFRESH_MAX_RHO]
__global__ __launch_bounds__(256) void factor_kernel(const double *__restrict__ part, int32_t slices, int32_t rho,
                                                     double *__restrict__ M)
{
    extern __shared__ __attribute__((aligned(16))) double refresh_lds[];
    double *S = refresh_lds, *E = S + REFRESH_MAX_RHO * REFRESH_LD, *diag0 = E + REFRESH_MAX_RHO * REFRESH_LD;
    const int tid = threadIdx.x;
    part += (int64_t)blockIdx.x * GRAM_SLICES * rho * rho; // one workgroup per matrix of the batch
    M += (int64_t)blockIdx.x * rho * rho;
    sum_partials(part, slices, rho, S);
    for (int e = tid; e < rho * rho; e += 256)
        E[(e / rho) * REFRESH_LD + e % rho] = (e / rho == e % rho) ? 1.0 : 0.0;
    __syncthreads();
    if (tid < rho)
        diag0[tid] = S[tid * REFRESH_LD + tid];
    __syncthreads();
    auto live = [&](int j) {
        const double d = S[j * REFRESH_LD + j];
        return d > 1e-13 * diag0[j] && d > 0.0 && d < 1e300;
    };
    for (int j = 0; j + 1 < rho; ++j) {
        if (live(j)) { // the same decision in every thread: S[j][j] is not written in this step
            const double inv = 1.0 / S[j * REFRESH_LD + j];
            const int below = rho - 1 - j, width = rho; // columns j+1 .. rho-1 of S and 0 .. j of E per row
            for (int e = tid; e < below * width; e += 256) {
                const int i = j + 1 + e / width, c = e % width;
                const double f = S[i * REFRESH_LD + j] * inv; // column j itself is left as it is
                if (c > j)
                    S[i * REFRESH_LD + c] -= f * S[j * REFRESH_LD + c];
                else
                    E[i * REFRESH_LD + c] -= f * E[j * REFRESH_LD + c];
            }
        }
        __syncthreads();
    }
    for (int e = tid; e < rho * rho; e += 256) {
        const int j = e / rho, c = e % rho;
        M[e] = (c <= j && live(j)) ? E[j * REFRESH_LD + c] / sqrt(S[j * REFRESH_LD + j]) : 0.0;
    }
}

// One workgroup: T = V diag(lambda) V^T by two-sided Jacobi rotations in double, rho / 2 disjoint pairs
// per round (round-robin pairing), a sweep = rho - 1 rounds; a pair is skipped once
// |T_pq| <= 1e-15 sqrt(T_pp T_qq), and a sweep without a rotation ends the iteration (at most 30 sweeps).
// M = the eigenvectors as rows in the order of decreasing eigenvalue, sigma = sqrt(max(lambda, 0)).
// dynamic LDS: double T[P][REFRESH_LD], V[P][REFRESH_LD], cs[REFRESH_MAX_RHO / 2], sn[...]; int pp[...], qq[...]
__global__ __launch_bounds__(256) void eig_kernel(const double *__restrict__ part, int32_t slices, int32_t rho,
                                                  double *__restrict__ M, float *__restrict__ sigma)
{
    extern __shared__ __attribute__((aligned(16))) double refresh_lds[];
    double *T = refresh_lds, *V = T + REFRESH_MAX_RHO * REFRESH_LD;
    double *cs = V + REFRESH_MAX_RHO * REFRESH_LD, *sn = cs + REFRESH_MAX_RHO / 2;
    int *pp = reinterpret_cast<int *>(sn + REFRESH_MAX_RHO / 2), *qq = pp + REFRESH_MAX_RHO / 2;
    __shared__ int rotated;
    const int tid = threadIdx.x;
    const int P = rho + (rho & 1), half = P / 2; // an odd size gets a zero row and column, which never rotate
    part += (int64_t)blockIdx.x * GRAM_SLICES * rho * rho; // one workgroup per matrix of the batch
    M += (int64_t)blockIdx.x * rho * rho;
    if (sigma)
        sigma += (int64_t)blockIdx.x * rho;
    for (int e = tid; e < REFRESH_MAX_RHO * REFRESH_LD; e += 256) {
        T[e] = 0.0;
        V[e] = (e / REFRESH_LD == e % REFRESH_LD) ? 1.0 : 0.0;
    }
    __syncthreads();
    sum_partials(part, slices, rho, T);
    __syncthreads();
    for (int sweep = 0; sweep < 30; ++sweep) {
        if (tid == 0)
            rotated = 0;
        __syncthreads();
        for (int rd = 0; rd < P - 1; ++rd) {
            if (tid < half) {
                int a, b;
                if (tid == 0) {
                    a = P - 1;
                    b = rd;
                } else {
                    a = (rd + tid) % (P - 1);
                    b = (rd - tid + (P - 1)) % (P - 1);
                }
                const int p = a < b ? a : b, q = a < b ? b : a;
                const double tpp = T[p * REFRESH_LD + p], tqq = T[q * REFRESH_LD + q], tpq = T[p * REFRESH_LD + q];
                double c = 1.0, s = 0.0;
                const double lim = 1e-15 * sqrt(fabs(tpp * tqq));
                if (fabs(tpq) > lim && fabs(tpq) > 0.0 && fabs(tpq) < 1e300) {
                    const double theta = (tqq - tpp) / (2.0 * tpq);
                    const double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                    c = 1.0 / sqrt(t * t + 1.0);
                    s = t * c;
                    atomicAdd(&rotated, 1);
                }
                pp[tid] = p;
                qq[tid] = q;
                cs[tid] = c;
                sn[tid] = s;
            }
            __syncthreads();
            // T <- J^T T J with J the product of the round's rotations: 2 x 2 blocks, one per pair of pairs
            for (int e = tid; e < half * half; e += 256) {
                const int ka = e / half, kb = e % half;
                const int pa = pp[ka], qa = qq[ka], pb = pp[kb], qb = qq[kb];
                const double ca = cs[ka], sa = sn[ka], cb = cs[kb], sb = sn[kb];
                const double x00 = T[pa * REFRESH_LD + pb], x01 = T[pa * REFRESH_LD + qb];
                const double x10 = T[qa * REFRESH_LD + pb], x11 = T[qa * REFRESH_LD + qb];
                const double w00 = ca * x00 - sa * x10, w01 = ca * x01 - sa * x11;
                const double w10 = sa * x00 + ca * x10, w11 = sa * x01 + ca * x11;
                T[pa * REFRESH_LD + pb] = cb * w00 - sb * w01;
                T[pa * REFRESH_LD + qb] = sb * w00 + cb * w01;
                T[qa * REFRESH_LD + pb] = cb * w10 - sb * w11;
                T[qa * REFRESH_LD + qb] = sb * w10 + cb * w11;
            }
            for (int e = tid; e < P * half; e += 256) { // V <- V J
                const int i = e / half, kb = e % half;
                const int pb = pp[kb], qb = qq[kb];
                const double cb = cs[kb], sb = sn[kb];
                const double v0 = V[i * REFRESH_LD + pb], v1 = V[i * REFRESH_LD + qb];
                V[i * REFRESH_LD + pb] = cb * v0 - sb * v1;
                V[i * REFRESH_LD + qb] = sb * v0 + cb * v1;
            }
            __syncthreads();
        }
        const int any = rotated;
        __syncthreads();
        if (any == 0)
            break;
    }
    if (tid < rho) {
        double lam = T[tid * REFRESH_LD + tid];
        lam = lam == lam ? lam : -1.0;
        int rank = 0;
        for (int j = 0; j < rho; ++j) {
            double lj = T[j * REFRESH_LD + j];
            lj = lj == lj ? lj : -1.0;
            rank += (lj > lam || (lj == lam && j < tid)) ? 1 : 0;
        }
        for (int j = 0; j < rho; ++j)
            M[rank * rho + j] = V[j * REFRESH_LD + tid];
        if (sigma)
            sigma[rank] = (float)sqrt(lam > 0.0 ? lam : 0.0);
    }
}

// X <- M X in place (M rho x rho in double, X rho x L in float): a workgroup owns 64 columns, four
// threads share a column and take every fourth row.
// dynamic LDS: double Ms[rho * rho]; float xs[rho][64]
__global__ __launch_bounds__(256) void transform_kernel(const double *__restrict__ M, float *__restrict__ X, int32_t rho,
                                                        int64_t L)
{
    extern __shared__ __attribute__((aligned(16))) double refresh_lds[];
    double *Ms = refresh_lds;
    float *xs = reinterpret_cast<float *>(Ms + rho * rho);
    const int tid = threadIdx.x, col = tid & 63, grp = tid >> 6;
    M += (int64_t)blockIdx.y * rho * rho; // matrix of the batch
    X += (int64_t)blockIdx.y * rho * L;
    const int64_t c = (int64_t)blockIdx.x * 64 + col;
    for (int e = tid; e < rho * rho; e += 256)
        Ms[e] = M[e];
    for (int j = grp; j < rho; j += 4)
        xs[j * 64 + col] = c < L ? X[(int64_t)j * L + c] : 0.f;
    __syncthreads(); // every row of the 64 columns is in LDS before any is overwritten
    for (int i = grp; i < rho; i += 4) {
        double acc = 0.0;
        for (int j = 0; j < rho; ++j)
            acc = __builtin_fma(Ms[i * rho + j], (double)xs[j * 64 + col], acc);
        if (c < L)
            X[(int64_t)i * L + c] = (float)acc;
    }
}

// a singular vector's sign is free: every row gets its largest-magnitude entry (the first among equals) positive
__global__ __launch_bounds__(256) void row_sign_kernel(float *__restrict__ B, int64_t m)
{
    __shared__ float bestv[256];
    __shared__ int64_t besti[256];
    float *row = B + (int64_t)blockIdx.x * m;
    float bv = -1.f;
    int64_t bi = 0;
    for (int64_t c = threadIdx.x; c < m; c += 256) {
        const float a = fabsf(row[c]);
        if (a > bv) {
            bv = a;
            bi = c;
        }
    }
    bestv[threadIdx.x] = bv;
    besti[threadIdx.x] = bi;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            const float ov = bestv[threadIdx.x + w];
            const int64_t oi = besti[threadIdx.x + w];
            if (ov > bestv[threadIdx.x] || (ov == bestv[threadIdx.x] && oi < besti[threadIdx.x])) {
                bestv[threadIdx.x] = ov;
                besti[threadIdx.x] = oi;
            }
        }
        __syncthreads();
    }
    const bool flip = bestv[0] > 0.f && row[besti[0]] < 0.f;
    __syncthreads();
    if (flip)
        for (int64_t c = threadIdx.x; c < m; c += 256)
            row[c] = -row[c];
}

// A start matrix may carry zero rows (the result of an earlier renewal on a gradient of lower rank): a zero
// row stays zero through every product, so it is given generic entries again - a fixed integer hash of
// its position, the same on every call - and takes part in the iteration like any other start vector.
__global__ __launch_bounds__(256) void reseed_zero_rows_kernel(float *__restrict__ B, int64_t m)
{
    __shared__ int any_s;
    float *row = B + (int64_t)blockIdx.x * m;
    if (threadIdx.x == 0)
        any_s = 0;
    __syncthreads();
    bool any = false;
    for (int64_t c = threadIdx.x; c < m; c += 256)
        any = any || !(row[c] == 0.f); // a NaN counts as content: it is not this kernel's to repair
    if (any)
        any_s = 1;
    __syncthreads();
    if (any_s)
        return;
    for (int64_t c = threadIdx.x; c < m; c += 256) {
        uint32_t h = (uint32_t)(blockIdx.x * 0x9e3779b9u) ^ (uint32_t)c * 0x85ebca6bu;
        h ^= h >> 16;
        h *= 0x7feb352du;
        h ^= h >> 15;
        h *= 0x846ca68bu;
        h ^= h >> 16;
        row[c] = ((float)(h >> 8) + 0.5f) * (1.0f / 8388608.0f) - 1.0f; // in (-1, 1)
    }
}

RefreshPlan refresh_plan(int32_t count, int32_t rho, int32_t m, int32_t n, bool g_bf16)
{
    auto up = [](size_t b) { return (b + 255) & ~(size_t)255; };
    RefreshPlan p;
    size_t off = 0;
    p.gt_off = off;
    off += up((size_t)count * m * n * (g_bf16 ? 2 : 4));
    p.z_off = off;
    off += up((size_t)count * rho * n * sizeof(float));
    p.part_off = off;
    off += up((size_t)count * GRAM_SLICES * rho * rho * sizeof(double));
    p.m_off = off;
    off += up((size_t)count * rho * rho * sizeof(double));
    p.outer_off = off;
    const size_t a = outer_plan(count, rho, m, n).ws_bytes, b = outer_plan(count, rho, n, m).ws_bytes;
    off += up(a > b ? a : b);
    p.ws_bytes = off;
    return p;
}

static hipError_t orthonormalise_rows(float *X, int32_t count, int32_t rho, int64_t L, double *part, double *M, bool ritz,
                                      float *sigma, hipStream_t s)
{
    const int64_t blocks = (L + GRAM_COLS - 1) / GRAM_COLS;
    const int slices = (int)(blocks < GRAM_SLICES ? blocks : GRAM_SLICES);
    gram_partial_kernel<<<dim3((unsigned)slices, (unsigned)count), 256, 0, s>>>(X, rho, L, part);
    if (ritz) {
        const size_t smem = (size_t)2 * REFRESH_MAX_RHO * REFRESH_LD * sizeof(double) +
                            REFRESH_MAX_RHO * (sizeof(double) + sizeof(int));
        const hipError_t e = raise_dynamic_lds(reinterpret_cast<const void *>(eig_kernel), smem);
        if (e != hipSuccess)
            return e;
        eig_kernel<<<dim3((unsigned)count), 256, smem, s>>>(part, slices, rho, M, sigma);
    } else {
        const size_t smem = (size_t)(2 * REFRESH_MAX_RHO * REFRESH_LD + REFRESH_MAX_RHO) * sizeof(double);
        const hipError_t e = raise_dynamic_lds(reinterpret_cast<const void *>(factor_kernel), smem);
        if (e != hipSuccess)
            return e;
        factor_kernel<<<dim3((unsigned)count), 256, smem, s>>>(part, slices, rho, M);
    }
    return hipGetLastError();
}

static hipError_t transform_rows(const double *M, float *X, int32_t count, int32_t rho, int64_t L, hipStream_t s)
{
    const size_t smem = (size_t)rho * rho * sizeof(double) + (size_t)rho * 64 * sizeof(float);
    transform_kernel<<<dim3((unsigned)((L + 63) / 64), (unsigned)count), 256, smem, s>>>(M, X, rho, L);
    return hipGetLastError();
}

hipError_t launch_outer_refresh(float *B, const void *G, bool g_bf16, int32_t count, int32_t rho, int32_t m, int32_t n,
                                int32_t iters, float *sigma, void *ws, hipStream_t s)
{
    const RefreshPlan pl = refresh_plan(count, rho, m, n, g_bf16);
    char *base = static_cast<char *>(ws);
    void *Gt = base + pl.gt_off;
    float *Z = reinterpret_cast<float *>(base + pl.z_off);
    double *part = reinterpret_cast<double *>(base + pl.part_off);
    double *M = reinterpret_cast<double *>(base + pl.m_off);
    void *ows = base + pl.outer_off;
    hipError_t e;
    {
        ProfileScope prof(KC_OUTER_REFRESH, s);
        if (iters > 0) // without a round nothing would orthonormalise the new rows
            reseed_zero_rows_kernel<<<dim3((unsigned)(rho * count)), 256, 0, s>>>(B, m);
        const int64_t tiles_x = (n + 31) / 32, tiles_y = (m + 31) / 32;
        const dim3 grid((unsigned)(tiles_x * tiles_y), (unsigned)count);
        if (g_bf16)
            transpose_kernel<uint16_t><<<grid, 256, 0, s>>>(static_cast<const uint16_t *>(G),
                                                            static_cast<uint16_t *>(Gt), m, n, (int32_t)tiles_x);
        else
            transpose_kernel<uint32_t><<<grid, 256, 0, s>>>(static_cast<const uint32_t *>(G),
                                                            static_cast<uint32_t *>(Gt), m, n, (int32_t)tiles_x);
        if ((e = hipGetLastError()) != hipSuccess)
            return e;
    }
    for (int32_t it = 0; it <= iters; ++it) {
        const bool last = it == iters;
        if ((e = launch_outer_project(B, G, g_bf16, count, rho, m, n, Z, ows, s)) != hipSuccess) // Z = Q G
            return e;
        {
            ProfileScope prof(KC_OUTER_REFRESH, s);
            if ((e = orthonormalise_rows(Z, count, rho, n, part, M, last, sigma, s)) != hipSuccess)
                return e;
            if (last) { // Rayleigh-Ritz: B = V^T Q, then the sign convention
                if ((e = transform_rows(M, B, count, rho, m, s)) != hipSuccess)
                    return e;
                row_sign_kernel<<<dim3((unsigned)(rho * count)), 256, 0, s>>>(B, m);
                return hipGetLastError();
            }
            if ((e = transform_rows(M, Z, count, rho, n, s)) != hipSuccess)
                return e;
        }
        if ((e = launch_outer_project(Z, Gt, g_bf16, count, rho, n, m, B, ows, s)) != hipSuccess) // Y = Z G^T
            return e;
        {
            ProfileScope prof(KC_OUTER_REFRESH, s);
            if ((e = orthonormalise_rows(B, count, rho, m, part, M, false, nullptr, s)) != hipSuccess)
                return e;
            if ((e = transform_rows(M, B, count, rho, m, s)) != hipSuccess)
                return e;
        }
    }
    return hipSuccess;
}

} // namespace sgc
