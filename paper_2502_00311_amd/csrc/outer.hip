// Outer projection of CESGC (paper Sec. 4.4): the gradient G (m x n) of a weight matrix is first
// compressed with B (rho x m; in the paper the leading left singular vectors of a gradient, refreshed
// every fixed number of steps and an input here), SGC runs on Gc = B G read row-major in chunks, and
// its update N (rho x n, sparse) is taken back: W <- W - lr * B^T N.
//
// With the paper's ranks (rho = 32) both products are skinny: 2 rho flop per 4 bytes of G, 2 rho per 8
// bytes of W. They are written as streaming kernels over G and W with the arithmetic on the float
// matrix cores, not as a tiled GEMM: a wavefront owns a strip of 128 columns, lane l holding the four
// adjacent columns 4 (l % 32) .. + 3 of row (l / 32) of a row pair as one 16-byte load, and feeds
// component e of that load to the MFMA of column block e, so that block e stands for the columns
// 4 j + e. The permutation costs nothing: for a fixed accumulator register the four blocks are again four
// adjacent columns, read and written as 16 bytes.
#include "sgc_internal.h"

namespace sgc {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int OUTER_STRIP = 128; // columns per wavefront
constexpr int OUTER_FLIGHT = 8;  // row pairs in flight per wavefront

// Partial products of one slice of rows of G: out[s][a][j] = sum over the slice's rows i of B[a][i] G[i][j]
// (the slices are summed in order by outer_reduce_kernel; a single slice writes Gc itself).
// grid (column strips, slices, blocks of 32 * RBLK rows of B); the four wavefronts share the slice's row
// pairs (pair p goes to wavefront p % 4) and add their accumulators up in wavefront order at the end.
template <int RBLK>
__global__ __launch_bounds__(256) void outer_project_kernel(const float *__restrict__ B, const float *__restrict__ G,
                                                            int32_t rho, int32_t m, int32_t n, int32_t slice,
                                                            float *__restrict__ out)
{
    extern __shared__ __attribute__((aligned(16))) float outer_lds[];
    constexpr int RB = 32 * RBLK, LDB = RB + 1; // odd stride: the transposing writes fall in distinct banks
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, l32 = lane & 31, lhalf = lane >> 5;
    const int32_t n0 = blockIdx.x * OUTER_STRIP, s = blockIdx.y, rho0 = blockIdx.z * RB;
    const int32_t m0 = s * slice;
    const int32_t mend = m0 + slice < m ? m0 + slice : m;
    const int32_t rows = mend - m0;

    // the slice of B, transposed: Bs[row of the slice][row of B], zero beyond either end
    for (int32_t e = tid; e < RB * slice; e += 256) {
        const int32_t a = e / slice, kk = e - a * slice;
        float v = 0.f;
        if (rho0 + a < rho && kk < rows)
            v = B[(int64_t)(rho0 + a) * m + m0 + kk];
        outer_lds[kk * LDB + a] = v;
    }
    __syncthreads();

    floatx16 acc[RBLK][4];
#pragma unroll
    for (int rb = 0; rb < RBLK; ++rb)
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[rb][e][v] = 0.f;

    const int32_t col = n0 + 4 * l32;
    const bool col_ok = col < n;
    const int32_t pairs = slice >> 1;
    for (int32_t p0 = w; p0 < pairs; p0 += 4 * OUTER_FLIGHT) {
        float4 g[OUTER_FLIGHT];
#pragma unroll
        for (int u = 0; u < OUTER_FLIGHT; ++u) {
            const int32_t row = m0 + 2 * (p0 + 4 * u) + lhalf;
            g[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row < mend && col_ok)
                g[u] = load_once_f4(G + (int64_t)row * n + col);
        }
#pragma unroll
        for (int u = 0; u < OUTER_FLIGHT; ++u) {
            const int32_t p = p0 + 4 * u;
            if (p < pairs) { // uniform over the wavefront
                const int32_t kk = 2 * p + lhalf;
                float a[RBLK];
#pragma unroll
                for (int rb = 0; rb < RBLK; ++rb)
                    a[rb] = outer_lds[kk * LDB + rb * 32 + l32];
#pragma unroll
                for (int rb = 0; rb < RBLK; ++rb) {
                    acc[rb][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[rb], g[u].x, acc[rb][0], 0, 0, 0);
                    acc[rb][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[rb], g[u].y, acc[rb][1], 0, 0, 0);
                    acc[rb][2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[rb], g[u].z, acc[rb][2], 0, 0, 0);
                    acc[rb][3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[rb], g[u].w, acc[rb][3], 0, 0, 0);
                }
            }
        }
    }

    // wavefronts 1..3 hand their accumulators to wavefront 0, one after the other (fixed order of the sums)
    __syncthreads();
    for (int ww = 1; ww < 4; ++ww) {
        if (w == ww) {
#pragma unroll
            for (int rb = 0; rb < RBLK; ++rb)
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        outer_lds[((rb * 4 + e) * 16 + v) * 64 + lane] = acc[rb][e][v];
        }
        __syncthreads();
        if (w == 0) {
#pragma unroll
            for (int rb = 0; rb < RBLK; ++rb)
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        acc[rb][e][v] += outer_lds[((rb * 4 + e) * 16 + v) * 64 + lane];
        }
        __syncthreads();
    }
    if (w == 0 && col_ok) {
        // accumulator register v of lane l: row 8 (v / 4) + v % 4 + 4 (l / 32) of the block
#pragma unroll
        for (int rb = 0; rb < RBLK; ++rb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int32_t a = rho0 + rb * 32 + 8 * (v >> 2) + (v & 3) + 4 * lhalf;
                if (a < rho)
                    *reinterpret_cast<float4 *>(out + ((int64_t)s * rho + a) * n + col) =
                        make_float4(acc[rb][0][v], acc[rb][1][v], acc[rb][2][v], acc[rb][3][v]);
            }
    }
}

// Gc = sum of the slices' partial products, in slice order
__global__ __launch_bounds__(256) void outer_reduce_kernel(const float *__restrict__ part, int32_t S, int64_t count4,
                                                           float *__restrict__ Gc)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= count4)
        return;
    float4 acc = reinterpret_cast<const float4 *>(part)[e];
    for (int32_t s = 1; s < S; ++s) {
        const float4 v = reinterpret_cast<const float4 *>(part)[(int64_t)s * count4 + e];
        acc.x += v.x;
        acc.y += v.y;
        acc.z += v.z;
        acc.w += v.w;
    }
    reinterpret_cast<float4 *>(Gc)[e] = acc;
}

__global__ __launch_bounds__(256) void outer_zero_kernel(float *__restrict__ p, int64_t count4)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e < count4)
        reinterpret_cast<float4 *>(p)[e] = make_float4(0.f, 0.f, 0.f, 0.f);
}

// W[i][j] -= lr * sum over a of B[a][i] Nd[a][j], Nd the update in the compressed space written out
// densely (rho x n, mostly zeros; it stays in the caches). grid (column strips, groups of `blocks`
// 32-row blocks of W); a wavefront takes every fourth block of its group: the rho-deep product of a
// 32 x 128 tile on the matrix cores, then one read-modify-write pass over the tile.
__global__ __launch_bounds__(256) void outer_back_kernel(float *__restrict__ W, const float *__restrict__ B,
                                                         const float *__restrict__ Nd, int32_t rho, int32_t m,
                                                         int32_t n, int32_t blocks, float lr)
{
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, l32 = lane & 31, lhalf = lane >> 5;
    const int32_t col = blockIdx.x * OUTER_STRIP + 4 * l32;
    const bool col_ok = col < n;
    for (int32_t q = w; q < blocks; q += 4) {
        const int32_t i0 = (blockIdx.y * blocks + q) * 32;
        if (i0 >= m)
            break;
        floatx16 acc[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[e][v] = 0.f;
        const bool row_ok = i0 + l32 < m;
        for (int32_t k0 = 0; k0 < rho; k0 += 2 * OUTER_FLIGHT) {
            float4 nv[OUTER_FLIGHT];
            float bv[OUTER_FLIGHT];
#pragma unroll
            for (int u = 0; u < OUTER_FLIGHT; ++u) {
                const int32_t a = k0 + 2 * u + lhalf;
                nv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                bv[u] = 0.f;
                if (a < rho) {
                    if (col_ok)
                        nv[u] = *reinterpret_cast<const float4 *>(Nd + (int64_t)a * n + col);
                    if (row_ok)
                        bv[u] = B[(int64_t)a * m + i0 + l32];
                }
            }
#pragma unroll
            for (int u = 0; u < OUTER_FLIGHT; ++u) {
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv[u], nv[u].x, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv[u], nv[u].y, acc[1], 0, 0, 0);
                acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv[u], nv[u].z, acc[2], 0, 0, 0);
                acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(bv[u], nv[u].w, acc[3], 0, 0, 0);
            }
        }
        if (col_ok) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int32_t row = i0 + 8 * (v >> 2) + (v & 3) + 4 * lhalf;
                if (row < m) {
                    float4 *p = reinterpret_cast<float4 *>(W + (int64_t)row * n + col);
                    float4 wv = *p;
                    wv.x -= lr * acc[0][v];
                    wv.y -= lr * acc[1][v];
                    wv.z -= lr * acc[2][v];
                    wv.w -= lr * acc[3][v];
                    *p = wv;
                }
            }
        }
    }
}

// ---- host side ----
// how the rows of G are cut in slices: enough workgroups to fill the chip, slices of at most 256 rows
// (the transposed slice of B has to fit the LDS) and a multiple of 8 (row pairs, four wavefronts)
OuterPlan outer_plan(int32_t rho, int32_t m, int32_t n)
{
    OuterPlan pl{};
    pl.rblk = rho <= 32 ? 1 : 2;
    pl.strips = (n + OUTER_STRIP - 1) / OUTER_STRIP;
    pl.rho_blocks = (rho + 32 * pl.rblk - 1) / (32 * pl.rblk);
    int64_t S = (1024 + (int64_t)pl.strips * pl.rho_blocks - 1) / ((int64_t)pl.strips * pl.rho_blocks);
    const int64_t most = (m + 63) / 64;
    S = S < 1 ? 1 : (S > most ? most : S);
    int64_t slice = ((m + S - 1) / S + 7) / 8 * 8;
    if (slice > 256)
        slice = 256;
    pl.slice = (int32_t)slice;
    pl.slices = (int32_t)((m + slice - 1) / slice);
    const size_t partial = pl.slices > 1 ? (size_t)pl.slices * rho * n * sizeof(float) : 0;
    const size_t dense = (size_t)rho * n * sizeof(float);
    pl.ws_bytes = ((partial > dense ? partial : dense) + 255) & ~(size_t)255;
    return pl;
}

hipError_t launch_outer_project(const float *B, const float *G, int32_t rho, int32_t m, int32_t n, float *Gc,
                                void *ws, hipStream_t s)
{
    const OuterPlan pl = outer_plan(rho, m, n);
    float *out = pl.slices > 1 ? static_cast<float *>(ws) : Gc;
    const dim3 grid((unsigned)pl.strips, (unsigned)pl.slices, (unsigned)pl.rho_blocks);
    const size_t stage = (size_t)pl.slice * (32 * pl.rblk + 1) * sizeof(float);
    const size_t handoff = (size_t)pl.rblk * 4 * 16 * 64 * sizeof(float);
    const size_t smem = stage > handoff ? stage : handoff;
    ProfileScope prof(KC_OUTER, s);
    if (pl.rblk == 1) {
        outer_project_kernel<1><<<grid, 256, smem, s>>>(B, G, rho, m, n, pl.slice, out);
    } else {
        static bool raised = false;
        if (!raised) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(outer_project_kernel<2>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
            if (e != hipSuccess)
                return e;
            raised = true;
        }
        outer_project_kernel<2><<<grid, 256, smem, s>>>(B, G, rho, m, n, pl.slice, out);
    }
    if (pl.slices > 1) {
        const int64_t count4 = (int64_t)rho * n / 4;
        outer_reduce_kernel<<<dim3((unsigned)((count4 + 255) / 256)), 256, 0, s>>>(out, pl.slices, count4, Gc);
    }
    return hipGetLastError();
}

hipError_t launch_outer_apply(float *W, const float *B, int32_t rho, int32_t m, int32_t n, int32_t d, int32_t k,
                              const int32_t *sel_m, const float *x_m, const int32_t *sel_v, const float *x_v,
                              float alpha, float eps, float lr, void *ws, hipStream_t s)
{
    float *Nd = static_cast<float *>(ws);
    const int64_t count4 = (int64_t)rho * n / 4;
    {
        ProfileScope prof(KC_OUTER, s);
        outer_zero_kernel<<<dim3((unsigned)((count4 + 255) / 256)), 256, 0, s>>>(Nd, count4);
    }
    // the update of the plain path applied to zeros with step -1 leaves N itself (0 - (-1) N is exact)
    hipError_t e = launch_apply(Nd, (int64_t)rho * n / d, d, k, sel_m, x_m, sel_v, x_v, alpha, eps, -1.0f, s);
    if (e != hipSuccess)
        return e;
    const int32_t strips = (n + OUTER_STRIP - 1) / OUTER_STRIP;
    const int32_t row_blocks = (m + 31) / 32;
    // eight blocks per workgroup (two per wavefront) unless that leaves the chip short of workgroups
    int32_t blocks = 8;
    while (blocks > 4 && (int64_t)strips * ((row_blocks + blocks - 1) / blocks) < 512)
        blocks -= 4;
    const dim3 grid((unsigned)strips, (unsigned)((row_blocks + blocks - 1) / blocks));
    ProfileScope prof(KC_OUTER, s);
    outer_back_kernel<<<grid, 256, 0, s>>>(W, B, Nd, rho, m, n, blocks, lr);
    return hipGetLastError();
}

} // namespace sgc
