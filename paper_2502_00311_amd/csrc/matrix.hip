// Utilities on the measurement matrix (paper Sec. 4.3): materialise the generated matrix, the
// reciprocal column norms used by the OMP selection rule of App. B, and the Gram matrix A^H A that
// App. B precomputes (here an optional table of the inner products between columns).
#include "philox_normal.h"
#include "sgc_internal.h"

namespace sgc {

__global__ __launch_bounds__(256) void matrix_fill_kernel(uint32_t key0, uint32_t key1, float scale, int32_t r,
                                                          int64_t row0, int64_t rows, float *__restrict__ out)
{
    const int32_t r4 = r >> 2;
    const int64_t total = rows * r4;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
        const int64_t row = e / r4;
        const int32_t jb = (int32_t)(e - row * r4);
        reinterpret_cast<float4 *>(out)[e] = matrix_quad((uint32_t)(row0 + row), (uint32_t)jb, key0, key1, scale);
    }
}

// one wavefront per column of A
template <bool GENERATED>
__global__ __launch_bounds__(256) void colnorm_kernel(MatrixView A, float *__restrict__ out)
{
    const int lane = threadIdx.x & 63;
    const int32_t i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= A.d)
        return;
    const int32_t r4 = A.r >> 2;
    double s = 0.0;
    for (int32_t jb = lane; jb < r4; jb += 64) {
        float4 a;
        if (GENERATED)
            a = matrix_quad((uint32_t)i, (uint32_t)jb, A.key0, A.key1, A.scale);
        else
            a = reinterpret_cast<const float4 *>(A.At + (int64_t)i * A.r)[jb];
        s += (double)a.x * a.x + (double)a.y * a.y + (double)a.z * a.z + (double)a.w * a.w;
    }
    s = wave_sum(s);
    if (lane == 0)
        out[i] = s > 0.0 ? (float)(1.0 / sqrt(s)) : 0.f;
}

// G = A^H A in double from the float entries (products of floats are exact in double), on the double
// matrix cores: 128 x 128 outputs per workgroup, 2 x 2 wavefronts, each a 64 x 64 sub-tile of 4 x 4
// blocks of v_mfma_f64_16x16x4f64. Operands: lane l supplies column (l % 16) of its block at depth l / 16;
// accumulator register v of lane l holds row l / 16 + 4 v, column l % 16 of the block. Only tiles on
// or above the diagonal are computed; every result is stored at (i, j) and (j, i).
constexpr int GRAM_B = 128, GRAM_BK = 16;
typedef double doublex4 __attribute__((ext_vector_type(4)));

template <bool GENERATED>
__global__ __launch_bounds__(256) void gram_kernel(MatrixView A, double *__restrict__ G)
{
    constexpr int LD = GRAM_BK + 1; // odd stride: the one-float fragment reads fall in distinct banks
    __shared__ float sa[2][GRAM_B * LD], sb[2][GRAM_B * LD];
    if (blockIdx.x < blockIdx.y)
        return; // below the diagonal
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int32_t d = A.d, r = A.r;
    const int32_t i0 = blockIdx.y * GRAM_B, j0 = blockIdx.x * GRAM_B;

    float4 ga[2], gb[2];
    auto fetch = [&](int32_t row, int32_t kk) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < d && kk < r) {
            if (GENERATED)
                v = matrix_quad((uint32_t)row, (uint32_t)(kk >> 2), A.key0, A.key1, A.scale);
            else
                v = *reinterpret_cast<const float4 *>(A.At + (int64_t)row * r + kk);
        }
        return v;
    };
    auto load_global = [&](int32_t k0) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int f = tid + 256 * u; // 128 rows x 4 quads
            ga[u] = fetch(i0 + (f >> 2), k0 + (f & 3) * 4);
            gb[u] = fetch(j0 + (f >> 2), k0 + (f & 3) * 4);
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int f = tid + 256 * u;
            float *pa = &sa[buf][(f >> 2) * LD + (f & 3) * 4];
            float *pb = &sb[buf][(f >> 2) * LD + (f & 3) * 4];
            pa[0] = ga[u].x; pa[1] = ga[u].y; pa[2] = ga[u].z; pa[3] = ga[u].w;
            pb[0] = gb[u].x; pb[1] = gb[u].y; pb[2] = gb[u].z; pb[3] = gb[u].w;
        }
    };

    doublex4 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
            acc[a][b] = doublex4{0.0, 0.0, 0.0, 0.0};

    const int nkb = (r + GRAM_BK - 1) / GRAM_BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    const int l16 = lane & 15, lq = lane >> 4;
    for (int kb = 0; kb < nkb; ++kb) {
        const int buf = kb & 1;
        if (kb + 1 < nkb)
            load_global((kb + 1) * GRAM_BK);
#pragma unroll
        for (int ks = 0; ks < GRAM_BK; ks += 4) {
            double av[4], bv[4];
#pragma unroll
            for (int a = 0; a < 4; ++a)
                av[a] = (double)sa[buf][(wm * 64 + a * 16 + l16) * LD + ks + lq];
#pragma unroll
            for (int b = 0; b < 4; ++b)
                bv[b] = (double)sb[buf][(wn * 64 + b * 16 + l16) * LD + ks + lq];
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[a], bv[b], acc[a][b], 0, 0, 0);
        }
        if (kb + 1 < nkb)
            store_lds(buf ^ 1);
        __syncthreads();
    }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int32_t gi = i0 + wm * 64 + a * 16 + lq + 4 * v;
                const int32_t gj = j0 + wn * 64 + b * 16 + l16;
                if (gi < d && gj < d) {
                    G[(int64_t)gi * d + gj] = acc[a][b][v];
                    G[(int64_t)gj * d + gi] = acc[a][b][v];
                }
            }
}

hipError_t launch_gram(const MatrixView &A, double *out, hipStream_t s)
{
    const unsigned tiles = (unsigned)((A.d + GRAM_B - 1) / GRAM_B);
    ProfileScope prof(KC_OTHER, s);
    if (A.generated)
        gram_kernel<true><<<dim3(tiles, tiles), 256, 0, s>>>(A, out);
    else
        gram_kernel<false><<<dim3(tiles, tiles), 256, 0, s>>>(A, out);
    return hipGetLastError();
}

hipError_t launch_matrix_fill(uint32_t key0, uint32_t key1, float scale, int32_t r, int64_t row0, int64_t rows,
                              float *out, hipStream_t s, int profile_class)
{
    if (rows == 0)
        return hipSuccess;
    const int64_t total = rows * (r >> 2);
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 32)
        blocks = 256 * 32;
    ProfileScope prof(profile_class, s);
    matrix_fill_kernel<<<dim3((unsigned)blocks), 256, 0, s>>>(key0, key1, scale, r, row0, rows, out);
    return hipGetLastError();
}

hipError_t launch_colnorms(const MatrixView &A, float *out, hipStream_t s)
{
    const unsigned blocks = (unsigned)((A.d + 3) / 4);
    ProfileScope prof(KC_OTHER, s);
    if (A.generated)
        colnorm_kernel<true><<<dim3(blocks), 256, 0, s>>>(A, out);
    else
        colnorm_kernel<false><<<dim3(blocks), 256, 0, s>>>(A, out);
    return hipGetLastError();
}

} // namespace sgc
