// Sparse projection (paper eq. 5-6, Alg. 2 line 1): p = A G~ and q = A G~^2 for the k-sparse
// G~ = Sparsify_k(G) of every chunk, as a gather-accumulate of k columns of A. Columns are rows
// of At (contiguous), so each thread owns four consecutive measurements and streams 16-byte
// pieces of the k selected rows; in generated mode the same four entries come from one Philox
// call instead of memory.
#include "philox_normal.h"
#include "sgc_internal.h"

namespace sgc {

constexpr int PROJ_THREADS = 256;
constexpr int PROJ_STAGE = 1024; // (position, value) pairs staged in LDS at a time

template <bool GENERATED>
__global__ __launch_bounds__(PROJ_THREADS) void project_kernel(const int32_t *__restrict__ idx,
                                                               const float *__restrict__ val, int32_t k,
                                                               MatrixView A, float *__restrict__ p,
                                                               float *__restrict__ q, float out_scale)
{
    __shared__ int32_t s_idx[PROJ_STAGE];
    __shared__ float s_val[PROJ_STAGE];
    const int64_t c = blockIdx.y;
    const int32_t r4 = A.r >> 2;
    const int32_t jb = blockIdx.x * PROJ_THREADS + threadIdx.x; // group of 4 measurements
    const bool active = jb < r4;
    float4 ap = make_float4(0.f, 0.f, 0.f, 0.f), aq = ap;
    for (int32_t t0 = 0; t0 < k; t0 += PROJ_STAGE) {
        const int32_t cnt = k - t0 < PROJ_STAGE ? k - t0 : PROJ_STAGE;
        __syncthreads();
        for (int32_t t = threadIdx.x; t < cnt; t += PROJ_THREADS) {
            s_idx[t] = idx[c * k + t0 + t];
            s_val[t] = val[c * k + t0 + t];
        }
        __syncthreads();
        if (active) {
            for (int32_t t = 0; t < cnt; ++t) {
                const int32_t i = s_idx[t];
                const float v = s_val[t];
                const float v2 = v * v;
                float4 a;
                if (GENERATED)
                    a = matrix_quad((uint32_t)i, (uint32_t)jb, A.key0, A.key1, A.scale);
                else
                    a = reinterpret_cast<const float4 *>(A.At + (int64_t)i * A.r)[jb];
                ap.x = __builtin_fmaf(a.x, v, ap.x);
                ap.y = __builtin_fmaf(a.y, v, ap.y);
                ap.z = __builtin_fmaf(a.z, v, ap.z);
                ap.w = __builtin_fmaf(a.w, v, ap.w);
                aq.x = __builtin_fmaf(a.x, v2, aq.x);
                aq.y = __builtin_fmaf(a.y, v2, aq.y);
                aq.z = __builtin_fmaf(a.z, v2, aq.z);
                aq.w = __builtin_fmaf(a.w, v2, aq.w);
            }
        }
    }
    if (active) {
        // out_scale is 1 for the projection (an exact multiplication); the re-projection scales its sum
        reinterpret_cast<float4 *>(p + c * A.r)[jb] =
            make_float4(ap.x * out_scale, ap.y * out_scale, ap.z * out_scale, ap.w * out_scale);
        if (q)
            reinterpret_cast<float4 *>(q + c * A.r)[jb] = aq;
    }
}

// Stored A and few chunks: the kernel above would launch C * r / 1024 workgroups, too few to keep the
// memory system busy (128 for 64 chunks of r = 2048). Here a workgroup owns 256 measurements of one
// chunk and its four wavefronts share the k rows (wavefront w takes rows w, w + 4, ...), eight 1-KiB
// row pieces in flight per wavefront; the four partial sums are added in wavefront order at the end.
constexpr int PROJ_FLIGHT = 8;

__global__ __launch_bounds__(PROJ_THREADS) void project_rows_split_kernel(const int32_t *__restrict__ idx,
                                                                          const float *__restrict__ val, int32_t k,
                                                                          MatrixView A, float *__restrict__ p,
                                                                          float *__restrict__ q, float out_scale)
{
    __shared__ int32_t s_idx[PROJ_STAGE];
    __shared__ float s_val[PROJ_STAGE];
    __shared__ float4 s_part[2][3][64];
    const int64_t c = blockIdx.y;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int32_t r4 = A.r >> 2;
    const int32_t jb = blockIdx.x * 64 + lane;
    const bool active = jb < r4;
    const float4 *base = reinterpret_cast<const float4 *>(A.At) + (active ? jb : 0);
    float4 ap = make_float4(0.f, 0.f, 0.f, 0.f), aq = ap;
    for (int32_t t0 = 0; t0 < k; t0 += PROJ_STAGE) {
        const int32_t cnt = k - t0 < PROJ_STAGE ? k - t0 : PROJ_STAGE;
        __syncthreads();
        for (int32_t t = threadIdx.x; t < cnt; t += PROJ_THREADS) {
            s_idx[t] = idx[c * k + t0 + t];
            s_val[t] = val[c * k + t0 + t];
        }
        __syncthreads();
        for (int32_t t = w; t < cnt; t += 4 * PROJ_FLIGHT) {
            float4 a[PROJ_FLIGHT];
            float v[PROJ_FLIGHT];
#pragma unroll
            for (int u = 0; u < PROJ_FLIGHT; ++u) {
                const int32_t tt = t + 4 * u;
                const bool on = tt < cnt;
                v[u] = on ? s_val[tt] : 0.f;
                a[u] = base[(int64_t)(on ? s_idx[tt] : s_idx[t]) * r4]; // past the end: a row already in flight, times 0
            }
#pragma unroll
            for (int u = 0; u < PROJ_FLIGHT; ++u) {
                const float v2 = v[u] * v[u];
                ap.x = __builtin_fmaf(a[u].x, v[u], ap.x);
                ap.y = __builtin_fmaf(a[u].y, v[u], ap.y);
                ap.z = __builtin_fmaf(a[u].z, v[u], ap.z);
                ap.w = __builtin_fmaf(a[u].w, v[u], ap.w);
                aq.x = __builtin_fmaf(a[u].x, v2, aq.x);
                aq.y = __builtin_fmaf(a[u].y, v2, aq.y);
                aq.z = __builtin_fmaf(a[u].z, v2, aq.z);
                aq.w = __builtin_fmaf(a[u].w, v2, aq.w);
            }
        }
    }
    if (w > 0) {
        s_part[0][w - 1][lane] = ap;
        s_part[1][w - 1][lane] = aq;
    }
    __syncthreads();
    if (w == 0 && active) {
#pragma unroll
        for (int o = 0; o < 3; ++o) {
            const float4 bp = s_part[0][o][lane], bq = s_part[1][o][lane];
            ap.x += bp.x; ap.y += bp.y; ap.z += bp.z; ap.w += bp.w;
            aq.x += bq.x; aq.y += bq.y; aq.z += bq.z; aq.w += bq.w;
        }
        reinterpret_cast<float4 *>(p + c * A.r)[jb] =
            make_float4(ap.x * out_scale, ap.y * out_scale, ap.z * out_scale, ap.w * out_scale);
        if (q)
            reinterpret_cast<float4 *>(q + c * A.r)[jb] = aq;
    }
}

hipError_t launch_project(const int32_t *idx, const float *val, int64_t C, int32_t k, const MatrixView &A,
                          float *p, float *q, hipStream_t s, float out_scale)
{
    if (C == 0)
        return hipSuccess;
    const int32_t r4 = A.r >> 2;
    const unsigned gx = (unsigned)((r4 + PROJ_THREADS - 1) / PROJ_THREADS);
    // gridDim.y is limited to 65535: walk the chunks in slabs
    for (int64_t c0 = 0; c0 < C; c0 += 65535) {
        const unsigned gy = (unsigned)(C - c0 < 65535 ? C - c0 : 65535);
        const dim3 grid(gx, gy);
        float *qq = q ? q + c0 * A.r : nullptr;
        ProfileScope prof(KC_PROJECT, s);
        if (!A.generated && (int64_t)gx * gy < 2048) {
            const dim3 sgrid((unsigned)((r4 + 63) / 64), gy);
            project_rows_split_kernel<<<sgrid, PROJ_THREADS, 0, s>>>(idx + c0 * k, val + c0 * k, k, A, p + c0 * A.r, qq,
                                                                     out_scale);
        } else if (A.generated)
            project_kernel<true><<<grid, PROJ_THREADS, 0, s>>>(idx + c0 * k, val + c0 * k, k, A, p + c0 * A.r, qq,
                                                               out_scale);
        else
            project_kernel<false><<<grid, PROJ_THREADS, 0, s>>>(idx + c0 * k, val + c0 * k, k, A, p + c0 * A.r, qq,
                                                                out_scale);
    }
    return hipGetLastError();
}

} // namespace sgc
