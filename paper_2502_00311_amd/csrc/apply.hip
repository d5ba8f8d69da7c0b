// Update in parameter space (paper eq. 11, Alg. 2 line 6, eq. 3): the recovered first and second
// moments are sparse vectors of R^d; on the support of the first,
//   W[i] -= lr * alpha * x_i / (sqrt(max(z_i, 0)) + eps),
// with z_i = 0 where the second recovery did not select position i.
#include "sgc_internal.h"

namespace sgc {

constexpr int APPLY_THREADS = 256;
constexpr int APPLY_MAXK = 4096;

__global__ __launch_bounds__(APPLY_THREADS) void apply_kernel(float *__restrict__ W, int32_t d, int32_t k,
                                                              const int32_t *__restrict__ sel_m,
                                                              const float *__restrict__ x_m,
                                                              const int32_t *__restrict__ sel_v,
                                                              const float *__restrict__ x_v, float alpha,
                                                              float eps, float lr)
{
    __shared__ int32_t s_pos[APPLY_MAXK];
    __shared__ float s_z[APPLY_MAXK];
    const int64_t c = blockIdx.x;
    for (int32_t t = threadIdx.x; t < k; t += APPLY_THREADS) {
        s_pos[t] = sel_v[c * k + t];
        s_z[t] = x_v[c * k + t];
    }
    __syncthreads();
    for (int32_t t = threadIdx.x; t < k; t += APPLY_THREADS) {
        const int32_t i = sel_m[c * k + t];
        const float x = x_m[c * k + t];
        float z = 0.f;
        for (int32_t u = 0; u < k; ++u)
            z = (s_pos[u] == i) ? s_z[u] : z;
        z = z > 0.f ? z : 0.f;
        if (x != 0.f && i >= 0 && i < d) { // a position outside the chunk (a recovery that gave up) updates nothing
            const float nv = alpha * x / (sqrtf(z) + eps);
            float *w = W + c * (int64_t)d + i;
            *w = *w - lr * nv;
        }
    }
}

hipError_t launch_apply(float *W, int64_t C, int32_t d, int32_t k, const int32_t *sel_m, const float *x_m,
                        const int32_t *sel_v, const float *x_v, float alpha, float eps, float lr,
                        hipStream_t s)
{
    if (C == 0)
        return hipSuccess;
    ProfileScope prof(KC_APPLY, s);
    apply_kernel<<<dim3((unsigned)C), APPLY_THREADS, 0, s>>>(W, d, k, sel_m, x_m, sel_v, x_v, alpha, eps, lr);
    return hipGetLastError();
}

} // namespace sgc
