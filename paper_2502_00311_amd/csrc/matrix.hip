// Utilities on the measurement matrix (paper Sec. 4.3): materialise the generated matrix, and
// the reciprocal column norms used by the OMP selection rule of App. B.
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
