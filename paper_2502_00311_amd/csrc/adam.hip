// Compressed AdamW moments (paper eq. 7-8 and Alg. 2 lines 2-5) on the r-dimensional
// measurements of every chunk: one fused elementwise pass, 32 bytes moved per state element.
#include "sgc_internal.h"

namespace sgc {

struct AdamCoef {
    float b1, omb1, b2, omb2, ibc1, ibc2;
};

__device__ __forceinline__ void adam_one(float p, float q, float &m, float &v, float &mh, float &vh,
                                         const AdamCoef &c)
{
    m = __builtin_fmaf(c.b1, m, c.omb1 * p);
    v = __builtin_fmaf(c.b2, v, c.omb2 * q);
    mh = m * c.ibc1;
    vh = v * c.ibc2;
}

__global__ __launch_bounds__(256) void adam_kernel(const float *__restrict__ p, const float *__restrict__ q,
                                                   float *__restrict__ m, float *__restrict__ v,
                                                   float *__restrict__ mhat, float *__restrict__ vhat,
                                                   int64_t count, AdamCoef c)
{
    const int64_t n4 = count >> 2;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
        const float4 pp = reinterpret_cast<const float4 *>(p)[i];
        const float4 qq = reinterpret_cast<const float4 *>(q)[i];
        float4 mm = reinterpret_cast<float4 *>(m)[i];
        float4 vv = reinterpret_cast<float4 *>(v)[i];
        float4 mh, vh;
        adam_one(pp.x, qq.x, mm.x, vv.x, mh.x, vh.x, c);
        adam_one(pp.y, qq.y, mm.y, vv.y, mh.y, vh.y, c);
        adam_one(pp.z, qq.z, mm.z, vv.z, mh.z, vh.z, c);
        adam_one(pp.w, qq.w, mm.w, vv.w, mh.w, vh.w, c);
        reinterpret_cast<float4 *>(m)[i] = mm;
        reinterpret_cast<float4 *>(v)[i] = vv;
        reinterpret_cast<float4 *>(mhat)[i] = mh;
        reinterpret_cast<float4 *>(vhat)[i] = vh;
    }
    // tail (count not a multiple of 4)
    const int64_t t = (n4 << 2) + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t < count) {
        float mm = m[t], vv = v[t], mh, vh;
        adam_one(p[t], q[t], mm, vv, mh, vh, c);
        m[t] = mm;
        v[t] = vv;
        mhat[t] = mh;
        vhat[t] = vh;
    }
}

hipError_t launch_adam(const float *p, const float *q, float *m, float *v, float *mhat, float *vhat,
                       int64_t count, float b1, float omb1, float b2, float omb2, float ibc1, float ibc2,
                       hipStream_t s)
{
    if (count == 0)
        return hipSuccess;
    const int64_t n4 = (count + 3) >> 2;
    int64_t blocks = (n4 + 255) / 256;
    if (blocks > 256 * 16)
        blocks = 256 * 16;
    if (blocks < 1)
        blocks = 1;
    ProfileScope prof(KC_ADAM, s);
    adam_kernel<<<dim3((unsigned)blocks), 256, 0, s>>>(p, q, m, v, mhat, vhat, count,
                                                       AdamCoef{b1, omb1, b2, omb2, ibc1, ibc2});
    return hipGetLastError();
}

} // namespace sgc
