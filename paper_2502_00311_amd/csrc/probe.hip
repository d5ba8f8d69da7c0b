// Machine probes (instrumentation, not a step of the method): small kernels that measure what the chip
// delivers for the resources the library's kernels are bound by, so that a fraction quoted against a
// published peak can be read next to the rate measured on the same machine. The caller times them.
//   SGC_PROBE_VALU   register-only chains of plain (non-packed) v_fma_f32: vector-ALU issue rate
//   SGC_PROBE_MFMA   register-only v_mfma_f32_32x32x2f32: float matrix-core rate
//   SGC_PROBE_MFMA_VALU4 / 8   the MFMA loop with 4 / 8 independent v_fma_f32 behind every MFMA
//   SGC_PROBE_SPLIT_BOTH / _MFMA / _VALU   workgroups of eight wavefronts, two per SIMD: four issue only the MFMAs
//                    of SGC_PROBE_MFMA, four only plain v_fma_f32 (256 per 16 MFMAs); both groups, or one of them alone
//   SGC_PROBE_READ   streaming read with non-temporal 16-byte loads
//   SGC_PROBE_RW44   four arrays read and four written, in the loop structure of the Adam kernel
//   SGC_PROBE_COPY   one array read, one written
#include "sgc_internal.h"

namespace sgc {

constexpr int PROBE_CHAINS = 16;

__global__ __launch_bounds__(256) void probe_valu_kernel(float *out, int32_t iters)
{
    float acc[PROBE_CHAINS];
    const float x = 1.0f + 1e-7f * (float)threadIdx.x, y = 1e-9f * (float)blockIdx.x;
#pragma unroll
    for (int c = 0; c < PROBE_CHAINS; ++c)
        acc[c] = (float)c;
    for (int32_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int c = 0; c < PROBE_CHAINS; ++c)
                asm volatile("v_fma_f32 %0, %1, %0, %2" : "+v"(acc[c]) : "v"(x), "v"(y));
        }
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < PROBE_CHAINS; ++c)
        s += acc[c];
    if (s == 123.456f) // never true: keeps the chains alive without a store per thread
        out[0] = s;
}

__global__ __launch_bounds__(256) void probe_mfma_kernel(float *out, int32_t iters)
{
    typedef float floatx16 __attribute__((ext_vector_type(16)));
    floatx16 a0 = {0}, a1 = {0}, a2 = {0}, a3 = {0};
    const float x = threadIdx.x * 1e-3f, y = blockIdx.x * 1e-3f;
    for (int32_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            a0 = __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, a0, 0, 0, 0);
            a1 = __builtin_amdgcn_mfma_f32_32x32x2f32(y, x, a1, 0, 0, 0);
            a2 = __builtin_amdgcn_mfma_f32_32x32x2f32(x, x, a2, 0, 0, 0);
            a3 = __builtin_amdgcn_mfma_f32_32x32x2f32(y, y, a3, 0, 0, 0);
        }
    }
    float s = 0.f;
    for (int v = 0; v < 16; ++v)
        s += a0[v] + a1[v] + a2[v] + a3[v];
    if (s == 123.456f)
        out[0] = s;
}

// per iteration 16 MFMAs and, between them, VALU_PER_MFMA independent v_fma_f32 each: does vector-ALU work ride in
// the shadow of the float matrix instructions of the same wavefront / SIMD, or does it add to their time?
template <int VALU_PER_MFMA>
__global__ __launch_bounds__(256) void probe_mix_kernel(float *out, int32_t iters)
{
    typedef float floatx16 __attribute__((ext_vector_type(16)));
    floatx16 a0 = {0}, a1 = {0}, a2 = {0}, a3 = {0};
    float acc[PROBE_CHAINS];
    const float x = threadIdx.x * 1e-3f, y = blockIdx.x * 1e-3f;
    const float fx = 1.0f + 1e-7f * (float)threadIdx.x, fy = 1e-9f * (float)blockIdx.x;
#pragma unroll
    for (int c = 0; c < PROBE_CHAINS; ++c)
        acc[c] = (float)c;
    for (int32_t i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            a0 = __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, a0, 0, 0, 0);
#pragma unroll
            for (int c = 0; c < VALU_PER_MFMA; ++c)
                asm volatile("v_fma_f32 %0, %1, %0, %2" : "+v"(acc[(4 * u * VALU_PER_MFMA + c) % PROBE_CHAINS]) : "v"(fx), "v"(fy));
            a1 = __builtin_amdgcn_mfma_f32_32x32x2f32(y, x, a1, 0, 0, 0);
#pragma unroll
            for (int c = 0; c < VALU_PER_MFMA; ++c)
                asm volatile("v_fma_f32 %0, %1, %0, %2" : "+v"(acc[((4 * u + 1) * VALU_PER_MFMA + c) % PROBE_CHAINS]) : "v"(fx), "v"(fy));
            a2 = __builtin_amdgcn_mfma_f32_32x32x2f32(x, x, a2, 0, 0, 0);
#pragma unroll
            for (int c = 0; c < VALU_PER_MFMA; ++c)
                asm volatile("v_fma_f32 %0, %1, %0, %2" : "+v"(acc[((4 * u + 2) * VALU_PER_MFMA + c) % PROBE_CHAINS]) : "v"(fx), "v"(fy));
            a3 = __builtin_amdgcn_mfma_f32_32x32x2f32(y, y, a3, 0, 0, 0);
#pragma unroll
            for (int c = 0; c < VALU_PER_MFMA; ++c)
                asm volatile("v_fma_f32 %0, %1, %0, %2" : "+v"(acc[((4 * u + 3) * VALU_PER_MFMA + c) % PROBE_CHAINS]) : "v"(fx), "v"(fy));
        }
    }
    float s = 0.f;
    for (int v = 0; v < 16; ++v)
        s += a0[v] + a1[v] + a2[v] + a3[v];
#pragma unroll
    for (int c = 0; c < PROBE_CHAINS; ++c)
        s += acc[c];
    if (s == 123.456f)
        out[0] = s;
}

// Does vector-ALU work of OTHER wavefronts on the same SIMD run beside float matrix instructions? Wavefronts 0-3 of a
// workgroup (one per SIMD) issue iters x 16 MFMAs, wavefronts 4-7 iters x 256 plain FMAs; WHICH: 0 both, 1 the
// MFMA wavefronts alone (the others leave at once), 2 the FMA wavefronts alone.
template <int WHICH>
__global__ __launch_bounds__(512) void probe_split_kernel(float *out, int32_t iters)
{
    typedef float floatx16 __attribute__((ext_vector_type(16)));
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    float s = 0.f;
    if (wave < 4) {
        if (WHICH == 2)
            return;
        floatx16 a0 = {0}, a1 = {0}, a2 = {0}, a3 = {0};
        const float x = threadIdx.x * 1e-3f, y = blockIdx.x * 1e-3f;
        for (int32_t i = 0; i < iters; ++i) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                a0 = __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, a0, 0, 0, 0);
                a1 = __builtin_amdgcn_mfma_f32_32x32x2f32(y, x, a1, 0, 0, 0);
                a2 = __builtin_amdgcn_mfma_f32_32x32x2f32(x, x, a2, 0, 0, 0);
                a3 = __builtin_amdgcn_mfma_f32_32x32x2f32(y, y, a3, 0, 0, 0);
            }
        }
        for (int v = 0; v < 16; ++v)
            s += a0[v] + a1[v] + a2[v] + a3[v];
    } else {
        if (WHICH == 1)
            return;
        float acc[PROBE_CHAINS];
        const float x = 1.0f + 1e-7f * (float)threadIdx.x, y = 1e-9f * (float)blockIdx.x;
#pragma unroll
        for (int c = 0; c < PROBE_CHAINS; ++c)
            acc[c] = (float)c;
        for (int32_t i = 0; i < iters; ++i) {
#pragma unroll
            for (int u = 0; u < 16; ++u) {
#pragma unroll
                for (int c = 0; c < PROBE_CHAINS; ++c)
                    asm volatile("v_fma_f32 %0, %1, %0, %2" : "+v"(acc[c]) : "v"(x), "v"(y));
            }
        }
#pragma unroll
        for (int c = 0; c < PROBE_CHAINS; ++c)
            s += acc[c];
    }
    if (s == 123.456f)
        out[0] = s;
}

__global__ __launch_bounds__(256) void probe_read_kernel(const float *__restrict__ a, float *out, int64_t n4)
{
    constexpr int U = 16;
    float s = 0.f;
    const int64_t per_pass = (int64_t)blockDim.x * U;
    for (int64_t base = (int64_t)blockIdx.x * per_pass; base < n4; base += (int64_t)gridDim.x * per_pass) {
        float4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + threadIdx.x + (int64_t)u * blockDim.x;
            v[u] = i < n4 ? load_once_f4(a + 4 * i) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
            s += v[u].x + v[u].y + v[u].z + v[u].w;
    }
    if (s == 123.456f)
        out[0] = s;
}

// STREAMS arrays of n4 quads read from a, STREAMS written to b (array j starts at j * n4 quads)
template <int STREAMS>
__global__ __launch_bounds__(256) void probe_rw_kernel(const float *__restrict__ a, float *__restrict__ b, int64_t n4)
{
    constexpr int U = 4;
    const int64_t per_pass = (int64_t)blockDim.x * U;
    for (int64_t base = (int64_t)blockIdx.x * per_pass; base < n4; base += (int64_t)gridDim.x * per_pass) {
        float4 v[STREAMS][U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + threadIdx.x + (int64_t)u * blockDim.x;
            if (i < n4) {
#pragma unroll
                for (int j = 0; j < STREAMS; ++j)
                    v[j][u] = load_once_f4(a + 4 * (j * n4 + i));
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = base + threadIdx.x + (int64_t)u * blockDim.x;
            if (i < n4) {
#pragma unroll
                for (int j = 0; j < STREAMS; ++j)
                    reinterpret_cast<float4 *>(b)[j * n4 + i] = v[j][u];
            }
        }
    }
}

} // namespace sgc

using namespace sgc;

extern "C" sgc_status sgc_probe(int32_t kind, const void *a, void *b, int64_t bytes, int32_t blocks, int32_t iters,
                                void *stream)
{
    hipStream_t s = (hipStream_t)stream;
    if (blocks <= 0 || blocks > (1 << 20) || iters < 0 || bytes < 0)
        return SGC_ERR_SHAPE;
    if (!b)
        return SGC_ERR_NULL;
    if (((uintptr_t)a & 15u) || ((uintptr_t)b & 15u))
        return SGC_ERR_ALIGN;
    switch (kind) {
    case SGC_PROBE_VALU:
        probe_valu_kernel<<<dim3((unsigned)blocks), 256, 0, s>>>((float *)b, iters);
        break;
    case SGC_PROBE_MFMA:
        probe_mfma_kernel<<<dim3((unsigned)blocks), 256, 0, s>>>((float *)b, iters);
        break;
    case SGC_PROBE_MFMA_VALU4:
        probe_mix_kernel<4><<<dim3((unsigned)blocks), 256, 0, s>>>((float *)b, iters);
        break;
    case SGC_PROBE_MFMA_VALU8:
        probe_mix_kernel<8><<<dim3((unsigned)blocks), 256, 0, s>>>((float *)b, iters);
        break;
    case SGC_PROBE_SPLIT_BOTH:
        probe_split_kernel<0><<<dim3((unsigned)blocks), 512, 0, s>>>((float *)b, iters);
        break;
    case SGC_PROBE_SPLIT_MFMA:
        probe_split_kernel<1><<<dim3((unsigned)blocks), 512, 0, s>>>((float *)b, iters);
        break;
    case SGC_PROBE_SPLIT_VALU:
        probe_split_kernel<2><<<dim3((unsigned)blocks), 512, 0, s>>>((float *)b, iters);
        break;
    case SGC_PROBE_READ:
        if (!a)
            return SGC_ERR_NULL;
        probe_read_kernel<<<dim3((unsigned)blocks), 256, 0, s>>>((const float *)a, (float *)b, bytes / 16);
        break;
    case SGC_PROBE_RW44:
        if (!a)
            return SGC_ERR_NULL;
        probe_rw_kernel<4><<<dim3((unsigned)blocks), 256, 0, s>>>((const float *)a, (float *)b, bytes / 16 / 8);
        break;
    case SGC_PROBE_COPY:
        if (!a)
            return SGC_ERR_NULL;
        probe_rw_kernel<1><<<dim3((unsigned)blocks), 256, 0, s>>>((const float *)a, (float *)b, bytes / 16 / 2);
        break;
    default:
        return SGC_ERR_DTYPE;
    }
    return hipGetLastError() == hipSuccess ? SGC_OK : SGC_ERR_DEVICE;
}
