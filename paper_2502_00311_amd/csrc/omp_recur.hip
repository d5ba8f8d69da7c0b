// The recovery with App. B's recurrence for the correlation vector (Alg. 3): with the table of column
// inner products G = A^H A at hand, p = A^H res is not recomputed by a contraction in every iteration
// but updated, p <- p - b_j a_j, where b_j = A^H q_j is the image of the new orthonormal direction
// q_j = A_Lambda F_:j and follows from the earlier ones, b_j = gamma_j (G_:lambda_j - sum_t c_t b_t), with
// c_t = <F_:t, w> the coordinates the least-squares update computes anyway and a_j = q_j^H y its new
// coefficient. Per right-hand side the vectors b_t are kept (d x k floats, the matrix B of App. B); an
// iteration streams the j vectors already there, one row of G, and p - no matrix-core work at all.
// Everything around it is the plain recovery: the same selection kernel (candidates near the maximum
// of p re-scored in double against the residual) and the same least-squares update.
#include "omp_internal.h"

namespace sgc {

// p0 = A^H y for every right-hand side, written out (the one contraction of a call): a wavefront takes
// 32 positions x 64 right-hand sides, operands straight from the caches (this runs once per call).
// grid (ceil(d / 128), ceil(N / 64)); rows of At resident; d % 4 == 0.
__global__ __launch_bounds__(256) void recur_init_kernel(MatrixView A, const float *__restrict__ Y, int32_t N,
                                                         float *__restrict__ p)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lhalf = lane >> 5;
    const int32_t d = A.d, r = A.r;
    const int32_t m0 = blockIdx.x * 128 + wave * 32, n0 = blockIdx.y * 64;
    const int32_t row = m0 + l32 < d ? m0 + l32 : d - 1; // clamped: results of rows past the end are dropped
    const float *arow = A.At + (int64_t)row * r;
    const float *yrow[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int32_t n = n0 + 32 * b + l32;
        yrow[b] = Y + (int64_t)(n < N ? n : N - 1) * r;
    }
    floatx16 acc[2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v)
            acc[b][v] = 0.f;
    for (int32_t kk = 0; kk < r; kk += 8) {
        const int32_t dep = kk + 4 * lhalf;      // this lane's four depths
        const bool valid = dep < r;              // r % 8 == 4: the upper half-wave has nothing in the last step
        const int32_t at = valid ? dep : kk;
        float4 a = *reinterpret_cast<const float4 *>(arow + at);
        float4 y0 = *reinterpret_cast<const float4 *>(yrow[0] + at);
        float4 y1 = *reinterpret_cast<const float4 *>(yrow[1] + at);
        if (!valid)
            a = make_float4(0.f, 0.f, 0.f, 0.f);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, y0.x, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, y1.x, acc[1], 0, 0, 0);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, y0.y, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, y1.y, acc[1], 0, 0, 0);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, y0.z, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, y1.z, acc[1], 0, 0, 0);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, y0.w, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, y1.w, acc[1], 0, 0, 0);
    }
    // accumulator register v of lane l: position 8 (v / 4) + 4 (l / 32) + v % 4, right-hand side l % 32
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int32_t n = n0 + 32 * b + l32;
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            const int32_t i = m0 + 8 * qd + 4 * lhalf;
            if (n < N && i < d)
                *reinterpret_cast<float4 *>(p + (int64_t)n * d + i) =
                    make_float4(acc[b][4 * qd], acc[b][4 * qd + 1], acc[b][4 * qd + 2], acc[b][4 * qd + 3]);
        }
    }
}

__device__ __forceinline__ void top2_put(uint64_t key, uint64_t &best, uint64_t &second)
{
    const uint64_t lo = key < best ? key : best;
    best = key > best ? key : best;
    second = lo > second ? lo : second;
}

struct RecurArgs {
    const double *gram;       // [d][d]
    const float *inv_colnorm; // [d]
    int32_t d, k, it;         // it: the iteration whose selection and update have just been made
    const int32_t *sel;       // [N][k]
    const double *F;          // inverse Cholesky factors (gamma_it on the diagonal of column it)
    int64_t f_stride;
    const double *avec;       // [N][k] coefficients a
    const double *cvec;       // [N][k] coordinates c of the iteration
    float *p;                 // [N][d]
    float *B;                 // [N][head][d]
    int32_t head;             // image vectors kept per right-hand side (iterations the recurrence serves)
    const uint32_t *bitmap;   // [N][words]
    int32_t words, tiles;     // tiles of 256 positions
    uint64_t *partial;        // [N][tiles][2]
};

// grid (N, ceil(d / 1024)): a workgroup takes 1024 positions of one right-hand side, a lane four adjacent
// ones. FIRST: only the two best (score, position) keys per tile of 256 positions are formed from p0;
// otherwise b_it is formed and stored, p updated, and the keys taken from the new p.
// The keys have the format of the contraction kernels' epilogue, which the selection kernel reads.
template <bool FIRST>
__global__ __launch_bounds__(256) void recur_step_kernel(RecurArgs R)
{
    __shared__ double c_s[1024];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t n = blockIdx.x;
    const int32_t d = R.d, k = R.k, it = R.it;
    const int32_t tile = blockIdx.y * 4 + wave;
    const int32_t pos = tile * 256 + lane * 4;
    const bool in = pos < d; // d % 4 == 0: a quad is inside or outside as a whole
    const int32_t at = in ? pos : 0;
    float *pn = R.p + n * d;
    float4 p4 = load_once_f4(pn + at);
    if (!FIRST) {
        for (int32_t t = tid; t < it; t += 256)
            c_s[t] = R.cvec[n * k + t];
        const int32_t lam = R.sel[n * k + it];
        const double gamma = R.F[n * R.f_stride + (int64_t)it * k + it], coef = R.avec[n * k + it];
        const double *grow = R.gram + (int64_t)lam * d + at;
        double a0 = grow[0], a1 = grow[1], a2 = grow[2], a3 = grow[3];
        __syncthreads();
        const float *Bn = R.B + (n * R.head) * (int64_t)d + at;
        int32_t t = 0;
        for (; t + 8 <= it; t += 8) {
            float4 b[8];
#pragma unroll
            for (int q = 0; q < 8; ++q)
                b[q] = load_once_f4(Bn + (int64_t)(t + q) * d);
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const double c = c_s[t + q];
                a0 -= c * b[q].x;
                a1 -= c * b[q].y;
                a2 -= c * b[q].z;
                a3 -= c * b[q].w;
            }
        }
        for (; t < it; ++t) {
            const float4 b = load_once_f4(Bn + (int64_t)t * d);
            const double c = c_s[t];
            a0 -= c * b.x;
            a1 -= c * b.y;
            a2 -= c * b.z;
            a3 -= c * b.w;
        }
        const float4 bn = make_float4((float)(gamma * a0), (float)(gamma * a1), (float)(gamma * a2), (float)(gamma * a3));
        p4.x = (float)((double)p4.x - coef * bn.x);
        p4.y = (float)((double)p4.y - coef * bn.y);
        p4.z = (float)((double)p4.z - coef * bn.z);
        p4.w = (float)((double)p4.w - coef * bn.w);
        if (in) { // neither is read again before the next iteration: past the caches
            typedef float floatx4_t __attribute__((ext_vector_type(4)));
            const floatx4_t bv = {bn.x, bn.y, bn.z, bn.w}, pv = {p4.x, p4.y, p4.z, p4.w};
            __builtin_nontemporal_store(bv, reinterpret_cast<floatx4_t *>(R.B + (n * R.head + it) * (int64_t)d + pos));
            __builtin_nontemporal_store(pv, reinterpret_cast<floatx4_t *>(pn + pos));
        }
    }
    // scores of the four positions, selected ones left out
    uint64_t best = 0, second = 0;
    if (in) {
        const float4 nv = *reinterpret_cast<const float4 *>(R.inv_colnorm + pos);
        const uint32_t mask = R.bitmap[n * R.words + (pos >> 5)] >> (pos & 31);
        const float sc[4] = {fabsf(p4.x) * nv.x, fabsf(p4.y) * nv.y, fabsf(p4.z) * nv.z, fabsf(p4.w) * nv.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint64_t key = ((mask >> e) & 1u) ? 0ull
                                                     : (((uint64_t)__float_as_uint(sc[e]) << 32) |
                                                        (uint64_t)(0xffffffffu - (uint32_t)(pos + e)));
            top2_put(key, best, second);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint64_t ob = shfl_xor_u64(best, off), os = shfl_xor_u64(second, off);
        top2_put(ob, best, second);
        top2_put(os, best, second);
    }
    if (lane == 0 && tile < R.tiles) {
        uint64_t *o = R.partial + (n * R.tiles + tile) * 2;
        o[0] = best;
        o[1] = second;
    }
}

hipError_t recur_init_launch(const MatrixView &A, const float *y, int32_t N, const OmpWorkspace &w, hipStream_t s)
{
    recur_init_kernel<<<dim3((unsigned)((A.d + 127) / 128), (unsigned)((N + 63) / 64)), 256, 0, s>>>(A, y, N, w.rc_p);
    return hipGetLastError();
}

hipError_t recur_step_launch(bool first, const MatrixView &A, int32_t N, int32_t k, int32_t it, const int32_t *sel,
                             const OmpWorkspace &w, int32_t tiles, hipStream_t s)
{
    RecurArgs R{A.gram, A.inv_colnorm, A.d, k, it, sel, w.F, w.f_stride, w.avec, w.cvec, w.rc_p, w.rc_B, w.rc_head,
                w.bitmap, w.words, tiles, w.partial};
    const dim3 grid((unsigned)N, (unsigned)((A.d + 1023) / 1024));
    if (first)
        recur_step_kernel<true><<<grid, 256, 0, s>>>(R);
    else
        recur_step_kernel<false><<<grid, 256, 0, s>>>(R);
    return hipGetLastError();
}

} // namespace sgc
