// Sparsify_k (paper Sec. 4.2; per chunk in Def. 1): for every chunk the k entries of largest
// magnitude, emitted in ascending position with their signed values.
//
// One workgroup per chunk. Float chunks of up to 65536 elements take the register-resident kernel
// (one HBM read); longer chunks and bfloat16 take the general kernel, which re-reads the chunk
// (from L2) in every pass. In both, the k-th largest magnitude key is found exactly by a most-significant-
// digit radix select over the sign-cleared bit patterns (integer work only, so the result is the
// unique one under the rule "larger magnitude first, lower position among equals"). The output is
// then written in position order without a sort: every wavefront owns a contiguous slice of the
// chunk, counts its keys above / equal to the threshold, and a second walk over the slice turns
// wavefront ballots into output slots.
#include "sgc_internal.h"

namespace sgc {

template <typename T>
struct Elem;

template <>
struct Elem<float> {
    static constexpr int kKeyBits = 31;
    static constexpr int kPasses = 3;
    __device__ static uint32_t key(float v) { return __float_as_uint(v) & 0x7fffffffu; }
    __device__ static float widen(float v) { return v; }
    __device__ static int shift(int pass) { return pass == 0 ? 20 : (pass == 1 ? 9 : 0); }
    __device__ static int bits(int pass) { return pass == 2 ? 9 : 11; }
};

template <>
struct Elem<uint16_t> { // bfloat16 bit patterns
    static constexpr int kKeyBits = 15;
    static constexpr int kPasses = 2;
    __device__ static uint32_t key(uint16_t v) { return (uint32_t)v & 0x7fffu; }
    __device__ static float widen(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
    __device__ static int shift(int pass) { return pass == 0 ? 4 : 0; }
    __device__ static int bits(int pass) { return pass == 0 ? 11 : 4; }
};

// inclusive prefix sum over the workgroup, in thread order
template <int THREADS>
__device__ __forceinline__ uint32_t block_inclusive_scan(uint32_t v, uint32_t *wave_tot)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_up(v, off, 64);
        if (lane >= off)
            v += t;
    }
    if (lane == 63)
        wave_tot[w] = v;
    __syncthreads();
    uint32_t add = 0;
    for (int u = 0; u < w; ++u)
        add += wave_tot[u];
    __syncthreads();
    return v + add;
}

template <typename T, int THREADS>
__global__ __launch_bounds__(THREADS) void topk_kernel(const T *__restrict__ g, int32_t d, int32_t k,
                                                       int32_t *__restrict__ idx, float *__restrict__ val)
{
    constexpr int NW = THREADS / 64;
    __shared__ uint32_t hist[2048];
    __shared__ uint32_t wave_tot[NW];
    __shared__ uint32_t s_bin, s_need;
    __shared__ uint32_t w_gt[NW], w_eq[NW];

    const int tid = threadIdx.x;
    const T *gc = g + (int64_t)blockIdx.x * d;
    int32_t *oidx = idx + (int64_t)blockIdx.x * k;
    float *oval = val + (int64_t)blockIdx.x * k;

    uint32_t prefix = 0;              // decided high bits of the threshold key
    uint32_t need = (uint32_t)k;      // entries still to take among keys that match the prefix
    int decided = Elem<T>::kKeyBits;  // bits [decided, kKeyBits) are fixed

    for (int pass = 0; pass < Elem<T>::kPasses; ++pass) {
        const int shift = Elem<T>::shift(pass);
        const int nb = 1 << Elem<T>::bits(pass);
        for (int b = tid; b < nb; b += THREADS)
            hist[b] = 0;
        __syncthreads();
        for (int32_t i = tid; i < d; i += THREADS) {
            const uint32_t key = Elem<T>::key(gc[i]);
            if (pass == 0 || (key >> decided) == prefix)
                atomicAdd(&hist[(key >> shift) & (uint32_t)(nb - 1)], 1u);
        }
        __syncthreads();
        // thread t owns `per` bins counted from the top: [nb-(t+1)*per, nb-t*per)
        const int per = (nb + THREADS - 1) / THREADS;
        const int hi = nb - tid * per;          // exclusive
        const int lo = hi - per < 0 ? 0 : hi - per;
        uint32_t local = 0;
        for (int b = hi - 1; b >= lo && b >= 0; --b)
            local += hist[b];
        const uint32_t incl = block_inclusive_scan<THREADS>(local, wave_tot);
        const uint32_t excl = incl - local;
        if (excl < need && need <= incl) { // exactly one thread
            uint32_t run = excl;
            for (int b = hi - 1; b >= lo; --b) {
                const uint32_t h = hist[b];
                if (run + h >= need) {
                    s_bin = (uint32_t)b;
                    s_need = need - run;
                    break;
                }
                run += h;
            }
        }
        __syncthreads();
        prefix = (prefix << Elem<T>::bits(pass)) | s_bin;
        need = s_need;
        decided = shift;
        __syncthreads();
    }
    const uint32_t thr = prefix; // the k-th largest key; `need` of the keys equal to it are kept

    // wavefront slices, multiples of 64 positions
    const int lane = tid & 63, w = tid >> 6;
    int32_t seg = (d + NW - 1) / NW;
    seg = (seg + 63) & ~63;
    const int32_t beg = w * seg < d ? w * seg : d;
    const int32_t end = beg + seg < d ? beg + seg : d;

    uint32_t cgt = 0, ceq = 0;
    for (int32_t i0 = beg; i0 < end; i0 += 64) {
        const int32_t i = i0 + lane;
        const uint32_t key = i < end ? Elem<T>::key(gc[i]) : 0u;
        const bool in = i < end;
        cgt += (uint32_t)__popcll(__ballot(in && key > thr));
        ceq += (uint32_t)__popcll(__ballot(in && key == thr));
    }
    if (lane == 0) {
        w_gt[w] = cgt;
        w_eq[w] = ceq;
    }
    __syncthreads();
    uint32_t run_gt = 0, run_eq = 0;
    for (int u = 0; u < w; ++u) {
        run_gt += w_gt[u];
        run_eq += w_eq[u];
    }
    const uint64_t below = (1ull << lane) - 1ull;
    for (int32_t i0 = beg; i0 < end; i0 += 64) {
        const int32_t i = i0 + lane;
        const bool in = i < end;
        const T raw = in ? gc[i] : T(0);
        const uint32_t key = Elem<T>::key(raw);
        const bool gt = in && key > thr, eq = in && key == thr;
        const uint64_t bgt = __ballot(gt), beq = __ballot(eq);
        const uint32_t gt_before = run_gt + (uint32_t)__popcll(bgt & below);
        const uint32_t eq_before = run_eq + (uint32_t)__popcll(beq & below);
        if (gt || (eq && eq_before < need)) {
            const uint32_t slot = gt_before + (eq_before < need ? eq_before : need);
            oidx[slot] = i;
            oval[slot] = Elem<T>::widen(raw);
        }
        run_gt += (uint32_t)__popcll(bgt);
        run_eq += (uint32_t)__popcll(beq);
    }
}

// Register-resident variant for float chunks of up to 16 * 4 * THREADS elements: the chunk is read
// from HBM exactly once (16-byte loads, each wavefront owning a contiguous slice), the three radix
// passes and the ordered emission run on registers. Positions at or beyond d are loaded as 0.0f:
// such entries carry the smallest key and the largest positions, so they never change the k-th
// largest key of the real entries and are never emitted.
template <int THREADS>
__global__ __launch_bounds__(THREADS) void topk_f32_regs_kernel(const float *__restrict__ g, int32_t d, int32_t k,
                                                                int32_t *__restrict__ idx, float *__restrict__ val,
                                                                int32_t vector_loads)
{
    constexpr int NW = THREADS / 64, ROWS = 16;
    __shared__ uint32_t hist[2048];
    __shared__ uint32_t wave_tot[NW];
    __shared__ uint32_t s_bin, s_need;
    __shared__ uint32_t w_gt[NW], w_eq[NW];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const float *gc = g + (int64_t)blockIdx.x * d;
    int32_t *oidx = idx + (int64_t)blockIdx.x * k;
    float *oval = val + (int64_t)blockIdx.x * k;
    const int32_t wbase = w * (ROWS * 256) + lane * 4; // element (j, e) of this lane sits at wbase + 256 j + e

    float4 v[ROWS];
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const int32_t i0 = wbase + j * 256;
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
        if (vector_loads && i0 + 3 < d) {
            t = *reinterpret_cast<const float4 *>(gc + i0);
        } else {
            if (i0 < d) t.x = gc[i0];
            if (i0 + 1 < d) t.y = gc[i0 + 1];
            if (i0 + 2 < d) t.z = gc[i0 + 2];
            if (i0 + 3 < d) t.w = gc[i0 + 3];
        }
        v[j] = t;
    }
    auto key_of = [](float f) { return __float_as_uint(f) & 0x7fffffffu; };

    uint32_t prefix = 0, need = (uint32_t)k;
    for (int pass = 0; pass < 3; ++pass) {
        const int shift = pass == 0 ? 20 : (pass == 1 ? 9 : 0);
        const int bits = pass == 2 ? 9 : 11;
        const int decided = pass == 0 ? 31 : (pass == 1 ? 20 : 9);
        const int nb = 1 << bits;
        for (int b = tid; b < nb; b += THREADS)
            hist[b] = 0;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < ROWS; ++j) {
            const float e4[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t key = key_of(e4[e]);
                if (pass == 0 || (key >> decided) == prefix)
                    atomicAdd(&hist[(key >> shift) & (uint32_t)(nb - 1)], 1u);
            }
        }
        __syncthreads();
        const int per = (nb + THREADS - 1) / THREADS;
        const int hi = nb - tid * per;
        const int lo = hi - per < 0 ? 0 : hi - per;
        uint32_t local = 0;
        for (int b = hi - 1; b >= lo && b >= 0; --b)
            local += hist[b];
        const uint32_t incl = block_inclusive_scan<THREADS>(local, wave_tot);
        const uint32_t excl = incl - local;
        if (excl < need && need <= incl) {
            uint32_t run = excl;
            for (int b = hi - 1; b >= lo; --b) {
                const uint32_t h = hist[b];
                if (run + h >= need) {
                    s_bin = (uint32_t)b;
                    s_need = need - run;
                    break;
                }
                run += h;
            }
        }
        __syncthreads();
        prefix = (prefix << bits) | s_bin;
        need = s_need;
        __syncthreads();
    }
    const uint32_t thr = prefix;

    // per-wavefront totals of keys above / equal to the threshold
    uint32_t cgt = 0, ceq = 0;
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const float e4[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t key = key_of(e4[e]);
            cgt += key > thr ? 1u : 0u;
            ceq += key == thr ? 1u : 0u;
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        cgt += __shfl_xor(cgt, off, 64);
        ceq += __shfl_xor(ceq, off, 64);
    }
    if (lane == 0) {
        w_gt[w] = cgt;
        w_eq[w] = ceq;
    }
    __syncthreads();
    uint32_t run_gt = 0, run_eq = 0;
    for (int u = 0; u < w; ++u) {
        run_gt += w_gt[u];
        run_eq += w_eq[u];
    }
    // ordered emission: position order inside the slice is (row j, lane, e)
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const float e4[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
        bool gt[4], eq[4];
        bool any = false;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t key = key_of(e4[e]);
            gt[e] = key > thr;
            eq[e] = key == thr;
            any = any || gt[e] || eq[e];
        }
        if (__ballot(any) == 0ull)
            continue;
        uint32_t gt_before = run_gt, eq_before = run_eq, tot_gt = 0, tot_eq = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint64_t bg = __ballot(gt[e]), be = __ballot(eq[e]);
            gt_before += __builtin_amdgcn_mbcnt_hi((uint32_t)(bg >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bg, 0u));
            eq_before += __builtin_amdgcn_mbcnt_hi((uint32_t)(be >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)be, 0u));
            tot_gt += (uint32_t)__popcll(bg);
            tot_eq += (uint32_t)__popcll(be);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (gt[e] || (eq[e] && eq_before < need)) {
                const uint32_t slot = gt_before + (eq_before < need ? eq_before : need);
                oidx[slot] = wbase + j * 256 + e;
                oval[slot] = e4[e];
            }
            gt_before += gt[e] ? 1u : 0u;
            eq_before += eq[e] ? 1u : 0u;
        }
        run_gt += tot_gt;
        run_eq += tot_eq;
    }
}

hipError_t launch_topk(const void *grad, int grad_type, int64_t C, int32_t d, int32_t k, int32_t *idx,
                       float *val, hipStream_t s)
{
    if (C == 0)
        return hipSuccess;
    const dim3 grid((unsigned)C);
    ProfileScope prof(KC_TOPK, s);
    if (grad_type == SGC_GRAD_F32) {
        const int32_t vec = (d % 4 == 0) ? 1 : 0; // every chunk then starts 16-byte aligned
        if (d <= 16 * 4 * 256)
            topk_f32_regs_kernel<256><<<grid, 256, 0, s>>>((const float *)grad, d, k, idx, val, vec);
        else if (d <= 16 * 4 * 1024)
            topk_f32_regs_kernel<1024><<<grid, 1024, 0, s>>>((const float *)grad, d, k, idx, val, vec);
        else
            topk_kernel<float, 1024><<<grid, 1024, 0, s>>>((const float *)grad, d, k, idx, val);
    } else {
        if (d <= 16384)
            topk_kernel<uint16_t, 256><<<grid, 256, 0, s>>>((const uint16_t *)grad, d, k, idx, val);
        else
            topk_kernel<uint16_t, 1024><<<grid, 1024, 0, s>>>((const uint16_t *)grad, d, k, idx, val);
    }
    return hipGetLastError();
}

} // namespace sgc
