// Sparsify_k (paper Sec. 4.2; per chunk in Def. 1): for every chunk the k entries of largest
// magnitude, emitted in ascending position with their signed values.
//
// One workgroup per chunk. Float chunks of up to 65536 elements take the register-resident kernel
// (one HBM read); bfloat16 chunks a two-sweep kernel that selects on a short list of candidates; everything
// else the general kernel, which re-reads the chunk (from L2) in every pass. In both, the k-th largest magnitude key is found exactly by a most-significant-
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

// General path: every pass re-reads the chunk from memory (L2 after the first pass). Works for any
// chunk length and element type; also the fallback of the register-resident kernel.
template <typename T, int THREADS>
__device__ __forceinline__ void topk_general(const T *__restrict__ gc, int32_t d, int32_t k,
                                             int32_t *__restrict__ oidx, float *__restrict__ oval)
{
    constexpr int NW = THREADS / 64;
    __shared__ uint32_t hist[2048];
    __shared__ uint32_t wave_tot[NW];
    __shared__ uint32_t s_bin, s_need;
    __shared__ uint32_t w_gt[NW], w_eq[NW];

    const int tid = threadIdx.x;

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

template <typename T, int THREADS>
__global__ __launch_bounds__(THREADS) void topk_kernel(const T *__restrict__ g, int32_t d, int32_t k,
                                                       int32_t *__restrict__ idx, float *__restrict__ val)
{
    topk_general<T, THREADS>(g + (int64_t)blockIdx.x * d, d, k, idx + (int64_t)blockIdx.x * k,
                             val + (int64_t)blockIdx.x * k);
}

constexpr uint32_t TOPK_CAND_CAP = 2048; // candidate entries kept in LDS

// The kth largest of n sign-cleared keys held in LDS (any float bit patterns; the sign bit is
// ignored), found by one wavefront: a bitwise binary search on the 31-bit key whose counts are
// wavefront ballots. Also returns how many keys are larger than / equal to the result.
__device__ __forceinline__ uint32_t wave_kth_largest(const uint32_t *keys, uint32_t n, uint32_t kth, uint32_t &gt,
                                                     uint32_t &eq, int key_bits = 31)
{
    const uint32_t lane = threadIdx.x & 63;
    uint32_t thr = 0;
    gt = 0;
    eq = 0;
    if (n <= 64 * 8) {
        // the usual case: the keys fit eight registers per lane, the search never touches LDS again
        uint32_t kr[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const uint32_t s = q * 64 + lane;
            kr[q] = s < n ? (keys[s] & 0x7fffffffu) : 0u; // padding keys are 0: never >= a candidate
        }
        for (int bit = key_bits - 1; bit >= 0; --bit) {
            const uint32_t cand = thr | (1u << bit);
            uint32_t cnt = 0;
#pragma unroll
            for (int q = 0; q < 8; ++q)
                cnt += (uint32_t)__popcll(__ballot(kr[q] >= cand));
            thr = cnt >= kth ? cand : thr;
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const bool in = q * 64 + lane < n;
            gt += (uint32_t)__popcll(__ballot(in && kr[q] > thr));
            eq += (uint32_t)__popcll(__ballot(in && kr[q] == thr));
        }
        return thr;
    }
    for (int bit = key_bits - 1; bit >= 0; --bit) {
        const uint32_t cand = thr | (1u << bit);
        uint32_t cnt = 0;
        for (uint32_t s0 = 0; s0 < n; s0 += 64) {
            const uint32_t s = s0 + lane;
            const bool ge = s < n && (keys[s] & 0x7fffffffu) >= cand;
            cnt += (uint32_t)__popcll(__ballot(ge));
        }
        thr = cnt >= kth ? cand : thr;
    }
    for (uint32_t s0 = 0; s0 < n; s0 += 64) {
        const uint32_t s = s0 + lane;
        const uint32_t key = s < n ? (keys[s] & 0x7fffffffu) : 0u;
        gt += (uint32_t)__popcll(__ballot(s < n && key > thr));
        eq += (uint32_t)__popcll(__ballot(s < n && key == thr));
    }
    return thr;
}

// Register-resident variant for float chunks of up to 16 * 4 * THREADS elements with k <= THREADS:
// the chunk is read from HBM once (16-byte loads, each wavefront owning a contiguous slice) and
// stays in registers. A lower bound of the threshold comes from the k-th largest of the per-thread
// maxima (at least k entries reach it); the entries that reach it - usually little more than k - go
// to an LDS list, and the exact k-th largest key is selected on the list. Both selections are done
// by one wavefront with ballots, so the path needs a handful of barriers. When the list overflows
// or entries tie at the threshold (tie-breaking needs position order), the workgroup falls back to
// the general path on the same chunk (then in L2); both paths compute the same unique result.
// Positions at or beyond d are loaded as 0.0f: the smallest key, never inside the k largest unless
// the threshold itself is 0, which is a tie case.
template <int THREADS, int MINBLOCKS>
__global__ __launch_bounds__(THREADS, MINBLOCKS) void topk_f32_regs_kernel(const float *__restrict__ g, int32_t d,
                                                                          int32_t k, int32_t *__restrict__ idx,
                                                                          float *__restrict__ val,
                                                                          int32_t vector_loads)
{
    constexpr int ROWS = 16;
    __shared__ uint32_t tmax_s[THREADS];
    __shared__ float cand_val[TOPK_CAND_CAP];
    __shared__ int32_t cand_pos[TOPK_CAND_CAP];
    __shared__ uint32_t s_thr, s_need, s_ties, s_ncand, s_nan;

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6); // wavefront index, kept scalar
    const float *gc = g + (int64_t)blockIdx.x * d;
    int32_t *oidx = idx + (int64_t)blockIdx.x * k;
    float *oval = val + (int64_t)blockIdx.x * k;
    const int32_t wslice = w * (ROWS * 256);  // first position of this wavefront's slice
    const int32_t wbase = wslice + lane * 4;  // element (j, e) of this lane sits at wbase + 256 j + e
    auto key_of = [](float f) { return __float_as_uint(f) & 0x7fffffffu; };

    float4 v[ROWS];
    if (vector_loads && wslice + ROWS * 256 <= d) {
        // the whole slice is inside the chunk: plain 16-byte loads off one scalar base
        const float *src = gc + wslice + lane * 4;
#pragma unroll
        for (int j = 0; j < ROWS; ++j)
            v[j] = load_once_f4(src + j * 256);
    } else {
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
    }
    uint32_t tmax = 0;
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const uint32_t a = key_of(v[j].x), b = key_of(v[j].y), c = key_of(v[j].z), e = key_of(v[j].w);
        const uint32_t ab = a > b ? a : b, ce = c > e ? c : e;
        const uint32_t m = ab > ce ? ab : ce;
        tmax = m > tmax ? m : tmax;
    }
    tmax_s[tid] = tmax;
    if (tid == 0) {
        s_ncand = 0;
        s_nan = 0;
    }
    __syncthreads();
    if (tmax > 0x7f800000u)
        s_nan = 1; // a NaN pattern in the chunk: its order is defined on the bits, not on float compares
    if (w == 0) {
        uint32_t gt, eq;
        const uint32_t bound = wave_kth_largest(tmax_s, THREADS, (uint32_t)k, gt, eq);
        if (lane == 0)
            s_thr = bound;
    }
    __syncthreads();
    const uint32_t bound = s_thr;
    // The candidate test is a float compare on |x| (one instruction per entry), which orders finite
    // values and infinities exactly like the keys; chunks with a NaN or with a subnormal / zero bound
    // take the general path.
    if (s_nan != 0u || bound < 0x00800000u) {
        topk_general<float, THREADS>(gc, d, k, oidx, oval);
        return;
    }
    const float boundf = __uint_as_float(bound);
#pragma unroll
    for (int j = 0; j < ROWS; ++j) {
        const float e4[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
        const uint64_t hits[4] = {__ballot(fabsf(e4[0]) >= boundf), __ballot(fabsf(e4[1]) >= boundf),
                                  __ballot(fabsf(e4[2]) >= boundf), __ballot(fabsf(e4[3]) >= boundf)};
        if ((hits[0] | hits[1] | hits[2] | hits[3]) == 0ull)
            continue;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint64_t bh = hits[e];
            if (bh == 0ull)
                continue;
            uint32_t base = 0;
            if (lane == 0)
                base = atomicAdd(&s_ncand, (uint32_t)__popcll(bh));
            base = __builtin_amdgcn_readfirstlane(base);
            const uint32_t mine = base + __builtin_amdgcn_mbcnt_hi((uint32_t)(bh >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bh, 0u));
            if (fabsf(e4[e]) >= boundf && mine < TOPK_CAND_CAP) {
                cand_val[mine] = e4[e];
                cand_pos[mine] = wbase + j * 256 + e;
            }
        }
    }
    __syncthreads();
    const uint32_t nc = s_ncand;
    const bool listed = nc <= TOPK_CAND_CAP;
    if (listed && w == 0) {
        uint32_t gt, eq;
        const uint32_t t = wave_kth_largest(reinterpret_cast<const uint32_t *>(cand_val), nc, (uint32_t)k, gt, eq);
        if (lane == 0) {
            s_thr = t;
            s_need = (uint32_t)k - gt;
            s_ties = eq;
        }
    }
    __syncthreads();
    if (listed && s_ties == s_need) {
        // exactly k listed entries have key >= thr: they are packed to the front of a second list
        // (wavefront-aggregated append; the order does not matter), then each goes to its rank by
        // position among those k
        const uint32_t thr = s_thr;
        if (tid == 0)
            s_ncand = 0;
        __syncthreads();
        int32_t *win_pos = cand_pos + TOPK_CAND_CAP / 2; // nc <= cap/2 is checked below
        float *win_val = cand_val + TOPK_CAND_CAP / 2;
        if (nc <= TOPK_CAND_CAP / 2) {
            for (uint32_t t0 = 0; t0 < nc; t0 += THREADS) {
                const uint32_t t = t0 + tid;
                const float cv = t < nc ? cand_val[t] : 0.f;
                const bool win = t < nc && key_of(cv) >= thr;
                const uint64_t bh = __ballot(win);
                if (bh != 0ull) {
                    uint32_t base = 0;
                    if (lane == 0)
                        base = atomicAdd(&s_ncand, (uint32_t)__popcll(bh));
                    base = __builtin_amdgcn_readfirstlane(base);
                    const uint32_t mine = base + __builtin_amdgcn_mbcnt_hi((uint32_t)(bh >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bh, 0u));
                    if (win) {
                        win_pos[mine] = cand_pos[t];
                        win_val[mine] = cv;
                    }
                }
            }
            __syncthreads();
            for (int32_t t = tid; t < k; t += THREADS) {
                const int32_t mine = win_pos[t];
                int32_t rank = 0;
                for (int32_t u = 0; u < k; ++u)
                    rank += win_pos[u] < mine ? 1 : 0;
                oidx[rank] = mine;
                oval[rank] = win_val[t];
            }
            return;
        }
        for (uint32_t t = tid; t < nc; t += THREADS) {
            const float mine_val = cand_val[t];
            if (key_of(mine_val) < thr)
                continue;
            const int32_t mine = cand_pos[t];
            int32_t rank = 0;
            for (uint32_t u = 0; u < nc; ++u)
                rank += (key_of(cand_val[u]) >= thr && cand_pos[u] < mine) ? 1 : 0;
            oidx[rank] = mine;
            oval[rank] = mine_val;
        }
        return;
    }
    topk_general<float, THREADS>(gc, d, k, oidx, oval);
}

// bfloat16 chunks (d % 8 == 0, k <= THREADS): two sweeps over the chunk with 16-byte loads instead of the general
// kernel's four with 2-byte loads and an LDS atomic per element. Sweep 1 takes every thread's largest key; the
// k-th largest of those maxima is a lower bound of the threshold that at least k entries reach (the maxima are
// k distinct entries). Sweep 2 collects the entries that reach the bound - a few per cent of the chunk for
// heavy-tailed data - into LDS: every wavefront owns a contiguous slice of the chunk and a segment of the list,
// and appends in position order (a prefix sum over the lanes' counts), so the list as a whole is in ascending
// position. The exact threshold is then a radix select over the list (15-bit keys: 11 + 4 bits), and the
// output is written by walking the list in order, exactly as the general kernel walks the chunk: entries
// above the threshold, and the first `need` of those equal to it. bfloat16 has so few distinct magnitudes
// that ties at the threshold are the rule; they cost nothing here. A segment that overflows (quantised or
// constant data: everything reaches the bound) or a bound of 0 sends the chunk to the general kernel.
// dynamic LDS: uint32_t pos[NW][SEG]; uint16_t raw[NW][SEG]
constexpr int TOPK_BF16_SEG = 1024; // list entries per wavefront

template <int THREADS>
__global__ __launch_bounds__(THREADS) void topk_bf16_list_kernel(const uint16_t *__restrict__ g, int32_t d, int32_t k,
                                                                 int32_t *__restrict__ idx, float *__restrict__ val)
{
    constexpr int NW = THREADS / 64;
    constexpr int SEG = TOPK_BF16_SEG;
    extern __shared__ __attribute__((aligned(16))) unsigned char topk_smem[];
    uint32_t *cand_pos = reinterpret_cast<uint32_t *>(topk_smem);           // [NW][SEG]
    uint16_t *cand_raw = reinterpret_cast<uint16_t *>(cand_pos + NW * SEG); // [NW][SEG]
    __shared__ uint32_t tmax_s[THREADS];
    __shared__ uint32_t hist[2048];
    __shared__ uint32_t wave_tot[NW];
    __shared__ uint32_t w_cnt[NW], w_gt[NW], w_eq[NW];
    __shared__ uint32_t s_bound, s_bin, s_need, s_overflow;

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const uint16_t *gc = g + (int64_t)blockIdx.x * d;
    int32_t *oidx = idx + (int64_t)blockIdx.x * k;
    float *oval = val + (int64_t)blockIdx.x * k;

    // wavefront slices in whole steps of 512 positions (64 lanes x 8)
    int32_t seg = (d + NW - 1) / NW;
    seg = (seg + 511) & ~511;
    const int32_t beg = w * seg < d ? w * seg : d;
    const int32_t end = beg + seg < d ? beg + seg : d;
    auto load8 = [&](int32_t i0, uint32_t (&key)[8], uint16_t (&raw)[8]) {
        // positions i0 .. i0 + 7 of the chunk (i0 % 8 == 0; d % 8 == 0, so the eight are inside or outside together)
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (i0 < end)
            v = *reinterpret_cast<const uint4 *>(gc + i0);
        const uint32_t wd[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            raw[2 * e] = (uint16_t)(wd[e] & 0xffffu);
            raw[2 * e + 1] = (uint16_t)(wd[e] >> 16);
            key[2 * e] = wd[e] & 0x7fffu;
            key[2 * e + 1] = (wd[e] >> 16) & 0x7fffu;
        }
    };

    // ---- sweep 1: the largest key of every thread ----
    uint32_t tmax = 0;
    for (int32_t i0 = beg + lane * 8; i0 < end; i0 += 8 * 512) {
        // eight 16-byte loads in flight per lane; the largest key of a 32-bit pair of entries without unpacking:
        // clear both sign bits, compare the halves
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int32_t i = i0 + u * 512;
            v[u] = i < end ? *reinterpret_cast<const uint4 *>(gc + i) : make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t wd[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t lo = wd[e] & 0x7fffu, hi = (wd[e] >> 16) & 0x7fffu;
                const uint32_t m = lo > hi ? lo : hi;
                tmax = m > tmax ? m : tmax;
            }
        }
    }
    tmax_s[tid] = tmax;
    if (tid == 0)
        s_overflow = 0;
    __syncthreads();
    if (w == 0) {
        uint32_t gt, eq;
        const uint32_t b = wave_kth_largest(tmax_s, THREADS, (uint32_t)k, gt, eq, 15);
        if (lane == 0)
            s_bound = b;
    }
    __syncthreads();
    const uint32_t bound = s_bound;
    if (bound == 0u) { // fewer than k threads saw a non-zero entry: no useful bound
        topk_general<uint16_t, THREADS>(gc, d, k, oidx, oval);
        return;
    }

    // ---- sweep 2: the entries that reach the bound, appended in position order to the wavefront's segment ----
    uint32_t count = 0; // entries of this wavefront so far (the same in every lane)
    constexpr int U2 = 4; // 16-byte loads in flight per lane
    for (int32_t s0 = beg; s0 < end; s0 += U2 * 512) {
        uint32_t key[U2][8];
        uint16_t raw[U2][8];
#pragma unroll
        for (int u = 0; u < U2; ++u)
            load8(s0 + u * 512 + lane * 8, key[u], raw[u]);
#pragma unroll
        for (int u = 0; u < U2; ++u) {
            uint32_t mine = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                mine += key[u][e] >= bound ? 1u : 0u;
            if (__ballot(mine != 0u) == 0ull)
                continue;
            uint32_t incl = mine; // inclusive prefix over the lanes
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t t = __shfl_up(incl, off, 64);
                if (lane >= off)
                    incl += t;
            }
            const uint32_t total = __shfl(incl, 63, 64);
            if (count + total > (uint32_t)SEG) {
                s_overflow = 1;
            } else {
                uint32_t slot = w * SEG + count + incl - mine;
                const int32_t p0 = s0 + u * 512 + lane * 8;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    if (key[u][e] >= bound) {
                        cand_pos[slot] = (uint32_t)(p0 + e);
                        cand_raw[slot] = raw[u][e];
                        ++slot;
                    }
                }
            }
            count += total;
        }
    }
    if (lane == 0)
        w_cnt[w] = count;
    __syncthreads();
    if (s_overflow != 0u) {
        topk_general<uint16_t, THREADS>(gc, d, k, oidx, oval);
        return;
    }

    // ---- the exact k-th largest key of the list: radix select, 11 then 4 bits ----
    uint32_t prefix = 0, need = (uint32_t)k;
    int decided = 15;
    for (int pass = 0; pass < 2; ++pass) {
        const int shift = pass == 0 ? 4 : 0;
        const int nb = pass == 0 ? 2048 : 16;
        for (int b = tid; b < nb; b += THREADS)
            hist[b] = 0;
        __syncthreads();
        for (int ww = 0; ww < NW; ++ww) {
            const uint32_t n = w_cnt[ww];
            for (uint32_t e = tid; e < n; e += THREADS) {
                const uint32_t key = (uint32_t)cand_raw[ww * SEG + e] & 0x7fffu;
                if (pass == 0 || (key >> decided) == prefix)
                    atomicAdd(&hist[(key >> shift) & (uint32_t)(nb - 1)], 1u);
            }
        }
        __syncthreads();
        // thread t owns `per` bins counted from the top
        const int per = (nb + THREADS - 1) / THREADS;
        const int hi = nb - tid * per;
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
        prefix = (prefix << (pass == 0 ? 11 : 4)) | s_bin;
        need = s_need;
        decided = shift;
        __syncthreads();
    }
    const uint32_t thr = prefix;

    // ---- emit: the list is in ascending position; every wavefront walks its own segment ----
    const uint32_t n_mine = w_cnt[w];
    uint32_t cgt = 0, ceq = 0;
    for (uint32_t e0 = 0; e0 < n_mine; e0 += 64) {
        const uint32_t e = e0 + lane;
        const bool in = e < n_mine;
        const uint32_t key = in ? ((uint32_t)cand_raw[w * SEG + e] & 0x7fffu) : 0u;
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
    for (uint32_t e0 = 0; e0 < n_mine; e0 += 64) {
        const uint32_t e = e0 + lane;
        const bool in = e < n_mine;
        const uint16_t raw = in ? cand_raw[w * SEG + e] : (uint16_t)0;
        const uint32_t key = (uint32_t)raw & 0x7fffu;
        const bool gt = in && key > thr, eq = in && key == thr;
        const uint64_t bgt = __ballot(gt), beq = __ballot(eq);
        const uint32_t gt_before = run_gt + (uint32_t)__popcll(bgt & below);
        const uint32_t eq_before = run_eq + (uint32_t)__popcll(beq & below);
        if (gt || (eq && eq_before < need)) {
            const uint32_t slot = gt_before + (eq_before < need ? eq_before : need);
            oidx[slot] = (int32_t)cand_pos[w * SEG + e];
            oval[slot] = Elem<uint16_t>::widen(raw);
        }
        run_gt += (uint32_t)__popcll(bgt);
        run_eq += (uint32_t)__popcll(beq);
    }
}

template <int THREADS>
static hipError_t launch_topk_bf16_list(const uint16_t *g, int64_t C, int32_t d, int32_t k, int32_t *idx, float *val,
                                        hipStream_t s)
{
    constexpr size_t smem = (size_t)(THREADS / 64) * TOPK_BF16_SEG * (sizeof(uint32_t) + sizeof(uint16_t));
    auto kern = topk_bf16_list_kernel<THREADS>;
    const hipError_t e = raise_dynamic_lds(reinterpret_cast<const void *>(kern), smem);
    if (e != hipSuccess)
        return e;
    kern<<<dim3((unsigned)C), THREADS, smem, s>>>(g, d, k, idx, val);
    return hipGetLastError();
}

// Second pass for long chunks (see launch_topk): the k largest of the S * k candidates that the register
// kernel kept for the S pieces of a chunk, one wavefront per chunk. The candidates of a piece are in
// ascending position and the pieces in order, so the list is in ascending position: the entries above
// the k-th largest key, and the first of those equal to it, taken in list order, are the result in its
// final order. Keys are sign-cleared bit patterns throughout, as in the first pass.
__global__ __launch_bounds__(64) void topk_merge_kernel(const int32_t *__restrict__ cand_i,
                                                        const float *__restrict__ cand_v, int32_t S, int32_t dsub,
                                                        int32_t k, int32_t *__restrict__ idx, float *__restrict__ val)
{
    __shared__ uint32_t keys[1024]; // S * k <= 1024
    const uint32_t lane = threadIdx.x;
    const uint32_t n = (uint32_t)(S * k);
    const int64_t base = (int64_t)blockIdx.x * n;
    for (uint32_t s = lane; s < n; s += 64)
        keys[s] = __float_as_uint(cand_v[base + s]);
    __syncthreads();
    uint32_t gt, eq;
    const uint32_t thr = wave_kth_largest(keys, n, (uint32_t)k, gt, eq);
    const uint32_t need = (uint32_t)k - gt; // entries equal to the threshold that belong to the result
    const uint64_t below = (1ull << lane) - 1ull;
    uint32_t out = 0, ties = 0;
    for (uint32_t s0 = 0; s0 < n; s0 += 64) {
        const uint32_t s = s0 + lane;
        const bool in = s < n;
        const uint32_t key = in ? (keys[s] & 0x7fffffffu) : 0u;
        const bool is_eq = in && key == thr;
        const uint64_t beq = __ballot(is_eq);
        const bool take = in && (key > thr || (is_eq && ties + (uint32_t)__popcll(beq & below) < need));
        const uint64_t bt = __ballot(take);
        if (take) {
            const uint32_t o = out + (uint32_t)__popcll(bt & below);
            idx[(int64_t)blockIdx.x * k + o] = (int32_t)(s / (uint32_t)k) * dsub + cand_i[base + s];
            val[(int64_t)blockIdx.x * k + o] = cand_v[base + s];
        }
        out += (uint32_t)__popcll(bt);
        ties += (uint32_t)__popcll(beq);
    }
}

hipError_t launch_topk(const void *grad, int grad_type, int64_t C, int32_t d, int32_t k, int32_t *idx,
                       float *val, hipStream_t s, int32_t *scratch_i, float *scratch_v, int64_t scratch_elems)
{
    if (C == 0)
        return hipSuccess;
    const dim3 grid((unsigned)C);
    ProfileScope prof(KC_TOPK, s);
    if (grad_type == SGC_GRAD_F32) {
        const int32_t vec = (d % 4 == 0) ? 1 : 0; // every chunk then starts 16-byte aligned
        // Chunks of more than 16384 floats: the register kernel for up to 65536 holds a whole chunk per
        // 1024-thread workgroup, one workgroup per CU, and loads and selects in turn (3.2 TB/s); beyond that
        // the general kernel makes several passes. With scratch for S * k candidates per chunk the chunk is
        // instead cut in S <= 16 pieces of at most 16384 that go through the 256-thread kernel, five
        // workgroups per CU, and a small second pass merges the (at most 1024) candidates.
        const int32_t S = (d + 16383) / 16384;
        // (k <= 128: the 256-thread kernel bounds the threshold by the k-th largest of its 256 per-thread
        // maxima, which is a useful bound only while k is well below 256)
        if (d > 16384 && S <= 16 && S * k <= 1024 && d % (4 * S) == 0 && k <= 128 && k <= d / S && scratch_i &&
            scratch_v &&
            (int64_t)C * S * k <= scratch_elems && (int64_t)C * S < (1ll << 31)) {
            const int32_t dsub = d / S;
            topk_f32_regs_kernel<256, 5><<<dim3((unsigned)(C * S)), 256, 0, s>>>((const float *)grad, dsub, k, scratch_i,
                                                                                 scratch_v, 1);
            topk_merge_kernel<<<grid, 64, 0, s>>>(scratch_i, scratch_v, S, dsub, k, idx, val);
            return hipGetLastError();
        }
        if (d <= 16 * 4 * 256 && k <= 256)
            topk_f32_regs_kernel<256, 5><<<grid, 256, 0, s>>>((const float *)grad, d, k, idx, val, vec);
        else if (d <= 16 * 4 * 1024 && k <= 1024)
            topk_f32_regs_kernel<1024, 1><<<grid, 1024, 0, s>>>((const float *)grad, d, k, idx, val, vec);
        else
            topk_kernel<float, 1024><<<grid, 1024, 0, s>>>((const float *)grad, d, k, idx, val);
    } else {
        const bool vec = d % 8 == 0; // every chunk then starts 16-byte aligned
        if (d <= 16384) {
            if (vec && k <= 256 && d >= 2048)
                return launch_topk_bf16_list<256>((const uint16_t *)grad, C, d, k, idx, val, s);
            topk_kernel<uint16_t, 256><<<grid, 256, 0, s>>>((const uint16_t *)grad, d, k, idx, val);
        } else {
            if (vec && k <= 1024)
                return launch_topk_bf16_list<1024>((const uint16_t *)grad, C, d, k, idx, val, s);
            topk_kernel<uint16_t, 1024><<<grid, 1024, 0, s>>>((const uint16_t *)grad, d, k, idx, val);
        }
    }
    return hipGetLastError();
}

} // namespace sgc
