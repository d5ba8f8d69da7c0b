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
#include <type_traits>

#include "sgc_internal.h"

namespace sgc {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int OUTER_STRIP = 128; // columns per wavefront

// Four adjacent entries of a row of G as loaded: 16 bytes of floats, or 8 bytes of bfloat16 bit patterns
// (widened to float, exactly, when they are used).
template <bool GBF16> struct OuterPiece { typedef float4 type; };
template <> struct OuterPiece<true> { typedef uint2 type; };

__device__ __forceinline__ float4 outer_load_g(const float *p) { return load_once_f4(p); }
__device__ __forceinline__ uint2 outer_load_g(const uint16_t *p)
{
    typedef unsigned int uintx2_t __attribute__((ext_vector_type(2)));
    const uintx2_t t = __builtin_nontemporal_load(reinterpret_cast<const uintx2_t *>(p));
    return make_uint2(t.x, t.y);
}
__device__ __forceinline__ float4 outer_widen(const float4 &v) { return v; }
__device__ __forceinline__ float4 outer_widen(const uint2 &v)
{
    return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u), __uint_as_float(v.y << 16),
                       __uint_as_float(v.y & 0xffff0000u));
}

// v where keep, else zero, as four selects (an `if` around a loaded value becomes a branch with a wait)
__device__ __forceinline__ float4 outer_keep(bool keep, float4 v)
{
    return make_float4(keep ? v.x : 0.f, keep ? v.y : 0.f, keep ? v.z : 0.f, keep ? v.w : 0.f);
}
constexpr int OUTER_FLIGHT = 8;  // row pairs in flight per wavefront

// Partial products of a run of rows of G: out[g][a][j] = sum over the rows i of run g of B[a][i] G[i][j]
// (the runs are summed in order by outer_reduce_kernel; a single run writes Gc itself).
// grid (column strips, runs, matrices of the batch x blocks of 32 * RBLK rows of B). A run is `reps`
// consecutive slices of 32 * NG rows; the workgroup takes them one after the other into the same
// accumulators. A slice is cut in groups of 8 rows, group q going to wavefront q % 4 (NG groups each):
//   - the slice of B goes through the LDS transposed (Bs[row of the slice][row of B], read back one
//     float per lane and MFMA);
//   - for the group at row k, lanes 0-31 read rows k .. k + 3 of G and lanes 32-63 rows k + 4 .. k + 7,
//     16 bytes each; MFMA j sums the depths k + j and k + 4 + j.
// Two sets of registers and two LDS buffers are used in turn: all loads of the next slice are issued
// before the MFMAs of the current one, and no load sits under a branch (addresses past an end are
// clamped, the values replaced by zero), so waits are counted and a group's MFMAs start as soon as its
// rows have arrived. One barrier per slice. The four wavefronts' accumulators are added in wavefront
// order at the end.
// FULL: m a multiple of the slice, rho of the block of rows of B, n of 128 (and offsets that fit 32 bits):
// no clamps or selects, and every address is a wavefront-uniform base plus a per-lane offset that
// never changes, so the loads cost no vector arithmetic (which would take its time from the MFMAs).
// GBF16: G holds bfloat16 bit patterns (8-byte pieces instead of 16-byte ones).
template <int RBLK, int NG, bool BVEC, bool FULL, bool GBF16>
__global__ __launch_bounds__(256) void outer_project_kernel(const float *__restrict__ B, const void *__restrict__ Gv,
                                                            int32_t rho, int32_t m, int32_t n, int32_t rho_blocks,
                                                            int32_t reps, float *__restrict__ out)
{
    typedef typename std::conditional<GBF16, uint16_t, float>::type GElem;
    typedef typename OuterPiece<GBF16>::type GPiece;
    const GElem *G = static_cast<const GElem *>(Gv);
    extern __shared__ __attribute__((aligned(16))) float outer_lds[]; // Bs x 2, later the accumulators of wavefronts 1..3
    constexpr int RB = 32 * RBLK, LDB = RB + 1, SLICE = 32 * NG, PIECES = RBLK * NG, BSZ = SLICE * LDB;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, l32 = lane & 31, lhalf = lane >> 5;
    const int32_t mat = blockIdx.z / rho_blocks; // matrix of the batch
    const int32_t n0 = blockIdx.x * OUTER_STRIP, rho0 = (blockIdx.z - mat * rho_blocks) * RB;
    B += (int64_t)mat * rho * m;
    G += (int64_t)mat * m * n;
    out += ((int64_t)mat * gridDim.y + blockIdx.y) * rho * n;
    const int32_t col = n0 + 4 * l32;
    const bool col_ok = col < n;
    const GElem *gcol = G + (col_ok ? col : n - 4);
    const int32_t slices = (m + SLICE - 1) / SLICE;
    const int32_t s_first = blockIdx.y * reps;
    const int32_t s_end = s_first + reps < slices ? s_first + reps : slices;

    float4 bp[2][PIECES];
    GPiece g[2][NG][4];
    const int wu = __builtin_amdgcn_readfirstlane(w);
    const uint32_t g_lane = (uint32_t)(4 * lhalf * n + col); // FULL: offsets in entries from a uniform base
    uint32_t b_lane[PIECES];
#pragma unroll
    for (int i = 0; i < PIECES; ++i) {
        const int e = tid + 256 * i;
        b_lane[i] = (uint32_t)((rho0 + e / (SLICE / 4)) * m + 4 * (e % (SLICE / 4)));
    }
    auto fetch = [&](int set, int32_t s) {
        const int32_t m0 = s * SLICE;
        if constexpr (FULL) {
#pragma unroll
            for (int i = 0; i < PIECES; ++i)
                bp[set][i] = *reinterpret_cast<const float4 *>(B + m0 + b_lane[i]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < NG; ++q)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    g[set][q][j] = outer_load_g(G + (int64_t)(m0 + 8 * (4 * q + wu) + j) * n + g_lane);
            __builtin_amdgcn_sched_barrier(0);
            return;
        }
        // 16-byte pieces of the slice of B: piece e is row e / (SLICE / 4) of the block, depths 4 (e % (SLICE / 4)) ..
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int e = tid + 256 * i;
            const int32_t a = rho0 + e / (SLICE / 4), k = m0 + 4 * (e % (SLICE / 4));
            const float *row = B + (int64_t)(a < rho ? a : rho - 1) * m;
            if (BVEC) {
                bp[set][i] = *reinterpret_cast<const float4 *>(row + (k + 3 < m ? k : m - 4));
            } else {
                bp[set][i].x = row[k < m ? k : m - 1];
                bp[set][i].y = row[k + 1 < m ? k + 1 : m - 1];
                bp[set][i].z = row[k + 2 < m ? k + 2 : m - 1];
                bp[set][i].w = row[k + 3 < m ? k + 3 : m - 1];
            }
        }
        __builtin_amdgcn_sched_barrier(0); // B first: its wait then leaves the loads of G in flight
#pragma unroll
        for (int q = 0; q < NG; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int32_t row = m0 + 8 * (4 * q + w) + 4 * lhalf + j;
                g[set][q][j] = outer_load_g(gcol + (int64_t)(row < m ? row : m - 1) * n);
            }
        __builtin_amdgcn_sched_barrier(0);
    };

    floatx16 acc[RBLK][4];
#pragma unroll
    for (int rb = 0; rb < RBLK; ++rb)
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[rb][e][v] = 0.f;

    auto work = [&](int set, int32_t s) { // slice s is in register set `set`; LDS buffer `set`
        const int32_t m0 = s * SLICE;
        float *bs = outer_lds + set * BSZ;
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int e = tid + 256 * i;
            const int32_t al = e / (SLICE / 4), kl = 4 * (e % (SLICE / 4));
            if constexpr (FULL) {
                bs[(kl + 0) * LDB + al] = bp[set][i].x;
                bs[(kl + 1) * LDB + al] = bp[set][i].y;
                bs[(kl + 2) * LDB + al] = bp[set][i].z;
                bs[(kl + 3) * LDB + al] = bp[set][i].w;
                continue;
            }
            const bool a_ok = rho0 + al < rho;
            bs[(kl + 0) * LDB + al] = (a_ok && m0 + kl + 0 < m) ? bp[set][i].x : 0.f;
            bs[(kl + 1) * LDB + al] = (a_ok && m0 + kl + 1 < m) ? bp[set][i].y : 0.f;
            bs[(kl + 2) * LDB + al] = (a_ok && m0 + kl + 2 < m) ? bp[set][i].z : 0.f;
            bs[(kl + 3) * LDB + al] = (a_ok && m0 + kl + 3 < m) ? bp[set][i].w : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < NG; ++q) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int32_t kl = 8 * (4 * q + w) + 4 * lhalf + j;
                // rows past the end of the matrix were read from a clamped address: they count as zero
                // (their depths of Bs are zero too, but zero times a non-finite entry would not be)
                const float4 gw = outer_widen(g[set][q][j]);
                const float4 gv = FULL ? gw : outer_keep(m0 + kl < m, gw);
#pragma unroll
                for (int rb = 0; rb < RBLK; ++rb) {
                    const float a = bs[kl * LDB + rb * 32 + l32];
                    acc[rb][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, gv.x, acc[rb][0], 0, 0, 0);
                    acc[rb][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, gv.y, acc[rb][1], 0, 0, 0);
                    acc[rb][2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, gv.z, acc[rb][2], 0, 0, 0);
                    acc[rb][3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, gv.w, acc[rb][3], 0, 0, 0);
                }
            }
        }
    };

    // A buffer of Bs written for slice s is read until the barrier of slice s + 1 and written again for
    // slice s + 2, after that barrier.
    // (pairs of slices in the loop and a possible last one after it: no branch around the MFMAs inside the
    // loop, so the accumulators stay where they are)
    fetch(0, s_first);
    int32_t s2 = s_first;
    for (; s2 + 1 < s_end; s2 += 2) {
        fetch(1, s2 + 1);
        work(0, s2);
        if (s2 + 2 < s_end)
            fetch(0, s2 + 2);
        work(1, s2 + 1);
    }
    if (s2 < s_end)
        work(0, s2);

    // wavefronts 1..3 hand their accumulators to wavefront 0, which adds them in wavefront order
    constexpr int PER_WAVE = RBLK * 4 * 16 * 64;
    __syncthreads();
    if (w > 0) {
#pragma unroll
        for (int rb = 0; rb < RBLK; ++rb)
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    outer_lds[(w - 1) * PER_WAVE + ((rb * 4 + e) * 16 + v) * 64 + lane] = acc[rb][e][v];
    }
    __syncthreads();
    if (w == 0 && col_ok) {
        // accumulator register v of lane l: row 8 (v / 4) + v % 4 + 4 (l / 32) of the block
#pragma unroll
        for (int rb = 0; rb < RBLK; ++rb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float o[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float t = acc[rb][e][v];
#pragma unroll
                    for (int ww = 0; ww < 3; ++ww)
                        t += outer_lds[ww * PER_WAVE + ((rb * 4 + e) * 16 + v) * 64 + lane];
                    o[e] = t;
                }
                const int32_t a = rho0 + rb * 32 + 8 * (v >> 2) + (v & 3) + 4 * lhalf;
                if (a < rho)
                    *reinterpret_cast<float4 *>(out + (int64_t)a * n + col) = make_float4(o[0], o[1], o[2], o[3]);
            }
    }
}

// Gc = sum of the slices' partial products, in slice order (the loads of four slices in flight);
// blockIdx.y: matrix of the batch
__global__ __launch_bounds__(256) void outer_reduce_kernel(const float *__restrict__ part, int32_t S, int64_t count4,
                                                           float *__restrict__ Gc)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= count4)
        return;
    const float4 *src = reinterpret_cast<const float4 *>(part) + (int64_t)blockIdx.y * S * count4 + e;
    Gc += (int64_t)blockIdx.y * count4 * 4;
    float4 acc = src[0];
    int32_t s = 1;
    for (; s + 4 <= S; s += 4) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            v[u] = src[(int64_t)(s + u) * count4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            acc.x += v[u].x;
            acc.y += v[u].y;
            acc.z += v[u].z;
            acc.w += v[u].w;
        }
    }
    for (; s < S; ++s) {
        const float4 v = src[(int64_t)s * count4];
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
// 32-row blocks of W); a wavefront takes every fourth block of its group, one wavefront per SIMD.
// Per block: the rho-deep product of the 32 x 128 tile on the matrix cores, then the tile of W is updated
// and stored; the loads of the next block's tile of W and of its values of B are issued before the
// product, so they are in flight while the matrix cores work. RHO32: rho <= 32, the strip of Nd is read
// once per wavefront and kept in registers for all its blocks. FULL: m % 32 == 0, n % 128 == 0 and, with
// RHO32, rho == 32: no bounds checks (so no branches around the loads and stores), and every address is
// a wavefront-uniform base plus a per-lane offset that never changes, which leaves the vector
// arithmetic to the update itself.
template <bool RHO32, bool FULL>
__global__ __launch_bounds__(256, 1) void outer_back_kernel(float *__restrict__ W, const float *__restrict__ B,
                                                            const float *__restrict__ Nd, int32_t rho, int32_t m,
                                                            int32_t n, int32_t blocks, float lr)
{
    constexpr int FL = OUTER_FLIGHT;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, l32 = lane & 31, lhalf = lane >> 5;
    const int32_t col = blockIdx.x * OUTER_STRIP + 4 * l32;
    const bool col_ok = FULL || col < n;
    W += (int64_t)blockIdx.z * m * n; // matrix of the batch
    B += (int64_t)blockIdx.z * rho * m;
    Nd += (int64_t)blockIdx.z * rho * n;
    float4 nfix[RHO32 ? 16 : 1];
    if (RHO32) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int32_t a = 2 * u + lhalf; // rows past rho: a clamped address, the value replaced by zero
            nfix[u] = outer_keep(a < rho, *reinterpret_cast<const float4 *>(Nd + (int64_t)(a < rho ? a : rho - 1) * n +
                                                                            (col_ok ? col : n - 4)));
        }
    }
    // two sets of tile registers, used in turn: one holds the block being worked on, the other receives
    // the next block's loads (no copies, so nothing waits for a load before its values are needed)
    float4 wt[2][16];
    float bt[2][RHO32 ? 16 : 1];
    const int wu = __builtin_amdgcn_readfirstlane(w);
    const uint32_t w_lane = (uint32_t)(4 * lhalf * n + col), b_lane = (uint32_t)(lhalf * m + l32);
    auto fetch = [&](int set, int32_t i0) { // the tile of W at rows i0.. and, RHO32, its values of B
        if constexpr (FULL) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                wt[set][v] = load_once_f4(W + (int64_t)(i0 + 8 * (v >> 2) + (v & 3)) * n + w_lane);
            if (RHO32) {
#pragma unroll
                for (int u = 0; u < 16; ++u)
                    bt[set][u] = (B + (int64_t)(2 * u) * m + i0)[b_lane];
            }
            return;
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int32_t row = i0 + 8 * (v >> 2) + (v & 3) + 4 * lhalf;
            if (FULL) {
                wt[set][v] = load_once_f4(W + (int64_t)row * n + col);
            } else {
                wt[set][v] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (row < m && col_ok)
                    wt[set][v] = load_once_f4(W + (int64_t)row * n + col);
            }
        }
        if (RHO32) {
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int32_t a = 2 * u + lhalf;
                const int32_t i = FULL || i0 + l32 < m ? i0 + l32 : m - 1;
                const float bval = B[(int64_t)(a < rho ? a : rho - 1) * m + i];
                bt[set][u] = (a < rho && (FULL || i0 + l32 < m)) ? bval : 0.f;
            }
        }
    };
    const int32_t first = blockIdx.y * blocks;
    if ((first + wu) * 32 < m && wu < blocks)
        fetch(0, (first + wu) * 32);
    for (int32_t q2 = wu; q2 < blocks; q2 += 8) {
#pragma unroll
      for (int ph = 0; ph < 2; ++ph) {
        const int32_t q = q2 + 4 * ph;
        const int32_t i0 = (first + q) * 32;
        if (q >= blocks || i0 >= m)
            break;
        if (q + 4 < blocks && i0 + 128 < m)
            fetch(ph ^ 1, i0 + 128);
        floatx16 acc[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[e][v] = 0.f;
        if (RHO32) {
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(bt[ph][u], nfix[u].x, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(bt[ph][u], nfix[u].y, acc[1], 0, 0, 0);
                acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(bt[ph][u], nfix[u].z, acc[2], 0, 0, 0);
                acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(bt[ph][u], nfix[u].w, acc[3], 0, 0, 0);
            }
        } else {
            const bool row_ok = FULL || i0 + l32 < m;
            for (int32_t k0 = 0; k0 < rho; k0 += 2 * FL) {
                float4 nv[FL];
                float bk[FL];
#pragma unroll
                for (int u = 0; u < FL; ++u) {
                    const int32_t a = k0 + 2 * u + lhalf;
                    nv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                    bk[u] = 0.f;
                    if (a < rho) {
                        if (col_ok)
                            nv[u] = *reinterpret_cast<const float4 *>(Nd + (int64_t)a * n + col);
                        if (row_ok)
                            bk[u] = B[(int64_t)a * m + i0 + l32];
                    }
                }
#pragma unroll
                for (int u = 0; u < FL; ++u) {
                    acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(bk[u], nv[u].x, acc[0], 0, 0, 0);
                    acc[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(bk[u], nv[u].y, acc[1], 0, 0, 0);
                    acc[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(bk[u], nv[u].z, acc[2], 0, 0, 0);
                    acc[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(bk[u], nv[u].w, acc[3], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int32_t row = i0 + 8 * (v >> 2) + (v & 3) + 4 * lhalf;
            if (FULL || (row < m && col_ok)) {
                float4 o = wt[ph][v];
                o.x -= lr * acc[0][v];
                o.y -= lr * acc[1][v];
                o.z -= lr * acc[2][v];
                o.w -= lr * acc[3][v];
                if constexpr (FULL) {
                    typedef float floatx4_t __attribute__((ext_vector_type(4)));
                    const floatx4_t ov = {o.x, o.y, o.z, o.w};
                    __builtin_nontemporal_store(
                        ov, reinterpret_cast<floatx4_t *>(W + (int64_t)(i0 + 8 * (v >> 2) + (v & 3)) * n + w_lane));
                }
                else
                    *reinterpret_cast<float4 *>(W + (int64_t)row * n + col) = o;
            }
        }
      }
    }
}

// ---- host side ----
// how the rows of G are cut: slices of 128 rows (64 with more than 32 rows of B; fewer when the matrix is too
// small to fill the chip with those), and runs of consecutive slices per workgroup, as long as possible while at least 512
// workgroups remain; with a large batch a run is the whole matrix and nothing partial is written
OuterPlan outer_plan(int32_t count, int32_t rho, int32_t m, int32_t n)
{
    OuterPlan pl{};
    pl.rblk = rho <= 32 ? 1 : 2;
    pl.strips = (n + OUTER_STRIP - 1) / OUTER_STRIP;
    pl.rho_blocks = (rho + 32 * pl.rblk - 1) / (32 * pl.rblk);
    const int64_t per_slice = (int64_t)pl.strips * pl.rho_blocks * count;
    int64_t slice = 64; // two sets of a slice's rows in registers, and room for two workgroups per CU
    while (slice > 32 && ((m + slice - 1) / slice) * per_slice < 512)
        slice >>= 1;
    const int64_t slices = (m + slice - 1) / slice;
    int64_t reps = slices * per_slice / 512;
    reps = reps < 1 ? 1 : (reps > slices ? slices : reps);
    pl.slice = (int32_t)slice;
    pl.reps = (int32_t)reps;
    pl.slices = (int32_t)((slices + reps - 1) / reps); // runs
    const size_t partial = pl.slices > 1 ? (size_t)count * pl.slices * rho * n * sizeof(float) : 0;
    const size_t dense = (size_t)count * rho * n * sizeof(float);
    pl.ws_bytes = ((partial > dense ? partial : dense) + 255) & ~(size_t)255;
    return pl;
}

hipError_t launch_outer_project(const float *B, const void *G, bool g_bf16, int32_t count, int32_t rho, int32_t m,
                                int32_t n, float *Gc, void *ws, hipStream_t s)
{
    const OuterPlan pl = outer_plan(count, rho, m, n);
    float *out = pl.slices > 1 ? static_cast<float *>(ws) : Gc;
    const dim3 grid((unsigned)pl.strips, (unsigned)pl.slices, (unsigned)(pl.rho_blocks * count));
    const size_t stage = (size_t)2 * pl.slice * (32 * pl.rblk + 1) * sizeof(float);
    const size_t handoff = (size_t)3 * pl.rblk * 4 * 16 * 64 * sizeof(float);
    const size_t smem = stage > handoff ? stage : handoff;
    const bool b_vec = m % 4 == 0 && ((uintptr_t)B & 15u) == 0;
    const bool full = b_vec && m % pl.slice == 0 && rho % (32 * pl.rblk) == 0 && n % OUTER_STRIP == 0 &&
                      (int64_t)rho * m < (1ll << 29) && (int64_t)n * 8 < (1ll << 29);
    typedef void (*Kernel)(const float *, const void *, int32_t, int32_t, int32_t, int32_t, int32_t, float *);
    Kernel kern = nullptr;
    const int ng = pl.slice / 32;
#define SGC_OUTER_PICK(R, N) \
    if (pl.rblk == R && ng == N) { \
        if (g_bf16) \
            kern = full ? outer_project_kernel<R, N, true, true, true> \
                        : (b_vec ? outer_project_kernel<R, N, true, false, true> \
                                 : outer_project_kernel<R, N, false, false, true>); \
        else \
            kern = full ? outer_project_kernel<R, N, true, true, false> \
                        : (b_vec ? outer_project_kernel<R, N, true, false, false> \
                                 : outer_project_kernel<R, N, false, false, false>); \
    }
    SGC_OUTER_PICK(1, 1) SGC_OUTER_PICK(1, 2) SGC_OUTER_PICK(1, 4)
    SGC_OUTER_PICK(2, 1) SGC_OUTER_PICK(2, 2)
#undef SGC_OUTER_PICK
    if (!kern)
        return hipErrorInvalidValue;
    if (smem > 48 * 1024) {
        const hipError_t e = raise_dynamic_lds(reinterpret_cast<const void *>(kern), smem);
        if (e != hipSuccess)
            return e;
    }
    ProfileScope prof(KC_OUTER_PROJECT, s);
    kern<<<grid, 256, smem, s>>>(B, G, rho, m, n, pl.rho_blocks, pl.reps, out);
    if (pl.slices > 1) {
        const int64_t count4 = (int64_t)rho * n / 4;
        outer_reduce_kernel<<<dim3((unsigned)((count4 + 255) / 256), (unsigned)count), 256, 0, s>>>(out, pl.slices,
                                                                                                   count4, Gc);
    }
    return hipGetLastError();
}

hipError_t launch_outer_apply(float *W, const float *B, int32_t count, int32_t rho, int32_t m, int32_t n, int32_t d,
                              int32_t k, const int32_t *sel_m, const float *x_m, const int32_t *sel_v,
                              const float *x_v, float alpha, float eps, float lr, void *ws, hipStream_t s)
{
    float *Nd = static_cast<float *>(ws);
    const int64_t count4 = (int64_t)count * rho * n / 4;
    {
        ProfileScope prof(KC_OUTER_APPLY, s);
        outer_zero_kernel<<<dim3((unsigned)((count4 + 255) / 256)), 256, 0, s>>>(Nd, count4);
    }
    // the update of the plain path applied to zeros with step -1 leaves N itself (0 - (-1) N is exact)
    hipError_t e = launch_apply(Nd, (int64_t)count * rho * n / d, d, k, sel_m, x_m, sel_v, x_v, alpha, eps, -1.0f, s);
    if (e != hipSuccess)
        return e;
    const int32_t strips = (n + OUTER_STRIP - 1) / OUTER_STRIP;
    const int32_t row_blocks = (m + 31) / 32;
    // sixteen blocks per workgroup (four per wavefront, so the next tile's loads overlap the product)
    // unless that leaves the chip short of workgroups
    int32_t blocks = 16;
    while (blocks > 4 && (int64_t)strips * ((row_blocks + blocks - 1) / blocks) * count < 256)
        blocks -= 4;
    const dim3 grid((unsigned)strips, (unsigned)((row_blocks + blocks - 1) / blocks), (unsigned)count);
    ProfileScope prof(KC_OUTER_APPLY, s);
    const bool full = m % 32 == 0 && n % OUTER_STRIP == 0 && (rho >= 32) && (int64_t)n * 8 < (1ll << 29) &&
                      (int64_t)m * 2 < (1ll << 29);
    if (rho <= 32) {
        if (full)
            outer_back_kernel<true, true><<<grid, 256, 0, s>>>(W, B, Nd, rho, m, n, blocks, lr);
        else
            outer_back_kernel<true, false><<<grid, 256, 0, s>>>(W, B, Nd, rho, m, n, blocks, lr);
    } else {
        if (full)
            outer_back_kernel<false, true><<<grid, 256, 0, s>>>(W, B, Nd, rho, m, n, blocks, lr);
        else
            outer_back_kernel<false, false><<<grid, 256, 0, s>>>(W, B, Nd, rho, m, n, blocks, lr);
    }
    return hipGetLastError();
}

} // namespace sgc
