// Batched orthogonal matching pursuit (paper Sec. 4.3 eq. 9; selection rule, inverse-Cholesky
// update and output of App. B) for N right-hand sides that share the measurement matrix A.
//
// Per iteration:
//   contraction    P = At * R for all right-hand sides at once: a dense float contraction on the
//                  matrix cores (32x32x2 MFMA, LDS-staged tiles; corr_pipelined_kernel for full
//                  position tiles of resident rows, corr_kernel for everything else). P is never
//                  written: the epilogue scales by 1/||A_:i||, leaves out selected positions and keeps
//                  the two best (score, position) pairs of every position tile per right-hand side.
//                  Optionally (a flag of the matrix) the same contraction on the bfloat16 matrix cores
//                  from operands split in two bfloat16 terms: corr_split_kernel, or the bfloat16 form
//                  of corr_pipelined_kernel on full tiles.
//   pick / factor / residual   re-score the near-maximal candidates in double (so the argmax does
//                  not depend on float rounding), append the winning column, extend F = L^-H
//                  (App. B) by mat-vecs only, and recompute the residual y - A_Lambda x in double.
// After the last iteration refit_kernel can fit a second right-hand side on the support found.
// App. B precomputes the Gram matrix A^H A (d x d) to avoid the contraction; here the contraction
// is kept (it is what the matrix cores are for) and only inner products with selected columns are
// formed, so memory stays O(N k r).
#include <type_traits>

#include "philox_normal.h"
#include "sgc_internal.h"

namespace sgc {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr float RESCORE_TOL = 0x1.0p-10f; // candidates within this relative distance of the float maximum

OmpWorkspace carve_workspace(void *base, int32_t N, int32_t d, int32_t r, int32_t k)
{
    OmpWorkspace w{};
    size_t off = 0;
    auto take = [&](size_t bytes) {
        void *p = base ? (void *)((char *)base + off) : nullptr;
        off += (bytes + 255) & ~(size_t)255;
        return p;
    };
    w.tiles_m = corr_tiles_m(d);
    w.words = (d + 31) / 32;
    w.res64 = (double *)take(sizeof(double) * (size_t)N * r);
    w.f_stride = (int64_t)k * k + 288;
    w.F = (double *)take(sizeof(double) * (size_t)N * w.f_stride);
    w.avec = (double *)take(sizeof(double) * (size_t)N * k);
    w.xs = (double *)take(sizeof(double) * (size_t)N * k * 2);
    w.xs_half = (int64_t)N * k;
    w.res32 = (float *)take(sizeof(float) * (size_t)N * r);
    w.res16 = reinterpret_cast<uint16_t *>(w.res32);
    w.cols = (float *)take(sizeof(float) * (size_t)N * k * r);
    w.partial = (uint64_t *)take(sizeof(uint64_t) * (size_t)N * w.tiles_m * 2);
    w.bitmap = (uint32_t *)take(sizeof(uint32_t) * (size_t)N * w.words);
    // Rows of a generated matrix, in whole tiles. A matrix of at most 64 MiB gets a panel of its own (it
    // then stays in the 256 MiB memory-side cache). A larger one is written out whole where the column
    // copies would be, if it is no larger than they are (d <= N k; the copies are not needed once the
    // rows are resident), else it goes through a 64 MiB panel that is refilled in every iteration.
    int64_t small_rows = ((int64_t)64 << 20) / ((int64_t)r * 4);
    small_rows = small_rows / 256 * 256;
    if (small_rows < 256)
        small_rows = 256;
    {
        const int64_t dpad = ((int64_t)d + 255) / 256 * 256;
        if (small_rows > dpad)
            small_rows = dpad;
        if (dpad > small_rows && dpad <= (int64_t)N * k) {
            w.panel_rows = (int32_t)dpad;
            w.panel = w.cols;
        } else {
            w.panel_rows = (int32_t)small_rows;
            w.panel = (float *)take(sizeof(float) * (size_t)small_rows * r);
        }
    }
    // bfloat16 planes of the matrix rows for the screening contraction: the whole matrix if that is at
    // most 2 GiB, else a 64 MiB panel's worth (larger resident matrices then keep the float contraction)
    {
        const int64_t dpad = ((int64_t)d + 127) / 128 * 128;
        w.a16_rows = dpad * r * 4 <= ((int64_t)2 << 30) ? (int32_t)dpad : (int32_t)small_rows;
        w.a16 = (uint16_t *)take(sizeof(float) * (size_t)w.a16_rows * r);
    }
    w.wv = (double *)take(sizeof(double) * (size_t)N * k);
    w.gb = (double *)take(sizeof(double) * (size_t)N * 2);
    w.bytes = off;
    return w;
}

// ----------------------------------------------------------------------------------------------
// a = hi + lo in bfloat16 (round to nearest even each), |a - hi - lo| <= 2^-17 |a|
__device__ __forceinline__ void split_bf16_1(float a, uint16_t &hi, uint16_t &lo)
{
    const __bf16 h = (__bf16)a;
    const __bf16 l = (__bf16)(a - (float)h);
    hi = *reinterpret_cast<const uint16_t *>(&h);
    lo = *reinterpret_cast<const uint16_t *>(&l);
}

// res_split != 0: the float copy of the residual is written in split32 format instead (see corr_split_kernel)
__global__ __launch_bounds__(256) void omp_init_kernel(const float *__restrict__ y, int32_t r, int32_t words,
                                                       double *__restrict__ res64, float *__restrict__ res32,
                                                       uint32_t *__restrict__ bitmap, int32_t res_split)
{
    const int64_t n = blockIdx.x;
    uint16_t *res16 = reinterpret_cast<uint16_t *>(res32);
    for (int32_t j = threadIdx.x; j < r; j += 256) {
        const float v = y[n * r + j];
        res64[n * r + j] = (double)v;
        if (res_split) { // split32 row: the same 4 r bytes as the float row
            uint16_t hi, lo;
            split_bf16_1(v, hi, lo);
            uint16_t *o = res16 + n * 2 * r + (j >> 5) * 64 + (j & 31);
            o[0] = hi;
            o[32] = lo;
        } else {
            res32[n * r + j] = v;
        }
    }
    for (int32_t w = threadIdx.x; w < words; w += 256)
        bitmap[n * words + w] = 0u;
}

// ----------------------------------------------------------------------------------------------
// keep the two largest keys seen
__device__ __forceinline__ void top2_insert(uint64_t key, uint64_t &best, uint64_t &second)
{
    const uint64_t lo = key < best ? key : best;
    best = key < best ? best : key;
    second = lo < second ? second : lo;
}

// Epilogue shared by the contraction kernels: scale the accumulators by the reciprocal column
// norms, mask selected positions and reduce to the two best packed (score, position) keys per
// right-hand side and tile. `red` is LDS scratch of WMW*BN*2 keys that is no longer in use.
template <int BM, int BN, int WMW, int WNW, int MB, int NB>
__device__ __forceinline__ void corr_epilogue(const MatrixView &A, floatx16 (&acc)[MB][NB], uint64_t *red, int32_t N,
                                              const uint32_t *__restrict__ bitmap, int32_t words,
                                              uint64_t *__restrict__ partial, int32_t tiles_m, int32_t m0, int32_t n0,
                                              int wm, int wn)
{
    const int tid = threadIdx.x, lane = tid & 63;
    const int l32 = lane & 31, lhalf = lane >> 5;
    const int32_t d = A.d;
    // reciprocal norms of this lane's MB x 16 positions (4 runs of 4 consecutive positions per block)
    // and the selection masks, fetched together before any of them is used
    float4 inv[MB][4];
    uint32_t msk[MB][NB];
#pragma unroll
    for (int a = 0; a < MB; ++a) {
        const int32_t ibase = m0 + wm * (BM / WMW) + a * 32;
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
            const int32_t i0 = ibase + 8 * qd + 4 * lhalf;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i0 + 3 < d) {
                v = *reinterpret_cast<const float4 *>(A.inv_colnorm + i0);
            } else {
                if (i0 < d) v.x = A.inv_colnorm[i0];
                if (i0 + 1 < d) v.y = A.inv_colnorm[i0 + 1];
                if (i0 + 2 < d) v.z = A.inv_colnorm[i0 + 2];
            }
            inv[a][qd] = v;
        }
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int32_t n = n0 + wn * (BN / WNW) + b * 32 + l32;
            msk[a][b] = (n < N && ibase < d) ? bitmap[(int64_t)n * words + (ibase >> 5)] : 0xffffffffu;
        }
    }
    __syncthreads();
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int nl = wn * (BN / WNW) + b * 32 + l32; // right-hand side within the tile
        uint64_t best = 0, second = 0;
#pragma unroll
        for (int a = 0; a < MB; ++a) {
            const int32_t ibase = m0 + wm * (BM / WMW) + a * 32;
            const uint32_t mask = msk[a][b];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int off = 8 * (v >> 2) + 4 * lhalf + (v & 3);
                const int32_t i = ibase + off;
                const float4 nv = inv[a][v >> 2];
                const float in = (v & 3) == 0 ? nv.x : ((v & 3) == 1 ? nv.y : ((v & 3) == 2 ? nv.z : nv.w));
                const float score = fabsf(acc[a][b][v]) * in;
                const bool ok = i < d && !((mask >> off) & 1u);
                const uint64_t key = ok ? (((uint64_t)__float_as_uint(score) << 32) | (uint64_t)(0xffffffffu - (uint32_t)i)) : 0ull;
                top2_insert(key, best, second);
            }
        }
        // the other half-wave holds the remaining positions of the same right-hand side
        const uint64_t ob = shfl_xor_u64(best, 32), os = shfl_xor_u64(second, 32);
        top2_insert(ob, best, second);
        top2_insert(os, best, second);
        if (lhalf == 0) {
            red[(wm * BN + nl) * 2 + 0] = best;
            red[(wm * BN + nl) * 2 + 1] = second;
        }
    }
    __syncthreads();
    if (tid < BN) {
        const int32_t n = n0 + tid;
        if (n < N) {
            uint64_t best = red[tid * 2], second = red[tid * 2 + 1];
#pragma unroll
            for (int w = 1; w < WMW; ++w) {
                top2_insert(red[(w * BN + tid) * 2], best, second);
                top2_insert(red[(w * BN + tid) * 2 + 1], best, second);
            }
            uint64_t *o = partial + ((int64_t)n * tiles_m + m0 / BM) * 2;
            o[0] = best;
            o[1] = second;
        }
    }
}

// Correlation contraction + fused selection epilogue.
//   grid.x = tiles over positions i (BM each), grid.y = tiles over right-hand sides (BN each)
//   WMW x WNW wavefronts; each owns a (BM/WMW) x (BN/WNW) sub-tile made of 32x32 MFMA blocks.
// MFMA 32x32x2 operands: lane l supplies At[row l%32][depth l/32] and R[rhs l%32][depth l/32]. Each
// lane reads four consecutive depths with one 16-byte LDS read; lanes 32..63 read depths +4..+7, so
// four MFMAs cover eight depths (the sum over depth does not depend on their order).
// Accumulator register v of lane l holds position 8*(v/4) + 4*(l/32) + v%4 of right-hand side l%32.
// LDS rows are padded by 4 floats: 16-byte aligned and conflict-free for the 16-byte reads.
template <bool GENERATED, int BM, int BN, int BK, int WMW, int WNW, int MINB>
__global__ __launch_bounds__(WMW * WNW * 64, MINB) void corr_kernel(MatrixView A, const float *__restrict__ R,
                                                                    int32_t N, const uint32_t *__restrict__ bitmap,
                                                                    int32_t words, uint64_t *__restrict__ partial,
                                                                    int32_t tiles_m)
{
    constexpr int T = WMW * WNW * 64;
    constexpr int LD = BK + 4;
    constexpr int MB = BM / WMW / 32, NB = BN / WNW / 32; // MFMA blocks per wavefront
    constexpr int LA = BM * BK / 4 / T, LB = BN * BK / 4 / T; // 16-byte pieces per thread per stage
    constexpr int C4 = BK / 4;
    static_assert(BM * BK / 4 % T == 0 && BN * BK / 4 % T == 0, "tile does not divide among the threads");
    extern __shared__ __attribute__((aligned(16))) float corr_lds[];
    float *lds_a = corr_lds;               // [2][BM*LD]
    float *lds_b = corr_lds + 2 * BM * LD; // [2][BN*LD]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WNW, wn = wave % WNW;
    const int32_t d = A.d, r = A.r;
    const int32_t m0 = A.row0 + blockIdx.x * BM; // row0 is a multiple of BM
    const int32_t n0 = blockIdx.y * BN;
    const float *At0 = A.At - (int64_t)A.row0 * r;

    float4 ga[LA], gb[LB];
    auto load_global = [&](int32_t k0) {
#pragma unroll
        for (int u = 0; u < LA; ++u) {
            const int f = tid + T * u;
            const int32_t i = m0 + f / C4, kk = k0 + (f % C4) * 4;
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i < d && kk < r) {
                if (GENERATED)
                    a = matrix_quad((uint32_t)i, (uint32_t)(kk >> 2), A.key0, A.key1, A.scale);
                else
                    a = *reinterpret_cast<const float4 *>(At0 + (int64_t)i * r + kk);
            }
            ga[u] = a;
        }
#pragma unroll
        for (int u = 0; u < LB; ++u) {
            const int f = tid + T * u;
            const int32_t n = n0 + f / C4, kk = k0 + (f % C4) * 4;
            float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
            if (n < N && kk < r)
                b = *reinterpret_cast<const float4 *>(R + (int64_t)n * r + kk);
            gb[u] = b;
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int u = 0; u < LA; ++u) {
            const int f = tid + T * u;
            *reinterpret_cast<float4 *>(&lds_a[buf * BM * LD + (f / C4) * LD + (f % C4) * 4]) = ga[u];
        }
#pragma unroll
        for (int u = 0; u < LB; ++u) {
            const int f = tid + T * u;
            *reinterpret_cast<float4 *>(&lds_b[buf * BN * LD + (f / C4) * LD + (f % C4) * 4]) = gb[u];
        }
    };

    floatx16 acc[MB][NB];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[a][b][v] = 0.f;

    const int nkb = (r + BK - 1) / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    const int l32 = lane & 31, lhalf = lane >> 5;
    for (int kb = 0; kb < nkb; ++kb) {
        const int buf = kb & 1;
        if (kb + 1 < nkb)
            load_global((kb + 1) * BK);
        const float *pa = &lds_a[buf * BM * LD + (wm * (BM / WMW) + l32) * LD + lhalf * 4];
        const float *pb = &lds_b[buf * BN * LD + (wn * (BN / WNW) + l32) * LD + lhalf * 4];
#pragma unroll
        for (int ks = 0; ks < BK; ks += 8) {
            float4 av[MB], bv[NB];
#pragma unroll
            for (int a = 0; a < MB; ++a)
                av[a] = *reinterpret_cast<const float4 *>(pa + a * 32 * LD + ks);
#pragma unroll
            for (int b = 0; b < NB; ++b)
                bv[b] = *reinterpret_cast<const float4 *>(pb + b * 32 * LD + ks);
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int a = 0; a < MB; ++a)
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        const float x = t == 0 ? av[a].x : (t == 1 ? av[a].y : (t == 2 ? av[a].z : av[a].w));
                        const float y = t == 0 ? bv[b].x : (t == 1 ? bv[b].y : (t == 2 ? bv[b].z : bv[b].w));
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, acc[a][b], 0, 0, 0);
                    }
        }
        if (kb + 1 < nkb)
            store_lds(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: normalise, mask, keep the two best per right-hand side ----
    corr_epilogue<BM, BN, WMW, WNW, MB, NB>(A, acc, reinterpret_cast<uint64_t *>(corr_lds), N, bitmap, words, partial,
                                            tiles_m, m0, n0, wm, wn);
}

// Screening variant of the contraction on the bfloat16 matrix cores (an option of the matrix, never the
// default). Every float operand is split into two bfloat16 terms, a = hi + lo with |a - hi - lo| <=
// 2^-17 |a|, and the product is taken as lo*hi + hi*lo + hi*hi in three v_mfma_f32_32x32x16_bf16 with
// float accumulation: scores agree with the float contraction to ~1e-5 relative, far inside the 2^-10
// band of near-maximal candidates that the selection kernel re-scores in double, so the selected
// support does not change while the matrix-core time drops by a factor of five (16 x the rate, three
// products).
// Split format ("split32", r % 32 == 0): a row of r floats becomes r/32 blocks of 128 bytes, each the 32
// high parts followed by the 32 low parts of 32 consecutive depths, so a row keeps its 4r bytes and a
// depth-32 stage of a row is one contiguous 128-byte piece, as for floats. The rows of At are split
// once per call (or per panel fill) into ws.a16, the residuals are written in this format by the
// update kernel.
// Kernel: 128 x 128 outputs per workgroup, 2 x 2 wavefronts of 64 x 64, depth 32 per stage; pieces are
// fetched two stages ahead into registers and copied to LDS as they are (rows padded to 144 bytes:
// 16-byte accesses without bank conflicts); a fragment is 16 bytes: lane l supplies row l % 32, depths
// 8 (l / 32) .. +7 of a 16-deep block, for both operands alike.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
constexpr int SPLIT_ROWB = 144; // bytes per LDS row: 32 high parts, 32 low parts, 16 bytes of padding

__device__ __forceinline__ void split_bf16(const float4 &a, uint2 &hi, uint2 &lo)
{
    const bf16x2 h0 = {(__bf16)a.x, (__bf16)a.y}, h1 = {(__bf16)a.z, (__bf16)a.w};
    const bf16x2 l0 = {(__bf16)(a.x - (float)h0[0]), (__bf16)(a.y - (float)h0[1])};
    const bf16x2 l1 = {(__bf16)(a.z - (float)h1[0]), (__bf16)(a.w - (float)h1[1])};
    hi = make_uint2(*reinterpret_cast<const uint32_t *>(&h0), *reinterpret_cast<const uint32_t *>(&h1));
    lo = make_uint2(*reinterpret_cast<const uint32_t *>(&l0), *reinterpret_cast<const uint32_t *>(&l1));
}

// byte offset, inside a split32 row, of the high parts of the float quad jb (depths 4 jb .. 4 jb + 3);
// the low parts sit 64 bytes further
__device__ __forceinline__ int64_t split32_quad_offset(int32_t jb)
{
    return (int64_t)(jb >> 3) * 128 + (jb & 7) * 8;
}

// As: rows of At in split32 format, row 0 = position A.row0; Rs: the residuals in split32 format.
__global__ __launch_bounds__(256, 2) void corr_split_kernel(MatrixView A, const unsigned char *__restrict__ As,
                                                            const unsigned char *__restrict__ Rs, int32_t N,
                                                            const uint32_t *__restrict__ bitmap, int32_t words,
                                                            uint64_t *__restrict__ partial, int32_t tiles_m)
{
    constexpr int BM = 128, BN = 128, MB = 2, NB = 2, LQ = 4; // LQ 16-byte pieces per thread, tile and stage
    constexpr int TILE = 128 * SPLIT_ROWB;
    extern __shared__ __attribute__((aligned(16))) float corr_lds[];
    unsigned char *lds = reinterpret_cast<unsigned char *>(corr_lds); // A tile, then R tile
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int32_t d = A.d, r = A.r;
    const int64_t rowb = (int64_t)r * 4; // bytes per row, as for floats
    const int32_t m0 = A.row0 + blockIdx.x * BM, n0 = blockIdx.y * BN;
    const unsigned char *As0 = As - (int64_t)A.row0 * rowb;

    uint4 ga[2][LQ], gb[2][LQ];
    auto load_global = [&](int set, int32_t kb) {
#pragma unroll
        for (int u = 0; u < LQ; ++u) {
            const int f = tid + 256 * u; // 128 rows x 8 pieces
            const int32_t row = f >> 3;
            const int64_t off = (int64_t)kb * 128 + (f & 7) * 16;
            uint4 a = make_uint4(0u, 0u, 0u, 0u), b = a;
            if (m0 + row < d)
                a = *reinterpret_cast<const uint4 *>(As0 + (int64_t)(m0 + row) * rowb + off);
            if (n0 + row < N)
                b = *reinterpret_cast<const uint4 *>(Rs + (int64_t)(n0 + row) * rowb + off);
            ga[set][u] = a;
            gb[set][u] = b;
        }
    };
    auto store_lds = [&](int set, int buf) { // LDS: two stage buffers, each the A tile then the R tile
#pragma unroll
        for (int u = 0; u < LQ; ++u) {
            const int f = tid + 256 * u;
            const int off = buf * 2 * TILE + (f >> 3) * SPLIT_ROWB + (f & 7) * 16;
            *reinterpret_cast<uint4 *>(lds + off) = ga[set][u];
            *reinterpret_cast<uint4 *>(lds + TILE + off) = gb[set][u];
        }
    };

    floatx16 acc[MB][NB];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[a][b][v] = 0.f;

    const int nkb = r / 32;
    const int l32 = lane & 31, lhalf = lane >> 5;
    const unsigned char *pa = lds + (wm * 64 + l32) * SPLIT_ROWB + lhalf * 16;
    const unsigned char *pb = lds + TILE + (wn * 64 + l32) * SPLIT_ROWB + lhalf * 16;
    // stage kb computes from LDS buffer kb & 1 while stage kb + 1 waits in registers (set (kb + 1) & 1)
    // and stage kb + 2 is being fetched into the set just emptied; one barrier per stage
    load_global(0, 0);
    store_lds(0, 0);
    if (nkb > 1)
        load_global(1, 1);
    if (nkb > 2)
        load_global(0, 2);
    __syncthreads();
    auto stage = [&](int kb, auto bufc) {
        constexpr int buf = decltype(bufc)::value; // also the register set that is being refilled: kb & 1
#pragma unroll
        for (int kq = 0; kq < 2; ++kq) {
            bf16x8 ah[MB], al[MB], bh[NB], bl[NB];
#pragma unroll
            for (int a = 0; a < MB; ++a) {
                ah[a] = *reinterpret_cast<const bf16x8 *>(pa + buf * 2 * TILE + a * 32 * SPLIT_ROWB + kq * 32);
                al[a] = *reinterpret_cast<const bf16x8 *>(pa + buf * 2 * TILE + a * 32 * SPLIT_ROWB + 64 + kq * 32);
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                bh[b] = *reinterpret_cast<const bf16x8 *>(pb + buf * 2 * TILE + b * 32 * SPLIT_ROWB + kq * 32);
                bl[b] = *reinterpret_cast<const bf16x8 *>(pb + buf * 2 * TILE + b * 32 * SPLIT_ROWB + 64 + kq * 32);
            }
            // the three products of a block are issued four MFMAs apart (no back-to-back dependency)
#pragma unroll
            for (int prod = 0; prod < 3; ++prod)
#pragma unroll
                for (int a = 0; a < MB; ++a)
#pragma unroll
                    for (int b = 0; b < NB; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(prod == 0 ? al[a] : ah[a],
                                                                            prod == 1 ? bl[b] : bh[b], acc[a][b], 0, 0, 0);
        }
        if (kb + 1 < nkb)
            store_lds(buf ^ 1, buf ^ 1); // stage kb + 1: register set (kb + 1) & 1 -> LDS buffer (kb + 1) & 1
        if (kb + 3 < nkb)
            load_global(buf ^ 1, kb + 3);
        __syncthreads();
    };
    for (int kb = 0; kb < nkb; kb += 2) {
        stage(kb, std::integral_constant<int, 0>{});
        if (kb + 1 < nkb)
            stage(kb + 1, std::integral_constant<int, 1>{});
    }
    corr_epilogue<BM, BN, 2, 2, MB, NB>(A, acc, reinterpret_cast<uint64_t *>(corr_lds), N, bitmap, words, partial,
                                        tiles_m, m0, n0, wm, wn);
}

// rows of floats -> split32 rows (count4 float quads, r4 quads per row)
__global__ __launch_bounds__(256) void split_rows_kernel(const float *__restrict__ src, int64_t count4, int32_t r4,
                                                         unsigned char *__restrict__ dst)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < count4; e += stride) {
        const int64_t row = e / r4;
        const int32_t jb = (int32_t)(e - row * r4);
        uint2 h, l;
        split_bf16(load_once_f4(src + 4 * e), h, l);
        unsigned char *o = dst + row * ((int64_t)r4 * 16) + split32_quad_offset(jb);
        *reinterpret_cast<uint2 *>(o) = h;
        *reinterpret_cast<uint2 *>(o + 64) = l;
    }
}

static void launch_split_rows(const float *src, int64_t rows, int32_t r, uint16_t *dst, hipStream_t s)
{
    const int64_t count4 = rows * (r >> 2);
    int64_t blocks = (count4 + 255) / 256;
    if (blocks > 256 * 32)
        blocks = 256 * 32;
    if (blocks > 0)
        split_rows_kernel<<<dim3((unsigned)blocks), 256, 0, s>>>(src, count4, r >> 2,
                                                                  reinterpret_cast<unsigned char *>(dst));
}

static hipError_t corr_split_launch(const MatrixView &A, const uint16_t *rows_split, int32_t rows, int32_t N,
                                    const OmpWorkspace &ws, int32_t tiles_m, hipStream_t s)
{
    constexpr size_t smem = (size_t)4 * 128 * SPLIT_ROWB;
    static bool raised = false;
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(corr_split_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess)
            return e;
        raised = true;
    }
    const dim3 grid((unsigned)((rows + 127) / 128), (unsigned)((N + 127) / 128));
    corr_split_kernel<<<grid, 256, smem, s>>>(A, reinterpret_cast<const unsigned char *>(rows_split),
                                              reinterpret_cast<const unsigned char *>(ws.res16), N, ws.bitmap, ws.words,
                                              ws.partial, tiles_m);
    return hipSuccess;
}

// One tiling of the contraction: sizes, and a launcher that raises the dynamic-LDS limit once.
template <bool GENERATED, int BM, int BN, int BK, int WMW, int WNW, int MINB>
static hipError_t corr_launch(const MatrixView &A, int32_t rows, const float *R, int32_t N, const OmpWorkspace &ws,
                              int32_t tiles_m, hipStream_t s)
{
    constexpr size_t smem = (size_t)2 * (BM + BN) * (BK + 4) * sizeof(float);
    auto kern = corr_kernel<GENERATED, BM, BN, BK, WMW, WNW, MINB>;
    static bool raised = false;
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess)
            return e;
        raised = true;
    }
    const dim3 grid((unsigned)((rows + BM - 1) / BM), (unsigned)((N + BN - 1) / BN));
    kern<<<grid, WMW * WNW * 64, smem, s>>>(A, R, N, ws.bitmap, ws.words, ws.partial, tiles_m);
    return hipSuccess;
}

// Software-pipelined contraction for full position tiles of a stored matrix (rows % 256 == 0,
// r % 64 == 0; a ragged last tile of right-hand sides computes on copies of the last one): 256 x 128 outputs per workgroup, one wavefront per SIMD, each wavefront a 128 x 64
// sub-tile (4 x 2 MFMA blocks, accumulators in AGPRs). A depth-32 stage is 4 groups of 32 MFMAs;
// every memory operation is issued in the shadow of an MFMA and the order is pinned:
//   group 0..2  fragment reads of the next group (double-buffered in registers)
//   group 2     LDS writes of the staged next stage (into the stage read one iteration earlier), then
//               the global loads two stages ahead into the registers just freed
//   barrier
//   group 3     fragment reads of the next stage's first group
// so the matrix pipe only waits for the barrier itself. Addresses are a uniform base plus one per-lane
// offset (no per-row bounds checks: tiles are full), and the depth loop is unrolled by two so that
// LDS stage offsets are immediates.
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

constexpr int CORRP_BM = 256;

// NB = 2: the 256 x 128 tile described above. NB = 1: a 256 x 64 tile for at most 64 right-hand sides
// (each wavefront 128 x 32, groups of 16 MFMAs; the LDS write and the global load of a staging piece
// follow the same MFMA of group 2, so the load still leads its use by a whole stage).
// BF16: the screening variant. At and R point to rows in split32 format (see corr_split_kernel: the same
// 4 r bytes per row, a depth-32 stage of a row is 32 high parts then 32 low parts), so the data movement is
// the float kernel's; a stage is two groups (16 depths each) of 3 * 8 MFMAs v_mfma_f32_32x32x16_bf16
// (low*high, high*low, high*high per block), and because a stage is five times shorter the global loads
// run three stages ahead through two sets of staging registers.
template <int NB, bool BF16>
__global__ __launch_bounds__(256, 1) void corr_pipelined_kernel(MatrixView A, const float *__restrict__ R, int32_t N,
                                                                const uint32_t *__restrict__ bitmap, int32_t words,
                                                                uint64_t *__restrict__ partial, int32_t tiles_m)
{
    constexpr int BM = CORRP_BM, BN = 64 * NB, BK = 32, LD = BK + 4, MB = 4;
    constexpr int WN = 32 * NB;            // right-hand sides per wavefront
    constexpr int GM = 4 * MB * NB;        // MFMAs per group (8 depths)
    constexpr int LA = 8, LB = 2 * NB;     // 16-byte pieces per thread per stage
    typedef float floatx4 __attribute__((ext_vector_type(4)));
    extern __shared__ __attribute__((aligned(16))) float corr_lds[];
    float *lds = corr_lds; // A stages [2][BM*LD], then R stages [2][BN*LD], then what the epilogue needs:
    float *inv_s = corr_lds + 2 * (BM + BN) * LD;                       // reciprocal norms of the BM positions
    uint32_t *msk_s = reinterpret_cast<uint32_t *>(inv_s + BM);         // selection words [BN][BM/32]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int32_t r = A.r;
    const int32_t m0 = A.row0 + blockIdx.x * BM, n0 = blockIdx.y * BN;
    const int l32 = lane & 31, lhalf = lane >> 5;
    const float *abase = A.At + (int64_t)(blockIdx.x * BM) * r;
    const float *bbase = R + (int64_t)n0 * r;
    const uint32_t lane_off = (uint32_t)((tid >> 3) * r + ((tid & 7) << 2));
    // right-hand sides past the end of a ragged last tile re-read the last one; their results are dropped
    uint32_t rhs_off[LB];
#pragma unroll
    for (int u = 0; u < LB; ++u) {
        const int32_t n = n0 + 32 * u + (tid >> 3);
        rhs_off[u] = (uint32_t)(((n < N ? n : N - 1) - n0) * r + ((tid & 7) << 2));
    }
    const int ldst0 = (tid >> 3) * LD + ((tid & 7) << 2);
    const int nkb = r / BK;

    constexpr int GS = BF16 ? 2 : 1; // staging register sets
    constexpr int FH = BF16 ? 2 : 1; // fragment parts (high, low)
    floatx4 g[GS][LA + LB];
    floatx4 fa[2][MB][FH], fb[2][NB][FH];
    floatx16 acc[MB][NB];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[a][b][v] = 0.f;
    const int ra = (wm * 128 + l32) * LD + lhalf * 4; // fragment read offsets (floats)
    const int rb = 2 * BM * LD + (wn * WN + l32) * LD + lhalf * 4;

    auto gload = [&](int u, int kb, int set = 0) { // staging piece u of stage kb (the last stage again beyond the end)
        const int kk = (kb < nkb ? kb : nkb - 1) * BK;
        if (u < LA)
            g[set][u] = *reinterpret_cast<const floatx4 *>(abase + ((int64_t)(32 * u) * r + kk) + lane_off);
        else
            g[set][u] = *reinterpret_cast<const floatx4 *>(bbase + kk + rhs_off[u < LA ? 0 : u - LA]);
    };
    auto lwrite = [&](int u, int buf, int set = 0) {
        const int off = u < LA ? buf * BM * LD + 32 * u * LD : 2 * BM * LD + buf * BN * LD + 32 * (u - LA) * LD;
        *reinterpret_cast<floatx4 *>(lds + ldst0 + off) = g[set][u];
    };
    // float: ks = 0..3, eight depths each. BF16: ks = 0..1, sixteen depths each, high parts and, 16 floats
    // (64 bytes) further in the row, low parts.
    auto fread = [&](int which, int op, int buf, int ks) { // op 0..3: block row of At, 4..5: block of R
#pragma unroll
        for (int h = 0; h < FH; ++h) {
            if (op < MB)
                fa[which][op][h] =
                    *reinterpret_cast<const floatx4 *>(lds + ra + buf * BM * LD + op * 32 * LD + ks * 8 + h * 16);
            else
                fb[which][op - MB][h] = *reinterpret_cast<const floatx4 *>(lds + rb + buf * BN * LD +
                                                                           (op - MB) * 32 * LD + ks * 8 + h * 16);
        }
    };
    auto mfma = [&](int which, int m) { // m = 0..GM-1: depth t of the fragment, then block row a, block column b
        const int t = m / (MB * NB), a = (m % (MB * NB)) / NB, b = m % NB;
        if constexpr (BF16) { // t = 0: low * high, 1: high * low, 2: high * high
            const floatx4 x4 = fa[which][a][t == 0 ? FH - 1 : 0], y4 = fb[which][b][t == 1 ? FH - 1 : 0];
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, x4),
                                                                __builtin_bit_cast(bf16x8, y4), acc[a][b], 0, 0, 0);
        } else {
            const floatx4 x4 = fa[which][a][0], y4 = fb[which][b][0];
            const float x = t == 0 ? x4.x : (t == 1 ? x4.y : (t == 2 ? x4.z : x4.w));
            const float y = t == 0 ? y4.x : (t == 1 ? y4.y : (t == 2 ? y4.z : y4.w));
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(x, y, acc[a][b], 0, 0, 0);
        }
    };

    // prologue: stage 0 -> LDS, stage 1 -> staging registers, fragments of (stage 0, group 0); the
    // epilogue's operands are fetched here too, so that it does not wait for memory at the end
    static_for<0, LA + LB>([&](auto uc) { gload(decltype(uc)::value, 0); });
    {
        const float nv = A.inv_colnorm[m0 + tid];
        uint32_t mw[BN * (BM / 32) / 256];
#pragma unroll
        for (int u = 0; u < BN * (BM / 32) / 256; ++u) {
            const int e = tid + 256 * u;
            const int32_t n = n0 + (e >> 3);
            mw[u] = bitmap[(int64_t)(n < N ? n : N - 1) * words + (m0 >> 5) + (e & 7)];
        }
        inv_s[tid] = nv;
#pragma unroll
        for (int u = 0; u < BN * (BM / 32) / 256; ++u)
            msk_s[tid + 256 * u] = mw[u];
    }
    static_for<0, LA + LB>([&](auto uc) { lwrite(decltype(uc)::value, 0); });
    static_for<0, LA + LB>([&](auto uc) { gload(decltype(uc)::value, 1, GS - 1); });
    if constexpr (BF16)
        static_for<0, LA + LB>([&](auto uc) { gload(decltype(uc)::value, 2, 0); });
    __syncthreads();
    static_for<0, MB + NB>([&](auto oc) { fread(0, decltype(oc)::value, 0, 0); });

    // BF16 stage kb (LDS buffer buf = kb & 1): stage kb + 1 waits in staging set buf ^ 1, stage kb + 2 in
    // set buf. Group 0 (first 16 depths, fragments read in the previous stage) reads the fragments of
    // group 1 and copies set buf ^ 1 into the other LDS buffer; barrier; group 1 reads the first
    // fragments of stage kb + 1 and refills set buf ^ 1 with stage kb + 3.
    auto stage_bf16 = [&](int kb, auto bufc) {
        constexpr int buf = decltype(bufc)::value;
        constexpr int G3 = 3 * MB * NB;
        static_for<0, G3>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            mfma(0, m);
            if constexpr (m < MB + NB)
                fread(1, m, buf, 1);
            else if constexpr (m < MB + NB + LA + LB)
                lwrite(m - (MB + NB), buf ^ 1, (buf ^ 1) & (GS - 1));
            __builtin_amdgcn_sched_barrier(0);
        });
        __syncthreads();
        static_for<0, G3>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            mfma(1, m);
            if constexpr (m < MB + NB)
                fread(0, m, buf ^ 1, 0);
            else if constexpr (m < MB + NB + LA + LB)
                gload(m - (MB + NB), kb + 3, (buf ^ 1) & (GS - 1));
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    auto stage = [&](int kb, auto bufc) {
        constexpr int buf = decltype(bufc)::value;
        static_for<0, GM>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            mfma(0, m);
            if constexpr (m < MB + NB)
                fread(1, m, buf, 1);
            __builtin_amdgcn_sched_barrier(0);
        });
        static_for<0, GM>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            mfma(1, m);
            if constexpr (m < MB + NB)
                fread(0, m, buf, 2);
            __builtin_amdgcn_sched_barrier(0);
        });
        static_for<0, GM>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            mfma(0, m);
            if constexpr (m < MB + NB) {
                fread(1, m, buf, 3);
            } else if constexpr (NB == 2) {
                if constexpr (m >= 6 && m < 6 + LA + LB)
                    lwrite(m - 6, buf ^ 1);
                else if constexpr (m >= 20 && m < 20 + LA + LB)
                    gload(m - 20, kb + 2);
            } else if constexpr (m < MB + NB + LA + LB) {
                lwrite(m - (MB + NB), buf ^ 1);
                gload(m - (MB + NB), kb + 2);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        __syncthreads();
        static_for<0, GM>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            mfma(1, m);
            if constexpr (m < MB + NB)
                fread(0, m, buf ^ 1, 0);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    for (int kb = 0; kb < nkb; kb += 2) {
        if constexpr (BF16) {
            stage_bf16(kb, std::integral_constant<int, 0>{});
            stage_bf16(kb + 1, std::integral_constant<int, 1>{});
        } else {
            stage(kb, std::integral_constant<int, 0>{});
            stage(kb + 1, std::integral_constant<int, 1>{});
        }
    }
    __syncthreads();

    // epilogue, one 32-row block of accumulators at a time (keeps the register peak low). Inside a
    // wavefront's 128 positions the two best are kept as 32-bit keys: the float score bits with the
    // low byte replaced by 255 - (position within the 128), so an unsigned max is the argmax with the
    // lower position winning among equal keys, and a selected position is key 0, below every live
    // one. Dropping 8 mantissa bits (2^-15 relative) is far inside the band of near-maximal
    // candidates that the selection kernel re-scores in double anyway.
    // Selected positions are left in on the first scan: their columns are orthogonal to the residual,
    // so they only reach the top two when the whole residual is rounding noise or zero; the two
    // winners are then tested against the selection bitmap and, if any lane of the wavefront holds a
    // selected one, the scan is repeated with the selected positions forced to key 0.
    uint64_t *red = reinterpret_cast<uint64_t *>(corr_lds);
    uint32_t best[NB], second[NB], msk[MB][NB];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
            msk[a][b] = msk_s[(wn * WN + b * 32 + l32) * (BM / 32) + wm * 4 + a];
    auto scan = [&](auto maskedc) {
        constexpr bool MASKED = decltype(maskedc)::value;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            best[b] = 0;
            second[b] = 0;
        }
#pragma unroll
        for (int a = 0; a < MB; ++a) {
            float4 inv[4];
#pragma unroll
            for (int qd = 0; qd < 4; ++qd)
                inv[qd] = *reinterpret_cast<const float4 *>(inv_s + wm * 128 + a * 32 + 8 * qd + 4 * lhalf);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                // this lane's 16 positions of the block are bits 8*(v/4) + v%4 of the shifted word
                const uint32_t mask = msk[a][b] >> (4 * lhalf);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int bit = 8 * (v >> 2) + (v & 3);
                    const float4 nv = inv[v >> 2];
                    const float in = (v & 3) == 0 ? nv.x : ((v & 3) == 1 ? nv.y : ((v & 3) == 2 ? nv.z : nv.w));
                    const float score = fabsf(acc[a][b][v]) * in;
                    // low byte: 255 - (a*32 + bit); the lane's own 4*lhalf is accounted for when widening
                    uint32_t key = (__float_as_uint(score) & 0xffffff00u) | (uint32_t)(255 - (a * 32 + bit));
                    if (MASKED)
                        key = ((mask >> bit) & 1u) ? 0u : key;
                    second[b] = max(second[b], min(key, best[b]));
                    best[b] = max(best[b], key);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    scan(std::false_type{});
    uint32_t hit = 0;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
#pragma unroll
        for (int which = 0; which < 2; ++which) {
            const uint32_t k32 = which ? second[b] : best[b];
            const uint32_t pos = 255u - (k32 & 0xffu) + 4u * (uint32_t)lhalf; // within the wavefront's 128
#pragma unroll
            for (int a = 0; a < MB; ++a) // straight-line: every block's word is tested
                hit |= ((msk[a][b] >> (pos & 31u)) & 1u) & (uint32_t)((pos >> 5) == (uint32_t)a);
        }
    }
    if (__builtin_amdgcn_ballot_w64(hit != 0u) != 0ull)
        scan(std::true_type{});
    const uint32_t pos0 = (uint32_t)(m0 + wm * 128);
    auto widen = [&](uint32_t k32) -> uint64_t { // (score bits, ~position) as the selection kernel reads it
        if (k32 == 0)
            return 0ull;
        const uint32_t i = pos0 + (255u - (k32 & 0xffu)) + 4u * (uint32_t)lhalf;
        return ((uint64_t)(k32 & 0xffffff00u) << 32) | (uint64_t)(0xffffffffu - i);
    };
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int nl = wn * WN + b * 32 + l32;
        uint64_t wb = widen(best[b]), ws2 = widen(second[b]);
        const uint64_t ob = shfl_xor_u64(wb, 32), os = shfl_xor_u64(ws2, 32);
        top2_insert(ob, wb, ws2);
        top2_insert(os, wb, ws2);
        if (lhalf == 0) {
            red[(wm * BN + nl) * 2 + 0] = wb;
            red[(wm * BN + nl) * 2 + 1] = ws2;
        }
    }
    __syncthreads();
    if (tid < BN && n0 + tid < N) {
        const int32_t n = n0 + tid;
        uint64_t b0 = red[tid * 2], s0 = red[tid * 2 + 1];
        top2_insert(red[(BN + tid) * 2], b0, s0);
        top2_insert(red[(BN + tid) * 2 + 1], b0, s0);
        uint64_t *o = partial + ((int64_t)n * tiles_m + m0 / BM) * 2;
        o[0] = b0;
        o[1] = s0;
    }
}

template <int NB, bool BF16 = false>
static hipError_t corr_pipelined_launch_nb(const MatrixView &A, int32_t rows, const float *R, int32_t N,
                                           const OmpWorkspace &ws, int32_t tiles_m, hipStream_t s)
{
    constexpr int BN = 64 * NB;
    constexpr size_t smem = (size_t)2 * (CORRP_BM + BN) * 36 * sizeof(float) + CORRP_BM * sizeof(float) +
                            (size_t)BN * (CORRP_BM / 32) * sizeof(uint32_t);
    static bool raised = false;
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(corr_pipelined_kernel<NB, BF16>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess)
            return e;
        raised = true;
    }
    const dim3 grid((unsigned)(rows / CORRP_BM), (unsigned)((N + BN - 1) / BN));
    corr_pipelined_kernel<NB, BF16><<<grid, 256, smem, s>>>(A, R, N, ws.bitmap, ws.words, ws.partial, tiles_m);
    return hipSuccess;
}

static hipError_t corr_pipelined_launch(const MatrixView &A, int32_t rows, const float *R, int32_t N,
                                        const OmpWorkspace &ws, int32_t tiles_m, hipStream_t s)
{
    if (N <= 64)
        return corr_pipelined_launch_nb<1>(A, rows, R, N, ws, tiles_m, s);
    return corr_pipelined_launch_nb<2>(A, rows, R, N, ws, tiles_m, s);
}

// the split rows through the pipelined kernel: its data movement reads them as rows of r floats
static hipError_t corr_screen_launch(bool pipelined, const MatrixView &A, const uint16_t *rows_split, int32_t rows,
                                     int32_t N, const OmpWorkspace &ws, int32_t tiles_m, hipStream_t s)
{
    if (!pipelined)
        return corr_split_launch(A, rows_split, rows, N, ws, tiles_m, s);
    MatrixView As = A;
    As.At = reinterpret_cast<const float *>(rows_split);
    return corr_pipelined_launch_nb<2, true>(As, rows, reinterpret_cast<const float *>(ws.res16), N, ws, tiles_m, s);
}

// whether the pipelined kernel covers this problem (full tiles of positions, stored rows, even number
// of stages; the last tile of right-hand sides may be ragged)
static bool corr_pipelined_ok(const MatrixView &A, int32_t N, int32_t panel_rows)
{
    // at most 64 right-hand sides and few position tiles: the general kernel's 128-row tiles give
    // twice the workgroups, which matters more than the schedule when the chip is far from full
    if (N <= 64 && A.d / CORRP_BM < 128)
        return false;
    return A.d % CORRP_BM == 0 && A.r % 64 == 0 && panel_rows % CORRP_BM == 0;
}

// The tiling in use: 128 x 128 outputs (128 x 64 when there are at most 64 right-hand sides), depth 32
// per stage, 2 x 2 wavefronts, two workgroups per CU.
// It is the general kernel: any d, N, r % 4 == 0, generated or stored A. (Other shapes of this
// compiler-scheduled kernel - 256 x 128 with 4 or 8 wavefronts, depth 16 or 64, LDS filled directly
// with global_load_lds - all measured within 2 % of it inside the full step.)
template <bool GENERATED>
static hipError_t corr_dispatch(const MatrixView &A, int32_t rows, const float *R, int32_t N, const OmpWorkspace &ws,
                                int32_t tiles_m, hipStream_t s)
{
    // a single half-width tile of right-hand sides (no matrix-core work on padding), or so few full tiles
    // that only half-width ones give every CU the two workgroups it can hold
    if (N <= 64 || (int64_t)corr_tiles_m(rows) * ((N + CORR_BN - 1) / CORR_BN) <= 256)
        return corr_launch<GENERATED, CORR_BM, 64, 32, 2, 2, 2>(A, rows, R, N, ws, tiles_m, s);
    return corr_launch<GENERATED, CORR_BM, CORR_BN, 32, 2, 2, 2>(A, rows, R, N, ws, tiles_m, s);
}

// ----------------------------------------------------------------------------------------------
// Selection and least-squares update, two kernels per iteration:
//   pick_kernel      re-scores the near-maximal candidates in double and fixes lambda; then
//                    w_t = <A_:lambda_t, A_:lambda> for the earlier selections (a row-major mat-vec over
//                    the selected columns, one wavefront per row, spread over several workgroups)
//   update_kernel    the small dense part of App. B: c = F^H w, gamma, the new coefficient, the new
//                    column of F and x = F a, all in double; then res = y - A_Lambda x in double (a
//                    column-major mat-vec over the selected columns), plus the float copy for the
//                    next contraction
constexpr int PICK_THREADS_WIDE = 512, PICK_THREADS_NARROW = 128; // narrow: short columns (r <= 512) and k <= 128
constexpr int PICK_CAND_CAP = 64;
constexpr int FACTOR_MAX_THREADS = 1024;

struct IterArgs {
    const float *y; // [N][r]
    int32_t k, it;  // sparsity, current iteration (0-based)
    int32_t *sel;   // [N][k]
    float *x;       // [N][k]
    OmpWorkspace ws;
    // rows of At resident in memory (a stored matrix, or a generated one produced whole into the
    // panel): the least-squares passes then fetch the selected columns from here through `sel`,
    // where a matrix shared by many right-hand sides stays in cache, and ws.cols is not used.
    // NULL: the selected columns are kept per right-hand side in ws.cols.
    const float *At_rows;
    int32_t share_table; // update_kernel: its dynamic LDS also holds the [wavefront][k] table of shares
    int32_t res_split;   // update_kernel: != 0: the residual's float copy goes out in split32 format
};

template <bool GENERATED>
__device__ __forceinline__ float4 column_quad(const MatrixView &A, int32_t i, int32_t jb)
{
    if (GENERATED)
        return matrix_quad((uint32_t)i, (uint32_t)jb, A.key0, A.key1, A.scale);
    return reinterpret_cast<const float4 *>(A.At + (int64_t)i * A.r)[jb];
}

// grid (N, slices). Every slice of a right-hand side repeats the (cheap) selection so that no
// grid-wide synchronisation is needed; slice 0 also stores the column and the scalars.
// dynamic LDS: float a_col[r]
template <bool GENERATED, int PICK_THREADS>
__global__ __launch_bounds__(PICK_THREADS) void pick_kernel(MatrixView A, IterArgs P)
{
    constexpr int PICK_WAVES = PICK_THREADS / 64;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *a_col = reinterpret_cast<float *>(smem);
    __shared__ uint64_t s_u64[PICK_WAVES];
    __shared__ double s_red[2][PICK_WAVES];
    __shared__ double s_cscore[PICK_WAVES];
    __shared__ int32_t s_cidx[PICK_WAVES];
    __shared__ int32_t s_cand[PICK_CAND_CAP];
    __shared__ int32_t s_lambda, s_ncand;

    const int32_t r = A.r, r4 = A.r >> 2, k = P.k, it = P.it;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t n = blockIdx.x;
    const int slice = blockIdx.y, nslices = gridDim.y;
    if (slice != 0 && slice * PICK_WAVES >= it)
        return; // no earlier selection falls to this slice
    const OmpWorkspace &W = P.ws;
    const int32_t np = W.tiles_m * 2;
    const uint64_t *part = W.partial + n * np;
    const double *res64 = W.res64 + n * r;

    // (1) float maximum over the tile partials
    uint64_t best = 0;
    for (int32_t e = tid; e < np; e += PICK_THREADS) {
        const uint64_t v = part[e];
        best = v > best ? v : best;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint64_t o = shfl_xor_u64(best, off);
        best = o > best ? o : best;
    }
    if (lane == 0)
        s_u64[wave] = best;
    if (tid == 0)
        s_ncand = 0;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < PICK_WAVES; ++u)
        best = s_u64[u] > best ? s_u64[u] : best;
    const float smax = __uint_as_float((uint32_t)(best >> 32));
    const float thr = smax * (1.0f - RESCORE_TOL);

    // (2) candidates: every kept pair whose float score is within the tolerance of the maximum
    for (int32_t e = tid; e < np; e += PICK_THREADS) {
        const uint64_t v = part[e];
        if (v != 0 && __uint_as_float((uint32_t)(v >> 32)) >= thr) {
            const int32_t slot = atomicAdd(&s_ncand, 1);
            if (slot < PICK_CAND_CAP)
                s_cand[slot] = (int32_t)(0xffffffffu - (uint32_t)v);
        }
    }
    __syncthreads();
    const int32_t ncand = s_ncand;

    // (3) a single candidate is the argmax; several are re-scored in double, one wavefront per
    //     candidate, winner = (score desc, position asc). More candidates than the list holds (an
    //     all-zero residual) are walked straight from the partials.
    double wbest = -1.0;
    int32_t widx = 0x7fffffff;
    if (ncand == 1) {
        wbest = 0.0;
        widx = s_cand[0];
    } else {
        const bool listed = ncand <= PICK_CAND_CAP;
        const int32_t count = listed ? ncand : np;
        for (int32_t e = wave; e < count; e += PICK_WAVES) {
            int32_t i;
            if (listed) {
                i = s_cand[e];
            } else {
                const uint64_t v = part[e];
                if (v == 0 || !(__uint_as_float((uint32_t)(v >> 32)) >= thr))
                    continue;
                i = (int32_t)(0xffffffffu - (uint32_t)v);
            }
            double dot = 0.0, nrm = 0.0;
            for (int32_t jb = lane; jb < r4; jb += 64) {
                const float4 a = column_quad<GENERATED>(A, i, jb);
                const double *rr = res64 + 4 * jb;
                dot += (double)a.x * rr[0] + (double)a.y * rr[1] + (double)a.z * rr[2] + (double)a.w * rr[3];
                nrm += (double)a.x * a.x + (double)a.y * a.y + (double)a.z * a.z + (double)a.w * a.w;
            }
            dot = __shfl(wave_sum(dot), 0, 64);
            nrm = __shfl(wave_sum(nrm), 0, 64);
            const double score = nrm > 0.0 ? fabs(dot) / sqrt(nrm) : 0.0;
            if (score > wbest || (score == wbest && i < widx)) {
                wbest = score;
                widx = i;
            }
        }
    }
    if (lane == 0) {
        s_cscore[wave] = wbest;
        s_cidx[wave] = widx;
    }
    __syncthreads();
    if (tid == 0) {
        double bs = s_cscore[0];
        int32_t bi = s_cidx[0];
        for (int u = 1; u < PICK_WAVES; ++u)
            if (s_cscore[u] > bs || (s_cscore[u] == bs && s_cidx[u] < bi)) {
                bs = s_cscore[u];
                bi = s_cidx[u];
            }
        // no candidate survives only when the scores are not numbers: fall back to the float
        // maximum so that every later access stays inside the matrix
        if (bi < 0 || bi >= A.d)
            bi = (int32_t)(0xffffffffu - (uint32_t)best);
        if (bi < 0 || bi >= A.d)
            bi = 0;
        s_lambda = bi;
    }
    __syncthreads();
    const int32_t lam = s_lambda;
    // with a table of column inner products, w_t = <A_:lambda_t, a> is a gather from its row lambda:
    // requested here, before the column itself is fetched, so that both travel at the same time
    constexpr int GQ = (1024 + PICK_THREADS - 1) / PICK_THREADS; // k <= 1024
    double gram_w[GQ];
    if (A.gram && slice == 0) {
        const double *grow = A.gram + (int64_t)lam * A.d;
        const int32_t *selq = P.sel + n * k;
#pragma unroll
        for (int q = 0; q < GQ; ++q) {
            const int32_t t = tid + q * PICK_THREADS;
            gram_w[q] = t < it ? grow[selq[t]] : 0.0;
        }
    }

    // (3) the new column to LDS; slice 0 stores it and g = ||a||^2, b = <a, y>
    float *cols = W.cols + (n * k) * (int64_t)r;
    {
        double g = 0.0, b = 0.0;
        const float *yy = P.y + n * r;
        for (int32_t jb = tid; jb < r4; jb += PICK_THREADS) {
            const float4 a = column_quad<GENERATED>(A, lam, jb);
            reinterpret_cast<float4 *>(a_col)[jb] = a;
            if (slice == 0) {
                if (!P.At_rows)
                    reinterpret_cast<float4 *>(cols + (int64_t)it * r)[jb] = a;
                const float4 yv = reinterpret_cast<const float4 *>(yy)[jb];
                g += (double)a.x * a.x + (double)a.y * a.y + (double)a.z * a.z + (double)a.w * a.w;
                b += (double)a.x * yv.x + (double)a.y * yv.y + (double)a.z * yv.z + (double)a.w * yv.w;
            }
        }
        if (slice == 0) {
            g = wave_sum(g);
            b = wave_sum(b);
            if (lane == 0) {
                s_red[0][wave] = g;
                s_red[1][wave] = b;
            }
        }
    }
    __syncthreads();
    if (slice == 0 && tid == 0) {
        double g = 0.0, b = 0.0;
        for (int u = 0; u < PICK_WAVES; ++u) {
            g += s_red[0][u];
            b += s_red[1][u];
        }
        W.gb[n * 2] = g;
        W.gb[n * 2 + 1] = b;
        P.sel[n * k + it] = lam;
        W.bitmap[n * W.words + (lam >> 5)] |= 1u << (lam & 31);
    }

    // (4) w_t = <A_:lambda_t, a>: from the table of column inner products if there is one, ...
    double *wv = W.wv + n * k;
    const int32_t *selp = P.sel + n * k;
    if (A.gram) {
        if (slice == 0) {
#pragma unroll
            for (int q = 0; q < GQ; ++q) {
                const int32_t t = tid + q * PICK_THREADS;
                if (t < it)
                    wv[t] = gram_w[q];
            }
        }
        return;
    }
    // ... else one wavefront per earlier selection, two rows in flight
    const int32_t gw = slice * PICK_WAVES + wave, GW = nslices * PICK_WAVES;
    for (int32_t t = gw; t < it; t += 2 * GW) {
        const int32_t t2 = t + GW;
        const bool two = t2 < it;
        const int32_t tb = two ? t2 : t;
        const float4 *c0 = reinterpret_cast<const float4 *>(
            P.At_rows ? P.At_rows + (int64_t)selp[t] * r : cols + (int64_t)t * r);
        const float4 *c1 = reinterpret_cast<const float4 *>(
            P.At_rows ? P.At_rows + (int64_t)selp[tb] * r : cols + (int64_t)tb * r);
        double s0 = 0.0, s1 = 0.0;
        for (int32_t jb = lane; jb < r4; jb += 64) {
            const float4 u0 = c0[jb];
            const float4 u1 = c1[jb];
            const float4 a = reinterpret_cast<const float4 *>(a_col)[jb];
            s0 += (double)u0.x * a.x + (double)u0.y * a.y + (double)u0.z * a.z + (double)u0.w * a.w;
            s1 += (double)u1.x * a.x + (double)u1.y * a.y + (double)u1.z * a.z + (double)u1.w * a.w;
        }
        s0 = wave_sum(s0);
        s1 = wave_sum(s1);
        if (lane == 0) {
            wv[t] = s0;
            if (two)
                wv[t2] = s1;
        }
    }
}

// grid (N, slices); 256 threads (k <= 128) or 1024. dynamic LDS: double w[k]; double fsum[k]; double a[k];
// scratch (the table of shares [wavefronts][k] if it fits, later the partial residuals)
// First the small dense part of App. B in one pass over F: a wavefront takes column t of F (entries
// 0..t, contiguous), forms c_t = <F_:t, w> (coordinate t of the new column in the orthonormal basis
// Q = A_Lambda F) and at once adds c_t F_:t to its share of F c; the shares are then summed in
// wavefront order. Then, in the same workgroup (the dependency is per right-hand side only),
// res = y - A_Lambda x as a column mat-vec in double: a thread owns four measurements; when there are
// fewer such quads than threads, several threads share one and take every G-th column, and their
// parts are added in a fixed order.
// ROWS = rows of F per lane (k <= 64 * ROWS); FLIGHT = columns in flight per wavefront
template <int FACTOR_ROWS, int FLIGHT>
__global__ __launch_bounds__(FACTOR_MAX_THREADS) void update_kernel(IterArgs P, int32_t r)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int32_t k = P.k, it = P.it;
    double *w_s = reinterpret_cast<double *>(smem);
    double *fsum = w_s + k;
    __shared__ double s_red[2][FACTOR_MAX_THREADS / 64];
    __shared__ double s_gamma, s_coef;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nthreads = blockDim.x, nwaves = blockDim.x >> 6;
    const int64_t n = blockIdx.x;
    const OmpWorkspace &W = P.ws;
    double *F = W.F + n * W.f_stride;
    double *avec = W.avec + n * k;
    // several workgroups (slices) may serve one right-hand side: each repeats the factor pass and takes
    // its share of the residual; slice 0 stores the factor and the solution. The solution is
    // double-buffered so that a late slice still reads the previous iteration's values.
    const int slice = blockIdx.y, nslices = gridDim.y;
    const bool writer = slice == 0;
    const double *xs = W.xs + (int64_t)((it + 1) & 1) * W.xs_half + n * k;
    double *xs_new = W.xs + (int64_t)(it & 1) * W.xs_half + n * k;

    // everything the update needs from memory besides F is fetched up front (one latency, not four)
    double *a_s = fsum + k;    // coefficients a_0 .. a_{it-1}
    double *scratch = a_s + k; // shares of F c, later partial residuals
    const double gb_g = W.gb[n * 2], gb_b = W.gb[n * 2 + 1];
    const double x_mine = tid < it ? xs[tid] : 0.0; // row tid of the solution (rows >= nthreads: read late)
    for (int32_t t = tid; t < it; t += nthreads) {
        w_s[t] = W.wv[n * k + t];
        a_s[t] = avec[t];
        fsum[t] = 0.0;
    }
    __syncthreads();
    const int nq = (it + 63) >> 6; // 64-row slabs in use
    double facc[FACTOR_ROWS];
#pragma unroll
    for (int q = 0; q < FACTOR_ROWS; ++q)
        facc[q] = 0.0;
    double cc = 0.0, ca = 0.0; // c.c and c.avec over this wavefront's columns
    for (int32_t t0 = wave; t0 < it; t0 += FLIGHT * nwaves) {
        // FLIGHT columns t0, t0 + nwaves, ... in flight: all loads are issued before any is used
        double v[FLIGHT][FACTOR_ROWS], dt[FLIGHT];
#pragma unroll
        for (int c = 0; c < FLIGHT; ++c) {
            const int32_t t = t0 + c * nwaves;
            const double *f = F + (int64_t)(t < it ? t : t0) * k;
#pragma unroll
            for (int q = 0; q < FACTOR_ROWS; ++q) {
                const int32_t u = q * 64 + lane;
                v[c][q] = (q < nq && t < it && u <= t) ? f[u] : 0.0;
            }
        }
#pragma unroll
        for (int c = 0; c < FLIGHT; ++c) {
            double acc = 0.0;
#pragma unroll
            for (int q = 0; q < FACTOR_ROWS; ++q) {
                const int32_t u = q * 64 + lane;
                acc += v[c][q] * ((q < nq && u < it) ? w_s[u] : 0.0);
            }
            dt[c] = __shfl(wave_sum(acc), 0, 64);
        }
#pragma unroll
        for (int c = 0; c < FLIGHT; ++c) {
            const int32_t t = t0 + c * nwaves;
#pragma unroll
            for (int q = 0; q < FACTOR_ROWS; ++q)
                facc[q] += v[c][q] * dt[c];
            cc += dt[c] * dt[c];
            ca += t < it ? dt[c] * a_s[t] : 0.0;
        }
    }
    if (lane == 0) {
        s_red[0][wave] = cc;
        s_red[1][wave] = ca;
    }
    // F c = sum of the wavefronts' shares, added in wavefront order (deterministic): through a
    // [wavefront][k] table when it fits (one barrier), else one wavefront after the other
    if (P.share_table) {
        double *share = scratch;
#pragma unroll
        for (int q = 0; q < FACTOR_ROWS; ++q) {
            const int32_t u = q * 64 + lane;
            if (q < nq && u < it)
                share[wave * k + u] = facc[q];
        }
        __syncthreads();
        for (int32_t u = tid; u < it; u += nthreads) {
            double a = 0.0;
            for (int wv = 0; wv < nwaves; ++wv)
                a += share[wv * k + u];
            fsum[u] = a;
        }
        __syncthreads();
    } else {
        for (int wv = 0; wv < nwaves; ++wv) {
            if (wave == wv) {
#pragma unroll
                for (int q = 0; q < FACTOR_ROWS; ++q) {
                    const int32_t u = q * 64 + lane;
                    if (q < nq && u < it)
                        fsum[u] += facc[q];
                }
            }
            __syncthreads();
        }
    }
    // gamma = 1/sqrt(g - c.c); new coefficient a_it = gamma (b - c.avec)
    if (tid == 0) {
        double tcc = 0.0, tca = 0.0;
        for (int u = 0; u < nwaves; ++u) {
            tcc += s_red[0][u];
            tca += s_red[1][u];
        }
        const double g = gb_g, b = gb_b;
        const double rem = g - tcc;
        const double gamma = rem > 0.0 ? 1.0 / sqrt(rem) : 0.0;
        const double coef = gamma * (b - tca);
        s_gamma = gamma;
        s_coef = coef;
        if (writer) {
            avec[it] = coef;
            F[(int64_t)it * k + it] = gamma;
        }
    }
    __syncthreads();
    const double gamma = s_gamma, coef = s_coef;
    // new column of F: -gamma F c on rows < it, and x <- [x; 0] + coef * F_:it
    // (w and fsum are dead from here: they become x and the float4 offsets of the selected columns)
    double *x_s = w_s;
    int64_t *row_s = reinterpret_cast<int64_t *>(fsum);
    const int32_t r4 = r >> 2;
    for (int32_t u = tid; u <= it; u += nthreads) {
        double xn;
        if (u < it) {
            const double f = -gamma * fsum[u];
            if (writer)
                F[(int64_t)it * k + u] = f;
            xn = (u == tid ? x_mine : xs[u]) + coef * f;
        } else {
            xn = coef * gamma;
        }
        if (writer) {
            xs_new[u] = xn;
            if (it == k - 1)
                P.x[n * k + u] = (float)xn;
        }
        x_s[u] = xn;
        row_s[u] = (P.At_rows ? (int64_t)P.sel[n * k + u] : (int64_t)u) * r4;
    }
    __syncthreads();

    // ---- residual ----
    const float4 *cbase = P.At_rows ? reinterpret_cast<const float4 *>(P.At_rows)
                                    : reinterpret_cast<const float4 *>(W.cols + (n * k) * (int64_t)r);
    // this slice's quads of measurements: [q0, q0 + nq4)
    const int32_t per = (r4 + nslices - 1) / nslices;
    const int32_t q0 = slice * per;
    const int32_t nq4 = q0 >= r4 ? 0 : (r4 - q0 < per ? r4 - q0 : per);
    const int32_t G = (nq4 > 0 && nq4 < nthreads) ? nthreads / nq4 : 1; // threads sharing one quad
    double *parts = scratch;                                              // [G-1][nq4][4]
    for (int32_t jb0 = 0; jb0 < nq4; jb0 += nthreads) {
        const int32_t jl = G > 1 ? tid % nq4 : jb0 + tid; // quad within the slice
        const int32_t jb = q0 + jl;
        const int32_t g = G > 1 ? tid / nq4 : 0;
        const bool active = jl < nq4 && g < G;
        double e0 = 0.0, e1 = 0.0, e2 = 0.0, e3 = 0.0;
        if (active) {
            if (g == 0) {
                const float4 yv = reinterpret_cast<const float4 *>(P.y + n * r)[jb];
                e0 = yv.x;
                e1 = yv.y;
                e2 = yv.z;
                e3 = yv.w;
            }
            const float4 *cj = cbase + jb;
            int32_t t = g;
            for (; t + 7 * G <= it; t += 8 * G) {
                float4 u[8];
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    u[q] = cj[row_s[t + q * G]];
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const double xt = x_s[t + q * G];
                    e0 -= xt * u[q].x;
                    e1 -= xt * u[q].y;
                    e2 -= xt * u[q].z;
                    e3 -= xt * u[q].w;
                }
            }
            for (; t <= it; t += G) {
                const float4 u = cj[row_s[t]];
                const double xt = x_s[t];
                e0 -= xt * u.x;
                e1 -= xt * u.y;
                e2 -= xt * u.z;
                e3 -= xt * u.w;
            }
        }
        if (G > 1) {
            if (active && g > 0) {
                double *o = parts + ((int64_t)(g - 1) * nq4 + jl) * 4;
                o[0] = e0;
                o[1] = e1;
                o[2] = e2;
                o[3] = e3;
            }
            __syncthreads();
            if (active && g == 0) {
                for (int32_t gg = 1; gg < G; ++gg) {
                    const double *o = parts + ((int64_t)(gg - 1) * nq4 + jl) * 4;
                    e0 += o[0];
                    e1 += o[1];
                    e2 += o[2];
                    e3 += o[3];
                }
            }
        }
        if (active && g == 0) {
            double *ro = W.res64 + n * r + 4 * jb;
            ro[0] = e0;
            ro[1] = e1;
            ro[2] = e2;
            ro[3] = e3;
            if (P.res_split) {
                uint16_t h[4], l[4];
                split_bf16_1((float)e0, h[0], l[0]);
                split_bf16_1((float)e1, h[1], l[1]);
                split_bf16_1((float)e2, h[2], l[2]);
                split_bf16_1((float)e3, h[3], l[3]);
                unsigned char *o = reinterpret_cast<unsigned char *>(W.res16) + n * ((int64_t)r * 4) + split32_quad_offset(jb);
                *reinterpret_cast<uint2 *>(o) = make_uint2(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16));
                *reinterpret_cast<uint2 *>(o + 64) = make_uint2(l[0] | ((uint32_t)l[1] << 16), l[2] | ((uint32_t)l[3] << 16));
            } else {
                reinterpret_cast<float4 *>(W.res32 + n * r)[jb] =
                    make_float4((float)e0, (float)e1, (float)e2, (float)e3);
            }
        }
    }
}

// Least-squares fit of a second right-hand side on the support already found (shared-support
// recovery): z = (A_L^T A_L)^-1 A_L^T y_fit = F (F^T (A_L^T y_fit)) with the finished inverse
// Cholesky factor F of the support (App. B), all in double. grid N; dynamic LDS: double b[k], u[k]
constexpr int REFIT_THREADS = 1024;
__global__ __launch_bounds__(REFIT_THREADS) void refit_kernel(IterArgs P, const float *__restrict__ y_fit,
                                                              float *__restrict__ z, int32_t r)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    double *b_s = reinterpret_cast<double *>(smem);
    double *u_s = b_s + P.k;
    const int32_t k = P.k, r4 = r >> 2;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int NW = REFIT_THREADS / 64;
    const int64_t n = blockIdx.x;
    const OmpWorkspace &W = P.ws;
    const int32_t *selp = P.sel + n * k;
    const float *cols = W.cols + (n * k) * (int64_t)r;
    const float4 *yy = reinterpret_cast<const float4 *>(y_fit + n * r);
    // b_t = <A_:lambda_t, y_fit>, one wavefront per selected column
    for (int32_t t = wave; t < k; t += NW) {
        const float4 *c = reinterpret_cast<const float4 *>(
            P.At_rows ? P.At_rows + (int64_t)selp[t] * r : cols + (int64_t)t * r);
        double acc = 0.0;
        for (int32_t jb = lane; jb < r4; jb += 64) {
            const float4 a = c[jb];
            const float4 yv = yy[jb];
            acc += (double)a.x * yv.x + (double)a.y * yv.y + (double)a.z * yv.z + (double)a.w * yv.w;
        }
        acc = wave_sum(acc);
        if (lane == 0)
            b_s[t] = acc;
    }
    __syncthreads();
    // u = F^T b: column t of F (rows 0..t, contiguous) against b
    const double *F = W.F + n * W.f_stride;
    for (int32_t t = wave; t < k; t += NW) {
        const double *f = F + (int64_t)t * k;
        double acc = 0.0;
        for (int32_t v = lane; v <= t; v += 64)
            acc += f[v] * b_s[v];
        acc = wave_sum(acc);
        if (lane == 0)
            u_s[t] = acc;
    }
    __syncthreads();
    // z = F u: row v of F holds the entries of columns t >= v
    for (int32_t v = tid; v < k; v += REFIT_THREADS) {
        double acc = 0.0;
        for (int32_t t = v; t < k; ++t)
            acc += F[(int64_t)t * k + v] * u_s[t];
        z[n * k + v] = (float)acc;
    }
}

// ---------------------------------------------------------------------------------------------
// Host side of the recovery.
struct OmpPlan {
    bool panels;     // generated A produced into ws.panel and consumed from there
    bool pipelined;  // full tiles of stored rows: corr_pipelined_kernel
    bool screen;     // resident rows that fit ws.a16 and the matrix asks for it: corr_split_kernel, or
    bool screen_pipelined; // on full tiles the bfloat16 form of corr_pipelined_kernel
    int32_t tiles_m; // position tiles of the contraction in use (stride of ws.partial)
    MatrixView Apick; // the view pick_kernel fetches columns from
    size_t pick_smem, factor_smem;
    bool factor_share_table; // update_kernel sums its wavefronts' shares through an LDS table
};

// the workspace as seen by the right-hand sides [n0, ...): every per-right-hand-side array shifted
static OmpWorkspace shift_workspace(const OmpWorkspace &ws, int32_t n0, int32_t r, int32_t k, int32_t tiles_m)
{
    OmpWorkspace w = ws;
    w.tiles_m = tiles_m;
    w.res64 += (int64_t)n0 * r;
    w.F += (int64_t)n0 * ws.f_stride;
    w.avec += (int64_t)n0 * k;
    w.xs += (int64_t)n0 * k;
    w.res32 += (int64_t)n0 * r;
    w.res16 += (int64_t)n0 * 2 * r;
    w.cols += (int64_t)n0 * k * r;
    w.partial += (int64_t)n0 * tiles_m * 2;
    w.bitmap += (int64_t)n0 * ws.words;
    w.wv += (int64_t)n0 * k;
    w.gb += (int64_t)n0 * 2;
    return w;
}

// One iteration for Ng right-hand sides whose arrays start at y / sel / x / w, enqueued on s:
// the contraction ...
static hipError_t omp_contraction(const OmpPlan &pl, const MatrixView &A, int32_t Ng, const OmpWorkspace &w,
                                  hipStream_t s)
{
    ProfileScope prof(KC_CORR, s);
    hipError_t e = hipSuccess;
    if (pl.panels) {
        for (int32_t p0 = 0; p0 < A.d && e == hipSuccess; p0 += w.panel_rows) {
            const int32_t rows = A.d - p0 < w.panel_rows ? A.d - p0 : w.panel_rows;
            if (w.panel_rows < A.d) { // a matrix larger than the panel is refilled panel by panel
                e = launch_matrix_fill(A.key0, A.key1, A.scale, A.r, p0, rows, w.panel, s, KC_FILL);
                if (e != hipSuccess)
                    break;
            }
            MatrixView Ap = A;
            Ap.generated = 0;
            Ap.At = w.panel;
            Ap.row0 = p0;
            if (pl.screen) {
                // a whole-matrix panel was split once per call; a refilled panel is split after each fill
                const bool whole = w.panel_rows >= A.d;
                if (!whole)
                    launch_split_rows(w.panel, rows, A.r, w.a16, s);
                e = corr_screen_launch(pl.screen_pipelined, Ap, w.a16, rows, Ng, w, pl.tiles_m, s);
            } else {
                e = pl.pipelined ? corr_pipelined_launch(Ap, rows, w.res32, Ng, w, pl.tiles_m, s)
                                 : corr_dispatch<false>(Ap, rows, w.res32, Ng, w, pl.tiles_m, s);
            }
        }
    } else if (A.generated) {
        e = corr_dispatch<true>(A, A.d, w.res32, Ng, w, pl.tiles_m, s);
    } else {
        e = pl.screen      ? corr_screen_launch(pl.screen_pipelined, A, w.a16, A.d, Ng, w, pl.tiles_m, s)
            : pl.pipelined ? corr_pipelined_launch(A, A.d, w.res32, Ng, w, pl.tiles_m, s)
                           : corr_dispatch<false>(A, A.d, w.res32, Ng, w, pl.tiles_m, s);
    }
    return e;
}

// ... then the selection and the least-squares update
static void omp_select_update(const OmpPlan &pl, const MatrixView &A, const float *y, int32_t Ng, int32_t k,
                              int32_t it, int32_t *sel, float *x, const OmpWorkspace &w, hipStream_t s)
{
    ProfileScope prof(KC_SELECT, s);
    // short columns: two wavefronts per right-hand side keep their lanes busy and let sixteen workgroups
    // share a CU, which hides the chain of dependent loads this kernel consists of
    const bool narrow = A.r <= 512 && k <= 128;
    int slices = 2048 / Ng;
    slices = slices < 1 ? 1 : (slices > 8 ? 8 : slices);
    if (pl.Apick.gram)
        slices = 1; // no pass over the selected columns to spread
    const dim3 pgrid((unsigned)Ng, (unsigned)slices);
    IterArgs P{y, k, it, sel, x, w, pl.Apick.generated ? nullptr : pl.Apick.At, pl.factor_share_table ? 1 : 0,
               pl.screen ? 1 : 0};
    if (narrow) {
        if (pl.Apick.generated)
            pick_kernel<true, PICK_THREADS_NARROW><<<pgrid, PICK_THREADS_NARROW, pl.pick_smem, s>>>(pl.Apick, P);
        else
            pick_kernel<false, PICK_THREADS_NARROW><<<pgrid, PICK_THREADS_NARROW, pl.pick_smem, s>>>(pl.Apick, P);
    } else {
        if (pl.Apick.generated)
            pick_kernel<true, PICK_THREADS_WIDE><<<pgrid, PICK_THREADS_WIDE, pl.pick_smem, s>>>(pl.Apick, P);
        else
            pick_kernel<false, PICK_THREADS_WIDE><<<pgrid, PICK_THREADS_WIDE, pl.pick_smem, s>>>(pl.Apick, P);
    }
    // One workgroup per right-hand side, two when there are so few that half the chip would idle
    // (each repeats the factor pass and takes half of the residual). More slices were measured
    // slower: the repeated passes over F cost more than the wider residual pass saves.
    const dim3 ugrid((unsigned)Ng, Ng <= 128 ? 2u : 1u);
    if (k <= 128)
        update_kernel<2, 4><<<ugrid, 256, pl.factor_smem, s>>>(P, A.r);
    else if (k <= 256)
        update_kernel<4, 6><<<ugrid, FACTOR_MAX_THREADS, pl.factor_smem, s>>>(P, A.r);
    else
        update_kernel<16, 1><<<ugrid, FACTOR_MAX_THREADS, pl.factor_smem, s>>>(P, A.r);
}

// A second stream (default priority) and two events per device, created on first use, so that the
// two halves of a large batch can run their iterations side by side: while one half is in its
// memory-bound selection / update kernels the other half's contraction keeps the matrix cores busy.
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    bool ok = false, tried = false;
};
static SideStream *side_stream()
{
    static SideStream per_device[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
        return nullptr;
    SideStream &ss = per_device[dev];
    if (!ss.tried) {
        ss.tried = true;
        ss.ok = hipStreamCreateWithFlags(&ss.stream, hipStreamNonBlocking) == hipSuccess &&
                hipEventCreateWithFlags(&ss.fork, hipEventDisableTiming) == hipSuccess &&
                hipEventCreateWithFlags(&ss.join, hipEventDisableTiming) == hipSuccess;
    }
    return ss.ok ? &ss : nullptr;
}

static hipError_t omp_iterations(const OmpPlan &pl, bool whole_matrix_panel, const float *y, int32_t N,
                                 const MatrixView &A, int32_t k, int32_t *sel, float *x, const OmpWorkspace &ws,
                                 hipStream_t s);

hipError_t launch_omp(const float *y, int32_t N, const MatrixView &A, int32_t k, int32_t *sel, float *x,
                      const OmpWorkspace &ws, hipStream_t s, const float *y_fit, float *z)
{
    // A generated matrix is written out once per call when the workspace has room for all of it. One
    // that does not fit is regenerated inside the contraction when few right-hand-side tiles share it;
    // with many tiles (each would regenerate all of A) it is produced panel by panel into a cache-sized
    // scratch in every iteration, and consumed from there.
    // Stored rows in full tiles take the pipelined kernel (256-row tiles), everything else the
    // general one (128-row tiles).
    OmpPlan pl{};
    pl.panels = A.generated && (ws.panel_rows >= A.d || (N + CORR_BN - 1) / CORR_BN >= 4);
    pl.pipelined = (!A.generated || pl.panels) && corr_pipelined_ok(A, N, ws.panel_rows);
    // the bfloat16 screening contraction needs resident rows; a matrix regenerated inside the
    // contraction keeps the float kernel (its time is the generator's anyway)
    pl.screen = (A.flags & SGC_MATRIX_FLAG_SCREEN_BF16) && A.r % 32 == 0 &&
                (A.generated ? pl.panels && ws.a16_rows >= (ws.panel_rows < A.d ? ws.panel_rows : A.d)
                             : ws.a16_rows >= A.d);
    pl.screen_pipelined = pl.screen && N > 64 && corr_pipelined_ok(A, N, ws.panel_rows);
    if (pl.screen)
        pl.pipelined = false;
    pl.tiles_m = pl.pipelined || pl.screen_pipelined ? A.d / CORRP_BM : corr_tiles_m(A.d);
    pl.pick_smem = ((size_t)A.r * 4 + 15) & ~(size_t)15;
    pl.factor_smem = 3 * sizeof(double) * (size_t)k;
    {
        const size_t threads = k <= 128 ? 256 : FACTOR_MAX_THREADS;
        const size_t table = sizeof(double) * (size_t)k * (threads / 64); // one row per wavefront
        const size_t parts = threads * 4 * sizeof(double); // partial residuals of threads sharing a quad
        pl.factor_share_table = pl.factor_smem + table <= 48 * 1024;
        const size_t scratch = pl.factor_share_table && table > parts ? table : parts;
        pl.factor_smem += scratch;
    }
    {
        ProfileScope prof(KC_OTHER, s);
        omp_init_kernel<<<dim3((unsigned)N), 256, 0, s>>>(y, A.r, ws.words, ws.res64, ws.res32, ws.bitmap,
                                                          pl.screen ? 1 : 0);
    }
    pl.Apick = A;
    const bool whole_matrix_panel = pl.panels && ws.panel_rows >= A.d;
    if (whole_matrix_panel) {
        hipError_t e = launch_matrix_fill(A.key0, A.key1, A.scale, A.r, 0, A.d, ws.panel, s, KC_FILL);
        if (e != hipSuccess)
            return e;
        pl.Apick.generated = 0;
        pl.Apick.At = ws.panel;
    }
    // screening contraction: the rows of At as bfloat16 planes, once per call where they fit
    if (pl.screen && (!A.generated || whole_matrix_panel)) {
        ProfileScope prof(KC_FILL, s);
        launch_split_rows(whole_matrix_panel ? ws.panel : A.At, A.d, A.r, ws.a16, s);
    }
    hipError_t e = omp_iterations(pl, whole_matrix_panel, y, N, A, k, sel, x, ws, s);
    if (e != hipSuccess || !y_fit)
        return e;
    {
        ProfileScope prof(KC_SELECT, s);
        const OmpWorkspace w = shift_workspace(ws, 0, A.r, k, pl.tiles_m);
        IterArgs P{y, k, k, sel, x, w, pl.Apick.generated ? nullptr : pl.Apick.At, 0, 0};
        refit_kernel<<<dim3((unsigned)N), REFIT_THREADS, 2 * sizeof(double) * (size_t)k, s>>>(P, y_fit, z, A.r);
    }
    return hipGetLastError();
}

static hipError_t omp_iterations(const OmpPlan &pl, bool whole_matrix_panel, const float *y, int32_t N,
                                 const MatrixView &A, int32_t k, int32_t *sel, float *x, const OmpWorkspace &ws,
                                 hipStream_t s)
{
    // two halves side by side when the batch is large (not while kernels are being timed one by one,
    // and not when both halves would have to share a panel that is refilled inside the iterations)
    const int32_t N0 = (N / 2 + CORR_BN - 1) / CORR_BN * CORR_BN;
    SideStream *ss = nullptr;
    if (N >= 4 * CORR_BN && N0 < N && !g_profile_on && !(pl.panels && !whole_matrix_panel))
        ss = side_stream();
    if (!ss) {
        const OmpWorkspace w = shift_workspace(ws, 0, A.r, k, pl.tiles_m);
        for (int32_t it = 0; it < k; ++it) {
            hipError_t e = omp_contraction(pl, A, N, w, s);
            if (e != hipSuccess)
                return e;
            omp_select_update(pl, A, y, N, k, it, sel, x, w, s);
        }
        return hipGetLastError();
    }
    const OmpWorkspace w0 = shift_workspace(ws, 0, A.r, k, pl.tiles_m);
    const OmpWorkspace w1 = shift_workspace(ws, N0, A.r, k, pl.tiles_m);
    if (hipEventRecord(ss->fork, s) != hipSuccess || hipStreamWaitEvent(ss->stream, ss->fork, 0) != hipSuccess)
        return hipErrorUnknown;
    hipError_t e = hipSuccess;
    for (int32_t it = 0; it < k && e == hipSuccess; ++it) {
        e = omp_contraction(pl, A, N0, w0, s);
        if (e != hipSuccess)
            break;
        omp_select_update(pl, A, y, N0, k, it, sel, x, w0, s);
        e = omp_contraction(pl, A, N - N0, w1, ss->stream);
        if (e != hipSuccess)
            break;
        omp_select_update(pl, A, y + (int64_t)N0 * A.r, N - N0, k, it, sel + (int64_t)N0 * k, x + (int64_t)N0 * k, w1,
                          ss->stream);
    }
    // join even after a failed launch so that the caller's stream never runs ahead of the side stream
    if (hipEventRecord(ss->join, ss->stream) != hipSuccess || hipStreamWaitEvent(s, ss->join, 0) != hipSuccess)
        return hipErrorUnknown;
    return e != hipSuccess ? e : hipGetLastError();
}

} // namespace sgc
