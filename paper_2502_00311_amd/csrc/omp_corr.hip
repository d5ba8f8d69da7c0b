// The correlation contraction of the batched recovery, P = At * R for all right-hand sides at once with a
// fused scale / mask / two-best epilogue (paper Sec. 4.3 eq. 9, selection rule of App. B): the general
// kernel, the hand-pipelined kernel for full tiles of resident rows (float, and its bfloat16 form), and the
// bfloat16 screening kernel on split operands. See omp.hip for the iteration around it.
#include <type_traits>

#include "omp_internal.h"
#include "philox_normal.h"

namespace sgc {

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

void launch_split_rows(const float *src, int64_t rows, int32_t r, uint16_t *dst, hipStream_t s)
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
    const hipError_t e = raise_dynamic_lds(reinterpret_cast<const void *>(corr_split_kernel), smem);
    if (e != hipSuccess)
        return e;
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
    const hipError_t e = raise_dynamic_lds(reinterpret_cast<const void *>(kern), smem);
    if (e != hipSuccess)
        return e;
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


// NB = 2: the 256 x 128 tile described above. NB = 1: a 256 x 64 tile for at most 64 right-hand sides
// (each wavefront 128 x 32, groups of 16 MFMAs; the LDS write and the global load of a staging piece
// follow the same MFMA of group 2, so the load still leads its use by a whole stage).
// BF16: the screening variant. At and R point to rows in split32 format (see corr_split_kernel: the same
// 4 r bytes per row, a depth-32 stage of a row is 32 high parts then 32 low parts), so the data movement is
// the float kernel's; a stage is two groups (16 depths each) of 3 * 8 MFMAs v_mfma_f32_32x32x16_bf16
// (low*high, high*low, high*high per block), and because a stage is five times shorter the global loads
// run three stages ahead through two sets of staging registers.
// PERSIST (float only): gridDim.x workgroups share total_tiles tiles (measured on 12352 tiles: 5.93 -> 5.87 ms per launch).
template <int NB, bool BF16, bool PERSIST>
__global__ __launch_bounds__(256, 1) void corr_pipelined_kernel(MatrixView A, const float *__restrict__ R, int32_t N,
                                                                const uint32_t *__restrict__ bitmap, int32_t words,
                                                                uint64_t *__restrict__ partial, int32_t tiles_m,
                                                                int32_t tiles_x, int32_t total_tiles)
{
    constexpr int BM = CORRP_BM, BN = 64 * NB, BK = 32, LD = BK + 4, MB = 4;
    constexpr int WN = 32 * NB;            // right-hand sides per wavefront
    constexpr int GM = 4 * MB * NB;        // MFMAs per group (8 depths)
    constexpr int LA = 8, LB = 2 * NB;     // 16-byte pieces per thread per stage
    typedef float floatx4 __attribute__((ext_vector_type(4)));
    extern __shared__ __attribute__((aligned(16))) float corr_lds[];
    float *lds = corr_lds; // A stages [2][BM*LD], then R stages [2][BN*LD], then what the epilogue needs, twice
    // (a workgroup that takes several tiles fetches the next tile's while it scans the current one's):
    constexpr int COPIES = PERSIST ? 2 : 1; // PERSIST: the workgroup goes on to further tiles
    float *inv_s = corr_lds + 2 * (BM + BN) * LD;                            // [COPIES][BM] reciprocal norms of the positions
    uint32_t *msk_s = reinterpret_cast<uint32_t *>(inv_s + COPIES * BM);     // [COPIES][BN][BM/32] selection words
    // [COPIES][2][BN][2] keys of the two halves of the tile; with one tile per workgroup they go where the stages were
    uint64_t *red = PERSIST ? reinterpret_cast<uint64_t *>(msk_s + COPIES * BN * (BM / 32)) : reinterpret_cast<uint64_t *>(corr_lds);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int32_t r = A.r;
    const int l32 = lane & 31, lhalf = lane >> 5;
    const uint32_t lane_off = (uint32_t)((tid >> 3) * r + ((tid & 7) << 2));
    const int ldst0 = (tid >> 3) * LD + ((tid & 7) << 2);
    const int nkb = r / BK;
    // The tiles of this workgroup: blockIdx.x, blockIdx.x + gridDim.x, ... (tile t = block row t % tiles_x of At,
    // block t / tiles_x of right-hand sides). With one tile per workgroup the loop below runs once. PERSIST: the
    // float kernel launched with a workgroup per CU; the depth loop then simply runs on across the tile
    // boundary - the last two stages of a tile load the first two of the next, so a new tile starts without
    // waiting for memory, and only the scan of the finished tile lies between two tiles' matrix instructions.
    struct Tile {
        int32_t m0, n0;     // first position, first right-hand side
        const float *abase; // its rows of At
        const float *bbase; // its right-hand sides
        uint32_t rhs_off[LB]; // right-hand sides past the end of a ragged last tile re-read the last one
    };
    auto set_tile = [&](Tile &c, int32_t t) {
        const int32_t bx = t % tiles_x, by = t / tiles_x;
        c.m0 = A.row0 + bx * BM;
        c.n0 = by * BN;
        c.abase = A.At + (int64_t)(bx * BM) * r;
        c.bbase = R + (int64_t)c.n0 * r;
#pragma unroll
        for (int u = 0; u < LB; ++u) {
            const int32_t n = c.n0 + 32 * u + (tid >> 3);
            c.rhs_off[u] = (uint32_t)(((n < N ? n : N - 1) - c.n0) * r + ((tid & 7) << 2));
        }
    };
    int32_t tile = blockIdx.x;
    Tile cur, nxt;
    set_tile(cur, tile);

    constexpr bool WIDE = BF16 && NB == 4;   // 128 x 128 outputs per wavefront: one staging set fits
    constexpr int GS = BF16 && !WIDE ? 2 : 1; // staging register sets
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

    auto gload_of = [&](const Tile &c, int u, int kb, int set) { // staging piece u of stage kb of tile c (the last stage again beyond the end)
        const int kk = (kb < nkb ? kb : nkb - 1) * BK;
        if (u < LA)
            g[set][u] = *reinterpret_cast<const floatx4 *>(c.abase + ((int64_t)(32 * u) * r + kk) + lane_off);
        else
            g[set][u] = *reinterpret_cast<const floatx4 *>(c.bbase + kk + c.rhs_off[u < LA ? 0 : u - LA]);
    };
    auto gload = [&](int u, int kb, int set = 0) { gload_of(cur, u, kb, set); };
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
        const float nv = A.inv_colnorm[cur.m0 + tid];
        uint32_t mw[BN * (BM / 32) / 256];
#pragma unroll
        for (int u = 0; u < BN * (BM / 32) / 256; ++u) {
            const int e = tid + 256 * u;
            const int32_t n = cur.n0 + (e >> 3);
            mw[u] = bitmap[(int64_t)(n < N ? n : N - 1) * words + (cur.m0 >> 5) + (e & 7)];
        }
        inv_s[tid] = nv;
#pragma unroll
        for (int u = 0; u < BN * (BM / 32) / 256; ++u)
            msk_s[tid + 256 * u] = mw[u];
    }
    static_for<0, LA + LB>([&](auto uc) { lwrite(decltype(uc)::value, 0); });
    static_for<0, LA + LB>([&](auto uc) { gload(decltype(uc)::value, 1, GS - 1); });
    if constexpr (WIDE) { // both LDS buffers filled, stage 2 in the staging registers
        static_for<0, LA + LB>([&](auto uc) { lwrite(decltype(uc)::value, 1); });
        static_for<0, LA + LB>([&](auto uc) { gload(decltype(uc)::value, 2); });
    } else if constexpr (BF16) {
        static_for<0, LA + LB>([&](auto uc) { gload(decltype(uc)::value, 2, 0); });
    }
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
    // WIDE stage kb: the other LDS buffer already holds stage kb + 1 and the one staging set stage kb + 2.
    // Group 0 reads the fragments of group 1; barrier, after which nobody reads this stage's buffer
    // again; group 1 reads the first fragments of stage kb + 1, copies the staging set into this stage's
    // buffer and refills it with stage kb + 3, which then has a whole stage to arrive.
    auto stage_wide = [&](int kb, auto bufc) {
        constexpr int buf = decltype(bufc)::value;
        constexpr int G3 = 3 * MB * NB;
        static_for<0, G3>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            mfma(0, m);
            if constexpr (m < MB + NB)
                fread(1, m, buf, 1);
            __builtin_amdgcn_sched_barrier(0);
        });
        __syncthreads();
        static_for<0, G3>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            mfma(1, m);
            if constexpr (m < MB + NB)
                fread(0, m, buf ^ 1, 0);
            else if constexpr (m < MB + NB + LA + LB)
                lwrite(m - (MB + NB), buf);
            else if constexpr (m < MB + NB + 2 * (LA + LB))
                gload(m - (MB + NB + LA + LB), kb + 3);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    // NEXT: the stage two ahead belongs to the workgroup's next tile (the last two stages of a tile)
    auto stage = [&](int kb, auto bufc, auto nextc) {
        constexpr int buf = decltype(bufc)::value;
        constexpr bool NEXT = decltype(nextc)::value;
        auto gahead = [&](int u) {
            if constexpr (NEXT)
                gload_of(nxt, u, kb + 2 - nkb, 0);
            else
                gload_of(cur, u, kb + 2, 0);
        };
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
                    gahead(m - 20);
            } else if constexpr (m < MB + NB + LA + LB) {
                lwrite(m - (MB + NB), buf ^ 1);
                gahead(m - (MB + NB));
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
    int half = 0; // which copy of inv_s / msk_s / red the current tile uses
    while (true) {
    const int32_t tile_next = tile + (int32_t)gridDim.x;
    const bool more = PERSIST && tile_next < total_tiles;
    if constexpr (PERSIST)
        set_tile(nxt, more ? tile_next : tile); // after the last tile its own first stages are loaded again, unused
    if constexpr (BF16) {
        for (int kb = 0; kb < nkb; kb += 2) {
            if constexpr (WIDE) {
                stage_wide(kb, std::integral_constant<int, 0>{});
                stage_wide(kb + 1, std::integral_constant<int, 1>{});
            } else {
                stage_bf16(kb, std::integral_constant<int, 0>{});
                stage_bf16(kb + 1, std::integral_constant<int, 1>{});
            }
        }
    } else if constexpr (PERSIST) {
        for (int kb = 0; kb < nkb - 2; kb += 2) {
            stage(kb, std::integral_constant<int, 0>{}, std::false_type{});
            stage(kb + 1, std::integral_constant<int, 1>{}, std::false_type{});
        }
        stage(nkb - 2, std::integral_constant<int, 0>{}, std::true_type{});
        stage(nkb - 1, std::integral_constant<int, 1>{}, std::true_type{});
    } else {
        for (int kb = 0; kb < nkb; kb += 2) {
            stage(kb, std::integral_constant<int, 0>{}, std::false_type{});
            stage(kb + 1, std::integral_constant<int, 1>{}, std::false_type{});
        }
    }
    __syncthreads();
    // the next tile's reciprocal norms and selection words: requested now, stored after the scan of this tile
    float nv_next = 0.f;
    uint32_t mw_next[BN * (BM / 32) / 256];
    if (more) {
        nv_next = A.inv_colnorm[nxt.m0 + tid];
#pragma unroll
        for (int u = 0; u < BN * (BM / 32) / 256; ++u) {
            const int e = tid + 256 * u;
            const int32_t n = nxt.n0 + (e >> 3);
            mw_next[u] = bitmap[(int64_t)(n < N ? n : N - 1) * words + (nxt.m0 >> 5) + (e & 7)];
        }
    }
    const int32_t m0 = cur.m0, n0 = cur.n0;
    const float *inv_h = inv_s + half * BM;
    const uint32_t *msk_h = msk_s + half * BN * (BM / 32);
    uint64_t *red_h = red + half * BN * 4;

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
    uint32_t best[NB], second[NB], msk[MB][NB];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
            msk[a][b] = msk_h[(wn * WN + b * 32 + l32) * (BM / 32) + wm * 4 + a];
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
                inv[qd] = *reinterpret_cast<const float4 *>(inv_h + wm * 128 + a * 32 + 8 * qd + 4 * lhalf);
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
            red_h[(wm * BN + nl) * 2 + 0] = wb;
            red_h[(wm * BN + nl) * 2 + 1] = ws2;
        }
    }
    __syncthreads();
    if (tid < BN && n0 + tid < N) {
        const int32_t n = n0 + tid;
        uint64_t b0 = red_h[tid * 2], s0 = red_h[tid * 2 + 1];
        top2_insert(red_h[(BN + tid) * 2], b0, s0);
        top2_insert(red_h[(BN + tid) * 2 + 1], b0, s0);
        uint64_t *o = partial + ((int64_t)n * tiles_m + m0 / BM) * 2;
        o[0] = b0;
        o[1] = s0;
    }
    if (!more)
        break;
    // on to the next tile: its first stage already lies in LDS, its second in the staging registers, and the
    // fragments of its first group were read at the end of the last stage
    half ^= 1;
    inv_s[half * BM + tid] = nv_next;
#pragma unroll
    for (int u = 0; u < BN * (BM / 32) / 256; ++u)
        msk_s[half * BN * (BM / 32) + tid + 256 * u] = mw_next[u];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                acc[a][b][v] = 0.f;
    cur = nxt;
    tile = tile_next;
    } // tiles of this workgroup
}

static int corr_cu_count()
{
    static int count[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
        return 0;
    if (count[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = -1;
        count[dev] = n;
    }
    return count[dev] > 0 ? count[dev] : 0;
}

template <int NB, bool BF16 = false>
static hipError_t corr_pipelined_launch_nb(const MatrixView &A, int32_t rows, const float *R, int32_t N,
                                           const OmpWorkspace &ws, int32_t tiles_m, hipStream_t s)
{
    constexpr int BN = 64 * NB;
    const int32_t tiles_x = rows / CORRP_BM, tiles_y = (N + BN - 1) / BN;
    const int64_t total = (int64_t)tiles_x * tiles_y;
    if (total > 0x7fffffff) // tile numbers are 32-bit (a launch of that size would run for days)
        return hipErrorInvalidValue;
    // The float kernel with more tiles than CUs: one workgroup per CU (all that fits anyway), each walking its share
    // of the tiles without a pause between them. Otherwise (and for the bfloat16 variants) a workgroup per tile.
    const int cus = BF16 ? 0 : corr_cu_count();
    if constexpr (!BF16) if (cus > 0 && total > cus) {
        constexpr size_t smem = (size_t)2 * (CORRP_BM + BN) * 36 * sizeof(float) + 2 * CORRP_BM * sizeof(float) +
                                (size_t)2 * BN * (CORRP_BM / 32) * sizeof(uint32_t) + (size_t)2 * BN * 4 * sizeof(uint64_t);
        const hipError_t e = raise_dynamic_lds(reinterpret_cast<const void *>(corr_pipelined_kernel<NB, BF16, true>), smem);
        if (e != hipSuccess)
            return e;
        corr_pipelined_kernel<NB, BF16, true><<<dim3((unsigned)cus), 256, smem, s>>>(A, R, N, ws.bitmap, ws.words, ws.partial,
                                                                                    tiles_m, tiles_x, (int32_t)total);
        return hipSuccess;
    }
    constexpr size_t smem = (size_t)2 * (CORRP_BM + BN) * 36 * sizeof(float) + CORRP_BM * sizeof(float) +
                            (size_t)BN * (CORRP_BM / 32) * sizeof(uint32_t);
    const hipError_t e = raise_dynamic_lds(reinterpret_cast<const void *>(corr_pipelined_kernel<NB, BF16, false>), smem);
    if (e != hipSuccess)
        return e;
    corr_pipelined_kernel<NB, BF16, false><<<dim3((unsigned)total), 256, smem, s>>>(A, R, N, ws.bitmap, ws.words, ws.partial,
                                                                                   tiles_m, tiles_x, (int32_t)total);
    return hipSuccess;
}

hipError_t corr_pipelined_launch(const MatrixView &A, int32_t rows, const float *R, int32_t N,
                                        const OmpWorkspace &ws, int32_t tiles_m, hipStream_t s)
{
    if (N <= 64)
        return corr_pipelined_launch_nb<1>(A, rows, R, N, ws, tiles_m, s);
    return corr_pipelined_launch_nb<2>(A, rows, R, N, ws, tiles_m, s);
}

// the split rows through the pipelined kernel: its data movement reads them as rows of r floats
hipError_t corr_screen_launch(bool pipelined, const MatrixView &A, const uint16_t *rows_split, int32_t rows,
                                     int32_t N, const OmpWorkspace &ws, int32_t tiles_m, hipStream_t s)
{
    if (!pipelined)
        return corr_split_launch(A, rows_split, rows, N, ws, tiles_m, s);
    MatrixView As = A;
    As.At = reinterpret_cast<const float *>(rows_split);
    const float *R = reinterpret_cast<const float *>(ws.res16);
    // 256 right-hand sides per workgroup (128 x 128 outputs per wavefront: a third less LDS traffic per
    // matrix-core instruction) once that still gives every CU a workgroup and wastes little on a ragged tile
    if (N >= 1024 && (int64_t)(rows / CORRP_BM) * ((N + 255) / 256) >= 256)
        return corr_pipelined_launch_nb<4, true>(As, rows, R, N, ws, tiles_m, s);
    return corr_pipelined_launch_nb<2, true>(As, rows, R, N, ws, tiles_m, s);
}

// whether the pipelined kernel covers this problem (full tiles of positions, stored rows, even number
// of stages; the last tile of right-hand sides may be ragged)
bool corr_pipelined_ok(const MatrixView &A, int32_t N, int32_t panel_rows)
{
    // fewer than 128 workgroups of 256 positions: the general kernel's smaller tiles give several times
    // the workgroups, which matters more than the schedule when the chip is far from full
    const int64_t rhs_tiles = N <= 64 ? 1 : (N + CORR_BN - 1) / CORR_BN;
    if ((int64_t)(A.d / CORRP_BM) * rhs_tiles < 128)
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
    // a matrix generated in the kernel: every tile of right-hand sides regenerates its 128 x r slice of A, so
    // the generator's vector-ALU time per flop falls with the tile's width: 256 right-hand sides per
    // workgroup halve it against the 128-wide tile. Float MFMAs and vector-ALU instructions of a SIMD do not
    // overlap on this chip (sgc_probe: their times add exactly), so the generator's time comes on top of the
    // matrix-core time whatever the schedule; sixteen wavefronts of 32 x 64 outputs (four per SIMD) hide
    // everything else - LDS reads, barriers, the loads of R - behind one another: measured at d = 262144,
    // r = 8192, N = 256: 9.9 ms per launch = 111 TFLOP/s, against 10.3 ms with eight wavefronts and 11.5 ms with four
    if (GENERATED && N > CORR_BN && (int64_t)corr_tiles_m(rows) * ((N + 255) / 256) >= 256)
        return corr_launch<GENERATED, CORR_BM, 256, 32, 4, 4, 1>(A, rows, R, N, ws, tiles_m, s);
    return corr_launch<GENERATED, CORR_BM, CORR_BN, 32, 2, 2, 2>(A, rows, R, N, ws, tiles_m, s);
}

// The contraction for very few measurements (r <= 16; the paper's memory-efficient setting has r = 8): at
// that depth a tile's matrix-core work is nothing and the tiled kernels spend their time on staging and
// on the cross-lane reduction of the epilogue. Here a thread owns two right-hand sides (their r residual
// entries in registers) and walks the 256 positions of the workgroup's tile, whose rows of At every
// lane reads from LDS at the same address (a broadcast; one read serves both right-hand sides): r FMAs
// per score, and the two best keys of the tile stay in the thread's own registers - no reduction across
// lanes at all. (Scalar loads of the rows instead of LDS measured slower: they return out of order and
// every use waits for all of them.) Keys as in the pipelined kernel's epilogue: score bits with the low
// byte replaced by 255 - (position in the tile).
// grid (tiles of 256 positions, ceil(N / 512)); rows of At resident; R4 = r / 4.
constexpr int NARROW_RHS = 2; // right-hand sides per thread
template <int R4>
__global__ __launch_bounds__(256) void corr_narrow_kernel(MatrixView A, int32_t rows, const float *__restrict__ R,
                                                          int32_t N, const uint32_t *__restrict__ bitmap, int32_t words,
                                                          uint64_t *__restrict__ partial, int32_t tiles_m)
{
    constexpr int RR = 4 * R4;
    __shared__ __attribute__((aligned(16))) float a_s[256 * RR];
    __shared__ float inv_s[256];
    const int tid = threadIdx.x;
    const int32_t local0 = blockIdx.x * 256;         // first row of the tile within At
    const int32_t m0 = A.row0 + local0;              // its position
    const int32_t live = rows - local0 < 256 ? rows - local0 : 256; // rows of the tile that exist
    // the tile's rows are contiguous in memory
    for (int e = tid; e < 256 * R4; e += 256) {
        const int row = e / R4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < live)
            v = reinterpret_cast<const float4 *>(A.At + (int64_t)local0 * RR)[e];
        reinterpret_cast<float4 *>(a_s)[e] = v;
    }
    inv_s[tid] = tid < live ? A.inv_colnorm[m0 + tid] : 0.f;
    int32_t n[NARROW_RHS];
    float y[NARROW_RHS][RR];
    uint32_t msk[NARROW_RHS][8];
#pragma unroll
    for (int u = 0; u < NARROW_RHS; ++u) {
        n[u] = blockIdx.y * (256 * NARROW_RHS) + 256 * u + tid;
        const int32_t nn = n[u] < N ? n[u] : N - 1; // past the end: the last right-hand side again, nothing stored
#pragma unroll
        for (int q = 0; q < R4; ++q) {
            const float4 v = reinterpret_cast<const float4 *>(R + (int64_t)nn * RR)[q];
            y[u][4 * q] = v.x;
            y[u][4 * q + 1] = v.y;
            y[u][4 * q + 2] = v.z;
            y[u][4 * q + 3] = v.w;
        }
#pragma unroll
        for (int w = 0; w < 8; ++w) {
            const int32_t word = (m0 >> 5) + w;
            msk[u][w] = word < words ? bitmap[(int64_t)nn * words + word] : 0xffffffffu;
            // positions of the tile past the last row count as selected
            const int32_t left = live - 32 * w;
            if (left < 32)
                msk[u][w] |= left <= 0 ? 0xffffffffu : ~((1u << left) - 1u);
        }
    }
    __syncthreads();
    // Selected positions are left in on the first scan (their columns are orthogonal to the residual, so
    // they reach the two best only when the residual is rounding noise or zero); if a winner of any lane
    // turns out to be selected, the scan is repeated with the selected positions forced to key 0. Positions
    // of the tile past the last row were marked as selected above and are caught the same way.
    uint32_t best[NARROW_RHS], second[NARROW_RHS];
    auto scan = [&](auto maskedc) {
        constexpr bool MASKED = decltype(maskedc)::value;
#pragma unroll
        for (int u = 0; u < NARROW_RHS; ++u)
            best[u] = second[u] = 0;
#pragma unroll
        for (int w = 0; w < 8; ++w) {
#pragma unroll 8
            for (int b = 0; b < 32; ++b) {
                const int i = 32 * w + b;
                float dot[NARROW_RHS];
#pragma unroll
                for (int u = 0; u < NARROW_RHS; ++u)
                    dot[u] = 0.f;
#pragma unroll
                for (int q = 0; q < R4; ++q) {
                    const float4 a = reinterpret_cast<const float4 *>(a_s)[i * R4 + q];
#pragma unroll
                    for (int u = 0; u < NARROW_RHS; ++u) {
                        dot[u] = __builtin_fmaf(a.x, y[u][4 * q], dot[u]);
                        dot[u] = __builtin_fmaf(a.y, y[u][4 * q + 1], dot[u]);
                        dot[u] = __builtin_fmaf(a.z, y[u][4 * q + 2], dot[u]);
                        dot[u] = __builtin_fmaf(a.w, y[u][4 * q + 3], dot[u]);
                    }
                }
                const float in = inv_s[i];
#pragma unroll
                for (int u = 0; u < NARROW_RHS; ++u) {
                    const float score = fabsf(dot[u]) * in;
                    uint32_t key = (__float_as_uint(score) & 0xffffff00u) | (uint32_t)(255 - i);
                    if (MASKED)
                        key = ((msk[u][w] >> b) & 1u) ? 0u : key;
                    second[u] = max(second[u], min(key, best[u]));
                    best[u] = max(best[u], key);
                }
            }
        }
    };
    scan(std::false_type{});
    uint32_t hit = 0;
#pragma unroll
    for (int u = 0; u < NARROW_RHS; ++u) {
#pragma unroll
        for (int which = 0; which < 2; ++which) {
            const uint32_t pos = 255u - ((which ? second[u] : best[u]) & 0xffu); // within the tile
#pragma unroll
            for (int w = 0; w < 8; ++w) // straight-line: every word is tested
                hit |= ((msk[u][w] >> (pos & 31u)) & 1u) & (uint32_t)((pos >> 5) == (uint32_t)w);
        }
    }
    if (__builtin_amdgcn_ballot_w64(hit != 0u) != 0ull)
        scan(std::true_type{});
    auto widen = [&](uint32_t k32) -> uint64_t { // (score bits, ~position) as the selection kernel reads it
        if (k32 == 0)
            return 0ull;
        const uint32_t i = (uint32_t)m0 + (255u - (k32 & 0xffu));
        return ((uint64_t)(k32 & 0xffffff00u) << 32) | (uint64_t)(0xffffffffu - i);
    };
#pragma unroll
    for (int u = 0; u < NARROW_RHS; ++u) {
        if (n[u] < N) {
            uint64_t *o = partial + ((int64_t)n[u] * tiles_m + m0 / 256) * 2;
            o[0] = widen(best[u]);
            o[1] = widen(second[u]);
        }
    }
}

bool corr_narrow_ok(int32_t r, int32_t N)
{
    return r <= 16 && N >= 128;
}

hipError_t corr_narrow_launch(const MatrixView &A, int32_t rows, const float *R, int32_t N, const OmpWorkspace &ws,
                              int32_t tiles_m, hipStream_t s)
{
    const dim3 grid((unsigned)((rows + 255) / 256), (unsigned)((N + 256 * NARROW_RHS - 1) / (256 * NARROW_RHS)));
    switch (A.r / 4) {
    case 1: corr_narrow_kernel<1><<<grid, 256, 0, s>>>(A, rows, R, N, ws.bitmap, ws.words, ws.partial, tiles_m); break;
    case 2: corr_narrow_kernel<2><<<grid, 256, 0, s>>>(A, rows, R, N, ws.bitmap, ws.words, ws.partial, tiles_m); break;
    case 3: corr_narrow_kernel<3><<<grid, 256, 0, s>>>(A, rows, R, N, ws.bitmap, ws.words, ws.partial, tiles_m); break;
    case 4: corr_narrow_kernel<4><<<grid, 256, 0, s>>>(A, rows, R, N, ws.bitmap, ws.words, ws.partial, tiles_m); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t corr_general_launch(bool generated, const MatrixView &A, int32_t rows, const float *R, int32_t N,
                               const OmpWorkspace &ws, int32_t tiles_m, hipStream_t s)
{
    return generated ? corr_dispatch<true>(A, rows, R, N, ws, tiles_m, s)
                     : corr_dispatch<false>(A, rows, R, N, ws, tiles_m, s);
}

} // namespace sgc
