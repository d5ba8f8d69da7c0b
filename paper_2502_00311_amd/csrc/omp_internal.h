// Declarations shared by the two translation units of the recovery (omp.hip: workspace, selection and
// update kernels, host side; omp_corr.hip: the contraction kernels).
#pragma once
#include "sgc_internal.h"

namespace sgc {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int CORRP_BM = 256; // positions per workgroup of the pipelined contraction

// a = hi + lo in bfloat16 (round to nearest even each), |a - hi - lo| <= 2^-17 |a|
__device__ __forceinline__ void split_bf16_1(float a, uint16_t &hi, uint16_t &lo)
{
    const __bf16 h = (__bf16)a;
    const __bf16 l = (__bf16)(a - (float)h);
    hi = *reinterpret_cast<const uint16_t *>(&h);
    lo = *reinterpret_cast<const uint16_t *>(&l);
}

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

// ---- contraction launchers (omp_corr.hip) ----
// rows of floats -> split32 rows
void launch_split_rows(const float *src, int64_t rows, int32_t r, uint16_t *dst, hipStream_t s);
// the float contraction: the pipelined kernel (full tiles of resident rows) or the general one
hipError_t corr_pipelined_launch(const MatrixView &A, int32_t rows, const float *R, int32_t N, const OmpWorkspace &ws,
                                 int32_t tiles_m, hipStream_t s);
hipError_t corr_general_launch(bool generated, const MatrixView &A, int32_t rows, const float *R, int32_t N,
                               const OmpWorkspace &ws, int32_t tiles_m, hipStream_t s);
// the bfloat16 screening contraction on split rows
hipError_t corr_screen_launch(bool pipelined, const MatrixView &A, const uint16_t *rows_split, int32_t rows, int32_t N,
                              const OmpWorkspace &ws, int32_t tiles_m, hipStream_t s);
// the correlation recurrence of App. B (omp_recur.hip): p0 = A^H y written out; then per iteration the new
// image vector, the update of p and the two best keys per tile of 256 positions (first: the keys only)
hipError_t recur_init_launch(const MatrixView &A, const float *y, int32_t N, const OmpWorkspace &w, hipStream_t s);
hipError_t recur_step_launch(bool first, const MatrixView &A, int32_t N, int32_t k, int32_t it, const int32_t *sel,
                             const OmpWorkspace &w, int32_t tiles, hipStream_t s);
// the contraction for r <= 16 on resident rows (a thread per right-hand side, no matrix cores)
bool corr_narrow_ok(int32_t r, int32_t N);
hipError_t corr_narrow_launch(const MatrixView &A, int32_t rows, const float *R, int32_t N, const OmpWorkspace &ws,
                              int32_t tiles_m, hipStream_t s);
// whether the pipelined kernel covers this problem
bool corr_pipelined_ok(const MatrixView &A, int32_t N, int32_t panel_rows);

} // namespace sgc
