// Internal declarations shared by the HIP translation units of libsgc (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/sgc.h"

namespace sgc {

// Device view of the measurement matrix.
struct MatrixView {
    const float *At;          // [d][r] or nullptr in generated mode
    const float *inv_colnorm; // [d] or nullptr
    const double *gram;       // [d][d] inner products of the columns of A, or nullptr
    int32_t d, r;
    uint32_t key0, key1; // Philox key
    float scale;         // (float)(1/sqrt((double)r))
    int32_t generated;   // 0 stored, 1 Philox
    int32_t row0;        // position held by At[0] (non-zero for a panel of a generated matrix)
    int32_t flags;       // SGC_MATRIX_FLAG_*
};

MatrixView make_view(const sgc_matrix *A);

// ---- correlation GEMM tiling (see omp.hip) ----
constexpr int CORR_BM = 128; // rows of At (positions i) per workgroup
constexpr int CORR_BN = 128; // right-hand sides per workgroup

inline int corr_tiles_m(int d) { return (d + CORR_BM - 1) / CORR_BM; }

// the single-launch recovery serves at most this many right-hand sides, with at most this many workgroups
constexpr int SMALL_MAX_RHS = 4;
constexpr int SMALL_MAX_GROUPS = 64;
constexpr int SMALL_XCHG_PAD = 8; // words after the r residual words of a right-hand side: [0] the selected position

// Workspace layout of sgc_recover_omp (all offsets 256-byte aligned).
struct OmpWorkspace {
    double *res64;     // [N][r] residual
    double *F;         // [N][f_stride] inverse Cholesky factor, column t of n at F[n*f_stride + t*k .. +t]
    int64_t f_stride;  // k*k plus a pad, so that equal columns of different right-hand sides (read at the
                       // same time by all workgroups) do not sit a power of two apart in memory
    double *avec;      // [N][k] coefficients in the orthonormal basis
    double *xs;        // [2][N][k] least-squares solution: iteration j reads half (j+1)&1, writes half j&1
    int64_t xs_half;   // elements between the two halves of xs
    float *res32;      // [N][r] residual rounded to float (operand of the contraction)
    uint16_t *res16;   // the same memory holding the residuals split in bfloat16 pairs (screening
                       // contraction; [N] rows of 4 r bytes, format in omp.hip)
    uint16_t *a16;     // [a16_rows] rows of At split the same way
    int32_t a16_rows;  // d (padded to whole tiles) if the matrix fits 2 GiB, else a 64 MiB panel's rows
    float *cols;       // [N][k][r] selected columns of A
    uint64_t *partial; // [N][tiles_m][2] best and second-best packed (score, position) per tile
    uint32_t *bitmap;  // [N][words] selected positions
    double *wv;        // [N][k] inner products of the new column with the earlier selections
    double *gb;        // [N][2] squared norm of the new column, its inner product with y
    float *panel;      // [panel_rows][r] rows of a generated matrix: all of them (written once per call; a
                       // matrix above 64 MiB then lies in the memory of `cols`, which is not needed with
                       // resident rows) or a 64 MiB panel refilled in every iteration
    int32_t panel_rows; // multiple of 256
    int32_t words;     // bitmap words per right-hand side
    int32_t tiles_m;
    size_t bytes;
    // only with the correlation recurrence of App. B (carve_recurrence), else null:
    float *rc_p;       // [N][d] correlation vector
    float *rc_B;       // [N][rc_head][d] images b_t = A^H q_t of the orthonormal directions
    int32_t rc_head;   // iterations served by the recurrence (the rest by the contraction)
    int32_t rc_d;      // d (row length of rc_p and rc_B)
    double *cvec;      // [N][k] coordinates c_t of the newest column, exported by update_kernel
    uint32_t *sync;    // [64] word 0: the give-up flag of the single-launch recovery for small batches
    uint64_t *xchg;    // [N][r + SMALL_XCHG_PAD] that kernel's exchange area (tagged residual words, selected position)
};
// `need`: which optional regions the matrix calls for. A stored matrix is read in place (no column copies, no
// panel); the bfloat16 planes exist only for a matrix that asks for the screening contraction.
enum : uint32_t { WS_NEED_GENERATED = 1u, WS_NEED_SCREEN = 2u, WS_NEED_WHOLE_MATRIX = 4u };
inline uint32_t workspace_need(int32_t mode, int32_t flags)
{
    return (mode == SGC_MATRIX_PHILOX ? WS_NEED_GENERATED : 0u) | ((flags & SGC_MATRIX_FLAG_SCREEN_BF16) ? WS_NEED_SCREEN : 0u) |
           ((flags & SGC_MATRIX_FLAG_MATERIALIZE) ? WS_NEED_WHOLE_MATRIX : 0u);
}
OmpWorkspace carve_workspace(void *base, int32_t N, int32_t d, int32_t r, int32_t k, uint32_t need);
// the same workspace followed by the three arrays of the recurrence; `bytes` covers both
OmpWorkspace carve_recurrence(void *base, int32_t N, int32_t d, int32_t r, int32_t k, int32_t head, uint32_t need);

// kernel classes of the optional per-kernel timing (see profile.hip)
enum KernelClass { KC_TOPK = 0, KC_PROJECT, KC_ADAM, KC_CORR, KC_SELECT, KC_APPLY, KC_OTHER, KC_FILL, KC_OUTER_PROJECT, KC_OUTER_APPLY, KC_OUTER_REFRESH };

// launchers (each returns hipGetLastError() of its launches)
// scratch_i / scratch_v: optional memory for scratch_elems candidates each (positions, values) that the
// call may overwrite; with it, long chunks take a faster two-pass path
hipError_t launch_topk(const void *grad, int grad_type, int64_t C, int32_t d, int32_t k, int32_t *idx,
                       float *val, hipStream_t s, int32_t *scratch_i = nullptr, float *scratch_v = nullptr,
                       int64_t scratch_elems = 0);
hipError_t launch_project(const int32_t *idx, const float *val, int64_t C, int32_t k, const MatrixView &A,
                          float *p, float *q, hipStream_t s, float out_scale = 1.0f);
hipError_t launch_adam(const float *p, const float *q, float *m, float *v, float *mhat, float *vhat,
                       int64_t count, float b1, float omb1, float b2, float omb2, float ibc1, float ibc2,
                       hipStream_t s);
hipError_t launch_matrix_fill(uint32_t key0, uint32_t key1, float scale, int32_t r, int64_t row0,
                              int64_t rows, float *out, hipStream_t s, int profile_class = KC_OTHER);
hipError_t launch_colnorms(const MatrixView &A, float *out, hipStream_t s);
hipError_t launch_gram(const MatrixView &A, double *out, hipStream_t s);
hipError_t launch_omp(const float *y, int32_t N, const MatrixView &A, int32_t k, int32_t *sel, float *x,
                      const OmpWorkspace &ws, hipStream_t s, const float *y_fit = nullptr, float *z = nullptr,
                      bool recurrence = false, bool one_stream = false);
hipError_t launch_apply(float *W, int64_t C, int32_t d, int32_t k, const int32_t *sel_m, const float *x_m,
                        const int32_t *sel_v, const float *x_v, float alpha, float eps, float lr,
                        hipStream_t s);

// outer projection of CESGC (see outer.hip)
struct OuterPlan {
    int32_t rblk;       // rows of B per workgroup / 32
    int32_t strips;     // column strips of 128
    int32_t rho_blocks; // blocks of 32 * rblk rows of B
    int32_t slice;      // rows of G per slice
    int32_t reps;       // consecutive slices per workgroup (a run)
    int32_t slices;     // runs: partial results per matrix
    size_t ws_bytes;
};
OuterPlan outer_plan(int32_t count, int32_t rho, int32_t m, int32_t n);
hipError_t launch_outer_project(const float *B, const void *G, bool g_bf16, int32_t count, int32_t rho, int32_t m,
                                int32_t n, float *Gc, void *ws, hipStream_t s);
hipError_t launch_outer_apply(float *W, const float *B, int32_t count, int32_t rho, int32_t m, int32_t n, int32_t d,
                              int32_t k, const int32_t *sel_m, const float *x_m, const int32_t *sel_v,
                              const float *x_v, float alpha, float eps, float lr, void *ws, hipStream_t s);

// ---- refresh of the CESGC projection matrix (refresh.hip) ----
constexpr int REFRESH_MAX_RHO = 64; // the rho x rho factorisations run in one workgroup's LDS, in double
struct RefreshPlan { // byte offsets into the workspace, 256-byte aligned; every region holds the whole batch
    size_t gt_off;    // G^T in G's own element type
    size_t z_off;     // rho x n floats
    size_t part_off;  // partial Gram matrices, doubles
    size_t m_off;     // the rho x rho transform, doubles
    size_t outer_off; // workspace of the two outer projections
    size_t ws_bytes;
};
RefreshPlan refresh_plan(int32_t count, int32_t rho, int32_t m, int32_t n, bool g_bf16);
hipError_t launch_outer_refresh(float *B, const void *G, bool g_bf16, int32_t count, int32_t rho, int32_t m, int32_t n,
                                int32_t iters, float *sigma, void *ws, hipStream_t s);

// ---- optional per-kernel timing (see profile.hip) ----
extern bool g_profile_on;
void profile_begin(int cls, hipStream_t s);
void profile_end(hipStream_t s);
struct ProfileScope {
    hipStream_t s;
    bool on;
    ProfileScope(int cls, hipStream_t st) : s(st), on(g_profile_on)
    {
        if (on)
            profile_begin(cls, s);
    }
    ~ProfileScope()
    {
        if (on)
            profile_end(s);
    }
};

// A named range around an entry point's launches, visible to rocprofv3 --marker-trace (a no-op when the marker
// library is not there).
struct RangeScope {
    bool on;
    explicit RangeScope(const char *name);
    ~RangeScope();
};

// Raise a kernel's dynamic-LDS limit to `bytes`, once per kernel and device (the attribute belongs to the
// device's copy of the code object). Host state without a lock, like the rest of the library.
hipError_t raise_dynamic_lds(const void *kernel, size_t bytes);

// ---- small device helpers ----
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
        v += __shfl_down(v, off, 64);
    return v; // valid in lane 0
}

// 16-byte load of data that is read once: marked non-temporal so that it streams past the caches
__device__ __forceinline__ float4 load_once_f4(const float *p)
{
    typedef float floatx4_t __attribute__((ext_vector_type(4)));
    const floatx4_t t = __builtin_nontemporal_load(reinterpret_cast<const floatx4_t *>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}

__device__ __forceinline__ uint64_t shfl_xor_u64(uint64_t v, int mask)
{
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    lo = __shfl_xor(lo, mask, 64);
    hi = __shfl_xor(hi, mask, 64);
    return ((uint64_t)hi << 32) | lo;
}

} // namespace sgc
