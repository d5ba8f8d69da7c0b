// C ABI of libsgc: host-side argument validation and kernel launches. Nothing here computes;
// every step of the path runs in the kernels of the sibling files.
#include <math.h>

#include <mutex>

#include "sgc_internal.h"

namespace sgc {

MatrixView make_view(const sgc_matrix *A)
{
    MatrixView v{};
    v.At = A->At;
    v.inv_colnorm = A->inv_colnorm;
    v.gram = A->gram;
    v.d = A->d;
    v.r = A->r;
    v.key0 = (uint32_t)(A->seed & 0xffffffffull);
    v.key1 = (uint32_t)(A->seed >> 32);
    v.scale = (float)(1.0 / sqrt((double)A->r));
    v.generated = A->mode == SGC_MATRIX_PHILOX ? 1 : 0;
    v.row0 = 0;
    v.flags = A->flags;
    return v;
}

static bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

static sgc_status check_matrix(const sgc_matrix *A, bool need_norms)
{
    if (!A)
        return SGC_ERR_NULL;
    if (A->mode != SGC_MATRIX_STORED && A->mode != SGC_MATRIX_PHILOX)
        return SGC_ERR_DTYPE;
    if (A->d <= 0 || A->r <= 0 || (A->r & 3) || A->d > (1 << 30))
        return SGC_ERR_SHAPE;
    if (A->mode == SGC_MATRIX_STORED) {
        if (!A->At)
            return SGC_ERR_NULL;
        if (!aligned16(A->At))
            return SGC_ERR_ALIGN;
    }
    if (need_norms && !A->inv_colnorm)
        return SGC_ERR_NULL;
    return SGC_OK;
}

static sgc_status from_hip(hipError_t e) { return e == hipSuccess ? SGC_OK : SGC_ERR_DEVICE; }

} // namespace sgc

using namespace sgc;

extern "C" {

const char *sgc_status_string(sgc_status s)
{
    switch (s) {
    case SGC_OK: return "ok";
    case SGC_ERR_NULL: return "required pointer is NULL";
    case SGC_ERR_SHAPE: return "invalid size";
    case SGC_ERR_DTYPE: return "unknown element type or matrix mode";
    case SGC_ERR_ALIGN: return "pointer not aligned";
    case SGC_ERR_WORKSPACE: return "workspace too small";
    case SGC_ERR_STEP: return "invalid step or hyper-parameter";
    case SGC_ERR_DEVICE: return "HIP error";
    default: return "unknown status";
    }
}

sgc_status sgc_matrix_fill(uint64_t seed, int32_t r, int64_t row0, int64_t rows, float *At_out, void *stream)
{
    if (!At_out)
        return SGC_ERR_NULL;
    if (r <= 0 || (r & 3) || rows < 0 || row0 < 0 || row0 + rows > (1ll << 30))
        return SGC_ERR_SHAPE;
    if (!aligned16(At_out))
        return SGC_ERR_ALIGN;
    const float scale = (float)(1.0 / sqrt((double)r));
    return from_hip(launch_matrix_fill((uint32_t)(seed & 0xffffffffull), (uint32_t)(seed >> 32), scale, r, row0,
                                       rows, At_out, (hipStream_t)stream));
}

sgc_status sgc_matrix_colnorms(const sgc_matrix *A, float *inv_colnorm_out, void *stream)
{
    sgc_status st = check_matrix(A, false);
    if (st != SGC_OK)
        return st;
    if (!inv_colnorm_out)
        return SGC_ERR_NULL;
    return from_hip(launch_colnorms(make_view(A), inv_colnorm_out, (hipStream_t)stream));
}

sgc_status sgc_matrix_gram(const sgc_matrix *A, double *gram_out, void *stream)
{
    sgc_status st = check_matrix(A, false);
    if (st != SGC_OK)
        return st;
    if (!gram_out)
        return SGC_ERR_NULL;
    if (A->d > 65536) // gridDim.y of the tile grid; a larger table would not fit in memory anyway
        return SGC_ERR_SHAPE;
    if (!aligned16(gram_out))
        return SGC_ERR_ALIGN;
    return from_hip(launch_gram(make_view(A), gram_out, (hipStream_t)stream));
}

sgc_status sgc_sparsify_project(const void *grad, int32_t grad_type, int64_t n, int32_t d, int32_t k,
                                const sgc_matrix *A, int32_t *idx, float *val, float *p, float *q, void *stream)
{
    if (!grad || !idx || !val || !p)
        return SGC_ERR_NULL;
    sgc_status st = check_matrix(A, false);
    if (st != SGC_OK)
        return st;
    if (grad_type != SGC_GRAD_F32 && grad_type != SGC_GRAD_BF16)
        return SGC_ERR_DTYPE;
    if (d <= 0 || d != A->d || k <= 0 || k > d || k > A->r || k > 4096 || n < 0 || n % d != 0)
        return SGC_ERR_SHAPE;
    if (!aligned16(grad) || !aligned16(p) || (q && !aligned16(q)))
        return SGC_ERR_ALIGN;
    const int64_t C = n / d;
    hipStream_t s = (hipStream_t)stream;
    RangeScope range("sgc_sparsify_project");
    // p and q are written by the projection afterwards: until then they are scratch for the top-k pass
    hipError_t e = launch_topk(grad, grad_type, C, d, k, idx, val, s, reinterpret_cast<int32_t *>(p), q,
                               q ? C * (int64_t)A->r : 0);
    if (e != hipSuccess)
        return SGC_ERR_DEVICE;
    return from_hip(launch_project(idx, val, C, k, make_view(A), p, q, s));
}

sgc_status sgc_adam_compressed(const float *p, const float *q, float *m, float *v, float *mhat, float *vhat,
                               int64_t count, int32_t step, const sgc_hyper *h, void *stream)
{
    if (!p || !q || !m || !v || !mhat || !vhat || !h)
        return SGC_ERR_NULL;
    if (count < 0)
        return SGC_ERR_SHAPE;
    if (step < 1 || !(h->beta1 >= 0.0 && h->beta1 < 1.0) || !(h->beta2 >= 0.0 && h->beta2 < 1.0))
        return SGC_ERR_STEP;
    if (!aligned16(p) || !aligned16(q) || !aligned16(m) || !aligned16(v) || !aligned16(mhat) || !aligned16(vhat))
        return SGC_ERR_ALIGN;
    const double c1 = 1.0 - pow(h->beta1, (double)step), c2 = 1.0 - pow(h->beta2, (double)step);
    RangeScope range("sgc_adam_compressed");
    return from_hip(launch_adam(p, q, m, v, mhat, vhat, count, (float)h->beta1, (float)(1.0 - h->beta1),
                                (float)h->beta2, (float)(1.0 - h->beta2), (float)(1.0 / c1), (float)(1.0 / c2),
                                (hipStream_t)stream));
}

static bool omp_sizes_ok(int32_t N, int32_t d, int32_t r, int32_t k)
{
    if (N <= 0 || d <= 0 || r <= 0 || (r & 3) || k <= 0 || k > d || k > r || k > 1024 || d > (1 << 30))
        return false;
    // LDS of the update kernel: one column (r floats) and two k-vectors of doubles
    if ((size_t)r * 4 + 16 + (size_t)k * 16 > 60 * 1024)
        return false;
    return true;
}

size_t sgc_omp_workspace_bytes(int32_t N, int32_t d, int32_t r, int32_t k)
{
    if (!omp_sizes_ok(N, d, r, k))
        return 0;
    // enough for a stored or a generated matrix without option flags
    return carve_workspace(nullptr, N, d, r, k, WS_NEED_GENERATED).bytes;
}

size_t sgc_omp_workspace_bytes_for(int32_t N, int32_t k, const sgc_matrix *A)
{
    if (check_matrix(A, false) != SGC_OK || !omp_sizes_ok(N, A->d, A->r, k))
        return 0;
    return carve_workspace(nullptr, N, A->d, A->r, k, workspace_need(A->mode, A->flags)).bytes;
}

sgc_status sgc_recover_omp(const float *y, int32_t N, const sgc_matrix *A, int32_t k, int32_t *sel, float *x,
                           void *ws, size_t ws_bytes, void *stream)
{
    if (!y || !sel || !x || !ws)
        return SGC_ERR_NULL;
    sgc_status st = check_matrix(A, true);
    if (st != SGC_OK)
        return st;
    if (!omp_sizes_ok(N, A->d, A->r, k))
        return SGC_ERR_SHAPE;
    if (!aligned16(y) || !aligned16(A->inv_colnorm) || ((uintptr_t)ws & 255u))
        return SGC_ERR_ALIGN;
    const OmpWorkspace w = carve_workspace(ws, N, A->d, A->r, k, workspace_need(A->mode, A->flags));
    if (ws_bytes < w.bytes)
        return SGC_ERR_WORKSPACE;
    RangeScope range("sgc_recover_omp");
    return from_hip(launch_omp(y, N, make_view(A), k, sel, x, w, (hipStream_t)stream));
}

// ---- recovery for callers that cannot allocate: the workspace is a static device array ----
// Every device the library runs on holds its own copy of the array at its own address; in host code the
// array's name is only a handle for hipGetSymbolAddress, never a pointer to hand to a kernel.
static __device__ __align__(256) unsigned char scratch[SGC_OMP_STATIC_WORKSPACE_BYTES];
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[64]; // per device, resolved on the first call made with that device current

static void *scratch_of_current_device()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
        return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr)
            return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

size_t sgc_omp_static_workspace_bytes(void) { return SGC_OMP_STATIC_WORKSPACE_BYTES; }

sgc_status sgc_recover_omp_static(const float *y, int32_t N, const sgc_matrix *A, int32_t k, int32_t *sel, float *x,
                                  void *stream)
{
    if (!y || !sel || !x)
        return SGC_ERR_NULL;
    sgc_status st = check_matrix(A, true);
    if (st != SGC_OK)
        return st;
    if (!omp_sizes_ok(N, A->d, A->r, k))
        return SGC_ERR_SHAPE;
    if (!aligned16(y) || !aligned16(A->inv_colnorm))
        return SGC_ERR_ALIGN;
    const uint32_t need = workspace_need(A->mode, A->flags);
    if (carve_workspace(nullptr, N, A->d, A->r, k, need).bytes > SGC_OMP_STATIC_WORKSPACE_BYTES)
        return SGC_ERR_WORKSPACE;
    void *ptr = scratch_of_current_device();
    if (!ptr)
        return SGC_ERR_DEVICE;
    // every region the kernels read is written earlier in the same call (the first kernel clears the
    // selection bitmaps and sets the residuals), so what the previous call left behind does not matter
    const OmpWorkspace w = carve_workspace(ptr, N, A->d, A->r, k, need);
    return from_hip(launch_omp(y, N, make_view(A), k, sel, x, w, (hipStream_t)stream, nullptr, nullptr, false,
                               /*one_stream=*/true));
}

size_t sgc_omp_recurrence_workspace_bytes(int32_t N, int32_t d, int32_t r, int32_t k, int32_t head)
{
    if (!omp_sizes_ok(N, d, r, k) || d % 4 != 0 || head < 1 || head > k)
        return 0;
    return carve_recurrence(nullptr, N, d, r, k, head, WS_NEED_GENERATED | WS_NEED_SCREEN | WS_NEED_WHOLE_MATRIX).bytes;
}

sgc_status sgc_recover_omp_recurrence(const float *y, int32_t N, const sgc_matrix *A, int32_t k, int32_t head,
                                      int32_t *sel, float *x, void *ws, size_t ws_bytes, void *stream)
{
    if (!y || !sel || !x || !ws)
        return SGC_ERR_NULL;
    sgc_status st = check_matrix(A, true);
    if (st != SGC_OK)
        return st;
    if (!A->gram)
        return SGC_ERR_NULL;
    if (!omp_sizes_ok(N, A->d, A->r, k) || A->d % 4 != 0 || head < 1 || head > k)
        return SGC_ERR_SHAPE;
    if (!aligned16(y) || !aligned16(A->inv_colnorm) || !aligned16(A->gram) || ((uintptr_t)ws & 255u))
        return SGC_ERR_ALIGN;
    const OmpWorkspace w = carve_recurrence(ws, N, A->d, A->r, k, head, WS_NEED_GENERATED | WS_NEED_SCREEN | WS_NEED_WHOLE_MATRIX);
    // a generated matrix must fit the workspace's panel as a whole: the selection reads its columns from there
    if (A->mode == SGC_MATRIX_PHILOX && w.panel_rows < A->d)
        return SGC_ERR_SHAPE;
    if (ws_bytes < w.bytes)
        return SGC_ERR_WORKSPACE;
    return from_hip(launch_omp(y, N, make_view(A), k, sel, x, w, (hipStream_t)stream, nullptr, nullptr, true));
}

sgc_status sgc_recover_omp_shared(const float *y_m, const float *y_v, int32_t C, const sgc_matrix *A, int32_t k,
                                  int32_t *sel, float *x, float *z, void *ws, size_t ws_bytes, void *stream)
{
    if (!y_m || !y_v || !sel || !x || !z || !ws)
        return SGC_ERR_NULL;
    sgc_status st = check_matrix(A, true);
    if (st != SGC_OK)
        return st;
    if (!omp_sizes_ok(C, A->d, A->r, k))
        return SGC_ERR_SHAPE;
    if (!aligned16(y_m) || !aligned16(y_v) || !aligned16(A->inv_colnorm) || ((uintptr_t)ws & 255u))
        return SGC_ERR_ALIGN;
    const OmpWorkspace w = carve_workspace(ws, C, A->d, A->r, k, workspace_need(A->mode, A->flags));
    if (ws_bytes < w.bytes)
        return SGC_ERR_WORKSPACE;
    RangeScope range("sgc_recover_omp_shared");
    return from_hip(launch_omp(y_m, C, make_view(A), k, sel, x, w, (hipStream_t)stream, y_v, z));
}

sgc_status sgc_reproject(const int32_t *sel, const float *x, int64_t N, int32_t k, const sgc_matrix *A_new,
                         double scale, float *out, void *stream)
{
    if (!sel || !x || !out)
        return SGC_ERR_NULL;
    sgc_status st = check_matrix(A_new, false);
    if (st != SGC_OK)
        return st;
    if (N < 0 || k <= 0 || k > A_new->d || k > 4096)
        return SGC_ERR_SHAPE;
    if (!aligned16(out))
        return SGC_ERR_ALIGN;
    return from_hip(launch_project(sel, x, N, k, make_view(A_new), out, nullptr, (hipStream_t)stream, (float)scale));
}

sgc_status sgc_reproject_moment(const int32_t *sel, const float *x, int64_t N, int32_t k, const sgc_matrix *A_new,
                                double beta, int32_t step, float *out, void *stream)
{
    if (step < 1 || !(beta >= 0.0 && beta < 1.0))
        return SGC_ERR_STEP;
    // the same expression as the bias correction of sgc_adam_compressed
    return sgc_reproject(sel, x, N, k, A_new, 1.0 - pow(beta, (double)step), out, stream);
}

sgc_status sgc_apply(float *W, int64_t C, int32_t d, int32_t k, const int32_t *sel_m, const float *x_m,
                     const int32_t *sel_v, const float *x_v, const sgc_hyper *h, void *stream)
{
    if (!W || !sel_m || !x_m || !sel_v || !x_v || !h)
        return SGC_ERR_NULL;
    if (C < 0 || d <= 0 || k <= 0 || k > d || k > 4096)
        return SGC_ERR_SHAPE;
    RangeScope range("sgc_apply");
    return from_hip(launch_apply(W, C, d, k, sel_m, x_m, sel_v, x_v, (float)h->alpha, (float)h->eps, (float)h->lr,
                                 (hipStream_t)stream));
}

static bool outer_sizes_ok(int32_t count, int32_t rho, int32_t m, int32_t n)
{
    const int32_t most = 1 << 22;
    // the batch and the blocks of rows of B share one grid dimension (at most 65535)
    return count > 0 && rho > 0 && m > 0 && n > 0 && rho <= (1 << 20) && m <= most && n <= most && (n & 3) == 0 &&
           (int64_t)count * ((rho + 31) / 32) <= 65535 && (int64_t)count * rho * n <= (1ll << 40);
}

size_t sgc_outer_workspace_bytes(int32_t count, int32_t rho, int32_t m, int32_t n)
{
    if (!outer_sizes_ok(count, rho, m, n))
        return 0;
    return outer_plan(count, rho, m, n).ws_bytes;
}

sgc_status sgc_outer_project(const float *B, const void *G, int32_t grad_type, int32_t count, int32_t rho, int32_t m,
                             int32_t n, float *Gc, void *ws, size_t ws_bytes, void *stream)
{
    if (!B || !G || !Gc || !ws)
        return SGC_ERR_NULL;
    if (grad_type != SGC_GRAD_F32 && grad_type != SGC_GRAD_BF16)
        return SGC_ERR_DTYPE;
    if (!outer_sizes_ok(count, rho, m, n))
        return SGC_ERR_SHAPE;
    if (!aligned16(G) || !aligned16(Gc) || ((uintptr_t)ws & 255u))
        return SGC_ERR_ALIGN;
    if (ws_bytes < outer_plan(count, rho, m, n).ws_bytes)
        return SGC_ERR_WORKSPACE;
    return from_hip(launch_outer_project(B, G, grad_type == SGC_GRAD_BF16, count, rho, m, n, Gc, ws,
                                         (hipStream_t)stream));
}

sgc_status sgc_outer_apply(float *W, const float *B, int32_t count, int32_t rho, int32_t m, int32_t n, int32_t d,
                           int32_t k, const int32_t *sel_m, const float *x_m, const int32_t *sel_v, const float *x_v,
                           const sgc_hyper *h, void *ws, size_t ws_bytes, void *stream)
{
    if (!W || !B || !sel_m || !x_m || !sel_v || !x_v || !h || !ws)
        return SGC_ERR_NULL;
    if (!outer_sizes_ok(count, rho, m, n) || d <= 0 || ((int64_t)rho * n) % d != 0 || k <= 0 || k > d || k > 4096)
        return SGC_ERR_SHAPE;
    if (!aligned16(W) || ((uintptr_t)ws & 255u))
        return SGC_ERR_ALIGN;
    if (ws_bytes < outer_plan(count, rho, m, n).ws_bytes)
        return SGC_ERR_WORKSPACE;
    return from_hip(launch_outer_apply(W, B, count, rho, m, n, d, k, sel_m, x_m, sel_v, x_v, (float)h->alpha,
                                       (float)h->eps, (float)h->lr, ws, (hipStream_t)stream));
}

static bool refresh_sizes_ok(int32_t count, int32_t rho, int32_t m, int32_t n)
{
    return outer_sizes_ok(count, rho, m, n) && outer_sizes_ok(count, rho, n, m) && rho <= REFRESH_MAX_RHO && rho <= m &&
           rho <= n && ((int64_t)((m + 31) / 32) * ((n + 31) / 32)) < (1ll << 31);
}

size_t sgc_outer_refresh_workspace_bytes(int32_t count, int32_t rho, int32_t m, int32_t n, int32_t grad_type)
{
    if (!refresh_sizes_ok(count, rho, m, n) || (grad_type != SGC_GRAD_F32 && grad_type != SGC_GRAD_BF16))
        return 0;
    return refresh_plan(count, rho, m, n, grad_type == SGC_GRAD_BF16).ws_bytes;
}

sgc_status sgc_outer_refresh(float *B, const void *G, int32_t grad_type, int32_t count, int32_t rho, int32_t m,
                             int32_t n, int32_t iters, float *sigma, void *ws, size_t ws_bytes, void *stream)
{
    if (!B || !G || !ws)
        return SGC_ERR_NULL;
    if (grad_type != SGC_GRAD_F32 && grad_type != SGC_GRAD_BF16)
        return SGC_ERR_DTYPE;
    if (!refresh_sizes_ok(count, rho, m, n) || iters < 0 || iters > 1000)
        return SGC_ERR_SHAPE;
    if (!aligned16(G) || !aligned16(B) || ((uintptr_t)ws & 255u))
        return SGC_ERR_ALIGN;
    if (ws_bytes < refresh_plan(count, rho, m, n, grad_type == SGC_GRAD_BF16).ws_bytes)
        return SGC_ERR_WORKSPACE;
    return from_hip(launch_outer_refresh(B, G, grad_type == SGC_GRAD_BF16, count, rho, m, n, iters, sigma, ws,
                                         (hipStream_t)stream));
}

} // extern "C"
