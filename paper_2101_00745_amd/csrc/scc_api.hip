// C ABI of the SCC library: argument validation, window arithmetic, kernel selection.
// Every check except the launch status happens on the host before any HIP call.
#include "scc.h"
#include "scc_common.h"

#include <cmath>
#include <limits>
#include <mutex>

// Scratch of scc_backward_weight_static: the K-split partials of grad-weight live here instead of in a
// caller-supplied workspace.  One copy per GPU, held until the process ends.  In host code the name is only a
// handle for hipGetSymbolAddress; the device address it resolves to is what the kernels get.
static __device__ __align__(256) unsigned char scratch[SCC_STATIC_SCRATCH_BYTES];

namespace {

using scc::Problem;

long long gcd_ll(long long a, long long b)
{
    while (b) {
        long long t = a % b;
        a = b;
        b = t;
    }
    return a;
}

// Algorithm 1 in closed form.  Returns SCC_OK or the status that rejects the arguments.
int make_problem(int N, int Cin, int Cout, int H, int W, int cg, double co, Problem* out)
{
    if (N <= 0 || Cin <= 0 || Cout <= 0 || H <= 0 || W <= 0 || cg < 1) return SCC_ERR_SHAPE;
    if (Cin % cg != 0) return SCC_ERR_SHAPE;
    if (!std::isfinite(co) || co < 0.0 || co > 1.0) return SCC_ERR_OVERLAP;
    const long long HW = (long long)H * W;
    const long long lim = std::numeric_limits<int>::max();
    // the kernels index columns, planes of one sample and the weight matrix with 32-bit ints
    if (HW > lim || HW * N > lim || HW * Cin > lim || HW * Cout > lim) return SCC_ERR_SHAPE;
    const int L = Cin / cg;
    if ((long long)Cout * L > lim) return SCC_ERR_SHAPE;
    const int ov = (int)(co * (double)L);  // truncation of the double product, as Algorithm 1 writes it
    const int stride = (L - ov) % Cin;     // L - ov == Cin only for cg == 1 with no overlap
    Problem p;
    p.N = N;
    p.Cin = Cin;
    p.Cout = Cout;
    p.HW = (int)HW;
    p.L = L;
    p.stride = stride;
    p.period = stride == 0 ? 1 : (int)(Cin / gcd_ll(stride, Cin));
    p.NQ = HW * N;
    *out = p;
    return SCC_OK;
}

bool dtype_ok(scc_dtype d) { return d == SCC_F32 || d == SCC_BF16; }

int launch_status(hipError_t e) { return e == hipSuccess ? SCC_OK : SCC_ERR_LAUNCH; }

// The launchers report hipGetLastError(), which also returns (and clears) an error an EARLIER, unrelated call of
// the process left behind.  Every entry point that launches drops such a leftover first, so that SCC_ERR_LAUNCH
// always speaks of this call's own kernels.
void drop_stale_error() { (void)hipGetLastError(); }

// Device address of `scratch` on the current device, resolved once per device (each GPU holds its own copy
// of the array at its own address).
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];

int scratch_of_current_device(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SCC_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SCC_ERR_LAUNCH;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SCC_OK;
}

}  // namespace

extern "C" {

int scc_window_params(int Cin, int Cout, int cg, double co, int* L, int* stride, int* period)
{
    Problem p;
    const int rc = make_problem(1, Cin, Cout, 1, 1, cg, co, &p);
    if (rc != SCC_OK) return rc;
    if (L) *L = p.L;
    if (stride) *stride = p.L - (int)(co * (double)p.L);
    if (period) *period = p.period < Cout ? p.period : Cout;
    return SCC_OK;
}

int scc_forward(const void* x, const void* w, void* y, int N, int Cin, int Cout, int H, int W, int cg, double co,
                scc_dtype dtype, void* stream)
{
    if (!x || !w || !y) return SCC_ERR_NULL;
    Problem p;
    const int rc = make_problem(N, Cin, Cout, H, W, cg, co, &p);
    if (rc != SCC_OK) return rc;
    if (!dtype_ok(dtype)) return SCC_ERR_DTYPE;
    drop_stale_error();
    hipStream_t st = (hipStream_t)stream;
    if (dtype == SCC_F32) {
        if (scc::forward_mfma_eligible(p))
            return launch_status(scc::launch_forward_mfma((const float*)x, (const float*)w, (float*)y, p, st));
        return launch_status(scc::launch_forward_generic((const float*)x, (const float*)w, (float*)y, p, st));
    }
    if (scc::forward_mfma_eligible(p))
        return launch_status(
            scc::launch_forward_mfma((const scc::bf16_t*)x, (const scc::bf16_t*)w, (scc::bf16_t*)y, p, st));
    return launch_status(
        scc::launch_forward_generic((const scc::bf16_t*)x, (const scc::bf16_t*)w, (scc::bf16_t*)y, p, st));
}

int scc_backward_input(const void* dy, const void* w, void* dx, int N, int Cin, int Cout, int H, int W, int cg,
                       double co, scc_dtype dtype, void* stream)
{
    if (!dy || !w || !dx) return SCC_ERR_NULL;
    Problem p;
    const int rc = make_problem(N, Cin, Cout, H, W, cg, co, &p);
    if (rc != SCC_OK) return rc;
    if (!dtype_ok(dtype)) return SCC_ERR_DTYPE;
    drop_stale_error();
    hipStream_t st = (hipStream_t)stream;
    if (dtype == SCC_F32) {
        if (scc::backward_input_mfma_eligible(p))
            return launch_status(scc::launch_backward_input_mfma((const float*)dy, (const float*)w, (float*)dx, p, st));
        return launch_status(scc::launch_backward_input_generic((const float*)dy, (const float*)w, (float*)dx, p, st));
    }
    if (scc::backward_input_mfma_eligible(p))
        return launch_status(
            scc::launch_backward_input_mfma((const scc::bf16_t*)dy, (const scc::bf16_t*)w, (scc::bf16_t*)dx, p, st));
    return launch_status(
        scc::launch_backward_input_generic((const scc::bf16_t*)dy, (const scc::bf16_t*)w, (scc::bf16_t*)dx, p, st));
}

size_t scc_backward_weight_workspace_bytes(int N, int Cin, int Cout, int H, int W, int cg, double co, scc_dtype dtype)
{
    Problem p;
    if (make_problem(N, Cin, Cout, H, W, cg, co, &p) != SCC_OK || !dtype_ok(dtype)) return 0;
    if (scc::backward_weight_mfma_eligible(p)) return scc::backward_weight_mfma_workspace(p);
    return 0;
}

int scc_backward_weight(const void* x, const void* dy, void* dw, int N, int Cin, int Cout, int H, int W, int cg,
                        double co, scc_dtype dtype, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !dy || !dw) return SCC_ERR_NULL;
    Problem p;
    const int rc = make_problem(N, Cin, Cout, H, W, cg, co, &p);
    if (rc != SCC_OK) return rc;
    if (!dtype_ok(dtype)) return SCC_ERR_DTYPE;
    const size_t need = scc_backward_weight_workspace_bytes(N, Cin, Cout, H, W, cg, co, dtype);
    if (need > 0 && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u) != 0))
        return SCC_ERR_WORKSPACE;
    drop_stale_error();
    hipStream_t st = (hipStream_t)stream;
    if (dtype == SCC_F32) {
        if (scc::backward_weight_mfma_eligible(p))
            return launch_status(scc::launch_backward_weight_mfma((const float*)x, (const float*)dy, (float*)dw,
                                                                  (float*)workspace, p, st));
        return launch_status(scc::launch_backward_weight_generic((const float*)x, (const float*)dy, (float*)dw, p, st));
    }
    if (scc::backward_weight_mfma_eligible(p))
        return launch_status(scc::launch_backward_weight_mfma((const scc::bf16_t*)x, (const scc::bf16_t*)dy, (float*)dw,
                                                              (float*)workspace, p, st));
    return launch_status(
        scc::launch_backward_weight_generic((const scc::bf16_t*)x, (const scc::bf16_t*)dy, (float*)dw, p, st));
}

size_t scc_backward_workspace_bytes(int N, int Cin, int Cout, int H, int W, int cg, double co, scc_dtype dtype)
{
    Problem p;
    if (make_problem(N, Cin, Cout, H, W, cg, co, &p) != SCC_OK || !dtype_ok(dtype)) return 0;
    // the fused kernel's need, or that of the separate grad-weight pass it may fall back to, whichever is larger
    size_t need = scc_backward_weight_workspace_bytes(N, Cin, Cout, H, W, cg, co, dtype);
    if (dtype == SCC_F32 && scc::backward_fused_eligible(p)) {
        const size_t fused = scc::backward_fused_workspace(p);
        need = fused > need ? fused : need;
    }
    return need;
}

int scc_backward(const void* x, const void* dy, const void* w, void* dx, void* dw, int N, int Cin, int Cout, int H,
                 int W, int cg, double co, scc_dtype dtype, void* workspace, size_t workspace_bytes, void* stream)
{
    if (!x || !dy || !w || !dx || !dw) return SCC_ERR_NULL;
    Problem p;
    const int rc = make_problem(N, Cin, Cout, H, W, cg, co, &p);
    if (rc != SCC_OK) return rc;
    if (!dtype_ok(dtype)) return SCC_ERR_DTYPE;
    const size_t need = scc_backward_workspace_bytes(N, Cin, Cout, H, W, cg, co, dtype);
    if (need > 0 && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u) != 0))
        return SCC_ERR_WORKSPACE;
    drop_stale_error();
    const bool aligned = (((uintptr_t)x | (uintptr_t)dy | (uintptr_t)dx) & 15u) == 0;
    if (dtype == SCC_F32 && aligned && scc::backward_fused_eligible(p))
        return launch_status(scc::launch_backward_fused((const float*)x, (const float*)dy, (const float*)w, (float*)dx,
                                                        (float*)dw, (float*)workspace, p, (hipStream_t)stream));
    // layers both matrix-core kernels take: their two grids as one launch
    if (dtype == SCC_F32) {
        if (scc::backward_merged_applicable((const float*)x, (const float*)dy, (const float*)dx, p))
            return launch_status(scc::launch_backward_merged((const float*)x, (const float*)dy, (const float*)w,
                                                             (float*)dx, (float*)dw, (float*)workspace, p,
                                                             (hipStream_t)stream));
    } else if (scc::backward_merged_applicable((const scc::bf16_t*)x, (const scc::bf16_t*)dy, (const scc::bf16_t*)dx, p)) {
        return launch_status(scc::launch_backward_merged((const scc::bf16_t*)x, (const scc::bf16_t*)dy,
                                                         (const scc::bf16_t*)w, (scc::bf16_t*)dx, (float*)dw,
                                                         (float*)workspace, p, (hipStream_t)stream));
    }
    // every other layer: the two passes one after the other
    const int r1 = scc_backward_input(dy, w, dx, N, Cin, Cout, H, W, cg, co, dtype, stream);
    if (r1 != SCC_OK) return r1;
    return scc_backward_weight(x, dy, dw, N, Cin, Cout, H, W, cg, co, dtype, workspace, workspace_bytes, stream);
}

// Geometry of the depthwise stage; SCC_ERR_SHAPE for a stride below 1 or maps too large for 32-bit pixel indices.
static int make_dw_geom(int C, int H, int W, int dw_stride, scc::DwGeom* g)
{
    if (C <= 0 || H <= 0 || W <= 0 || dw_stride < 1) return SCC_ERR_SHAPE;
    if ((long long)H * W * C > std::numeric_limits<int>::max()) return SCC_ERR_SHAPE;
    g->H = H;
    g->W = W;
    g->s = dw_stride;
    g->Ho = (H - 1) / dw_stride + 1;
    g->Wo = (W - 1) / dw_stride + 1;
    return SCC_OK;
}

int scc_depthwise3x3_out(int size, int dw_stride)
{
    if (size <= 0 || dw_stride < 1) return SCC_ERR_SHAPE;
    return (size - 1) / dw_stride + 1;
}

int scc_depthwise3x3_forward(const void* x, const void* kdw, void* z, int N, int C, int H, int W, int dw_stride,
                             scc_dtype dtype, void* stream)
{
    if (!x || !kdw || !z) return SCC_ERR_NULL;
    scc::DwGeom g;
    if (N <= 0) return SCC_ERR_SHAPE;
    const int rc = make_dw_geom(C, H, W, dw_stride, &g);
    if (rc != SCC_OK) return rc;
    if ((long long)N * H * W > std::numeric_limits<int>::max()) return SCC_ERR_SHAPE;
    if (!dtype_ok(dtype)) return SCC_ERR_DTYPE;
    drop_stale_error();
    if (dtype == SCC_F32)
        return launch_status(
            scc::launch_depthwise3x3((const float*)x, (const float*)kdw, (float*)z, N, C, g, (hipStream_t)stream));
    return launch_status(scc::launch_depthwise3x3((const scc::bf16_t*)x, (const scc::bf16_t*)kdw, (scc::bf16_t*)z, N, C,
                                                  g, (hipStream_t)stream));
}

size_t scc_depthwise3x3_backward_workspace_bytes(int N, int C, int H, int W, int dw_stride, scc_dtype dtype)
{
    scc::DwGeom g;
    if (N <= 0 || make_dw_geom(C, H, W, dw_stride, &g) != SCC_OK || !dtype_ok(dtype)) return 0;
    return scc::depthwise3x3_backward_workspace(N, C, g);
}

int scc_depthwise3x3_backward(const void* x, const void* kdw, const void* dz, void* dx, void* dkdw, int N, int C, int H,
                              int W, int dw_stride, scc_dtype dtype, void* workspace, size_t workspace_bytes,
                              void* stream)
{
    if (!dz || (!dx && !dkdw) || (dx && !kdw) || (dkdw && !x)) return SCC_ERR_NULL;
    scc::DwGeom g;
    if (N <= 0) return SCC_ERR_SHAPE;
    const int rc = make_dw_geom(C, H, W, dw_stride, &g);
    if (rc != SCC_OK) return rc;
    if ((long long)N * H * W > std::numeric_limits<int>::max()) return SCC_ERR_SHAPE;
    if (!dtype_ok(dtype)) return SCC_ERR_DTYPE;
    const size_t need = dkdw ? scc::depthwise3x3_backward_workspace(N, C, g) : 0;
    if (need > 0 && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u) != 0))
        return SCC_ERR_WORKSPACE;
    drop_stale_error();
    if (dtype == SCC_F32)
        return launch_status(scc::launch_depthwise3x3_backward((const float*)x, (const float*)kdw, (const float*)dz,
                                                               (float*)dx, (float*)dkdw, (float*)workspace, N, C, g,
                                                               (hipStream_t)stream));
    return launch_status(scc::launch_depthwise3x3_backward((const scc::bf16_t*)x, (const scc::bf16_t*)kdw,
                                                           (const scc::bf16_t*)dz, (scc::bf16_t*)dx, (float*)dkdw,
                                                           (float*)workspace, N, C, g, (hipStream_t)stream));
}

// Problem of the SCC behind the depthwise stage (it sees the Ho x Wo map) and the stage's geometry.
static int make_dw_problem(int N, int Cin, int Cout, int H, int W, int dw_stride, int cg, double co, Problem* p,
                           scc::DwGeom* g)
{
    if (N <= 0) return SCC_ERR_SHAPE;
    int rc = make_dw_geom(Cin, H, W, dw_stride, g);
    if (rc != SCC_OK) return rc;
    if ((long long)N * H * W > std::numeric_limits<int>::max()) return SCC_ERR_SHAPE;
    return make_problem(N, Cin, Cout, g->Ho, g->Wo, cg, co, p);
}

size_t scc_dw_forward_workspace_bytes(int N, int Cin, int Cout, int H, int W, int dw_stride, int cg, double co,
                                      scc_dtype dtype)
{
    Problem p;
    scc::DwGeom g;
    if (make_dw_problem(N, Cin, Cout, H, W, dw_stride, cg, co, &p, &g) != SCC_OK || !dtype_ok(dtype)) return 0;
    if (dtype == SCC_F32 && scc::dw_forward_fused_preferred(p)) return 0;
    return (size_t)p.NQ * Cin * (dtype == SCC_F32 ? 4 : 2);   // the depthwise stage's output
}

int scc_dw_forward_fusable(int N, int Cin, int Cout, int H, int W, int dw_stride, int cg, double co, scc_dtype dtype)
{
    Problem p;
    scc::DwGeom g;
    const int rc = make_dw_problem(N, Cin, Cout, H, W, dw_stride, cg, co, &p, &g);
    if (rc != SCC_OK) return rc;
    if (!dtype_ok(dtype)) return SCC_ERR_DTYPE;
    return dtype == SCC_F32 && scc::dw_forward_fused_eligible(p) ? 1 : 0;
}

int scc_dw_forward(const void* x, const void* kdw, const void* w, void* y, int N, int Cin, int Cout, int H, int W,
                   int dw_stride, int cg, double co, scc_dtype dtype, void* workspace, size_t workspace_bytes,
                   void* stream)
{
    if (!x || !kdw || !w || !y) return SCC_ERR_NULL;
    Problem p;
    scc::DwGeom g;
    const int rc = make_dw_problem(N, Cin, Cout, H, W, dw_stride, cg, co, &p, &g);
    if (rc != SCC_OK) return rc;
    if (!dtype_ok(dtype)) return SCC_ERR_DTYPE;
    const size_t need = scc_dw_forward_workspace_bytes(N, Cin, Cout, H, W, dw_stride, cg, co, dtype);
    // without a workspace the fused kernel runs wherever it can, also where the two stages would be faster
    const bool fused = dtype == SCC_F32 && (need == 0 || (!workspace && scc::dw_forward_fused_eligible(p)));
    if (!fused && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255u) != 0))
        return SCC_ERR_WORKSPACE;
    if (fused) {
        drop_stale_error();
        return launch_status(scc::launch_dw_forward_fused((const float*)x, (const float*)kdw, (const float*)w, (float*)y,
                                                          p, g, (hipStream_t)stream));
    }
    // every other layer: the depthwise stage into the workspace, then the SCC forward on it
    const int r1 = scc_depthwise3x3_forward(x, kdw, workspace, N, Cin, H, W, dw_stride, dtype, stream);
    if (r1 != SCC_OK) return r1;
    return scc_forward(workspace, w, y, N, Cin, Cout, g.Ho, g.Wo, cg, co, dtype, stream);
}

int scc_backward_weight_static(const void* x, const void* dy, void* dw, int N, int Cin, int Cout, int H, int W, int cg,
                               double co, scc_dtype dtype, void* stream)
{
    if (!x || !dy || !dw) return SCC_ERR_NULL;
    Problem p;
    const int rc = make_problem(N, Cin, Cout, H, W, cg, co, &p);
    if (rc != SCC_OK) return rc;
    if (!dtype_ok(dtype)) return SCC_ERR_DTYPE;
    const size_t need = scc_backward_weight_workspace_bytes(N, Cin, Cout, H, W, cg, co, dtype);
    if (need > (size_t)SCC_STATIC_SCRATCH_BYTES) return SCC_ERR_SCRATCH;
    void* ptr = nullptr;
    if (need > 0) {
        const int sc = scratch_of_current_device(&ptr);
        if (sc != SCC_OK) return sc;
    }
    return scc_backward_weight(x, dy, dw, N, Cin, Cout, H, W, cg, co, dtype, ptr, need, stream);
}

const char* scc_status_string(int status)
{
    switch (status) {
        case SCC_OK: return "SCC_OK";
        case SCC_ERR_NULL: return "SCC_ERR_NULL: a required pointer is NULL";
        case SCC_ERR_SHAPE: return "SCC_ERR_SHAPE: non-positive dimension, cg < 1, Cin not divisible by cg, or tensor too large";
        case SCC_ERR_OVERLAP: return "SCC_ERR_OVERLAP: co must be finite and within [0, 1]";
        case SCC_ERR_DTYPE: return "SCC_ERR_DTYPE: dtype must be SCC_F32 or SCC_BF16";
        case SCC_ERR_WORKSPACE: return "SCC_ERR_WORKSPACE: workspace missing, misaligned or too small";
        case SCC_ERR_LAUNCH: return "SCC_ERR_LAUNCH: the HIP runtime refused the kernel launch";
        case SCC_ERR_SCRATCH:
            return "SCC_ERR_SCRATCH: the problem needs more scratch than the library's static buffer holds";
        default: return "unknown scc status";
    }
}

}  // extern "C"
