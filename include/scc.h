/*
 * scc.h - C ABI of the MI355X (gfx950) sliding-channel convolution library.
 *
 * Sliding-channel convolution (SCC) is the cross-channel step of a depthwise
 * separable block in DSXplore (Section 3.1 of the paper): output channel
 * ("filter") k is a weighted sum, at every pixel, over a window of
 *     L = Cin / cg
 * consecutive input channels.  Adjacent filters' windows overlap by
 *     ov = int(co * L)                      (Algorithm 1: C truncation of the double product)
 * channels, so the window of filter k starts at
 *     s_k = (k * (L - ov)) mod Cin          (Algorithm 1 walked filter by filter; Algorithm 2)
 * and wraps from channel Cin-1 to channel 0 (the "channel circle", Section 3.1).
 * Weight j of filter k multiplies channel (s_k + j) mod Cin.
 *
 * Conventions shared by every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The library
 *     allocates nothing, keeps no state between calls and never frees or
 *     modifies an input.  (scc_backward_weight_static alone uses a buffer the
 *     library holds itself; see there.)
 *   - Tensors are dense, row-major:  x, dx : [N][Cin][H][W]
 *                                    y, dy : [N][Cout][H][W]
 *                                    w, dw : [Cout][L]
 *     No spatial offset, padding or stride: output pixel (h, w) reads input
 *     pixel (h, w) (Section 4.2, forward pass).  Only H*W matters.
 *   - Outputs are overwritten, never accumulated into.  An output must not
 *     alias an input.
 *   - dtype SCC_F32: all tensors are IEEE binary32 and all sums are binary32.
 *     Products are binary32 products, or (forward, grad-input and the fused
 *     backward on the matrix cores) six of the nine partial products of an
 *     exact three-way bfloat16 split of both factors, which differ from the
 *     binary32 product by less than 2^-23 of it.
 *     Finite inputs: a filter never sees a channel outside its window, and
 *     all-zero weights give exact zeros.  Non-finite inputs: an Inf or NaN
 *     element gives NaN where binary32 arithmetic would give Inf, and in the
 *     forward and grad-input passes it may also turn outputs of OTHER filters
 *     or channels at the same sample and pixel into NaN (inside a tile zero
 *     weights multiply it); it never reaches another sample or pixel.  In
 *     grad-weight, which sums over all samples and pixels, it may reach any
 *     weight gradient.
 *     Operands below about 2^-110 in magnitude lose the low pieces of the
 *     split to underflow: the error is then bounded by a fraction of the
 *     smallest normal number instead of 2^-23 of the product (scc_backward_weight
 *     multiplies in binary32 and is not affected).
 *     dtype SCC_BF16: x, w, y, dy, dx are bfloat16 (upper half of a binary32,
 *     results rounded to nearest even), products accumulated in binary32;
 *     dw is written as binary32 in BOTH dtypes.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work and return; nothing synchronises the device.
 *   - Return value: SCC_OK, or a negative scc_status.  Everything except
 *     SCC_ERR_LAUNCH is decided on the host before any GPU call is made, so an
 *     invalid call touches no memory.  Nothing is printed, nothing aborts.
 *     A call that launches first discards any error an earlier HIP call of the
 *     process left pending (hipGetLastError), so SCC_ERR_LAUNCH always refers
 *     to this call's own kernels.
 *   - co is a double so that int(co * L) truncates exactly as Algorithm 1 does.
 */
#ifndef SCC_H
#define SCC_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SCC_F32 = 0, SCC_BF16 = 1 } scc_dtype;

typedef enum {
    SCC_OK = 0,
    SCC_ERR_NULL = -1,      /* a required pointer is NULL */
    SCC_ERR_SHAPE = -2,     /* a dimension <= 0, cg < 1, Cin % cg != 0, or a tensor too large to index */
    SCC_ERR_OVERLAP = -3,   /* co is not finite or lies outside [0, 1] */
    SCC_ERR_DTYPE = -4,     /* dtype is neither SCC_F32 nor SCC_BF16 */
    SCC_ERR_WORKSPACE = -5, /* workspace missing, misaligned or smaller than the query says */
    SCC_ERR_LAUNCH = -6,    /* the HIP runtime refused a launch (hipGetLastError != hipSuccess) */
    SCC_ERR_SCRATCH = -7    /* scc_backward_weight_static: the problem needs more than SCC_STATIC_SCRATCH_BYTES */
} scc_status;

/* Size of the device buffer the library itself holds, per GPU, for scc_backward_weight_static. */
#define SCC_STATIC_SCRATCH_BYTES (8u << 20)

/*
 * Window arithmetic of Algorithm 1, host only (no GPU call).
 *   L      <- Cin / cg
 *   stride <- L - int(co * L)             distance between adjacent filters' window starts
 *   period <- number of distinct windows among the Cout filters: the "cyclic
 *             distance" of the channel-cyclic pattern (Section 4.2), i.e.
 *             min(Cout, Cin / gcd(stride mod Cin, Cin)), and 1 when stride mod Cin == 0.
 * Any output pointer may be NULL.  Errors: SCC_ERR_SHAPE, SCC_ERR_OVERLAP.
 */
int scc_window_params(int Cin, int Cout, int cg, double co, int* L, int* stride, int* period);

/*
 * Forward pass (Section 4.2, "Output-Centric Forward Pass"):
 *     y[n,k,h,w] = sum_{j<L} w[k,j] * x[n, (s_k + j) mod Cin, h, w]
 * x: in, N*Cin*H*W elements.  w: in, Cout*L elements.  y: out, N*Cout*H*W elements.
 */
int scc_forward(const void* x, const void* w, void* y,
                int N, int Cin, int Cout, int H, int W, int cg, double co,
                scc_dtype dtype, void* stream);

/*
 * Gradient with respect to the input (Section 4.2, "Input-Centric Backward Pass"):
 * each input-gradient element gathers from the filters whose window covers its channel,
 *     dx[n,c,h,w] = sum_{k : (c - s_k) mod Cin < L} w[k, (c - s_k) mod Cin] * dy[n,k,h,w]
 * No atomics are used.  dy: in, N*Cout*H*W.  w: in, Cout*L.  dx: out, N*Cin*H*W.
 * A channel no window covers (possible when Cout is small) receives zeros.
 */
int scc_backward_input(const void* dy, const void* w, void* dx,
                       int N, int Cin, int Cout, int H, int W, int cg, double co,
                       scc_dtype dtype, void* stream);

/*
 * Bytes of device scratch scc_backward_weight needs for this problem (may be 0).
 * Returns 0 as well when the arguments are invalid; scc_backward_weight reports the error.
 */
size_t scc_backward_weight_workspace_bytes(int N, int Cin, int Cout, int H, int W, int cg, double co,
                                           scc_dtype dtype);

/*
 * Gradient with respect to the weights (Section 4.2 names it among the trainable
 * parameters' gradients; it is the derivative of the forward definition):
 *     dw[k,j] = sum_{n,h,w} dy[n,k,h,w] * x[n, (s_k + j) mod Cin, h, w]
 * x: in, N*Cin*H*W.  dy: in, N*Cout*H*W.  dw: out, Cout*L binary32 values (both dtypes).
 * workspace: device scratch of at least scc_backward_weight_workspace_bytes(...) bytes,
 * 256-byte aligned, owned by the caller, contents undefined before and after; may be NULL
 * when the query returns 0.  The reduction order is fixed: two calls on the same inputs
 * give bitwise identical results.
 */
int scc_backward_weight(const void* x, const void* dy, void* dw,
                        int N, int Cin, int Cout, int H, int W, int cg, double co,
                        scc_dtype dtype, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Bytes of device scratch scc_backward needs for this problem (may be 0; 0 as well when the
 * arguments are invalid, scc_backward then reports the error).
 */
size_t scc_backward_workspace_bytes(int N, int Cin, int Cout, int H, int W, int cg, double co,
                                    scc_dtype dtype);

/*
 * Both gradients of one layer in one call (Section 4.2, backward pass: the gradients with respect
 * to the input feature map and to the trainable weights are the two results of a layer's backward
 * step):
 *     dx as scc_backward_input computes it, dw as scc_backward_weight computes it.
 * For fp32 layers whose windows start on multiples of 32 channels and are 64 channels long, with
 * at most 32 filters per window, H*W a multiple of 4 and 16-byte aligned tensors, one kernel reads
 * dy and x from memory once and produces both (a third less memory traffic than the two passes;
 * all products are binary32 products).  Every other layer runs the two passes one after the other.
 * x: in, N*Cin*H*W.  dy: in, N*Cout*H*W.  w: in, Cout*L.  dx: out, N*Cin*H*W.
 * dw: out, Cout*L binary32 values (both dtypes).  workspace: device scratch of at least
 * scc_backward_workspace_bytes(...) bytes, 256-byte aligned, owned by the caller, contents
 * undefined before and after; may be NULL when the query returns 0.  Two calls on the same inputs
 * give bitwise identical results.
 */
int scc_backward(const void* x, const void* dy, const void* w, void* dx, void* dw,
                 int N, int Cin, int Cout, int H, int W, int cg, double co,
                 scc_dtype dtype, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Depthwise 3x3 stage of a DW + SCC block (Eq. 2 of the paper):
 *     z[n,a,m,q] = sum_{i,j in 0..2} kdw[a,i,j] * x[n,a, s*m + i - 1, s*q + j - 1],   s = dw_stride,
 * pixels outside the H x W map counting as zero (the filter is centred on input pixel (s*m, s*q), no
 * flip).  The output map has scc_depthwise3x3_out(H, s) x scc_depthwise3x3_out(W, s) pixels,
 * (size-1)/s + 1 each.  x: in, N*C*H*W.  kdw: in, C*9 values, [C][3][3] row-major, same dtype as x.
 * z: out, N*C*Ho*Wo, same dtype.  Sums are binary32.  Errors: SCC_ERR_NULL, SCC_ERR_SHAPE (a dimension
 * <= 0, dw_stride < 1, a map too large to index), SCC_ERR_DTYPE, SCC_ERR_LAUNCH.
 */
int scc_depthwise3x3_out(int size, int dw_stride);   /* rows (columns) produced, or SCC_ERR_SHAPE */
int scc_depthwise3x3_forward(const void* x, const void* kdw, void* z,
                             int N, int C, int H, int W, int dw_stride, scc_dtype dtype, void* stream);

/*
 * Gradients of the depthwise 3x3 stage (the derivatives of Eq. 2; the paper trains DW + SCC blocks end to end
 * and gives no formula for them).  With dz the gradient of the loss with respect to the stage's output z:
 *     dx[n,a,r,c]   = sum over taps (i,j) and outputs (m,q) with s*m+i-1 = r, s*q+j-1 = c of kdw[a,i,j] * dz[n,a,m,q]
 *     dkdw[a,i,j]   = sum_{n,m,q} dz[n,a,m,q] * x[n,a, s*m+i-1, s*q+j-1]        (pixels outside the map: zero)
 * x: in, N*C*H*W (needed for dkdw).  kdw: in, C*9 (needed for dx).  dz: in, N*C*Ho*Wo.  dx: out, N*C*H*W, dtype of x.
 * dkdw: out, C*9 binary32 values in BOTH dtypes.  Either of dx, dkdw may be NULL: that gradient is skipped (and the
 * input only it needs may be NULL too).  Sums are binary32; dkdw is summed in a fixed order (per thread, per
 * workgroup, then over slices of the batch), so two calls give bitwise identical results.  workspace: device
 * scratch of at least scc_depthwise3x3_backward_workspace_bytes(...) bytes when dkdw is wanted, 256-byte aligned,
 * owned by the caller, contents undefined before and after; may be NULL when the query returns 0.
 * Errors: SCC_ERR_NULL, SCC_ERR_SHAPE, SCC_ERR_DTYPE, SCC_ERR_WORKSPACE, SCC_ERR_LAUNCH.
 */
size_t scc_depthwise3x3_backward_workspace_bytes(int N, int C, int H, int W, int dw_stride, scc_dtype dtype);
int scc_depthwise3x3_backward(const void* x, const void* kdw, const void* dz, void* dx, void* dkdw,
                              int N, int C, int H, int W, int dw_stride, scc_dtype dtype,
                              void* workspace, size_t workspace_bytes, void* stream);

/*
 * Forward of a whole DW + SCC block (Section 3.1: the SCC takes the place of the pointwise convolution
 * behind the depthwise one of Eq. 2):
 *     y = scc_forward(scc_depthwise3x3_forward(x, kdw), w)
 * on the Ho x Wo map the depthwise stage produces.  x: in, N*Cin*H*W.  kdw: in, Cin*9.  w: in, Cout*L.
 * y: out, N*Cout*Ho*Wo.
 * Two paths.  Fused (fp32 layers with Cin a multiple of 16 and at most 1104 channels): one kernel keeps the
 * depthwise output of a tile of pixels for all channels on chip and feeds the SCC from there; x is read
 * once, y written once, the intermediate never reaches memory (and is not rounded to the storage type).
 * Two stages (every layer): scc_depthwise3x3_forward into `workspace`, then scc_forward on it; `workspace`
 * then holds the depthwise output (N*Cin*Ho*Wo values of the dtype).
 * scc_dw_forward_workspace_bytes(...) returns 0 for the layers the library runs fused by its own choice
 * (fusable and at least 16384 output pixels over the batch, where fusing is the faster path) and the size
 * of the depthwise output for all others.  A call with a workspace of at least that size (256-byte aligned,
 * owned by the caller, contents undefined afterwards) takes the path the library prefers.  A call with
 * workspace == NULL runs fused whenever scc_dw_forward_fusable(...) returns 1, also where two stages would
 * be faster, and is refused with SCC_ERR_WORKSPACE otherwise.
 * scc_dw_forward_fusable: 1 or 0, or a negative scc_status for invalid arguments.
 * Errors: as scc_forward and scc_depthwise3x3_forward, SCC_ERR_WORKSPACE.
 */
size_t scc_dw_forward_workspace_bytes(int N, int Cin, int Cout, int H, int W, int dw_stride,
                                      int cg, double co, scc_dtype dtype);
int scc_dw_forward_fusable(int N, int Cin, int Cout, int H, int W, int dw_stride,
                           int cg, double co, scc_dtype dtype);
int scc_dw_forward(const void* x, const void* kdw, const void* w, void* y,
                   int N, int Cin, int Cout, int H, int W, int dw_stride, int cg, double co,
                   scc_dtype dtype, void* workspace, size_t workspace_bytes, void* stream);

/*
 * scc_backward_weight for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels, arithmetic and summation order as scc_backward_weight (results are bitwise
 * equal), but the scratch is a buffer of SCC_STATIC_SCRATCH_BYTES that the library holds in
 * device memory on every GPU it runs on, from load until the process ends.  The call allocates
 * and frees nothing; its first use on a device looks the buffer's address up once (do that
 * before starting a capture), later calls only enqueue kernels.
 * Errors: those of scc_backward_weight, and SCC_ERR_SCRATCH when the problem needs more scratch
 * than the buffer holds (then scc_backward_weight_workspace_bytes(...) > SCC_STATIC_SCRATCH_BYTES;
 * decided on the host, nothing is launched).
 * All calls on one GPU share that GPU's buffer: two calls that may run at the same time there
 * (different streams, or different host threads on different streams) race on it.  Calls ordered
 * on one stream are safe; nothing in the buffer needs to survive or be cleared between calls.
 */
int scc_backward_weight_static(const void* x, const void* dy, void* dw,
                               int N, int Cin, int Cout, int H, int W, int cg, double co,
                               scc_dtype dtype, void* stream);

/* Static, human-readable name of a status code (never NULL). */
const char* scc_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* SCC_H */
