// Shared declarations of the gfx950 SCC kernels: problem description, storage-type
// conversion, launch prototypes.  Internal to the library (the public C ABI is include/scc.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace scc {

// One SCC layer, as the kernels see it.  Window arithmetic follows Algorithm 1 of the
// paper in closed form: filter k starts at (k * stride) mod Cin and spans L channels.
struct Problem {
    int N, Cin, Cout, HW;
    int L;        // window length Cin / cg
    int stride;   // (L - int(co*L)) mod Cin, in [0, Cin)
    int period;   // distinct window starts over all k >= 0: Cin / gcd(stride, Cin), 1 if stride == 0
    long long NQ; // N * HW: number of (sample, pixel) columns
};

// Geometry of the depthwise 3x3 stage in front of an SCC (Eq. 2): input map H x W, spatial stride s, output map
// Ho x Wo with Ho = (H-1)/s + 1 (taps centred on input pixel (s*m, s*q), zero outside the map).
struct DwGeom {
    int H, W, Ho, Wo, s;
};

typedef uint16_t bf16_t;  // bfloat16 storage: the upper 16 bits of a binary32

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
// round to nearest, ties to even; NaN stays NaN (quiet bit forced)
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v)
{
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// One bf16 matrix instruction over K = 2*KC: each lane passes KC bf16 values (packed in pairs, low half
// first) of its A row and of its B column; lanes 0-31 and 32-63 hold different K values.  KC is 8
// (v_mfma_f32_32x32x16_bf16) or 4 (v_mfma_f32_32x32x8_bf16_1k).  Accumulation is binary32.
template <int KC>
__device__ __forceinline__ float __attribute__((ext_vector_type(16)))
mfma_bf16(const uint32_t (&a)[KC / 2], const uint32_t (&b)[KC / 2], float __attribute__((ext_vector_type(16))) acc)
{
    static_assert(KC == 8 || KC == 4, "a chunk is 8 or 4 K-steps");
    if constexpr (KC == 8) {
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
        const u32x4 av = {a[0], a[1], a[2], a[3]}, bv = {b[0], b[1], b[2], b[3]};
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, bv),
                                                       acc, 0, 0, 0);
    } else {
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        typedef short s16x4 __attribute__((ext_vector_type(4)));
        const u32x2 av = {a[0], a[1]}, bv = {b[0], b[1]};
        return __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(__builtin_bit_cast(s16x4, av), __builtin_bit_cast(s16x4, bv), acc,
                                                        0, 0, 0);
    }
}

// Exact split of KC binary32 values into bf16 pieces: v = hi + mid + lo with hi = v truncated to bf16,
// mid = (v - hi) truncated, lo = v - hi - mid (at most 8 significant bits left, so it is a bf16 value).
// Pieces of values 2e and 2e+1 are packed into one register, low half first, as mfma_bf16 takes them.
// Seven vector instructions per pair of values: a byte permute packs the two upper halves (the truncations),
// and v_dot2c_f32_bf16 (d += a.lo*b.lo + a.hi*b.hi on packed bf16 pairs) with b = (-1, -0) or (-0, -1)
// subtracts one half of the packed pair from the binary32 value it was cut from: an exact subtraction, the
// other half only adds a signed zero.  (The constants carry -0.0 in the unused half so that they are literals:
// as an inline constant -1.0 the operand was observed to reach the wrong half.)
template <int KC, typename F>
__device__ __forceinline__ void split3(F get, uint32_t (&hi)[KC / 2], uint32_t (&mid)[KC / 2], uint32_t (&lo)[KC / 2])
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    const bf16x2 kLow = __builtin_bit_cast(bf16x2, 0x8000bf80u);    // (-1.0, -0.0): minus the value in the low half
    const bf16x2 kHigh = __builtin_bit_cast(bf16x2, 0xbf808000u);   // (-0.0, -1.0): minus the value in the high half
#pragma unroll
    for (int e = 0; e < KC / 2; ++e) {
        const float v0 = get(2 * e), v1 = get(2 * e + 1);
        // upper halves of (x1, x0) side by side: bytes 2,3 of x0 then bytes 2,3 of x1
        hi[e] = __builtin_amdgcn_perm(__float_as_uint(v1), __float_as_uint(v0), 0x07060302u);
        const bf16x2 h2 = __builtin_bit_cast(bf16x2, hi[e]);
        const float r0 = __builtin_amdgcn_fdot2_f32_bf16(h2, kLow, v0, false);
        const float r1 = __builtin_amdgcn_fdot2_f32_bf16(h2, kHigh, v1, false);
        mid[e] = __builtin_amdgcn_perm(__float_as_uint(r1), __float_as_uint(r0), 0x07060302u);
        const bf16x2 m2 = __builtin_bit_cast(bf16x2, mid[e]);
        const float l0 = __builtin_amdgcn_fdot2_f32_bf16(m2, kLow, r0, false);
        const float l1 = __builtin_amdgcn_fdot2_f32_bf16(m2, kHigh, r1, false);
        lo[e] = __builtin_amdgcn_perm(__float_as_uint(l1), __float_as_uint(l0), 0x07060302u);
    }
}

// Generic (any shape) VALU kernels: scc_generic.hip
template <typename T> hipError_t launch_forward_generic(const T* x, const T* w, T* y, const Problem& p, hipStream_t st);
template <typename T> hipError_t launch_backward_input_generic(const T* dy, const T* w, T* dx, const Problem& p, hipStream_t st);
template <typename T> hipError_t launch_backward_weight_generic(const T* x, const T* dy, float* dw, const Problem& p, hipStream_t st);

// Matrix-core kernels: scc_mfma_*.hip
bool forward_mfma_eligible(const Problem& p);
template <typename T> hipError_t launch_forward_mfma(const T* x, const T* w, T* y, const Problem& p, hipStream_t st);
// Forward with the activation operand shared by four tiles through LDS, fp32 (scc_fwd_shared.hip)
bool forward_shared_eligible(const float* x, const float* w, const float* y, const Problem& p);
double forward_shared_gain(const Problem& p);   // channel fetches saved: own spans / shared walks
bool forward_shared_preferred(const float* x, const float* w, const float* y, const Problem& p);   // ... and faster
hipError_t launch_forward_shared(const float* x, const float* w, float* y, const Problem& p, hipStream_t st);
bool backward_input_mfma_eligible(const Problem& p);
template <typename T> hipError_t launch_backward_input_mfma(const T* dy, const T* w, T* dx, const Problem& p, hipStream_t st);
// Grad-input with the dy operand shared by four channel blocks through LDS, fp32 (scc_bwi_shared.hip)
bool backward_input_shared_eligible(const float* dy, const float* dx, const Problem& p);
bool backward_input_shared_preferred(const float* dy, const float* dx, const Problem& p);   // ... and faster
hipError_t launch_backward_input_shared(const float* dy, const float* w, float* dx, const Problem& p, hipStream_t st);
bool backward_weight_mfma_eligible(const Problem& p);
size_t backward_weight_mfma_workspace(const Problem& p);  // bytes of K-split partials (0 when not split)
template <typename T>
hipError_t launch_backward_weight_mfma(const T* x, const T* dy, float* dw, float* workspace, const Problem& p,
                                       hipStream_t st);

// dw[e] = sum over K-splits of part[ks][e], e < count, in a fixed order (scc_mfma_bww.hip)
hipError_t launch_weight_reduce(const float* part, float* dw, int count, int KS, hipStream_t st);

// Fused backward pass, fp32 (scc_lds_bwd.hip): dx and dw from one read of dy and x
bool backward_fused_eligible(const Problem& p);
size_t backward_fused_workspace(const Problem& p);  // bytes of K-split partials (0 when not split)
hipError_t launch_backward_fused(const float* x, const float* dy, const float* w, float* dx, float* dw,
                                 float* workspace, const Problem& p, hipStream_t st);

// Both gradients in one launch, the two matrix-core kernels side by side in one grid (scc_bwd_merged.hip);
// needs the workspace of the grad-weight pass
template <typename T> bool backward_merged_applicable(const T* x, const T* dy, const T* dx, const Problem& p);
template <typename T>
hipError_t launch_backward_merged(const T* x, const T* dy, const T* w, T* dx, float* dw, float* workspace,
                                  const Problem& p, hipStream_t st);

// Depthwise 3x3 stage and the fused DW + SCC forward (scc_dw_fwd.hip); `p` describes the SCC on the Ho x Wo map
// flip: the filters turned by 180 degrees (tap (i, j) takes the weight of tap (2-i, 2-j)): at stride 1 that is the
// stage's gradient with respect to its input, applied to dz
template <typename T>
hipError_t launch_depthwise3x3(const T* x, const T* kdw, T* z, int N, int C, const DwGeom& g, hipStream_t st,
                               bool flip = false);

// Gradients of the depthwise stage (scc_dw_bwd.hip).  dx and dk may each be null (that gradient is skipped).
size_t depthwise3x3_backward_workspace(int N, int C, const DwGeom& g);
template <typename T>
hipError_t launch_depthwise3x3_backward(const T* x, const T* kdw, const T* dz, T* dx, float* dk, float* workspace, int N,
                                        int C, const DwGeom& g, hipStream_t st);
bool dw_forward_fused_eligible(const Problem& p);    // the fused kernel can run the layer
bool dw_forward_fused_preferred(const Problem& p);   // ... and is the faster path for it
hipError_t launch_dw_forward_fused(const float* x, const float* kdw, const float* w, float* y, const Problem& p,
                                   const DwGeom& g, hipStream_t st);

}  // namespace scc
