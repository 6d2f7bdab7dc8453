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

// Generic (any shape) VALU kernels: scc_generic.hip
template <typename T> hipError_t launch_forward_generic(const T* x, const T* w, T* y, const Problem& p, hipStream_t st);
template <typename T> hipError_t launch_backward_input_generic(const T* dy, const T* w, T* dx, const Problem& p, hipStream_t st);
template <typename T> hipError_t launch_backward_weight_generic(const T* x, const T* dy, float* dw, const Problem& p, hipStream_t st);

// Matrix-core (fp32 MFMA) kernels: scc_mfma_*.hip
bool forward_mfma_eligible(const Problem& p);
template <typename T> hipError_t launch_forward_mfma(const T* x, const T* w, T* y, const Problem& p, hipStream_t st);
bool backward_input_mfma_eligible(const Problem& p);
template <typename T> hipError_t launch_backward_input_mfma(const T* dy, const T* w, T* dx, const Problem& p, hipStream_t st);
bool backward_weight_mfma_eligible(const Problem& p);
size_t backward_weight_mfma_workspace(const Problem& p);  // bytes of K-split partials (0 when not split)
template <typename T>
hipError_t launch_backward_weight_mfma(const T* x, const T* dy, float* dw, float* workspace, const Problem& p,
                                       hipStream_t st);

}  // namespace scc
