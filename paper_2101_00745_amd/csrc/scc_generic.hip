// Shape-agnostic SCC kernels for gfx950: plain vector-ALU code that is correct for every
// (N, Cin, Cout, HW, cg, co), used for shapes the tiled matrix-core kernels do not take.
//
// A "column" is one (sample, pixel) pair, q = n*HW + p.  Lanes of a wavefront hold 64
// consecutive columns, so global accesses along a channel plane are coalesced whenever
// HW >= 64, and the filter / channel index is uniform across the wavefront: weights are
// fetched through the scalar cache and the cyclic wrap is a scalar compare, not a table.
#include "scc_common.h"

namespace scc {

namespace {

constexpr int kWaves = 4;        // wavefronts per workgroup
constexpr int kRowsPerBlock = 16;  // output rows (filters or channels) one workgroup walks

__device__ __forceinline__ int wave_id() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

// Forward (Section 4.2, output-centric): y[n,k,p] = sum_j w[k,j] * x[n,(s_k+j) mod Cin,p].
template <typename T>
__global__ __launch_bounds__(kWaves * 64) void forward_generic(const T* __restrict__ x, const T* __restrict__ w,
                                                              T* __restrict__ y, Problem P)
{
    const int lane = threadIdx.x & 63;
    const long long q = (long long)blockIdx.x * 64 + lane;
    const bool live = q < P.NQ;
    const long long qc = live ? q : 0;
    const int n = (int)(qc / P.HW), p = (int)(qc % P.HW);
    const T* xcol = x + (long long)n * P.Cin * P.HW + p;
    T* ycol = y + (long long)n * P.Cout * P.HW + p;
    for (int k0 = blockIdx.y * kRowsPerBlock; k0 < P.Cout; k0 += gridDim.y * kRowsPerBlock) {   // grid.y is capped
    const int k_end = min(P.Cout, k0 + kRowsPerBlock);
    for (int k = k0 + wave_id(); k < k_end; k += kWaves) {
        int c = (int)(((long long)k * P.stride) % P.Cin);  // window start, uniform
        const T* wk = w + (long long)k * P.L;
        float acc = 0.f;
        for (int j = 0; j < P.L; ++j) {
            acc = fmaf(to_f32(wk[j]), to_f32(xcol[(long long)c * P.HW]), acc);
            c = (c + 1 == P.Cin) ? 0 : c + 1;
        }
        if (live) ycol[(long long)k * P.HW] = from_f32<T>(acc);
    }
    }
}

// Grad-input (Section 4.2, input-centric): channel c pulls from every filter whose window
// covers it; position of c inside window k is (c - s_k) mod Cin.  No atomics.
template <typename T>
__global__ __launch_bounds__(kWaves * 64) void backward_input_generic(const T* __restrict__ dy, const T* __restrict__ w,
                                                                     T* __restrict__ dx, Problem P)
{
    const int lane = threadIdx.x & 63;
    const long long q = (long long)blockIdx.x * 64 + lane;
    const bool live = q < P.NQ;
    const long long qc = live ? q : 0;
    const int n = (int)(qc / P.HW), p = (int)(qc % P.HW);
    const T* gcol = dy + (long long)n * P.Cout * P.HW + p;
    T* dcol = dx + (long long)n * P.Cin * P.HW + p;
    for (int c0 = blockIdx.y * kRowsPerBlock; c0 < P.Cin; c0 += gridDim.y * kRowsPerBlock) {     // grid.y is capped
    const int c_end = min(P.Cin, c0 + kRowsPerBlock);
    for (int c = c0 + wave_id(); c < c_end; c += kWaves) {
        float acc = 0.f;
        int j = c;  // (c - s_0) mod Cin with s_0 = 0
        for (int k = 0; k < P.Cout; ++k) {
            if (j < P.L) acc = fmaf(to_f32(w[(long long)k * P.L + j]), to_f32(gcol[(long long)k * P.HW]), acc);
            j -= P.stride;  // s_{k+1} = s_k + stride (mod Cin)
            if (j < 0) j += P.Cin;
        }
        if (live) dcol[(long long)c * P.HW] = from_f32<T>(acc);
    }
    }
}

// Grad-weight: dw[k,j] = sum_{n,p} dy[n,k,p] * x[n,(s_k+j) mod Cin,p].  One wavefront per
// weight; lanes stride over the columns, then a fixed-order butterfly over the 64 lanes.
template <typename T>
__global__ __launch_bounds__(kWaves * 64) void backward_weight_generic(const T* __restrict__ x, const T* __restrict__ dy,
                                                                      float* __restrict__ dw, Problem P)
{
    const int lane = threadIdx.x & 63;
    const long long e = (long long)blockIdx.x * kWaves + wave_id();  // flat weight index k*L + j
    if (e >= (long long)P.Cout * P.L) return;
    const int k = (int)(e / P.L), j = (int)(e % P.L);
    const int c = (int)((((long long)k * P.stride) % P.Cin + j) % P.Cin);
    float acc = 0.f;
    for (int n = 0; n < P.N; ++n) {
        const T* g = dy + ((long long)n * P.Cout + k) * P.HW;
        const T* xi = x + ((long long)n * P.Cin + c) * P.HW;
        for (int p = lane; p < P.HW; p += 64) acc = fmaf(to_f32(g[p]), to_f32(xi[p]), acc);
    }
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) dw[e] = acc;
}

inline dim3 column_grid(const Problem& p, int rows)
{
    // grid.y may not exceed 65535: the kernels stride over the row blocks beyond that
    const long long row_blocks = (rows + kRowsPerBlock - 1) / kRowsPerBlock;
    return dim3((unsigned)((p.NQ + 63) / 64), (unsigned)(row_blocks < 65535 ? row_blocks : 65535), 1);
}

}  // namespace

template <typename T>
hipError_t launch_forward_generic(const T* x, const T* w, T* y, const Problem& p, hipStream_t st)
{
    hipLaunchKernelGGL(forward_generic<T>, column_grid(p, p.Cout), dim3(kWaves * 64), 0, st, x, w, y, p);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_backward_input_generic(const T* dy, const T* w, T* dx, const Problem& p, hipStream_t st)
{
    hipLaunchKernelGGL(backward_input_generic<T>, column_grid(p, p.Cin), dim3(kWaves * 64), 0, st, dy, w, dx, p);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_backward_weight_generic(const T* x, const T* dy, float* dw, const Problem& p, hipStream_t st)
{
    const long long weights = (long long)p.Cout * p.L;
    hipLaunchKernelGGL(backward_weight_generic<T>, dim3((unsigned)((weights + kWaves - 1) / kWaves)), dim3(kWaves * 64),
                       0, st, x, dy, dw, p);
    return hipGetLastError();
}

template hipError_t launch_forward_generic<float>(const float*, const float*, float*, const Problem&, hipStream_t);
template hipError_t launch_forward_generic<bf16_t>(const bf16_t*, const bf16_t*, bf16_t*, const Problem&, hipStream_t);
template hipError_t launch_backward_input_generic<float>(const float*, const float*, float*, const Problem&, hipStream_t);
template hipError_t launch_backward_input_generic<bf16_t>(const bf16_t*, const bf16_t*, bf16_t*, const Problem&, hipStream_t);
template hipError_t launch_backward_weight_generic<float>(const float*, const float*, float*, const Problem&, hipStream_t);
template hipError_t launch_backward_weight_generic<bf16_t>(const bf16_t*, const bf16_t*, float*, const Problem&, hipStream_t);

}  // namespace scc
