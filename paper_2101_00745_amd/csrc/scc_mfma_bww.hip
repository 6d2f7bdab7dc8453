// Grad-weight of SCC on the gfx950 matrix cores with a fixed-order reduction: fp32 MFMA for fp32
// tensors, bf16 MFMA (exact products, fp32 accumulation) for bf16 tensors.
//
// dw[k,j] = sum_{n,p} dy[n,k,p] * x[n,(s_k+j) mod Cin,p]     (the derivative of the forward
// definition with respect to w; Section 4.2 lists it among the backward work without
// describing a kernel).
//
// Per tile of 32 filters (TM window starts x TI filters per start, see scc_band.h) and a chunk
// of 64 span positions u (channel (lo+u) mod Cin), the product D[f][u] = sum_q dy[q,k_f]*x[q,ch(u)]
// is a GEMM whose contraction runs over the columns q = (n,p).  Both operands are contiguous
// along p in memory while a lane of the MFMA operand wants successive K values of ONE row, so
// the rows go through LDS: a wavefront reads 32 columns of its 96 operand rows (32 dy rows,
// 64 x rows) with fully coalesced 16-byte loads (8 rows x 128 bytes per instruction), parks
// them in a private, padded LDS block and reads them back in operand layout.  The global loads
// of the next 32 columns are in flight while the matrix instructions of the current ones issue.
//
// bf16 rows are parked as stored (2 bytes per column); a 16-byte LDS read then is one lane's 8 consecutive
// K values of v_mfma_f32_32x32x16_bf16, so 32 columns take 2 matrix instructions per tile instead of 16.
//
// The columns are split over workgroups (K-split) and again over the 4 wavefronts of a
// workgroup.  Wavefront partials are summed through LDS in wave order, workgroup partials go to
// the workspace in the layout of dw and a second kernel sums them in split order: no atomics,
// bitwise reproducible.
#include "scc_mfma_bww_kernel.h"

namespace scc {

namespace {

using namespace bww;

template <typename T_, int kPosTiles, bool VEC>
__global__ __launch_bounds__(kWaves * 64) void backward_weight_mfma32(const T_* __restrict__ x,
                                                                      const T_* __restrict__ dy,
                                                                      float* __restrict__ out, Problem P, BwwTiling T)
{
    backward_weight_body<T_, kPosTiles, VEC>(x, dy, out, P, T, (int)blockIdx.x);
}

// dw[e] = sum over K-splits of part[ks][e].  A workgroup owns 64 weights; its 4 wavefronts take the
// splits ks = w, w+4, ... (all loads of a thread are independent and in flight together), then the
// four sums are added in wavefront order: the summation tree is fixed, so results are reproducible.
__global__ __launch_bounds__(256) void backward_weight_reduce(const float* __restrict__ part, float* __restrict__ dw,
                                                              int count, int KS)
{
    __shared__ float sums[4][64];
    const int el = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int e = blockIdx.x * 64 + el;
    float s = 0.f;
    if (e < count) {
        int ks = w;
        for (; ks + 28 < KS; ks += 32) {      // 8 loads in flight per trip
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = part[(size_t)(ks + 4 * u) * count + e];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += v[u];
        }
        for (; ks < KS; ks += 4) s += part[(size_t)ks * count + e];
    }
    sums[w][el] = s;
    __syncthreads();
    if (w == 0 && e < count) dw[e] = ((sums[0][el] + sums[1][el]) + sums[2][el]) + sums[3][el];
}

template <typename T_, int NPT, bool VEC>
hipError_t launch_tile(dim3 grid, dim3 block, hipStream_t st, const T_* x, const T_* dy, float* out, const Problem& p,
                       const BwwTiling& t)
{
    constexpr size_t kLds = lds_bytes_of(NPT, (int)sizeof(T_));
    if (kLds > 64 * 1024) {
        // more than 64 KiB of LDS per workgroup has to be allowed once (per process: the library drives one GPU)
        static const hipError_t allowed = hipFuncSetAttribute((const void*)backward_weight_mfma32<T_, NPT, VEC>,
                                                              hipFuncAttributeMaxDynamicSharedMemorySize,
                                                              (int)kLds);
        if (allowed != hipSuccess) return allowed;
    }
    backward_weight_mfma32<T_, NPT, VEC><<<grid, block, kLds, st>>>(x, dy, out, p, t);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_weight_reduce(const float* part, float* dw, int count, int KS, hipStream_t st)
{
    backward_weight_reduce<<<dim3((unsigned)((count + 63) / 64)), dim3(256), 0, st>>>(part, dw, count, KS);
    return hipGetLastError();
}

bool backward_weight_mfma_eligible(const Problem& p)
{
    const long long rows = p.Cin > p.Cout ? p.Cin : p.Cout;
    return p.L >= 8 && p.NQ >= 256 && p.Cout >= 8 && p.Cin < 65536 &&
           (long long)p.NQ * rows * 4 < (1ll << 32) && (long long)p.Cout * p.L * 4 < (1ll << 31);
}

size_t backward_weight_mfma_workspace(const Problem& p)
{
    const BwwTiling t = make_tiling(p);
    return t.KS > 1 ? (size_t)t.KS * p.Cout * p.L * sizeof(float) : 0;
}

template <typename T_>
hipError_t launch_backward_weight_mfma(const T_* x, const T_* dy, float* dw, float* workspace, const Problem& p,
                                       hipStream_t st)
{
    const BwwTiling t = make_tiling(p);
    const long long blocks = (long long)8 * t.chunk;
    float* out = t.KS > 1 ? workspace : dw;
    const dim3 grid((unsigned)blocks), block(kWaves * 64);
    hipError_t e = hipSuccess;
    // vector loads of 4 columns need planes whose size is a multiple of 4 and tensors aligned to 4 elements
    const bool vec = p.HW % 4 == 0 && (((uintptr_t)x | (uintptr_t)dy) & (4 * sizeof(T_) - 1)) == 0;
    if (t.NPT == 1)
        e = vec ? launch_tile<T_, 1, true>(grid, block, st, x, dy, out, p, t)
                : launch_tile<T_, 1, false>(grid, block, st, x, dy, out, p, t);
    else if (t.NPT == 2)
        e = vec ? launch_tile<T_, 2, true>(grid, block, st, x, dy, out, p, t)
                : launch_tile<T_, 2, false>(grid, block, st, x, dy, out, p, t);
    else
        e = vec ? launch_tile<T_, 3, true>(grid, block, st, x, dy, out, p, t)
                : launch_tile<T_, 3, false>(grid, block, st, x, dy, out, p, t);
    if (e != hipSuccess) return e;
    e = hipGetLastError();
    if (e != hipSuccess || t.KS == 1) return e;
    return launch_weight_reduce(workspace, dw, p.Cout * p.L, t.KS, st);
}

template hipError_t launch_backward_weight_mfma<float>(const float*, const float*, float*, float*, const Problem&,
                                                       hipStream_t);
template hipError_t launch_backward_weight_mfma<bf16_t>(const bf16_t*, const bf16_t*, float*, float*, const Problem&,
                                                        hipStream_t);

}  // namespace scc
