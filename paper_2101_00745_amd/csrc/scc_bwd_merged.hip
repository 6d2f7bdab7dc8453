// Both gradients of one SCC layer in ONE launch, for the layers the fused backward kernel (scc_lds_bwd.hip) does
// not take: the workgroups of the grad-weight kernel (scc_mfma_bww_kernel.h) and those of the grad-input kernel
// (scc_mfma_bwi_kernel.h) are two ranges of one grid and run side by side.
//
//   dx[n,c,p] = sum over filters k covering c of w[k,(c-s_k) mod Cin] * dy[n,k,p]    (Section 4.2, input-centric)
//   dw[k,j]   = sum_{n,p} dy[n,k,p] * x[n,(s_k+j) mod Cin,p]
//
// Nothing about either computation changes: same tiles, same arithmetic, same summation order, so the results
// are bitwise those of the two separate passes (one exception: a split of the columns into only two slices is
// dropped here, see bww::make_tiling, so dw is then one summation chain instead of two).  What changes is time: one launch instead of two, no drained
// chip between them, and on layers with few columns (where each pass alone leaves most of the chip waiting on
// latencies) the two passes overlap.  The grad-weight range comes first in the grid (its partial sums still have
// to be reduced by a second kernel, so it should not finish last); both ranges are a multiple of 8 workgroups,
// which keeps workgroup index mod 8 = XCD true inside each of them.
#include "scc_mfma_bwi_kernel.h"
#include "scc_mfma_bww_kernel.h"

namespace scc {

namespace {

template <typename T_, int CT, bool VEC, int S, int NPT>
__global__ __launch_bounds__(256) void backward_merged(const T_* __restrict__ x, const T_* __restrict__ dy,
                                                       const T_* __restrict__ w, T_* __restrict__ dx,
                                                       float* __restrict__ out, Problem P, bwi::BwiTiling TI,
                                                       bww::BwwTiling TW, int nbww)
{
    // the dynamic LDS is the grad-weight range's staging area; the grad-input range, which a workgroup never is at
    // the same time, adds its shared tiles' partial sums in it
    extern __shared__ __attribute__((aligned(16))) float lds_dyn[];
    const int bid = (int)blockIdx.x;
    if (bid < nbww)
        bww::backward_weight_body<T_, NPT, true>(x, dy, out, P, TW, bid);
    else
        bwi::backward_input_body<T_, CT, 8, VEC, S, 4, true>(dy, w, dx, P, TI, bid - nbww, lds_dyn);
}

template <typename T_, int CT, bool VEC, int S, int NPT>
hipError_t launch_variant(const T_* x, const T_* dy, const T_* w, T_* dx, float* out, const Problem& p,
                          const bwi::BwiTiling& ti, long long nbwi, const bww::BwwTiling& tw, hipStream_t st)
{
    constexpr size_t kNeedW = bww::lds_bytes_of(NPT, (int)sizeof(T_)), kNeedI = bwi::reduce_bytes<CT, S, 4>();
    constexpr size_t kLds = kNeedW > kNeedI ? kNeedW : kNeedI;
    if (kLds > 48 * 1024) {
        // more than 64 KiB of LDS per workgroup has to be allowed once
        static const hipError_t allowed = hipFuncSetAttribute((const void*)backward_merged<T_, CT, VEC, S, NPT>,
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLds);
        if (allowed != hipSuccess) return allowed;
    }
    const long long nbww = (long long)8 * tw.chunk;
    backward_merged<T_, CT, VEC, S, NPT><<<dim3((unsigned)(nbww + nbwi)), dim3(256), kLds, st>>>(x, dy, w, dx, out, p, ti,
                                                                                               tw, (int)nbww);
    return hipGetLastError();
}

}  // namespace

// Layers the merged launch takes: both passes on the matrix-core kernels, 4 columns of a plane loadable as a vector
// (planes that are a multiple of 4 pixels, tensors aligned to 4 values) and the grad-input variant with 4 wavefronts
// per workgroup (the 8-wavefront variant is for grids the fused backward kernel takes anyway).
template <typename T_>
bool backward_merged_applicable(const T_* x, const T_* dy, const T_* dx, const Problem& p)
{
    if (!backward_input_mfma_eligible(p) || !backward_weight_mfma_eligible(p)) return false;
    if (p.HW % 4 != 0 || (((uintptr_t)x | (uintptr_t)dy) & (4 * sizeof(T_) - 1)) != 0) return false;
    bool four = false;
    bwi::select_backward_input(dy, dx, p, [&](auto, auto, auto, auto wpb, const bwi::BwiTiling&, long long) {
        four = decltype(wpb)::value == 4;
    });
    return four && (long long)8 * bww::make_tiling(p, true).chunk < (1ll << 30);
}

template <typename T_>
hipError_t launch_backward_merged(const T_* x, const T_* dy, const T_* w, T_* dx, float* dw, float* workspace,
                                  const Problem& p, hipStream_t st)
{
    const bww::BwwTiling tw = bww::make_tiling(p, true);
    float* out = tw.KS > 1 ? workspace : dw;
    hipError_t e = hipErrorInvalidValue;
    bwi::select_backward_input(dy, dx, p, [&](auto ct, auto vec, auto s, auto wpb, const bwi::BwiTiling& ti, long long nbwi) {
        constexpr int CT = decltype(ct)::value, S = decltype(s)::value, WPB = decltype(wpb)::value;
        constexpr bool VEC = decltype(vec)::value;
        if constexpr (WPB == 4) {
            if (tw.NPT == 1)
                e = launch_variant<T_, CT, VEC, S, 1>(x, dy, w, dx, out, p, ti, nbwi, tw, st);
            else if (tw.NPT == 2)
                e = launch_variant<T_, CT, VEC, S, 2>(x, dy, w, dx, out, p, ti, nbwi, tw, st);
            else
                e = launch_variant<T_, CT, VEC, S, 3>(x, dy, w, dx, out, p, ti, nbwi, tw, st);
        }
    });
    if (e != hipSuccess || tw.KS == 1) return e;
    return launch_weight_reduce(workspace, dw, p.Cout * p.L, tw.KS, st);
}

template bool backward_merged_applicable<float>(const float*, const float*, const float*, const Problem&);
template bool backward_merged_applicable<bf16_t>(const bf16_t*, const bf16_t*, const bf16_t*, const Problem&);
template hipError_t launch_backward_merged<float>(const float*, const float*, const float*, float*, float*, float*,
                                                  const Problem&, hipStream_t);
template hipError_t launch_backward_merged<bf16_t>(const bf16_t*, const bf16_t*, const bf16_t*, bf16_t*, float*, float*,
                                                   const Problem&, hipStream_t);

}  // namespace scc
