// Grad-input of SCC on the gfx950 matrix cores (bf16 matrix instructions with fp32 sums: directly for bf16
// tensors, on an exact three-way bf16 split of each value for fp32 tensors), as a per-input-channel gather.
//
// dx[n,c,p] = sum over filters k whose window covers c of w[k,(c-s_k) mod Cin] * dy[n,k,p]
// (Section 4.2, input-centric backward: every input-gradient element PULLS from the filters
// covering its channel, so nothing is accumulated with atomics).
//
// A tile is 32 consecutive input channels c0..c0+31 times 32*CT columns.  The filters that can
// cover any of those channels are the ones whose window start s lies in (c0-L, c0+31] on the
// channel circle; starts are the multiples g*m (see scc_band.h), so the contraction runs over
// the grid (mm, i): window m = mlo+mm, i-th filter of that window, k = r(m) + P*i.  The A
// operand of a K-slot is row k of the weight matrix read at consecutive positions by
// consecutive channels (one coalesced 128-byte read per half-wave), zero where the window
// does not reach the channel; the B operand is the plane dy[n,k,:].
#include "scc_mfma_bwi_kernel.h"

namespace scc {

namespace {

template <typename T_, int CT, int KC, bool VEC, int S, int WPB>
__global__ __launch_bounds__(WPB * 64) void backward_input_mfma32(const T_* __restrict__ dy, const T_* __restrict__ w,
                                                             T_* __restrict__ dx, Problem P, bwi::BwiTiling T)
{
    bwi::backward_input_body<T_, CT, KC, VEC, S, WPB>(dy, w, dx, P, T, (int)blockIdx.x);
}

}  // namespace

bool backward_input_mfma_eligible(const Problem& p)
{
    const long long rows = p.Cin > p.Cout ? p.Cin : p.Cout;
    // (window, filter) slots of one block, (L+30)/g + 1 windows at most, must fit an int
    const Band b = make_band(p);
    if (((long long)(p.L + 30) / b.g + 1) * b.F > (1 << 28)) return false;
    return p.L >= 8 && p.NQ >= 64 && p.Cin >= 8 && p.Cin < 65536 && (long long)p.NQ * rows * 4 < (1ll << 32) &&
           (long long)p.Cout * p.L * 4 < (1ll << 31);
}

template <typename T_>
hipError_t launch_backward_input_mfma(const T_* dy, const T_* w, T_* dx, const Problem& p, hipStream_t st)
{
    if constexpr (sizeof(T_) == 4) {
        if (backward_input_shared_preferred((const float*)dy, (const float*)dx, p))
            return launch_backward_input_shared((const float*)dy, (const float*)w, (float*)dx, p, st);
    }
    bwi::select_backward_input(dy, dx, p, [&](auto ct, auto vec, auto s, auto wpb, const bwi::BwiTiling& t, long long blocks) {
        constexpr int CT = decltype(ct)::value, S = decltype(s)::value, WPB = decltype(wpb)::value;
        constexpr bool VEC = decltype(vec)::value;
        backward_input_mfma32<T_, CT, 8, VEC, S, WPB><<<dim3((unsigned)blocks), dim3(WPB * 64), 0, st>>>(dy, w, dx, p, t);
    });
    return hipGetLastError();
}

template hipError_t launch_backward_input_mfma<float>(const float*, const float*, float*, const Problem&, hipStream_t);
template hipError_t launch_backward_input_mfma<bf16_t>(const bf16_t*, const bf16_t*, bf16_t*, const Problem&, hipStream_t);

}  // namespace scc
