// Strips of the depthwise 3x3 stage (Eq. 2 of the paper): the unit of work of the stand-alone stage, of the fused
// DW + SCC forward and of the stage's gradients.
#pragma once
#include "scc_common.h"

namespace scc {

namespace dw {

// The nine taps of channel a's filter as binary32, tap t of the result taking weight 8 - t when `flip` is set (the
// filter turned by 180 degrees).  A vector memory instruction costs the same address-processing time whatever
// its width, and the taps are a third to a half of a strip's instructions: binary32 taps are fetched with two
// 16-byte loads and one 4-byte load (the address is only 4-byte aligned, which global loads allow).
template <typename T_>
__device__ __forceinline__ void load_taps(const T_* kdw, int a, bool flip, float (&k)[9])
{
    float raw[9];
    if constexpr (sizeof(T_) == 4) {
        typedef float f32x4u __attribute__((ext_vector_type(4), aligned(4)));
        const float* src = (const float*)kdw + a * 9;
        const f32x4u lo = *(const f32x4u*)src, hi = *(const f32x4u*)(src + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            raw[i] = lo[i];
            raw[4 + i] = hi[i];
        }
        raw[8] = src[8];
    } else {
#pragma unroll
        for (int i = 0; i < 9; ++i) raw[i] = to_f32(kdw[a * 9 + i]);
    }
#pragma unroll
    for (int i = 0; i < 9; ++i) k[i] = flip ? raw[8 - i] : raw[i];
}

// Input rows of a strip: RB consecutive output rows x 4 consecutive output columns of one channel at spatial stride
// S (1 or 2) need NR = S*(RB-1)+3 input rows of 4*S+2 pixels each; pixel e of row t is input pixel
// (S*r0 - 1 + t, S*cw - 1 + e).  Each row is read once: 4*S pixels from the strip's first input column on (one or
// two 16-byte loads for binary32); the pixel left of them and, for S == 1, the pixel right of them are the last
// and first pixel of what the NEIGHBOURING LANES loaded for the same row: lane l-1 must own the strip to the left and
// lane l+1 the strip to the right (same channel, same rows) whenever `left` / `right` is set and `lo` / `hi` is
// not; they are fetched with a lane shuffle (single misaligned 4-byte loads measured 40 % of the whole stage).
//   xc       input pixel (S*r0, S*cw) of the channel: centre of the strip's first output
//   W        pixels per input row
//   rowmask  bit t set: input row S*r0 - 1 + t lies inside the map (bit 1 always is)
//   left     the input column left of the strip exists; right (S == 1): the column right of it exists
//   lo, hi   the lane has no lane below / above it in the wavefront that owns the neighbouring strip: it loads
//            the edge pixel itself
// Rows and columns outside the map are read at an address inside it and replaced by zero.  Every lane of the
// wavefront must call this together (the shuffles are wavefront-wide).
template <int S, typename T_>
__device__ __forceinline__ void strip_row(const T_* xc, int W, int t, uint32_t rowmask, bool left, bool right, bool lo,
                                          bool hi, float (&v)[4 * S + 2])
{
    typedef T_ tvec __attribute__((ext_vector_type(4)));
    const bool ok = (rowmask >> t) & 1u;
    const T_* row = ok ? xc + (t - 1) * W : xc;
    float raw[4 * S];
#pragma unroll
    for (int h = 0; h < S; ++h) {
        const tvec m = *(const tvec*)(row + 4 * h);
#pragma unroll
        for (int e = 0; e < 4; ++e) raw[4 * h + e] = to_f32(m[e]);
    }
    float lv = __shfl_up(raw[4 * S - 1], 1, 64);
    if (lo && left) lv = to_f32(row[-1]);
    v[0] = (ok && left) ? lv : 0.f;
#pragma unroll
    for (int e = 0; e < 4 * S; ++e) v[1 + e] = ok ? raw[e] : 0.f;
    if constexpr (S == 1) {
        float rv = __shfl_down(raw[0], 1, 64);
        if (hi && right) rv = to_f32(row[4]);
        v[5] = (ok && right) ? rv : 0.f;
    } else {
        v[4 * S + 1] = 0.f;   // never used: the last tap of the last output reads v[S*3 + 2] = v[8]
    }
}

// The strip's outputs: out[rr][i] = sum over taps (di, dj) of k[di*3 + dj] * pixel (S*rr + di, S*i + dj) of the rows above.
template <int S, int RB, typename T_>
__device__ __forceinline__ void dw_strip(const T_* xc, int W, const float (&k)[9], uint32_t rowmask, bool left, bool right,
                                         bool lo, bool hi, float (&out)[RB][4])
{
    constexpr int NR = S * (RB - 1) + 3;
#pragma unroll
    for (int rr = 0; rr < RB; ++rr)
#pragma unroll
        for (int i = 0; i < 4; ++i) out[rr][i] = 0.f;
#pragma unroll
    for (int t = 0; t < NR; ++t) {
        float v[4 * S + 2];
        strip_row<S>(xc, W, t, rowmask, left, right, lo, hi, v);
#pragma unroll
        for (int rr = 0; rr < RB; ++rr) {
            const int di = t - S * rr;   // tap row of output row rr that this input row feeds
            if (di < 0 || di > 2) continue;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 3; ++j) out[rr][i] += k[di * 3 + j] * v[S * i + j];
        }
    }
}

// Input rows a strip of output rows [r0, r0 + RB) has inside the map, as the mask strip_row takes.
template <int S, int RB>
__device__ __forceinline__ uint32_t strip_rowmask(int r0, int Ho)
{
    uint32_t m = (1u << (S * (RB - 1) + 3)) - 1;
    if (r0 == 0) m &= ~1u;
    if (S == 1 && r0 + RB == Ho) m &= ~(1u << (RB + 1));
    return m;
}

}  // namespace dw

}  // namespace scc
