// Forward SCC on the gfx950 matrix cores (fp32 MFMA, exact fp32 products and sums).
//
// y[n,k,p] = sum_j w[k,j] * x[n,(s_k+j) mod Cin,p]   (Section 4.2, output-centric forward)
// is computed as banded GEMM tiles: a tile of 32 filters (TM adjacent window starts x TI
// filters per start, see scc_band.h) times a span of U = L + g*(TM-1) channels, for 32*CT
// columns (a column is one (sample, pixel) pair).  When TM == 1 the tile is dense.
//
// One wavefront owns one tile.  v_mfma_f32_32x32x2_f32 contracts two K-slots per issue,
// one per half-wave; half h walks the channels lo + h*Uh + t, t = 0..Uh-1, so that a lane's
// successive A values are CONSECUTIVE weights of one filter (16-byte loads straight from
// the weight matrix, which stays L2 resident) and its B values are one channel plane after
// another at a fixed column (each half-wave reads 128 contiguous bytes of the plane).
// The cyclic wrap is a compare-and-subtract on the channel index; nothing is copied.
#include "scc_band.h"
#include "scc_common.h"

namespace scc {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4u __attribute__((ext_vector_type(4), aligned(4)));

struct FwdTiling {
    Band b;
    int TI, TM;    // tile = TM starts x TI filters per start; TI*TM <= 32 (TM is capped by P)
    int IB, MB;    // tiles along i and m
    int Uh;        // K-steps per tile (multiple of 4); each half-wave covers Uh channels
    int NCT;       // column tiles (of 32*CT columns), padded to a multiple of 8
    int FG;        // workgroups per column tile = ceil(IB*MB / 4)
};

template <int CT>
__global__ __launch_bounds__(256) void forward_mfma32(const float* __restrict__ x, const float* __restrict__ w,
                                                      float* __restrict__ y, Problem P, FwdTiling T)
{
    // workgroup -> (column tile, filter-tile group); all groups of a column tile share blockIdx % 8,
    // i.e. one XCD and its L2, because they re-read the same channel planes.
    const int bid = blockIdx.x;
    const int xcd = bid & 7, slot = bid >> 3;
    const int ct = (slot / T.FG) * 8 + xcd;
    const int fg = slot % T.FG;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int tile = fg * 4 + wave;
    if (tile >= T.IB * T.MB || (long long)ct * (32 * CT) >= P.NQ) return;
    const int mb = tile / T.IB, ib = tile % T.IB;

    const int lane = threadIdx.x & 63;
    const int f = lane & 31, h = lane >> 5;

    // ---- A side: this lane's filter -------------------------------------------------------
    const int mi = f / T.TI, ii = f % T.TI;
    const int m = mb * T.TM + mi, i = ib * T.TI + ii;
    const int k = (int)(((long long)m * T.b.inv) % T.b.P) + T.b.P * i;
    const bool fvalid = (mi < T.TM) && (m < T.b.P) && (k < P.Cout);
    const int off = T.b.g * mi;                      // this filter's window starts `off` channels into the span
    const float* wk = w + (long long)(fvalid ? k : 0) * P.L;
    const int lo = T.b.g * mb * T.TM;                // first channel of the span (< Cin)

    // ---- B side: this lane's columns ---------------------------------------------------------
    const float* xcol[CT];
    bool live[CT];
    long long ycol[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) {
        const long long q = ((long long)ct * CT + c) * 32 + f;
        live[c] = q < P.NQ;
        const long long qq = live[c] ? q : 0;
        const int n = (int)(qq / P.HW), p = (int)(qq % P.HW);
        xcol[c] = x + (long long)n * P.Cin * P.HW + p;
        ycol[c] = (long long)n * P.Cout * P.HW + p;
    }
    int ch = (lo + h * T.Uh) % P.Cin;                // channel this half-wave reads at step 0
    int jj = h * T.Uh - off;                         // weight index of this lane at step 0

    f32x16 acc[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;

    for (int t = 0; t < T.Uh; t += 4) {
        float a[4];
        if (fvalid && jj >= 0 && jj + 3 < P.L) {
            const f32x4u a4 = *(const f32x4u*)(wk + jj);
            a[0] = a4[0]; a[1] = a4[1]; a[2] = a4[2]; a[3] = a4[3];
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int j = jj + s;
                a[s] = (fvalid && j >= 0 && j < P.L) ? wk[j] : 0.f;
            }
        }
        float b[4][CT];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const long long roff = (long long)ch * P.HW;
#pragma unroll
            for (int c = 0; c < CT; ++c) b[s][c] = xcol[c][roff];
            ch = (ch + 1 == P.Cin) ? 0 : ch + 1;
        }
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int c = 0; c < CT; ++c)
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], b[s][c], acc[c], 0, 0, 0);
        jj += 4;
    }

    // ---- store: register v of the accumulator holds tile row 8*(v/4) + 4*h + v%4, column f ----
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int fr = 8 * (v >> 2) + 4 * h + (v & 3);
        const int mr = mb * T.TM + fr / T.TI, ir = ib * T.TI + fr % T.TI;
        const int kr = (int)(((long long)mr * T.b.inv) % T.b.P) + T.b.P * ir;
        if (fr / T.TI < T.TM && mr < T.b.P && kr < P.Cout) {
#pragma unroll
            for (int c = 0; c < CT; ++c)
                if (live[c]) y[ycol[c] + (long long)kr * P.HW] = acc[c][v];
        }
    }
}

int pow2_floor(int v)
{
    int p = 1;
    while (p * 2 <= v) p *= 2;
    return p;
}

}  // namespace

// Whether the matrix-core forward takes this problem (otherwise the generic kernel does).
bool forward_mfma_eligible(const Problem& p)
{
    // enough contraction depth and columns for a 32x32 tile to pay; everything else is exact for any shape
    return p.L >= 8 && p.NQ >= 64 && p.Cout >= 8;
}

hipError_t launch_forward_mfma(const float* x, const float* w, float* y, const Problem& p, hipStream_t st)
{
    constexpr int CT = 2;
    FwdTiling t;
    t.b = make_band(p);
    t.TI = pow2_floor(t.b.F < 32 ? t.b.F : 32);
    t.TM = 32 / t.TI < t.b.P ? 32 / t.TI : t.b.P;
    t.IB = (t.b.F + t.TI - 1) / t.TI;
    t.MB = (t.b.P + t.TM - 1) / t.TM;
    const int U = p.L + t.b.g * (t.TM - 1);
    t.Uh = (((U + 1) / 2) + 3) / 4 * 4;
    const long long nct = (p.NQ + 32 * CT - 1) / (32 * CT);
    t.NCT = (int)((nct + 7) / 8 * 8);
    t.FG = (t.IB * t.MB + 3) / 4;
    const long long blocks = (long long)t.NCT * t.FG;
    hipLaunchKernelGGL(forward_mfma32<CT>, dim3((unsigned)blocks), dim3(256), 0, st, x, w, y, p, t);
    return hipGetLastError();
}

}  // namespace scc
