// Grad-weight of SCC on the gfx950 matrix cores (fp32 MFMA) with a fixed-order reduction.
//
// dw[k,j] = sum_{n,p} dy[n,k,p] * x[n,(s_k+j) mod Cin,p]     (the derivative of the forward
// definition with respect to w; Section 4.2 lists it among the backward work without
// describing a kernel).
//
// Per tile of 32 filters (TM window starts x TI filters per start, see scc_band.h) and a chunk
// of 64 span positions u (channel (lo+u) mod Cin), the product D[f][u] = sum_q dy[q,k_f]*x[q,ch(u)]
// is a GEMM whose contraction runs over the columns q = (n,p).  Both operands are contiguous
// along p, which is what a lane of the A/B operand wants: each lane reads 16 bytes (4 pixels)
// of its own row per load, the two half-waves take alternate 16-byte groups, so one plane
// line is consumed by four back-to-back loads.
//
// The columns are split over workgroups (K-split) and again over the 8 wavefronts of a
// workgroup.  Wavefront partials are summed through LDS in wave order, workgroup partials go to
// the workspace in the layout of dw and a second kernel sums them in split order: no atomics,
// bitwise reproducible.
#include "scc_band.h"
#include "scc_common.h"

namespace scc {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 8;   // wavefronts per workgroup
constexpr int kPosTiles = 2;  // span positions per wavefront tile = 32 * kPosTiles
constexpr int kG = 4;       // 16-byte groups per operand row per pipelined chunk (one 128-byte line per row)

struct BwwTiling {
    Band b;
    int TI, TM;   // tile = TM starts x TI filters per start
    int IB, MB;   // tiles along i and m
    int U;        // span positions of a tile: L + g*(TM-1)
    int NSC;      // span chunks of 64 positions
    int KS;       // K-splits (workgroups per tile and span chunk)
    int NQ4;      // groups of 4 consecutive columns: N*HW/4
};

__device__ __forceinline__ void tile_filter(const BwwTiling& T, const Problem& P, int mb, int ib, int f, int& k,
                                            int& off, bool& valid)
{
    const int mi = f / T.TI, ii = f % T.TI;
    const int m = mb * T.TM + mi, i = ib * T.TI + ii;
    k = (int)(((uint32_t)m * (uint32_t)T.b.inv) % (uint32_t)T.b.P) + T.b.P * i;
    valid = (mi < T.TM) && (m < T.b.P) && (k < P.Cout);
    off = T.b.g * mi;
}

__global__ __launch_bounds__(kWaves * 64) void backward_weight_mfma32(const float* __restrict__ x,
                                                                      const float* __restrict__ dy,
                                                                      float* __restrict__ out, Problem P, BwwTiling T)
{
    __shared__ float red[kWaves][32][32 * kPosTiles];

    // workgroup -> (K-split, tile, span chunk); workgroups of one K-split share blockIdx % 8, i.e. an
    // XCD and its L2: they read the same dy columns and overlapping x windows at about the same time.
    const int ntile = T.IB * T.MB * T.NSC;
    const int bid = blockIdx.x;
    const int xcd = bid & 7, slot = bid >> 3;
    const int ks = (slot / ntile) * 8 + xcd;
    const int tix = slot % ntile;
    if (ks >= T.KS) return;   // whole workgroup leaves: no barrier is reached by anyone
    const int sc = tix % T.NSC, tile = tix / T.NSC;
    const int mb = tile / T.IB, ib = tile % T.IB;

    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = threadIdx.x & 63;
    const int f = lane & 31, h = lane >> 5;

    int k, off;
    bool fvalid;
    tile_filter(T, P, mb, ib, f, k, off, fvalid);
    const int lo = T.b.g * mb * T.TM;

    // operand rows of this lane: A = dy row k; B[c] = x row of span position sc*64 + c*32 + f
    const uint32_t plane = (uint32_t)P.HW * 4u;
    const uint32_t rowA = (uint32_t)(fvalid ? k : 0) * plane;
    uint32_t rowB[kPosTiles];
#pragma unroll
    for (int c = 0; c < kPosTiles; ++c)
        rowB[c] = (uint32_t)((lo + sc * (32 * kPosTiles) + c * 32 + f) % P.Cin) * plane;

    // column groups [qb, qe) of this wavefront: the K-split's share, split again over the waves
    const long long per_ks = ((long long)T.NQ4 + T.KS - 1) / T.KS;
    const long long ks_b = (long long)ks * per_ks;
    const long long ks_e = ks_b + per_ks < T.NQ4 ? ks_b + per_ks : T.NQ4;
    const long long span = ks_e > ks_b ? ks_e - ks_b : 0;
    const long long per_w = (span + kWaves - 1) / kWaves;
    const int qb = (int)(ks_b + (long long)wave * per_w);
    const int qe = (int)((ks_b + (long long)(wave + 1) * per_w) < ks_e ? (ks_b + (long long)(wave + 1) * per_w) : ks_e);

    // this half-wave takes groups qb + h, qb + h + 2, ...
    int qg = qb + h;
    const uint32_t col = (uint32_t)qg * 4u;                      // first column of the group
    uint32_t n = col / (uint32_t)P.HW, p = col % (uint32_t)P.HW;
    uint32_t offA = (n * (uint32_t)P.Cout * (uint32_t)P.HW + p) * 4u;   // without the row
    uint32_t offB = (n * (uint32_t)P.Cin * (uint32_t)P.HW + p) * 4u;
    const uint32_t dn = 8u / (uint32_t)P.HW, dp = 8u % (uint32_t)P.HW;    // advance of 8 columns
    const uint32_t stepA = (dn * (uint32_t)P.Cout * (uint32_t)P.HW + dp) * 4u;
    const uint32_t stepB = (dn * (uint32_t)P.Cin * (uint32_t)P.HW + dp) * 4u;
    const uint32_t wrapA = ((uint32_t)P.Cout - 1u) * plane, wrapB = ((uint32_t)P.Cin - 1u) * plane;
    const char* ab = (const char*)dy;
    const char* bb = (const char*)x;

    f32x16 acc[kPosTiles];
#pragma unroll
    for (int c = 0; c < kPosTiles; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;

    auto load_chunk = [&](f32x4 (&ad)[kG], f32x4 (&bd)[kG][kPosTiles], uint32_t& vm) {
        vm = 0;
#pragma unroll
        for (int s = 0; s < kG; ++s) {
            const bool in = qg < qe;
            vm |= in ? (1u << s) : 0u;
            ad[s] = *(const f32x4*)(ab + (in ? offA + rowA : 0u));
#pragma unroll
            for (int c = 0; c < kPosTiles; ++c) bd[s][c] = *(const f32x4*)(bb + (in ? offB + rowB[c] : 0u));
            qg += 2;
            p += dp;
            const bool wr = p >= (uint32_t)P.HW;       // crossed into the next sample
            p -= wr ? (uint32_t)P.HW : 0u;
            offA += stepA + (wr ? wrapA : 0u);
            offB += stepB + (wr ? wrapB : 0u);
        }
    };
    auto mma_chunk = [&](const f32x4 (&as)[kG], const f32x4 (&bs)[kG][kPosTiles], uint32_t vm) {
#pragma unroll
        for (int s = 0; s < kG; ++s) {
            const bool in = (vm >> s) & 1u;          // a group past the end of the range contributes 0 * 0
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float av = in ? as[s][e] : 0.f;
#pragma unroll
                for (int c = 0; c < kPosTiles; ++c)
                    acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, in ? bs[s][c][e] : 0.f, acc[c], 0, 0, 0);
            }
        }
    };

    // each chunk covers 2*kG column groups; an even number of chunks, software pipelined
    const int groups = qe > qb ? qe - qb : 0;
    const int nch = ((groups + 2 * kG - 1) / (2 * kG) + 1) / 2 * 2;
    if (nch > 0) {
        f32x4 a0[kG], a1[kG], b0[kG][kPosTiles], b1[kG][kPosTiles];
        uint32_t v0, v1;
        load_chunk(a0, b0, v0);
        for (int cix = 0; cix + 2 < nch; cix += 2) {
            load_chunk(a1, b1, v1);
            mma_chunk(a0, b0, v0);
            load_chunk(a0, b0, v0);
            mma_chunk(a1, b1, v1);
        }
        load_chunk(a1, b1, v1);
        mma_chunk(a0, b0, v0);
        mma_chunk(a1, b1, v1);
    }

    // wavefront partials -> LDS; accumulator register v holds row 8*(v/4) + 4*h + v%4, column f
#pragma unroll
    for (int c = 0; c < kPosTiles; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[wave][8 * (v >> 2) + 4 * h + (v & 3)][c * 32 + f] = acc[c][v];
    __syncthreads();

    // fixed-order sum over the wavefronts, written in the layout of dw
    float* dst = out + (size_t)ks * ((size_t)P.Cout * P.L);
    for (int e = threadIdx.x; e < 32 * 32 * kPosTiles; e += kWaves * 64) {
        const int fr = e / (32 * kPosTiles), uc = e % (32 * kPosTiles);
        float s = 0.f;
#pragma unroll
        for (int wv = 0; wv < kWaves; ++wv) s += red[wv][fr][uc];
        int kr, offr;
        bool vr;
        tile_filter(T, P, mb, ib, fr, kr, offr, vr);
        const int j = sc * (32 * kPosTiles) + uc - offr;
        if (vr && j >= 0 && j < P.L) dst[(size_t)kr * P.L + j] = s;
    }
}

// dw[e] = sum over K-splits of part[ks][e], in split order
__global__ __launch_bounds__(256) void backward_weight_reduce(const float* __restrict__ part, float* __restrict__ dw,
                                                              int count, int KS)
{
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= count) return;
    float s = 0.f;
    for (int ks = 0; ks < KS; ++ks) s += part[(size_t)ks * count + e];
    dw[e] = s;
}

int pow2_floor(int v)
{
    int p = 1;
    while (p * 2 <= v) p *= 2;
    return p;
}

BwwTiling make_tiling(const Problem& p)
{
    BwwTiling t;
    t.b = make_band(p);
    t.TI = pow2_floor(t.b.F < 32 ? t.b.F : 32);
    t.TM = 32 / t.TI < t.b.P ? 32 / t.TI : t.b.P;
    t.IB = (t.b.F + t.TI - 1) / t.TI;
    t.MB = (t.b.P + t.TM - 1) / t.TM;
    t.U = p.L + t.b.g * (t.TM - 1);
    t.NSC = (t.U + 32 * kPosTiles - 1) / (32 * kPosTiles);
    t.NQ4 = (int)(p.NQ / 4);
    // enough workgroups to fill 256 CUs about twice, but at least 16 column groups per wavefront
    const long long tiles = (long long)t.IB * t.MB * t.NSC;
    long long ks = (512 + tiles - 1) / tiles;
    const long long ks_max = t.NQ4 / (16 * kWaves);
    if (ks > ks_max) ks = ks_max;
    if (ks < 1) ks = 1;
    t.KS = (int)ks;
    return t;
}

}  // namespace

bool backward_weight_mfma_eligible(const Problem& p)
{
    const long long rows = p.Cin > p.Cout ? p.Cin : p.Cout;
    return p.HW % 4 == 0 && p.L >= 8 && p.NQ >= 256 && p.Cout >= 8 && p.Cin < 65536 &&
           (long long)p.NQ * rows * 4 < (1ll << 32) && (long long)p.Cout * p.L * 4 < (1ll << 31);
}

size_t backward_weight_mfma_workspace(const Problem& p)
{
    const BwwTiling t = make_tiling(p);
    return t.KS > 1 ? (size_t)t.KS * p.Cout * p.L * sizeof(float) : 0;
}

hipError_t launch_backward_weight_mfma(const float* x, const float* dy, float* dw, float* workspace, const Problem& p,
                                       hipStream_t st)
{
    const BwwTiling t = make_tiling(p);
    const long long ntile = (long long)t.IB * t.MB * t.NSC;
    const long long blocks = (long long)((t.KS + 7) / 8 * 8) * ntile;
    float* out = t.KS > 1 ? workspace : dw;
    backward_weight_mfma32<<<dim3((unsigned)blocks), dim3(kWaves * 64), 0, st>>>(x, dy, out, p, t);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || t.KS == 1) return e;
    const int count = p.Cout * p.L;
    backward_weight_reduce<<<dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st>>>(workspace, dw, count, t.KS);
    return hipGetLastError();
}

}  // namespace scc
