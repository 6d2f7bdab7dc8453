// Depthwise 3x3 stage (Eq. 2 of the paper) and the forward of a DW + SCC block (Section 3.1: the SCC takes the
// place of the pointwise convolution behind the depthwise one) in one kernel.
//
//   z[n,a,m,q] = sum_{i,j<3} kdw[a,i,j] * x[n,a, s*m+i-1, s*q+j-1]      (pixels outside the H x W map count as zero)
//   y[n,k,p]   = sum_{j<L}  w[k,j] * z[n,(s_k+j) mod Cin,p]             (Section 4.2, output-centric forward)
//
// The fused kernel never writes z: a workgroup owns 32*CP columns (a column is one (sample, output pixel) pair),
// computes z for ALL Cin channels of those columns into LDS (phase 1, vector ALU, binary32), and then its four
// wavefronts walk over the 32-filter tiles of scc_band.h and contract them against the LDS tile on the matrix
// cores (phase 2).  Products use the exact three-way bf16 split of scc_common.h (six bf16 matrix instructions
// per 16 channels, binary32 sums), like the stand-alone forward.  HBM sees x once and y once.
#include "scc_band.h"
#include "scc_common.h"

namespace scc {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct DwTiling {
    Band b;
    int TI, TM;     // filter tile = TM window starts x TI filters per start (TI * TM <= 32)
    int IB, MB;     // tiles along i and m
    int ntiles;     // IB * MB
    int U;          // channels a tile spans: L + g * (TM - 1)
    long long nct;  // column tiles
    long long chunk;  // consecutive column tiles given to one XCD: ceil(nct / 8)
};

int pow2_floor_dw(int v)
{
    int p = 1;
    while (p * 2 <= v) p *= 2;
    return p;
}

// ---------------------------------------------------------------------------------------------------------
// Stand-alone depthwise stage: one thread per output value (VEC: per 4 consecutive values of one output row,
// for spatial stride 1 and rows that are a multiple of 4 pixels).  Sums are binary32, taps in row-major order.
template <typename T_, bool VEC>
__global__ __launch_bounds__(256) void depthwise3x3_kernel(const T_* __restrict__ x, const T_* __restrict__ kdw,
                                                           T_* __restrict__ z, int C, DwGeom G, long long items)
{
    const long long HWi = (long long)G.H * G.W, HWo = (long long)G.Ho * G.Wo;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < items; e += (long long)gridDim.x * 256) {
        if constexpr (VEC) {
            const int W4 = G.Wo / 4;
            const int cw = (int)(e % W4) * 4;
            long long t = e / W4;
            const int r = (int)(t % G.Ho);
            t /= G.Ho;                       // t = n*C + a
            const int a = (int)(t % C);
            const T_* xc = x + t * HWi + (long long)r * G.W + cw;
            float k[9];
#pragma unroll
            for (int i = 0; i < 9; ++i) k[i] = to_f32(kdw[a * 9 + i]);
            float out[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int dr = -1; dr <= 1; ++dr) {
                const int rr = r + dr;
                if (rr < 0 || rr >= G.H) continue;
                const T_* row = xc + dr * G.W;
                float v[6];
                v[0] = cw > 0 ? to_f32(row[-1]) : 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i) v[1 + i] = to_f32(row[i]);
                v[5] = cw + 4 < G.W ? to_f32(row[4]) : 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 3; ++j) out[i] += k[(dr + 1) * 3 + j] * v[i + j];
            }
            T_* zo = z + t * HWo + (long long)r * G.Wo + cw;
#pragma unroll
            for (int i = 0; i < 4; ++i) zo[i] = from_f32<T_>(out[i]);
        } else {
            const int q = (int)(e % G.Wo);
            long long t = e / G.Wo;
            const int m = (int)(t % G.Ho);
            t /= G.Ho;
            const int a = (int)(t % C);
            const T_* xc = x + t * HWi;
            float out = 0.f;
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                const int rr = G.s * m + i - 1;
                if (rr < 0 || rr >= G.H) continue;
#pragma unroll
                for (int j = 0; j < 3; ++j) {
                    const int cc = G.s * q + j - 1;
                    if (cc < 0 || cc >= G.W) continue;
                    out += to_f32(kdw[a * 9 + i * 3 + j]) * to_f32(xc[(long long)rr * G.W + cc]);
                }
            }
            z[e] = from_f32<T_>(out);
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// Fused DW + SCC forward, fp32.
//   CP    column groups of 32 per workgroup (the LDS tile is Cin x 32*CP binary32 values)
//   AL4   g and L are multiples of 4: groups of four weights are wholly inside or outside a window and 16-byte
//         aligned, so the A operand is read with 16-byte loads
//   FAST  spatial stride 1, rows that are a multiple of 4 pixels, x aligned to 16 bytes: a thread's 4 columns
//         are 4 consecutive pixels of one row and each row of the stencil is one 16-byte load plus two edge values
//
// LDS layout: zl[c / 4][column][c % 4] (16 bytes per (channel quad, column)): a lane of phase 2 reads the 8
// channels of its half of a 16-channel chunk at its column with two 16-byte reads, 16 lanes covering all banks.
template <int CP, bool AL4, bool FAST>
__global__ __launch_bounds__(256) void dw_scc_forward_lds(const float* __restrict__ x, const float* __restrict__ kdw,
                                                          const float* __restrict__ w, float* __restrict__ y, Problem P,
                                                          DwGeom G, DwTiling T)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    float* zl = (float*)lds_raw;
    constexpr int TP = 32 * CP;
    constexpr int G4 = TP / 4;           // groups of 4 columns per tile
    constexpr int CSTEP = 256 / G4;      // channels the workgroup covers per trip of phase 1

    // workgroup -> column tile; blockIdx % 8 names the XCD, and every XCD takes a contiguous run of column
    // tiles, so the rows of x that neighbouring tiles of one sample both need meet in one L2
    const long long tile = (long long)(blockIdx.x & 7) * T.chunk + (blockIdx.x >> 3);
    if (tile >= T.nct) return;
    const long long q0 = tile * TP;
    const int tid = threadIdx.x;
    const int HWi = G.H * G.W;

    // ---------------- phase 1: z of all channels for this tile's columns
    {
        const int g4 = tid % G4;
        const long long qa = q0 + 4 * g4;
        if constexpr (FAST) {
            // the 4 columns qa..qa+3 are pixels p..p+3 of one row of one sample (HW % 4 == 0, so NQ % 4 == 0)
            const bool live = qa < P.NQ;
            const long long qs = live ? qa : 0;
            const int n = (int)(qs / P.HW), p = (int)(qs % P.HW);
            const int r = p / G.W, cw = p % G.W;
            const float* xb = x + (size_t)n * P.Cin * HWi + p;
            const bool rowok[3] = {live && r > 0, live, live && r + 1 < G.H};
            const bool left = cw > 0, right = cw + 4 < G.W;
            for (int c = tid / G4; c < P.Cin; c += CSTEP) {
                const float* xc = xb + (size_t)c * HWi;
                float k[9];
#pragma unroll
                for (int i = 0; i < 9; ++i) k[i] = kdw[c * 9 + i];
                float out[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int dr = 0; dr < 3; ++dr) {
                    // rows outside the map are read at the centre row (always inside) and discarded
                    const float* row = rowok[dr] ? xc + (dr - 1) * G.W : xc;
                    const f32x4 mid = *(const f32x4*)row;
                    const float lv = row[left ? -1 : 0], rv = row[right ? 4 : 3];
                    float v[6];
                    v[0] = (rowok[dr] && left) ? lv : 0.f;
                    v[1] = rowok[dr] ? mid[0] : 0.f;
                    v[2] = rowok[dr] ? mid[1] : 0.f;
                    v[3] = rowok[dr] ? mid[2] : 0.f;
                    v[4] = rowok[dr] ? mid[3] : 0.f;
                    v[5] = (rowok[dr] && right) ? rv : 0.f;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int j = 0; j < 3; ++j) out[i] += k[dr * 3 + j] * v[i + j];
                }
                float* zo = zl + ((size_t)(c >> 2) * TP + 4 * g4) * 4 + (c & 3);
#pragma unroll
                for (int i = 0; i < 4; ++i) zo[4 * i] = out[i];
            }
        } else {
            // any stride and map size: each of the thread's 4 columns has its own sample and pixel
            long long base[4];     // offset of the stencil's centre pixel in channel 0 of the column's sample
            uint32_t taps[4];      // bit 3*i+j: tap (i, j) falls inside the map
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const long long q = qa + i4;
                taps[i4] = 0;
                base[i4] = 0;
                if (q < P.NQ) {
                    const int n = (int)(q / P.HW), p = (int)(q % P.HW);
                    const int m = p / G.Wo, qq = p % G.Wo;
                    base[i4] = (long long)n * P.Cin * HWi + (long long)(G.s * m) * G.W + G.s * qq;
#pragma unroll
                    for (int i = 0; i < 3; ++i)
#pragma unroll
                        for (int j = 0; j < 3; ++j) {
                            const int rr = G.s * m + i - 1, cc = G.s * qq + j - 1;
                            if (rr >= 0 && rr < G.H && cc >= 0 && cc < G.W) taps[i4] |= 1u << (3 * i + j);
                        }
                }
            }
            for (int c = tid / G4; c < P.Cin; c += CSTEP) {
                float k[9];
#pragma unroll
                for (int i = 0; i < 9; ++i) k[i] = kdw[c * 9 + i];
                float* zo = zl + ((size_t)(c >> 2) * TP + 4 * g4) * 4 + (c & 3);
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const float* xc = x + base[i4] + (long long)c * HWi;
                    float out = 0.f;
#pragma unroll
                    for (int i = 0; i < 3; ++i)
#pragma unroll
                        for (int j = 0; j < 3; ++j)
                            if (taps[i4] & (1u << (3 * i + j))) out += k[3 * i + j] * xc[(i - 1) * G.W + (j - 1)];
                    zo[4 * i4] = out;
                }
            }
        }
    }
    __syncthreads();

    // ---------------- phase 2: the SCC tiles of this column tile, B operand from LDS
    const int lane = tid & 63, wave = tid >> 6, col = lane & 31, kg = lane >> 5;
    const f32x4* zl4 = (const f32x4*)zl;
    const Band& b = T.b;
    const int f = lane & 31;  // this lane's A row (filter of the tile)

    // where this lane's columns go in y
    long long ycol[CP];
    bool live[CP];
#pragma unroll
    for (int c = 0; c < CP; ++c) {
        const long long q = q0 + 32 * c + col;
        live[c] = q < P.NQ;
        const long long qs = live[c] ? q : 0;
        ycol[c] = (qs / P.HW) * (long long)P.Cout * P.HW + qs % P.HW;
    }

    for (int ft = wave; ft < T.ntiles; ft += 4) {
        const int ib = ft % T.IB, mb = ft / T.IB;
        const int m = mb * T.TM + f / T.TI, i = ib * T.TI + f % T.TI;
        long long kf = -1;
        if (m < b.P) {
            kf = (long long)(((long long)m * b.inv) % b.P) + (long long)b.P * i;
            if (kf >= P.Cout) kf = -1;
        }
        const int sf = b.g * m;                 // window start of this lane's filter
        const int c0 = b.g * mb * T.TM;         // window start of the tile's first filter column
        const int cend = c0 + T.U;              // one past the tile's span (unwrapped channel axis)
        const float* wrow = w + (kf >= 0 ? kf : 0) * P.L;

        f32x16 acc[CP];
#pragma unroll
        for (int c = 0; c < CP; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;

        for (int cb = c0 & ~15; cb < cend; cb += 64) {
            // A operand of up to 4 chunks of 16 channels: this lane's 8 weights per chunk, cut into bf16 pieces
            uint32_t ah[4][4], am[4][4], al[4][4];
#pragma unroll
            for (int ch = 0; ch < 4; ++ch) {
                const int j0 = cb + 16 * ch + 8 * kg - sf;   // weight index of the lane's first channel
                float a[8];
                if constexpr (AL4) {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int j = j0 + 4 * h;
                        const bool in = kf >= 0 && j >= 0 && j < P.L;
                        const f32x4 v = *(const f32x4*)(wrow + (in ? j : 0));
#pragma unroll
                        for (int e = 0; e < 4; ++e) a[4 * h + e] = in ? v[e] : 0.f;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int j = j0 + e;
                        const bool in = kf >= 0 && j >= 0 && j < P.L;
                        const float v = wrow[in ? j : 0];
                        a[e] = in ? v : 0.f;
                    }
                }
                split3<8>([&](int e) { return a[e]; }, ah[ch], am[ch], al[ch]);
            }
#pragma unroll
            for (int ch = 0; ch < 4; ++ch) {
                const int cu = cb + 16 * ch;
                if (cu >= cend) break;          // uniform over the wavefront
                int cw = cu;
                while (cw >= P.Cin) cw -= P.Cin;   // Cin and the chunk start are multiples of 16: a chunk never straddles the wrap
                const int quad = (cw + 8 * kg) >> 2;
#pragma unroll
                for (int c = 0; c < CP; ++c) {
                    const f32x4 b0 = zl4[(size_t)quad * TP + 32 * c + col];
                    const f32x4 b1 = zl4[(size_t)(quad + 1) * TP + 32 * c + col];
                    const float bv[8] = {b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
                    uint32_t bh[4], bm[4], bl[4];
                    split3<8>([&](int e) { return bv[e]; }, bh, bm, bl);
                    acc[c] = mfma_bf16<8>(al[ch], bh, acc[c]);
                    acc[c] = mfma_bf16<8>(ah[ch], bl, acc[c]);
                    acc[c] = mfma_bf16<8>(am[ch], bm, acc[c]);
                    acc[c] = mfma_bf16<8>(am[ch], bh, acc[c]);
                    acc[c] = mfma_bf16<8>(ah[ch], bm, acc[c]);
                    acc[c] = mfma_bf16<8>(ah[ch], bh, acc[c]);
                }
            }
        }

        // accumulator register v of a lane holds tile row (v/4)*8 + kg*4 + v%4 at the lane's column
        const int kmine = (int)kf;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = (v >> 2) * 8 + kg * 4 + (v & 3);
            const int kr = __shfl(kmine, row, 64);   // lane `row` computed that filter's index
            if (kr < 0) continue;
#pragma unroll
            for (int c = 0; c < CP; ++c)
                if (live[c]) __builtin_nontemporal_store(acc[c][v], y + ycol[c] + (long long)kr * P.HW);
        }
    }
}

DwTiling make_dw_tiling(const Problem& p, int TP)
{
    DwTiling t;
    t.b = make_band(p);
    t.TI = pow2_floor_dw(t.b.F < 32 ? t.b.F : 32);
    t.TM = 32 / t.TI < t.b.P ? 32 / t.TI : t.b.P;
    t.IB = (t.b.F + t.TI - 1) / t.TI;
    t.MB = (t.b.P + t.TM - 1) / t.TM;
    t.ntiles = t.IB * t.MB;
    t.U = p.L + t.b.g * (t.TM - 1);
    t.nct = (p.NQ + TP - 1) / TP;
    t.chunk = (t.nct + 7) / 8;
    return t;
}

// columns per workgroup: as many groups of 32 (4, 2 or 1) as leave every CU a workgroup and fit 64 KiB of LDS,
// else the most that fit 128 KiB
int pick_cp(const Problem& p)
{
    for (int cp = 4; cp >= 1; cp /= 2) {
        const long long lds = (long long)p.Cin * 32 * cp * 4;
        if (lds <= 64 * 1024 && (p.NQ + 32 * cp - 1) / (32 * cp) >= 256) return cp;
    }
    for (int cp = 4; cp >= 1; cp /= 2)
        if ((long long)p.Cin * 32 * cp * 4 <= 64 * 1024) return cp;
    return 1;
}

template <int CP, bool AL4, bool FAST>
hipError_t launch_fused(const float* x, const float* kdw, const float* w, float* y, const Problem& p, const DwGeom& g,
                        hipStream_t st)
{
    const DwTiling t = make_dw_tiling(p, 32 * CP);
    const size_t lds = (size_t)p.Cin * 32 * CP * sizeof(float);
    if (lds > 64 * 1024) {
        // more than 64 KiB of LDS per workgroup has to be allowed once per kernel (per process: one GPU is driven)
        static const hipError_t allowed = hipFuncSetAttribute((const void*)dw_scc_forward_lds<CP, AL4, FAST>,
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
        if (allowed != hipSuccess) return allowed;
    }
    dw_scc_forward_lds<CP, AL4, FAST><<<dim3((unsigned)(8 * t.chunk)), dim3(256), lds, st>>>(x, kdw, w, y, p, g, t);
    return hipGetLastError();
}

template <int CP>
hipError_t launch_fused_cp(const float* x, const float* kdw, const float* w, float* y, const Problem& p, const DwGeom& g,
                           hipStream_t st)
{
    const Band b = make_band(p);
    const bool al4 = b.g % 4 == 0 && p.L % 4 == 0 && ((uintptr_t)w & 15) == 0;
    const bool fast = g.s == 1 && g.W % 4 == 0 && ((uintptr_t)x & 15) == 0;
    if (al4)
        return fast ? launch_fused<CP, true, true>(x, kdw, w, y, p, g, st)
                    : launch_fused<CP, true, false>(x, kdw, w, y, p, g, st);
    return fast ? launch_fused<CP, false, true>(x, kdw, w, y, p, g, st)
                : launch_fused<CP, false, false>(x, kdw, w, y, p, g, st);
}

}  // namespace

template <typename T>
hipError_t launch_depthwise3x3(const T* x, const T* kdw, T* z, int N, int C, const DwGeom& g, hipStream_t st)
{
    const long long outs = (long long)N * C * g.Ho * g.Wo;
    const bool vec = g.s == 1 && g.W % 4 == 0;
    const long long items = vec ? outs / 4 : outs;
    long long blocks = (items + 255) / 256;
    if (blocks > (1ll << 20)) blocks = 1ll << 20;   // the kernel strides over what is left
    if (vec)
        depthwise3x3_kernel<T, true><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(x, kdw, z, C, g, items);
    else
        depthwise3x3_kernel<T, false><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(x, kdw, z, C, g, items);
    return hipGetLastError();
}

template hipError_t launch_depthwise3x3<float>(const float*, const float*, float*, int, int, const DwGeom&, hipStream_t);
template hipError_t launch_depthwise3x3<bf16_t>(const bf16_t*, const bf16_t*, bf16_t*, int, int, const DwGeom&,
                                                hipStream_t);

// The fused kernel takes layers whose channel count is a multiple of 16 (a 16-channel chunk of the matrix
// instruction then never straddles the cyclic wrap) and whose z tile of 32 columns fits 128 KiB of LDS.
bool dw_forward_fused_eligible(const Problem& p)
{
    return p.Cin % 16 == 0 && (long long)p.Cin * 32 * 4 <= 128 * 1024 && p.L >= 8 && p.Cin < 65536 &&
           (long long)p.NQ * p.Cout * 4 < (1ll << 40);
}

hipError_t launch_dw_forward_fused(const float* x, const float* kdw, const float* w, float* y, const Problem& p,
                                   const DwGeom& g, hipStream_t st)
{
    const int cp = pick_cp(p);
    if (cp == 4) return launch_fused_cp<4>(x, kdw, w, y, p, g, st);
    if (cp == 2) return launch_fused_cp<2>(x, kdw, w, y, p, g, st);
    return launch_fused_cp<1>(x, kdw, w, y, p, g, st);
}

}  // namespace scc
