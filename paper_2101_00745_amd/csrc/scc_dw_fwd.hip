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
#include "scc_dw_strip.h"

namespace scc {

namespace {

using dw::dw_strip;

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
    int al4;        // g and L are multiples of 4 and w is 16-byte aligned: a lane's groups of four weights are wholly
                    // inside or outside a window and are read with 16-byte loads
};

int pow2_floor_dw(int v)
{
    int p = 1;
    while (p * 2 <= v) p *= 2;
    return p;
}

// Stand-alone depthwise stage on strips (see scc_dw_strip.h): stride 1 or 2, input maps of exactly S times the
// output size, RB dividing the output rows, output rows of whole quads of pixels, tensors aligned to 4 values.
template <typename T_, int S, int RB>
__global__ __launch_bounds__(256) void depthwise3x3_strips(const T_* __restrict__ x, const T_* __restrict__ kdw,
                                                           T_* __restrict__ z, int C, DwGeom G, long long items,
                                                           int flip)
{
    typedef T_ tvec __attribute__((ext_vector_type(4)));
    const size_t HWi = (size_t)G.H * G.W, HWo = (size_t)G.Ho * G.Wo;
    const uint32_t W4 = G.Wo / 4, SB = G.Ho / RB;
    // 32-bit index arithmetic (the launcher sends fewer than 2^31 strips here): 64-bit divisions in every lane
    // cost more than the stencil itself.  All lanes of a wavefront run the same number of trips (the strip
    // routine shuffles between lanes); lanes past the end compute strip 0 again and store nothing.
    const uint32_t lane = threadIdx.x & 63;
    for (uint32_t e0 = blockIdx.x * 256u; e0 < (uint32_t)items; e0 += gridDim.x * 256u) {
        const uint32_t ee = e0 + threadIdx.x;
        const bool live = ee < (uint32_t)items;
        const uint32_t e = live ? ee : 0;
        const int cw = (int)(e % W4) * 4;
        uint32_t t = e / W4;
        const int r0 = (int)(t % SB) * RB;
        t /= SB;                          // t = n*C + a
        const int a = (int)(t % (uint32_t)C);
        float k[9];
        dw::load_taps(kdw, a, flip != 0, k);
        const uint32_t rowmask = dw::strip_rowmask<S, RB>(r0, G.Ho);
        float out[RB][4];
        // consecutive strips of a row are consecutive lanes; the first and last lane of the wavefront and the
        // last live one have no neighbour to ask
        dw_strip<S, RB>(x + t * HWi + (size_t)(S * r0) * G.W + S * cw, G.W, k, rowmask, cw > 0, cw + 4 < G.Wo, lane == 0,
                        lane == 63 || ee + 1 >= (uint32_t)items, out);
        if (!live) continue;
        T_* zo = z + t * HWo + (size_t)r0 * G.Wo + cw;
#pragma unroll
        for (int rr = 0; rr < RB; ++rr) {
            tvec o;
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] = from_f32<T_>(out[rr][i]);
            __builtin_nontemporal_store(o, (tvec*)(zo + rr * G.Wo));
        }
    }
}

// Stand-alone depthwise stage at stride 1 for rows of any length: a thread owns ONE column of RB consecutive output
// rows, consecutive lanes own consecutive pixels of the row-major map, so every load instruction reads consecutive
// values; the pixels left and right of a lane's column are what its neighbouring lanes loaded (lane shuffle), and
// each input row is loaded once per strip.  1 + 2/RB loads per output instead of the nine of the kernel below.
template <typename T_, int RB>
__global__ __launch_bounds__(256) void depthwise3x3_columns(const T_* __restrict__ x, const T_* __restrict__ kdw,
                                                            T_* __restrict__ z, int C, DwGeom G, long long items,
                                                            int flip)
{
    const size_t HW = (size_t)G.H * G.W;
    const uint32_t W = (uint32_t)G.W, SB = (uint32_t)G.H / RB;
    const uint32_t lane = threadIdx.x & 63;
    // all lanes of a wavefront run the same number of trips (they shuffle); lanes past the end redo item 0 and store nothing
    for (uint32_t e0 = blockIdx.x * 256u; e0 < (uint32_t)items; e0 += gridDim.x * 256u) {
        const uint32_t ee = e0 + threadIdx.x;
        const bool live = ee < (uint32_t)items;
        const uint32_t e = live ? ee : 0;
        const int c = (int)(e % W);
        uint32_t t = e / W;
        const int r0 = (int)(t % SB) * RB;
        t /= SB;                          // t = n*C + a
        float k[9];
        dw::load_taps(kdw, (int)(t % (uint32_t)C), flip != 0, k);
        const T_* xc = x + t * HW + (size_t)r0 * W + c;      // input pixel (r0, c)
        const bool left = c > 0, right = c + 1 < (int)W;
        const bool lo = lane == 0, hi = lane == 63 || ee + 1 >= (uint32_t)items;
        float out[RB];
#pragma unroll
        for (int rr = 0; rr < RB; ++rr) out[rr] = 0.f;
#pragma unroll
        for (int tr = 0; tr < RB + 2; ++tr) {
            const int r = r0 - 1 + tr;
            const bool ok = r >= 0 && r < G.H;
            const T_* row = ok ? xc + (tr - 1) * (int)W : xc;
            const float mid = to_f32(row[0]);
            float lv = __shfl_up(mid, 1, 64), rv = __shfl_down(mid, 1, 64);
            if (lo && left) lv = to_f32(row[-1]);
            if (hi && right) rv = to_f32(row[1]);
            const float v0 = (ok && left) ? lv : 0.f, v1 = ok ? mid : 0.f, v2 = (ok && right) ? rv : 0.f;
#pragma unroll
            for (int rr = 0; rr < RB; ++rr) {
                const int di = tr - rr;
                if (di < 0 || di > 2) continue;
                out[rr] += k[di * 3] * v0 + k[di * 3 + 1] * v1 + k[di * 3 + 2] * v2;
            }
        }
        if (!live) continue;
        T_* zo = z + t * HW + (size_t)r0 * W + c;
#pragma unroll
        for (int rr = 0; rr < RB; ++rr) __builtin_nontemporal_store(from_f32<T_>(out[rr]), zo + rr * (int)W);
    }
}

// Stand-alone depthwise stage, any stride and map size: one thread per output value, taps in row-major order.
// IDX is the type of the flat output index: 32 bits whenever the tensor allows it (64-bit divisions in every lane
// cost several times the stencil).
template <typename T_, typename IDX>
__global__ __launch_bounds__(256) void depthwise3x3_kernel(const T_* __restrict__ x, const T_* __restrict__ kdw,
                                                           T_* __restrict__ z, int C, DwGeom G, long long items,
                                                           int flip)
{
    const size_t HWi = (size_t)G.H * G.W;
    for (IDX e = (IDX)blockIdx.x * 256 + threadIdx.x; e < (IDX)items; e += (IDX)gridDim.x * 256) {
        const int q = (int)(e % (IDX)G.Wo);
        IDX t = e / (IDX)G.Wo;
        const int m = (int)(t % (IDX)G.Ho);
        t /= (IDX)G.Ho;
        const int a = (int)(t % (IDX)C);
        const T_* xc = x + (size_t)t * HWi;
        float out = 0.f;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int rr = G.s * m + i - 1;
            if (rr < 0 || rr >= G.H) continue;
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const int cc = G.s * q + j - 1;
                if (cc < 0 || cc >= G.W) continue;
                out += to_f32(kdw[a * 9 + (flip ? 8 - (i * 3 + j) : i * 3 + j)]) * to_f32(xc[(size_t)rr * G.W + cc]);
            }
        }
        z[e] = from_f32<T_>(out);
    }
}

// ---------------------------------------------------------------------------------------------------------
// Fused DW + SCC forward, fp32.
//   CP    column groups of 32 per workgroup (the LDS tile is Cin x 32*CP binary32 values)
//   S,RB  phase 1 on strips (dw_strip): spatial stride S (1 or 2), RB output rows per strip; the tile is then whole
//         output rows (32*CP is a multiple of the row length) cut into strips that do not straddle samples.
//         S == 0: any stride and map size, every thread computes its 4 columns tap by tap.
//
// LDS layout: zl[c / 4][column][c % 4] (16 bytes per (channel quad, column)), a quad's row padded by one column:
// a lane of phase 2 reads the 8 channels of its half of a 16-channel chunk at its column with two 16-byte reads
// (16 lanes cover all banks), and the writes of phase 1 (lanes differ in channel and column group) spread over
// all banks too.
template <int CP, int S, int RB>
__global__ __launch_bounds__(256) void dw_scc_forward_lds(const float* __restrict__ x, const float* __restrict__ kdw,
                                                          const float* __restrict__ w, float* __restrict__ y, Problem P,
                                                          DwGeom G, DwTiling T)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    float* zl = (float*)lds_raw;
    constexpr int TP = 32 * CP;
    constexpr int TPP = TP + 1;          // padded row of a channel quad, in columns

    // workgroup -> column tile; blockIdx % 8 names the XCD, and every XCD takes a contiguous run of column
    // tiles, so the rows of x that neighbouring tiles of one sample both need meet in one L2
    const long long tile = (long long)(blockIdx.x & 7) * T.chunk + (blockIdx.x >> 3);
    if (tile >= T.nct) return;
    const long long q0 = tile * TP;
    const int tid = threadIdx.x;
    const int HWi = G.H * G.W;

    // ---------------- phase 2's A operand is requested one step ahead of its use; the first step's before phase 1
    // A step is one chunk of a filter tile: the 16 channels one matrix instruction contracts.
    const int lane = tid & 63, wave = tid >> 6, col = lane & 31, kg = lane >> 5;
    const Band& b = T.b;
    struct Step {
        int ft, cb;        // filter tile and first channel (unwrapped axis) of the block; ft >= ntiles: past the end
        int cend;          // one past the tile's span
        int sf;            // window start of this lane's filter
        long long kf;      // this lane's filter (A row lane & 31 of the tile), -1 if the tile has none there
    };
    auto tile_of = [&](int ft) {
        Step st;
        st.ft = ft;
        const int ib = ft % T.IB, mb = ft / T.IB;
        const int f = lane & 31;
        const int m = mb * T.TM + f / T.TI, i = ib * T.TI + f % T.TI;
        st.kf = -1;
        if (ft < T.ntiles && m < b.P) {
            st.kf = (long long)(((long long)m * b.inv) % b.P) + (long long)b.P * i;
            if (st.kf >= P.Cout) st.kf = -1;
        }
        st.sf = b.g * m;
        const int c0 = b.g * mb * T.TM;     // window start of the tile's first filter column
        st.cb = c0 & ~15;
        st.cend = c0 + T.U;
        return st;
    };
    auto next_of = [&](const Step& st) {
        if (st.cb + 16 < st.cend) {
            Step n = st;
            n.cb += 16;
            return n;
        }
        return tile_of(st.ft + 4);
    };
    // the lane's 8 weights of the chunk, zero outside the filter's window
    auto load_a = [&](const Step& st, float (&a)[8]) {
        const float* wrow = w + (st.kf >= 0 ? st.kf : 0) * P.L;
        {
            const int j0 = st.cb + 8 * kg - st.sf;   // weight index of the lane's first channel
            if (T.al4) {      // uniform over the grid
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int j = j0 + 4 * h;
                    const bool in = st.kf >= 0 && j >= 0 && j < P.L;
                    const f32x4 v = *(const f32x4*)(wrow + (in ? j : 0));
#pragma unroll
                    for (int e = 0; e < 4; ++e) a[4 * h + e] = in ? v[e] : 0.f;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int j = j0 + e;
                    const bool in = st.kf >= 0 && j >= 0 && j < P.L;
                    const float v = wrow[in ? j : 0];
                    a[e] = in ? v : 0.f;
                }
            }
        }
    };
    Step cur = tile_of(wave);
    float araw[8];
    load_a(cur, araw);

    // ---------------- phase 1: z of all channels for this tile's columns
    if constexpr (S > 0) {
        // the tile is TP / Wo whole output rows; a thread owns one strip of it (RB rows x 4 columns) and walks
        // over the channels.  NQ is a multiple of the strip's row block, so a strip is wholly live or wholly not.
        constexpr int IPC = TP / (4 * RB);       // strips per channel
        constexpr int CSTEP = 256 / IPC;         // channels the workgroup covers per trip
        const int item = tid % IPC;
        const int W4 = G.Wo / 4;
        const int cw = (item % W4) * 4, srow = (item / W4) * RB;      // first column / first tile row of the strip
        const long long qa = q0 + (long long)srow * G.Wo + cw;        // first column (sample, pixel) of the strip
        const bool live = qa < P.NQ;
        const long long qs = live ? qa : 0;
        const int n = (int)(qs / P.HW), r0 = (int)(qs % P.HW) / G.Wo;
        const float* xb = x + (size_t)n * P.Cin * HWi + (size_t)(S * r0) * G.W + S * cw;
        const uint32_t rowmask = live ? dw::strip_rowmask<S, RB>(r0, G.Ho) : 0u;
        const bool left = cw > 0, right = cw + 4 < G.Wo;
        const int colbase = srow * G.Wo + cw;    // column of the strip's first output inside the tile
#pragma unroll 2
        for (int c = tid / IPC; c < P.Cin; c += CSTEP) {
            float k[9];
            dw::load_taps(kdw, c, false, k);
            float out[RB][4];
            dw_strip<S, RB>(xb + (size_t)c * HWi, G.W, k, rowmask, left, right, false, false, out);
            float* zo = zl + ((size_t)(c >> 2) * TPP + colbase) * 4 + (c & 3);
#pragma unroll
            for (int rr = 0; rr < RB; ++rr)
#pragma unroll
                for (int i = 0; i < 4; ++i) zo[(rr * G.Wo + i) * 4] = out[rr][i];
        }
    } else {
        // any stride and map size: each of the thread's 4 columns has its own sample and pixel
        constexpr int G4 = TP / 4;           // groups of 4 columns per tile
        constexpr int CSTEP = 256 / G4;      // channels the workgroup covers per trip
        const int g4 = tid % G4;
        const long long qa = q0 + 4 * g4;
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
            dw::load_taps(kdw, c, false, k);
            float* zo = zl + ((size_t)(c >> 2) * TPP + 4 * g4) * 4 + (c & 3);
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
    __syncthreads();

    // ---------------- phase 2: the SCC tiles of this column tile, B operand from LDS
    const f32x4* zl4 = (const f32x4*)zl;

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

    f32x16 acc[CP];
#pragma unroll
    for (int c = 0; c < CP; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;

    while (cur.ft < T.ntiles) {       // uniform over the wavefront
        // this step's A operand, cut into bf16 pieces; then the next step's weights are requested
        uint32_t ah[4], am[4], al[4];
        split3<8>([&](int e) { return araw[e]; }, ah, am, al);
        const Step nxt = next_of(cur);
        load_a(nxt, araw);            // past the end: reads row 0 of w and is never used

        {
            int cw = cur.cb;
            while (cw >= P.Cin) cw -= P.Cin;   // Cin and the chunk start are multiples of 16: a chunk never straddles the wrap
            const int quad = (cw + 8 * kg) >> 2;
#pragma unroll
            for (int c = 0; c < CP; ++c) {
                const f32x4 b0 = zl4[(size_t)quad * TPP + 32 * c + col];
                const f32x4 b1 = zl4[(size_t)(quad + 1) * TPP + 32 * c + col];
                const float bv[8] = {b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
                uint32_t bh[4], bm[4], bl[4];
                split3<8>([&](int e) { return bv[e]; }, bh, bm, bl);
                acc[c] = mfma_bf16<8>(al, bh, acc[c]);
                acc[c] = mfma_bf16<8>(ah, bl, acc[c]);
                acc[c] = mfma_bf16<8>(am, bm, acc[c]);
                acc[c] = mfma_bf16<8>(am, bh, acc[c]);
                acc[c] = mfma_bf16<8>(ah, bm, acc[c]);
                acc[c] = mfma_bf16<8>(ah, bh, acc[c]);
            }
        }

        if (nxt.ft != cur.ft) {
            // the tile is complete: accumulator register v of a lane holds tile row (v/4)*8 + kg*4 + v%4 at the
            // lane's column
            const int kmine = (int)cur.kf;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = (v >> 2) * 8 + kg * 4 + (v & 3);
                const int kr = __shfl(kmine, row, 64);   // lane `row` computed that filter's index
                if (kr < 0) continue;
#pragma unroll
                for (int c = 0; c < CP; ++c)
                    if (live[c]) __builtin_nontemporal_store(acc[c][v], y + ycol[c] + (long long)kr * P.HW);
            }
#pragma unroll
            for (int c = 0; c < CP; ++c)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;
        }
        cur = nxt;
    }
}

DwTiling make_dw_tiling(const Problem& p, int TP, const float* w)
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
    t.al4 = t.b.g % 4 == 0 && p.L % 4 == 0 && ((uintptr_t)w & 15) == 0;
    return t;
}

size_t fused_lds_bytes(const Problem& p, int cp) { return (size_t)4 * p.Cin * (32 * cp + 1); }

// Rows per strip (4 or 2) when phase 1 can run on strips for tiles of 32*cp columns, else 0: stride 1 or 2, output
// rows that are a multiple of 4 pixels and divide the tile, input maps of exactly stride times the output size,
// and a strip height that divides both the rows of a tile and the rows of a map.
int strip_rows(const DwGeom& g, int cp, const float* x)
{
    const int TP = 32 * cp;
    if ((g.s != 1 && g.s != 2) || g.Wo % 4 != 0 || TP % g.Wo != 0 || g.H != g.s * g.Ho || g.W != g.s * g.Wo ||
        ((uintptr_t)x & 15) != 0)
        return 0;
    const int rt = TP / g.Wo;
    if (rt % 4 == 0 && g.Ho % 4 == 0) return 4;
    if (rt % 2 == 0 && g.Ho % 2 == 0) return 2;
    return 0;
}

// Columns per workgroup, in groups of 32 (2 or 1): two workgroups per CU where the LDS tile allows it (80 KiB each),
// the wider tile when it still leaves every CU two workgroups, and a width on which phase 1 can run on strips
// if there is one.
int pick_cp(const Problem& p, const DwGeom& g, const float* x)
{
    int first = 0;
    for (int cp = 2; cp >= 1; --cp) {
        const bool fits = fused_lds_bytes(p, cp) <= 80 * 1024 || cp == 1;
        const bool enough = (p.NQ + 32 * cp - 1) / (32 * cp) >= 512 || cp == 1;
        if (!fits || !enough) continue;
        if (!first) first = cp;
        if (strip_rows(g, cp, x) > 0) return cp;
    }
    // no width of that choice runs on strips: a wider tile may (rows of 64 pixels need 64 columns)
    if (fused_lds_bytes(p, 2) <= 80 * 1024 && strip_rows(g, 2, x) > 0) return 2;
    return first;
}

template <int CP, int S, int RB>
hipError_t launch_fused(const float* x, const float* kdw, const float* w, float* y, const Problem& p, const DwGeom& g,
                        hipStream_t st)
{
    const DwTiling t = make_dw_tiling(p, 32 * CP, w);
    const size_t lds = fused_lds_bytes(p, CP);
    if (lds > 64 * 1024) {
        // more than 64 KiB of LDS per workgroup has to be allowed once per kernel (per process: one GPU is driven)
        static const hipError_t allowed = hipFuncSetAttribute((const void*)dw_scc_forward_lds<CP, S, RB>,
                                                              hipFuncAttributeMaxDynamicSharedMemorySize, 144 * 1024);
        if (allowed != hipSuccess) return allowed;
    }
    dw_scc_forward_lds<CP, S, RB><<<dim3((unsigned)(8 * t.chunk)), dim3(256), lds, st>>>(x, kdw, w, y, p, g, t);
    return hipGetLastError();
}

template <int CP>
hipError_t launch_fused_cp(const float* x, const float* kdw, const float* w, float* y, const Problem& p, const DwGeom& g,
                           hipStream_t st)
{
    const int rb = strip_rows(g, CP, x);
    if (rb == 0) return launch_fused<CP, 0, 1>(x, kdw, w, y, p, g, st);
    if (g.s == 1)
        return rb == 4 ? launch_fused<CP, 1, 4>(x, kdw, w, y, p, g, st) : launch_fused<CP, 1, 2>(x, kdw, w, y, p, g, st);
    return rb == 4 ? launch_fused<CP, 2, 4>(x, kdw, w, y, p, g, st) : launch_fused<CP, 2, 2>(x, kdw, w, y, p, g, st);
}

template <typename T, int S>
hipError_t launch_strips(const T* x, const T* kdw, T* z, int N, int C, const DwGeom& g, hipStream_t st, int flip)
{
    // taller strips read fewer halo rows per output; small problems take shorter ones to have enough threads
    const long long w4 = g.Wo / 4;
    int rb = g.Ho % 4 == 0 ? 4 : g.Ho % 2 == 0 ? 2 : 1;
    while (rb > 1 && (long long)N * C * (g.Ho / rb) * w4 < 256 * 1024) rb /= 2;
    const long long items = (long long)N * C * (g.Ho / rb) * w4;
    long long blocks = (items + 255) / 256;
    if (blocks > (1ll << 20)) blocks = 1ll << 20;   // the kernel strides over what is left
    const dim3 grid((unsigned)blocks), block(256);
    if (rb == 4)
        depthwise3x3_strips<T, S, 4><<<grid, block, 0, st>>>(x, kdw, z, C, g, items, flip);
    else if (rb == 2)
        depthwise3x3_strips<T, S, 2><<<grid, block, 0, st>>>(x, kdw, z, C, g, items, flip);
    else
        depthwise3x3_strips<T, S, 1><<<grid, block, 0, st>>>(x, kdw, z, C, g, items, flip);
    return hipGetLastError();
}

}  // namespace

template <typename T>
hipError_t launch_depthwise3x3(const T* x, const T* kdw, T* z, int N, int C, const DwGeom& g, hipStream_t st, bool flip)
{
    const bool sized = (g.s == 1 || g.s == 2) && g.H == g.s * g.Ho && g.W == g.s * g.Wo &&
                       (long long)N * C * g.Ho * ((g.Wo + 3) / 4) < (1ll << 31);
    const bool vec = g.Wo % 4 == 0 && (((uintptr_t)x | (uintptr_t)z) & (4 * sizeof(T) - 1)) == 0;
    if (sized && vec)
        return g.s == 1 ? launch_strips<T, 1>(x, kdw, z, N, C, g, st, flip) : launch_strips<T, 2>(x, kdw, z, N, C, g, st, flip);
    if (g.s == 1 && (long long)N * C * g.H * g.W < (1ll << 31)) {       // rows of any length
        const int rb = g.H % 4 == 0 ? 4 : g.H % 2 == 0 ? 2 : 1;
        const long long items = (long long)N * C * (g.H / rb) * g.W;
        long long blocks = (items + 255) / 256;
        if (blocks > (1ll << 20)) blocks = 1ll << 20;   // the kernel strides over what is left
        const dim3 grid((unsigned)blocks), block(256);
        if (rb == 4)
            depthwise3x3_columns<T, 4><<<grid, block, 0, st>>>(x, kdw, z, C, g, items, flip);
        else if (rb == 2)
            depthwise3x3_columns<T, 2><<<grid, block, 0, st>>>(x, kdw, z, C, g, items, flip);
        else
            depthwise3x3_columns<T, 1><<<grid, block, 0, st>>>(x, kdw, z, C, g, items, flip);
        return hipGetLastError();
    }
    const long long items = (long long)N * C * g.Ho * g.Wo;
    long long blocks = (items + 255) / 256;
    if (blocks > (1ll << 20)) blocks = 1ll << 20;
    if (items + (1ll << 28) < (1ll << 32))      // the index plus one grid stride still fits 32 bits
        depthwise3x3_kernel<T, uint32_t><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(x, kdw, z, C, g, items, flip);
    else
        depthwise3x3_kernel<T, unsigned long long><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(x, kdw, z, C, g, items, flip);
    return hipGetLastError();
}

template hipError_t launch_depthwise3x3<float>(const float*, const float*, float*, int, int, const DwGeom&, hipStream_t,
                                               bool);
template hipError_t launch_depthwise3x3<bf16_t>(const bf16_t*, const bf16_t*, bf16_t*, int, int, const DwGeom&,
                                                hipStream_t, bool);

// The fused kernel takes layers whose channel count is a multiple of 16 (a 16-channel chunk of the matrix
// instruction then never straddles the cyclic wrap) and whose z tile of 32 columns fits 144 KiB of LDS.
bool dw_forward_fused_eligible(const Problem& p)
{
    return p.Cin % 16 == 0 && fused_lds_bytes(p, 1) <= 144 * 1024 && p.Cin < 65536;
}

// Where it also pays: a workgroup computes every filter tile of its columns, so the grid has one workgroup per 32
// or 64 columns; measured against the two stages run one after the other it wins from 16384 columns up (two
// workgroups per CU) and loses below (the deep layers of the MobileNet-shaped stack: 512 to 8192 columns).
bool dw_forward_fused_preferred(const Problem& p) { return dw_forward_fused_eligible(p) && p.NQ >= 16384; }

hipError_t launch_dw_forward_fused(const float* x, const float* kdw, const float* w, float* y, const Problem& p,
                                   const DwGeom& g, hipStream_t st)
{
    if (pick_cp(p, g, x) == 2) return launch_fused_cp<2>(x, kdw, w, y, p, g, st);
    return launch_fused_cp<1>(x, kdw, w, y, p, g, st);
}

}  // namespace scc
