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
#pragma once
#include "scc_band.h"
#include "scc_common.h"

namespace scc {

namespace bww {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kWaves = 4;     // wavefronts per workgroup
constexpr int kLd = 36;       // floats per staged fp32 row: 32 columns + 4 of padding (bank spread, 16-byte aligned)
constexpr int kRowBytes32 = kLd * 4;   // bytes per staged fp32 row
constexpr int kRowBytes16 = 80;        // bytes per staged bf16 row: 32 columns (64 bytes) + 16 of padding

// NPT = span positions per wavefront tile / 32 (1, 2 or 3): the tile is 32 filters x 32*NPT positions
constexpr int rows_of(int npt) { return 32 * (1 + npt); }            // operand rows: 32 of dy, 32*NPT of x
constexpr int row_bytes_of(int esz) { return esz == 2 ? kRowBytes16 : kRowBytes32; }
// staging blocks of the wavefronts, reused for the cross-wavefront sum (whichever is larger), + the row tables
constexpr size_t region_bytes_of(int npt, int esz)
{
    const size_t stage = (size_t)kWaves * rows_of(npt) * row_bytes_of(esz), red = (size_t)kWaves * 32 * 32 * npt * 4;
    return stage > red ? stage : red;
}
constexpr size_t lds_bytes_of(int npt, int esz) { return region_bytes_of(npt, esz) + 2 * 32 * 4; }

struct BwwTiling {
    Band b;
    int TI, TM;   // tile = TM starts x TI filters per start
    int IB, MB;   // tiles along i and m
    int U;        // span positions of a tile: L + g*(TM-1)
    int NPT;      // span positions per wavefront tile / 32
    int NSC;      // span chunks of 32*NPT positions
    int KS;       // K-splits (workgroups per tile and span chunk)
    int NQ4;      // groups of 4 consecutive columns: ceil(N*HW / 4)
    int per_ks;   // column groups per K-split: ceil(NQ4 / KS)
    int chunk;    // consecutive workgroups of the (K-split, tile) order given to one XCD: ceil(KS * tiles / 8)
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

// T_ is the storage type of x and dy (float or bf16_t); staged values, products, sums and dw are binary32.
// VEC: H*W is a multiple of 4 and the tensors are aligned to 4 elements, so a lane's 4 consecutive columns
// lie in one sample and are one vector load; otherwise they are 4 scalar loads with their own addresses.
template <typename T_, int kPosTiles, bool VEC>
__device__ __forceinline__ void backward_weight_body(const T_* __restrict__ x, const T_* __restrict__ dy,
                                                     float* __restrict__ out, const Problem& P, const BwwTiling& T,
                                                     const int bid)
{
    typedef T_ ldvec __attribute__((ext_vector_type(4)));   // 4 consecutive columns of one row, as stored
    constexpr uint32_t ES = sizeof(T_);
    constexpr int kRows = rows_of(kPosTiles);
    constexpr int kRowB = row_bytes_of((int)ES);
    // per-wavefront staging blocks, reused after the K loop for the cross-wavefront sum; then the filter
    // and span offset of each tile row (k = -1: no such filter)
    extern __shared__ __attribute__((aligned(16))) float lds[];
    int* row_k = (int*)((char*)lds + region_bytes_of(kPosTiles, (int)ES));
    int* row_off = row_k + 32;

    // workgroup -> (K-split, tile, span chunk), tile fastest.  bid is the workgroup's index in a launch whose first
    // workgroup is a multiple of 8, so bid % 8 names the XCD and each XCD takes
    // a contiguous run of that order, so the tiles of one K-split, which read the same dy columns and
    // overlapping x windows at about the same time, share an XCD and its L2.
    const int ntile = T.IB * T.MB * T.NSC;
    const int xcd = bid & 7, slot = bid >> 3;
    const int logical = xcd * T.chunk + slot;
    if (slot >= T.chunk || logical >= T.KS * ntile) return;   // whole workgroup leaves: nobody reaches a barrier
    const int ks = logical / ntile;
    const int tix = logical % ntile;
    const int sc = tix % T.NSC, tile = tix / T.NSC;
    const int mb = tile / T.IB, ib = tile % T.IB;

    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = threadIdx.x & 63;
    const int f = lane & 31, h = lane >> 5;   // operand view: row f, half-wave h
    const int lr = lane >> 3, lc = lane & 7;  // load view: row lr of a group of 8, 16-byte column lc of 8
    const int lo = T.b.g * mb * T.TM;

    // this lane's tile row: filter k_f (one modulo per lane; other rows' filters come by lane exchange)
    int k_f, off_f;
    bool valid_f;
    tile_filter(T, P, mb, ib, f, k_f, off_f, valid_f);
    if (threadIdx.x < 32) {
        row_k[f] = valid_f ? k_f : -1;
        row_off[f] = off_f;
    }

    // byte offsets (inside one sample) of the 12 rows this lane loads: rows 8*it + lr of the block;
    // block rows 0..31 are dy rows of the tile's filters, rows 32..95 are x rows of the span chunk
    const uint32_t plane = (uint32_t)P.HW * ES;
    uint32_t rowoff[kRows / 8];
    const int ksafe = valid_f ? k_f : 0;       // rows of filters that do not exist are loaded but never stored
    const int cbase = (lo + sc * (32 * kPosTiles)) % P.Cin;
#pragma unroll
    for (int it = 0; it < kRows / 8; ++it) {
        const int row = 8 * it + lr;
        if (it < 4) {
            rowoff[it] = (uint32_t)__shfl(ksafe, row, 64) * plane;
        } else {
            int c = cbase + (row - 32);
            if (P.Cin >= 32 * kPosTiles) {     // at most one wrap
                c -= (c >= P.Cin) ? P.Cin : 0;
            } else {
                c %= P.Cin;
            }
            rowoff[it] = (uint32_t)c * plane;
        }
    }

    // column groups [qb, qe) of this wavefront: the K-split's share, split again over the waves
    const int ks_b = ks * T.per_ks < T.NQ4 ? ks * T.per_ks : T.NQ4;          // NQ4 + per_ks fits an int
    const int ks_e = ks_b + T.per_ks < T.NQ4 ? ks_b + T.per_ks : T.NQ4;
    const int per_w = (ks_e - ks_b + kWaves - 1) / kWaves;
    const int wb_ = ks_b + wave * per_w, we_ = wb_ + per_w;
    const int qb = wb_ < ks_e ? wb_ : ks_e;
    const int qe = we_ < ks_e ? we_ : ks_e;
    const int nchunk = (qe - qb + 7) / 8;     // chunks of 8 groups = 32 columns

    // this lane's column group in chunk 0, advanced by 8 groups (32 columns) per chunk; one (sample, pixel)
    // position for the whole group when it is a vector, one per column otherwise
    constexpr int NE = VEC ? 1 : 4;
    uint32_t cp[NE], offA[NE], offB[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) {
        const uint32_t col = (uint32_t)(qb + lc) * 4u + e;
        const uint32_t cn = col / (uint32_t)P.HW;
        cp[e] = col % (uint32_t)P.HW;
        offA[e] = (cn * (uint32_t)P.Cout * (uint32_t)P.HW + cp[e]) * ES;
        offB[e] = (cn * (uint32_t)P.Cin * (uint32_t)P.HW + cp[e]) * ES;
    }
    const uint32_t dn = 32u / (uint32_t)P.HW, dp = 32u % (uint32_t)P.HW;
    const uint32_t stepA = (dn * (uint32_t)P.Cout * (uint32_t)P.HW + dp) * ES;
    const uint32_t stepB = (dn * (uint32_t)P.Cin * (uint32_t)P.HW + dp) * ES;
    const uint32_t wrapA = ((uint32_t)P.Cout - 1u) * plane, wrapB = ((uint32_t)P.Cin - 1u) * plane;
    int qnext = qb + lc;                       // column group the next load_chunk call takes

    const char* ab = (const char*)dy;
    const char* bb = (const char*)x;
    char* stage = (char*)lds + wave * (kRows * kRowB);

    f32x16 acc[kPosTiles];
#pragma unroll
    for (int c = 0; c < kPosTiles; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;

    // global -> registers: 4 columns of each of this lane's rows; `rin` gets one bit per column that exists
    auto load_chunk = [&](ldvec (&r)[kRows / 8], uint32_t& rin) {
        const bool gin = qnext < qe;
        if (VEC) {
            rin = gin ? 0xfu : 0u;
            const uint32_t ca = gin ? offA[0] : 0u, cb = gin ? offB[0] : 0u;
#pragma unroll
            for (int it = 0; it < kRows / 8; ++it)
                r[it] = it < 4 ? *(const ldvec*)(ab + (ca + rowoff[it])) : *(const ldvec*)(bb + (cb + rowoff[it]));
        } else {
            rin = 0;
#pragma unroll
            for (int e = 0; e < NE; ++e) {
                const bool in = gin && (long long)qnext * 4 + e < P.NQ;
                rin |= in ? (1u << e) : 0u;
                const uint32_t ca = in ? offA[e] : 0u, cb = in ? offB[e] : 0u;
#pragma unroll
                for (int it = 0; it < kRows / 8; ++it)
                    r[it][e] = it < 4 ? *(const T_*)(ab + (ca + rowoff[it])) : *(const T_*)(bb + (cb + rowoff[it]));
            }
        }
        qnext += 8;
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            cp[e] += dp;
            const bool wr = cp[e] >= (uint32_t)P.HW;             // crossed into the next sample
            cp[e] -= wr ? (uint32_t)P.HW : 0u;
            offA[e] += stepA + (wr ? wrapA : 0u);
            offB[e] += stepB + (wr ? wrapB : 0u);
        }
    };
    auto park_chunk = [&](const ldvec (&r)[kRows / 8], uint32_t rin, bool full) {   // registers -> LDS
#pragma unroll
        for (int it = 0; it < kRows / 8; ++it) {
            char* dst = stage + (8 * it + lr) * kRowB + (int)(4 * ES) * lc;
            if constexpr (ES == 2) {                             // bf16: as stored; zeros past the range
                ldvec v = r[it];
                if (!full) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (rin >> e) & 1u ? r[it][e] : (T_)0;
                }
                *(ldvec*)dst = v;
            } else {                                             // fp32 (or widened): zeros past the range
                f32x4 v;
                if (full) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = to_f32((T_)r[it][e]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (rin >> e) & 1u ? to_f32((T_)r[it][e]) : 0.f;
                }
                *(f32x4*)dst = v;
            }
        }
    };
    auto mma_chunk = [&]() {                  // LDS -> operand layout -> matrix cores
        if constexpr (ES == 2) {
#pragma unroll
            for (int s = 0; s < 2; ++s) {     // 16 columns per instruction: half-wave h takes columns 16*s + 8*h .. +7
                const int cb = 32 * s + 16 * h;
                const bf16x8 av = __builtin_bit_cast(bf16x8, *(const u16x8*)(stage + f * kRowB + cb));
#pragma unroll
                for (int c = 0; c < kPosTiles; ++c) {
                    const bf16x8 bv = __builtin_bit_cast(bf16x8, *(const u16x8*)(stage + (32 + 32 * c + f) * kRowB + cb));
                    acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc[c], 0, 0, 0);
                }
            }
        } else {
#pragma unroll
            for (int s = 0; s < 4; ++s) {     // half-wave h takes 16-byte column 2*s + h
                const f32x4 av = *(const f32x4*)(stage + f * kRowB + 16 * (2 * s + h));
                f32x4 bv[kPosTiles];
#pragma unroll
                for (int c = 0; c < kPosTiles; ++c)
                    bv[c] = *(const f32x4*)(stage + (32 + 32 * c + f) * kRowB + 16 * (2 * s + h));
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int c = 0; c < kPosTiles; ++c)
                        acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[e], bv[c][e], acc[c], 0, 0, 0);
            }
        }
    };

    // One chunk of global loads is in flight while the matrix instructions of the previous one issue; the
    // LDS block is private to the wavefront, so the K loop needs no barrier.  (Measured: with four chunks,
    // 48 KB per wavefront, queued the first data arrives ~6 us after issue whatever the wait policy and the
    // kernel is 3 us slower: more loads in flight than bandwidth x latency only queue up.  Parking the next
    // chunk in a second LDS block during the matrix instructions was also slower.)
    ldvec r[kRows / 8];
    uint32_t in = 0;
    if (nchunk > 0) load_chunk(r, in);
    for (int ci = 0; ci < nchunk; ++ci) {
        park_chunk(r, in, qb + 8 * (ci + 1) <= qe && (long long)(qb + 8 * (ci + 1)) * 4 <= P.NQ);
        if (ci + 1 < nchunk) load_chunk(r, in);
        mma_chunk();
    }
    __syncthreads();                           // everyone is done with the staging blocks

    // wavefront partials -> LDS; accumulator register v holds row 8*(v/4) + 4*h + v%4, column f
    float* red = lds;
#pragma unroll
    for (int c = 0; c < kPosTiles; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v)
            red[(wave * 32 + 8 * (v >> 2) + 4 * h + (v & 3)) * (32 * kPosTiles) + c * 32 + f] = acc[c][v];
    __syncthreads();

    // fixed-order sum over the wavefronts, written in the layout of dw
    float* dst = out + (size_t)ks * ((size_t)P.Cout * P.L);
    for (int e = threadIdx.x; e < 32 * 32 * kPosTiles; e += kWaves * 64) {
        const int fr = e / (32 * kPosTiles), uc = e % (32 * kPosTiles);
        float s = 0.f;
#pragma unroll
        for (int wv = 0; wv < kWaves; ++wv) s += red[(wv * 32 + fr) * (32 * kPosTiles) + uc];
        const int kr = row_k[fr];
        const int j = sc * (32 * kPosTiles) + uc - row_off[fr];
        if (kr >= 0 && j >= 0 && j < P.L) dst[(size_t)kr * P.L + j] = s;
    }
}

// ---- host side: tiling of a layer -------------------------------------------------------------------------

inline int pow2_floor(int v)
{
    int p = 1;
    while (p * 2 <= v) p *= 2;
    return p;
}

// side_by_side: the kernel shares its grid with the grad-input kernel (scc_backward's merged launch).  A split
// into only two slices is then dropped: the longer main kernel hides behind the grad-input range and the reduction
// kernel goes away (measured on the 4x4 layers of the stack: 19.7 against 22.7 us; alone it is 18 against 13.6).
inline BwwTiling make_tiling(const Problem& p, bool side_by_side = false)
{
    BwwTiling t;
    t.b = make_band(p);
    t.TI = pow2_floor(t.b.F < 32 ? t.b.F : 32);
    t.TM = 32 / t.TI < t.b.P ? 32 / t.TI : t.b.P;
    t.IB = (t.b.F + t.TI - 1) / t.TI;
    t.MB = (t.b.P + t.TM - 1) / t.TM;
    t.U = p.L + t.b.g * (t.TM - 1);
    // positions per wavefront tile: the fewest operand rows over all span chunks, ties to the smaller tile
    t.NPT = 1;
    long long best = -1;
    for (int npt = 1; npt <= 3; ++npt) {
        const long long chunks = (t.U + 32 * npt - 1) / (32 * npt);
        const long long rows = chunks * (1 + npt);
        if (best < 0 || rows < best) {
            best = rows;
            t.NPT = npt;
        }
    }
    // layers with few columns are bound by latencies, not by operand rows: the narrow tile gives them more
    // workgroups per K-split (so fewer splits to reduce) and a third less LDS per workgroup, which lets more of
    // them, and of the grad-input workgroups that share their grid in scc_backward, be resident (measured on
    // the 2x2 to 8x8 layers of the stack: 1-3 us per pass, except for spans of 512 channels)
    if (p.NQ <= 8192 && t.U <= 256) t.NPT = 1;
    t.NSC = (t.U + 32 * t.NPT - 1) / (32 * t.NPT);
    t.NQ4 = (int)((p.NQ + 3) / 4);   // the last group is partial when N*H*W is not a multiple of 4
    // about one workgroup per CU (one wavefront per SIMD, deep prefetch), at least 32 column groups per wavefront
    const long long tiles = (long long)t.IB * t.MB * t.NSC;
    long long ks = (256 + tiles - 1) / tiles;
    const long long ks_max = t.NQ4 / (32 * kWaves);
    if (ks > ks_max) ks = ks_max;
    if (ks < 1) ks = 1;
    if (side_by_side && ks <= 2) ks = 1;
    t.KS = (int)ks;
    t.per_ks = (t.NQ4 + t.KS - 1) / t.KS;
    t.chunk = (int)((t.KS * tiles + 7) / 8);
    return t;
}

}  // namespace bww

}  // namespace scc
