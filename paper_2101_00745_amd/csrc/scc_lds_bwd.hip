// Fused backward pass of SCC on gfx950: grad-input and grad-weight from ONE read of dy and x.
//
//   dx[n,c,p] = sum over filters k whose window covers c of w[k,(c-s_k) mod Cin] * dy[n,k,p]
//   dw[k,j]   = sum_{n,p} dy[n,k,p] * x[n,(s_k+j) mod Cin,p]
// (Section 4.2: the input-centric gather, without atomics, and the derivative of the forward definition with
// respect to the weights.)  Run as two passes, dy crosses HBM twice; here every workgroup stages the dy rows
// and x rows it needs in LDS once and takes both products from them.
//
// Layers this kernel takes (launch_backward_fused_eligible): fp32, window starts on multiples of 32 channels
// (g == 32 in the notation of scc_band.h) and windows of L == 64 channels, so that window m covers exactly the
// channel blocks m and m+1 (cyclically), a block of 32 channels is covered by exactly the windows m-1 and m,
// and, with at most 32 filters per window, a window's filters are one 32-row tile.  The metric layer
// (256 -> 256 channels, cg = 4, co = 0.5) and the 14x14 late-stage layer are of this kind.  Other layers run
// grad-input and grad-weight as separate passes.
//
// Work item of a workgroup: (K-split ks, channel block b).  The K-split's columns (a column is one (sample,
// pixel) pair) are walked in chunks of 128, four sub-chunks of 32.  A sub-chunk is 128 rows of 32 columns:
// the dy planes of the filters of windows b-1 and b (2 x 32 rows), then the x planes of channel blocks b and
// b+1 (64 rows).  The rows go from global memory STRAIGHT INTO LDS (global_load_lds_dwordx4: no registers, no
// store instructions) into one of two 64 KB buffers, so chunk c+1 is in flight while chunk c is multiplied.
// One load instruction moves 8 rows x 128 bytes; lane 8r+c writes the c-th 16 bytes of row r's 128 and FETCHES
// piece c ^ r of the row, so piece p of row R sits at R*128 + 16*(p ^ (R & 7)) and both ways of reading a
// sub-chunk, along a row (grad-weight operands: 16 bytes = 4 consecutive columns of one row per lane) and
// across rows (grad-input operand: one column per lane), are free of bank conflicts.
//
// Eight wavefronts, two per SIMD.  Wavefronts 0-3 fetch the dy rows of sub-chunk w and then compute its dx
// tile; wavefronts 4-7 fetch the x rows of sub-chunk w-4 and compute its dw tile: the two wavefronts of a SIMD
// work on the same staged rows, one fills the matrix pipe while the other waits for LDS or issues stores.
// Per sub-chunk:
//   dx tile  [32 channels of block b] x [32 columns]  = W'(32 x 64) * dy rows(64 x 32)     -> stored at once
//   dw tile  [32 filters of window b] x [64 positions] += dy rows(32 x 32 cols) * x rows(64 x 32 cols)^T
// Both run on the bf16 matrix instruction with every binary32 operand cut EXACTLY into three bf16 pieces
// (v = hi + mid + lo) and six of the nine partial products taken (the dropped mid*lo, lo*mid, lo*lo are below
// 2^-23 of the product, the size of one binary32 rounding; sums are binary32): 6 x 32 cycles per 16 K values
// against 8 x 64 for v_mfma_f32_32x32x2_f32, paid for with about 5.5 vector instructions per value cut.
// Measured, a SIMD's matrix instructions, vector instructions and incoming loads overlap only in part, and
// this kernel is bound by their sum, not by memory: fp32 matrix instructions for both tiles measured 4 us
// slower, fp32 for the dw tile only 2.5 us slower.
// W' (the weights that multiply each (channel, filter) pair) is loaded once per wavefront, cut into its pieces
// once and stays in registers.  The dw tiles of the four wavefronts are summed through LDS in wavefront order, the K-split slices
// go to the workspace in the layout of dw and a second kernel adds them in split order: no floating-point
// atomics, bitwise reproducible.
#include "scc_band.h"
#include "scc_common.h"

namespace scc {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 8;                  // wavefronts per workgroup: 4 for dx, 4 for dw
constexpr int kSub = 4;                    // sub-chunks of 32 columns per chunk
constexpr int kRows = 128;                 // rows of a sub-chunk: 64 of dy, 64 of x
constexpr int kSubB = kRows * 128;         // bytes of a staged sub-chunk
constexpr int kBufB = kSub * kSubB;        // bytes of a buffer (one chunk)
constexpr int kInstr = 8;                  // load instructions per wavefront and chunk (64 rows of one sub-chunk)
constexpr int kStores = 16;                // dx store instructions per sub-chunk
constexpr size_t kLdsBytes = 2 * (size_t)kBufB + 32 * sizeof(int);

// 16 bytes of zeros in device memory: what lanes past the end of the column range fetch, so that a chunk is
// always kInstr loads per wavefront and columns that do not exist add nothing to dw
__device__ __attribute__((aligned(16))) float zero16[4];

struct FusedTiling {
    Band b;       // g == 32: window m starts at channel 32*m; P windows and P channel blocks
    int KS;       // K-splits (workgroups per channel block)
    int NQ4;      // groups of 4 consecutive columns: N*HW / 4
    int per_ks;   // column groups per K-split: ceil(NQ4 / KS)
    int chunk;    // consecutive workgroups of the (K-split, block) order given to one XCD: ceil(KS * P / 8)
};

__global__ __launch_bounds__(kWaves * 64) void backward_fused_lds32(const float* __restrict__ x,
                                                                    const float* __restrict__ dy,
                                                                    const float* __restrict__ w,
                                                                    float* __restrict__ dx, float* __restrict__ dwout,
                                                                    Problem P, FusedTiling T)
{
    extern __shared__ __attribute__((aligned(16))) float lds[];
    int* row_k = (int*)((char*)lds + 2 * (size_t)kBufB);

    // workgroup -> (K-split, channel block), block fastest.  blockIdx % 8 names the XCD and each XCD takes a
    // contiguous run of that order, so the blocks of one K-split, which read the same dy columns and overlapping
    // x windows at about the same time, share an XCD and its L2.
    const int nb = T.b.P;
    const int bid = blockIdx.x;
    const int xcd = bid & 7, slot = bid >> 3;
    const int logical = xcd * T.chunk + slot;
    if (slot >= T.chunk || logical >= T.KS * nb) return;      // whole workgroup leaves: nobody reaches a barrier
    const int ks = logical / nb;
    const int b = logical % nb;
    const int bm1 = b == 0 ? nb - 1 : b - 1;

    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const bool dx_role = wave < 4;            // else dw
    const int sub = wave & 3;                 // this wavefront's sub-chunk
    const int lane = threadIdx.x & 63;
    const int f = lane & 31, h = lane >> 5;   // operand view: row or column f, half-wave h
    const int lr = lane >> 3, lc = lane & 7;  // load view: row lr of a group of 8, LDS piece lc of that row

    // filters of window m: k = r(m) + P*i, r(m) = (m * inv) mod P (scc_band.h)
    const int r_b = (int)(((uint32_t)b * (uint32_t)T.b.inv) % (uint32_t)nb);
    const int r_bm1 = (int)(((uint32_t)bm1 * (uint32_t)T.b.inv) % (uint32_t)nb);
    if (threadIdx.x < 32) {
        const int k = r_b + nb * f;            // row f of the dw tile
        row_k[f] = k < P.Cout ? k : -1;
    }

    // byte offsets (inside one sample) of the rows this lane loads: rows 8*it + lr of the dy half (wavefronts
    // 0-3) or of the x half (wavefronts 4-7) of a sub-chunk.  Rows of filters that do not exist load plane 0;
    // they meet zero weights in dx and are never stored in dw.
    const uint32_t plane = (uint32_t)P.HW * 4u;
    uint32_t rowoff[kInstr];
#pragma unroll
    for (int it = 0; it < kInstr; ++it) {
        const int row = 8 * it + lr;           // 0..63 inside the half
        if (dx_role) {
            const int k = (it < 4 ? r_bm1 : r_b) + nb * (row & 31);
            rowoff[it] = (uint32_t)(k < P.Cout ? k : 0) * plane;
        } else {
            int c = 32 * b + row;
            c -= (c >= P.Cin) ? P.Cin : 0;     // block b+1 of the last window is block 0
            rowoff[it] = (uint32_t)c * plane;
        }
    }

    // column groups [ks_b, ks_e) of this K-split; chunk c is groups [ks_b + 32c, +32), this wavefront's
    // sub-chunk the 8 groups from ks_b + 32c + 8*sub
    const int ks_b = ks * T.per_ks < T.NQ4 ? ks * T.per_ks : T.NQ4;
    const int ks_e = ks_b + T.per_ks < T.NQ4 ? ks_b + T.per_ks : T.NQ4;
    const int nchunk = (ks_e - ks_b + 31) / 32;
    const int q0 = ks_b + 8 * sub;

    // load view: this lane's column group in chunk 0 (piece lc ^ lr of the sub-chunk's 128 bytes per row)
    const uint32_t tensor_rows = dx_role ? (uint32_t)P.Cout : (uint32_t)P.Cin;   // planes per sample of what is loaded
    int qload = q0 + (lc ^ lr);
    uint32_t cpl, offL;
    {
        const uint32_t col = (uint32_t)qload * 4u;
        const uint32_t cn = col / (uint32_t)P.HW;
        cpl = col % (uint32_t)P.HW;
        offL = (cn * tensor_rows * (uint32_t)P.HW + cpl) * 4u;
    }
    // store view (dx wavefronts): this lane's column in chunk 0 (column f of the sub-chunk)
    int qstore = q0 + (f >> 2);
    uint32_t cps, offD;
    {
        const uint32_t col = (uint32_t)q0 * 4u + (uint32_t)f;
        const uint32_t cn = col / (uint32_t)P.HW;
        cps = col % (uint32_t)P.HW;
        offD = (cn * (uint32_t)P.Cin * (uint32_t)P.HW + cps) * 4u;
    }
    const uint32_t dn = 128u / (uint32_t)P.HW, dp = 128u % (uint32_t)P.HW;   // a chunk further: 128 columns
    const uint32_t stepL = (dn * tensor_rows * (uint32_t)P.HW + dp) * 4u, wrapL = (tensor_rows - 1u) * plane;
    const uint32_t stepD = (dn * (uint32_t)P.Cin * (uint32_t)P.HW + dp) * 4u, wrapD = ((uint32_t)P.Cin - 1u) * plane;

    const char* lb = dx_role ? (const char*)dy : (const char*)x;
    char* db = (char*)dx + (size_t)(32 * b) * plane;           // first plane of channel block b
    // this wavefront's half of its sub-chunk inside a buffer, and the whole sub-chunk it computes on
    const int ld_ofs = sub * kSubB + (dx_role ? 0 : 64 * 128);
    const int sub_ofs = sub * kSubB;

    typedef const __attribute__((address_space(1))) void* gptr_t;
    typedef __attribute__((address_space(3))) void* lptr_t;
    const char* const zeros = (const char*)zero16;
    auto issue = [&](int buf) {                // this wavefront's 64 rows of one chunk: global -> LDS buffer `buf`
        const bool gin = qload < ks_e;
        const char* const base = gin ? lb + offL : zeros;      // one 64-bit select per chunk, no branches
        const uint32_t keep = gin ? 0xffffffffu : 0u;
        char* sb = (char*)lds + buf * kBufB + ld_ofs;
#pragma unroll
        for (int it = 0; it < kInstr; ++it)
            __builtin_amdgcn_global_load_lds((gptr_t)(base + (rowoff[it] & keep)), (lptr_t)(sb + it * 1024), 16, 0, 0);
        qload += 32;
        cpl += dp;
        const bool wr = cpl >= (uint32_t)P.HW;  // crossed into the next sample
        cpl -= wr ? (uint32_t)P.HW : 0u;
        offL += stepL + (wr ? wrapL : 0u);
    };

    // W' (dx wavefronts): the K values of a matrix instruction are 16 stage rows; lane (f, h) holds, for K group
    // gk, the weights that multiply stage rows 16gk + 8h + e, e < 8 (filters of window b-1 for rows 0..31, of
    // window b for rows 32..63) into channel 32b+f: position 32+f of the former window's filters, position f of
    // the latter's.  Cut into bf16 pieces once.
    // The weights are requested first (loads complete in order: behind the first chunk they would arrive
    // last), then the first chunk; the pieces are cut while the chunk is in flight.
    float wv[4][8];
#pragma unroll
    for (int gk = 0; gk < 4; ++gk)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int row = 16 * gk + 8 * h + e;
            const int k = (gk < 2 ? r_bm1 : r_b) + nb * (row & 31);
            const int j = (gk < 2 ? 32 : 0) + f;
            wv[gk][e] = (dx_role && k < P.Cout) ? w[(size_t)k * 64 + j] : 0.f;
        }
    __builtin_amdgcn_sched_barrier(0);
    if (nchunk > 0) issue(0);
    __builtin_amdgcn_sched_barrier(0);
    uint32_t a_hi[4][4], a_mid[4][4], a_lo[4][4];
#pragma unroll
    for (int gk = 0; gk < 4; ++gk) split3<8>([&](int e) { return wv[gk][e]; }, a_hi[gk], a_mid[gk], a_lo[gk]);

    f32x16 acc_w[2];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc_w[c][v] = 0.f;

    // LDS byte offsets of this lane's operand reads inside a staged sub-chunk
    // grad-input: row 16gk + 8h + e, column f -> piece (f>>2) ^ e (the row number mod 8 is e), word f & 3
    const int dx_rd = 8 * h * 128 + 4 * (f & 3);
    const int dx_piece = f >> 2;
    // grad-weight: rows 32+f (dy) and 64+32c+f (x); K group gk of half-wave h is columns 16gk + 8h .. +7 of the
    // sub-chunk: the 16-byte pieces 4gk + 2h and 4gk + 2h + 1, at positions piece ^ (f & 7)
    const int dw_a = (32 + f) * 128, dw_b = (64 + f) * 128;

    auto compute_dx = [&](int buf) -> bool {   // returns whether the tile was stored
        const char* sb = (const char*)lds + buf * kBufB + sub_ofs;
        // two accumulators, so that a matrix instruction does not wait for the one right before it
        f32x16 acc, acc2;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = acc2[v] = 0.f;
        // all 32 operand values of the tile are requested from LDS at once; then the pieces of K group gk+1 are
        // cut (vector ALU) while the matrix instructions of group gk run
        float bv[4][8];
#pragma unroll
        for (int gk = 0; gk < 4; ++gk)
#pragma unroll
            for (int e = 0; e < 8; ++e)
                bv[gk][e] = *(const float*)(sb + dx_rd + (16 * gk + e) * 128 + 16 * (dx_piece ^ e));
        uint32_t bh[2][4], bm[2][4], bl[2][4];
        split3<8>([&](int e) { return bv[0][e]; }, bh[0], bm[0], bl[0]);
#pragma unroll
        for (int gk = 0; gk < 4; ++gk) {
            const int cur = gk & 1, nxt = cur ^ 1;
            if (gk + 1 < 4) split3<8>([&](int e) { return bv[gk + 1][e]; }, bh[nxt], bm[nxt], bl[nxt]);
            acc = mfma_bf16<8>(a_lo[gk], bh[cur], acc);
            acc2 = mfma_bf16<8>(a_hi[gk], bl[cur], acc2);
            acc = mfma_bf16<8>(a_mid[gk], bm[cur], acc);
            acc2 = mfma_bf16<8>(a_mid[gk], bh[cur], acc2);
            acc = mfma_bf16<8>(a_hi[gk], bm[cur], acc);
            acc2 = mfma_bf16<8>(a_hi[gk], bh[cur], acc2);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] += acc2[v];
        const bool any = __builtin_amdgcn_readfirstlane(qstore - (f >> 2)) < ks_e;   // the sub-chunk's first group exists
        if (qstore < ks_e) {
            // accumulator register v holds channel 32b + 8*(v/4) + 4*h + v%4, column f of the sub-chunk
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const uint32_t ch = (uint32_t)(8 * (v >> 2) + 4 * h + (v & 3));
                __builtin_nontemporal_store(acc[v], (float*)(db + (offD + ch * plane)));   // written once, never re-read
            }
        }
        qstore += 32;
        cps += dp;
        const bool wr = cps >= (uint32_t)P.HW;
        cps -= wr ? (uint32_t)P.HW : 0u;
        offD += stepD + (wr ? wrapD : 0u);
        return any;
    };
    auto compute_dw = [&](int buf) {
        const char* sb = (const char*)lds + buf * kBufB + sub_ofs;
        // all operand rows of the chunk are requested from LDS at once (12 reads of 16 bytes per lane); then the
        // pieces of K group 1 are cut while the matrix instructions of group 0 run
        f32x4 ra[2][2], rb[2][2][2];           // [K group][16-byte piece], [K group][position tile][piece]
#pragma unroll
        for (int gk = 0; gk < 2; ++gk) {
            const int p0 = 16 * ((4 * gk + 2 * h) ^ (f & 7)), p1 = 16 * ((4 * gk + 2 * h + 1) ^ (f & 7));
            ra[gk][0] = *(const f32x4*)(sb + dw_a + p0);
            ra[gk][1] = *(const f32x4*)(sb + dw_a + p1);
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                rb[gk][c][0] = *(const f32x4*)(sb + dw_b + c * 32 * 128 + p0);
                rb[gk][c][1] = *(const f32x4*)(sb + dw_b + c * 32 * 128 + p1);
            }
        }
        uint32_t ah[2][4], am[2][4], al[2][4], bh[2][2][4], bm[2][2][4], bl[2][2][4];
        auto cut = [&](int gk) {
            split3<8>([&](int e) { return e < 4 ? ra[gk][0][e] : ra[gk][1][e - 4]; }, ah[gk], am[gk], al[gk]);
#pragma unroll
            for (int c = 0; c < 2; ++c)
                split3<8>([&](int e) { return e < 4 ? rb[gk][c][0][e] : rb[gk][c][1][e - 4]; }, bh[gk][c], bm[gk][c],
                          bl[gk][c]);
        };
        cut(0);
#pragma unroll
        for (int gk = 0; gk < 2; ++gk) {
            if (gk == 0) cut(1);
            // the two position tiles take turns, so that no matrix instruction waits for the one right before it
            acc_w[0] = mfma_bf16<8>(al[gk], bh[gk][0], acc_w[0]);
            acc_w[1] = mfma_bf16<8>(al[gk], bh[gk][1], acc_w[1]);
            acc_w[0] = mfma_bf16<8>(ah[gk], bl[gk][0], acc_w[0]);
            acc_w[1] = mfma_bf16<8>(ah[gk], bl[gk][1], acc_w[1]);
            acc_w[0] = mfma_bf16<8>(am[gk], bm[gk][0], acc_w[0]);
            acc_w[1] = mfma_bf16<8>(am[gk], bm[gk][1], acc_w[1]);
            acc_w[0] = mfma_bf16<8>(am[gk], bh[gk][0], acc_w[0]);
            acc_w[1] = mfma_bf16<8>(am[gk], bh[gk][1], acc_w[1]);
            acc_w[0] = mfma_bf16<8>(ah[gk], bm[gk][0], acc_w[0]);
            acc_w[1] = mfma_bf16<8>(ah[gk], bm[gk][1], acc_w[1]);
            acc_w[0] = mfma_bf16<8>(ah[gk], bh[gk][0], acc_w[0]);
            acc_w[1] = mfma_bf16<8>(ah[gk], bh[gk][1], acc_w[1]);
        }
    };

    // Two buffers.  Per chunk: wait for this wavefront's loads of chunk c; barrier (now every wavefront's loads
    // of chunk c have landed, and every wavefront is done reading the other buffer); request chunk c+1 into the
    // other buffer; multiply chunk c.  Completion of vector memory instructions is reported in issue order, and a
    // dx wavefront issues, per chunk, its loads and then either kStores stores or none, so waiting until at
    // most kStores (or 0) instructions are outstanding leaves the stores to drain during the next chunk.
    // (The two kinds of wavefront run their own copy of the loop, so that each keeps its own accumulators in
    // place; both execute the same number of barriers.)
    if (dx_role) {
        bool stored_prev = false;
        for (int c = 0; c < nchunk; ++c) {
            if (stored_prev)
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kStores) : "memory");
            else
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            if (c + 1 < nchunk) issue((c + 1) & 1);
            stored_prev = compute_dx(c & 1);
        }
    } else {
        for (int c = 0; c < nchunk; ++c) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            if (c + 1 < nchunk) issue((c + 1) & 1);
            compute_dw(c & 1);
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();              // everyone is done with the staging buffers
    asm volatile("" ::: "memory");

    // wavefront partials of the dw tile -> LDS; accumulator register v holds row 8*(v/4) + 4*h + v%4, column f
    float* red = lds;
    if (!dx_role) {
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                red[(sub * 32 + 8 * (v >> 2) + 4 * h + (v & 3)) * 64 + c * 32 + f] = acc_w[c][v];
    }
    __syncthreads();

    // fixed-order sum over the four dw wavefronts, written in the layout of dw (this K-split's slice, or dw itself)
    float* dst = dwout + (size_t)ks * ((size_t)P.Cout * 64);
    for (int e = threadIdx.x; e < 32 * 64; e += kWaves * 64) {
        const int fr = e >> 6, j = e & 63;
        float s = 0.f;
#pragma unroll
        for (int wv = 0; wv < 4; ++wv) s += red[(wv * 32 + fr) * 64 + j];
        const int kr = row_k[fr];
        if (kr >= 0) dst[(size_t)kr * 64 + j] = s;
    }
}

FusedTiling make_fused_tiling(const Problem& p)
{
    FusedTiling t;
    t.b = make_band(p);
    t.NQ4 = (int)(p.NQ / 4);
    // about one workgroup per CU (its staging buffers fill the LDS), at least two chunks of 128 columns each
    long long ks = (256 + t.b.P - 1) / t.b.P;
    const long long ks_max = t.NQ4 / 64;
    if (ks > ks_max) ks = ks_max;
    if (ks < 1) ks = 1;
    t.KS = (int)ks;
    t.per_ks = (t.NQ4 + t.KS - 1) / t.KS;
    t.chunk = (int)(((long long)t.KS * t.b.P + 7) / 8);
    return t;
}

}  // namespace

bool backward_fused_eligible(const Problem& p)
{
    if (p.L != 64 || p.stride == 0 || p.HW % 4 != 0 || p.NQ < 256) return false;
    const Band b = make_band(p);
    if (b.g != 32 || b.P < 2 || b.F > 32) return false;       // P >= 2: windows b-1 and b are different windows
    const long long rows = p.Cin > p.Cout ? p.Cin : p.Cout;
    return (long long)p.NQ * rows * 4 < (1ll << 32) && (long long)p.Cout * p.L * 4 < (1ll << 31);
}

size_t backward_fused_workspace(const Problem& p)
{
    const FusedTiling t = make_fused_tiling(p);
    return t.KS > 1 ? (size_t)t.KS * p.Cout * p.L * sizeof(float) : 0;
}

hipError_t launch_backward_fused(const float* x, const float* dy, const float* w, float* dx, float* dw,
                                 float* workspace, const Problem& p, hipStream_t st)
{
    const FusedTiling t = make_fused_tiling(p);
    static const hipError_t allowed = hipFuncSetAttribute((const void*)backward_fused_lds32,
                                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes);
    if (allowed != hipSuccess) return allowed;
    float* out = t.KS > 1 ? workspace : dw;
    backward_fused_lds32<<<dim3((unsigned)(8 * t.chunk)), dim3(kWaves * 64), kLdsBytes, st>>>(x, dy, w, dx, out, p, t);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || t.KS == 1) return e;
    return launch_weight_reduce(workspace, dw, p.Cout * p.L, t.KS, st);
}

}  // namespace scc
