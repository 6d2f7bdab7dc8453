// Forward SCC on the gfx950 matrix cores for layers in which MANY 32-filter tiles read the same channels
// (few, long windows: cg <= 2; many filters per window; windows that start on every channel, as in the
// channel-expanding layers): the activation operand goes through LDS once per workgroup.
//
// y[n,k,p] = sum_j w[k,j] * x[n,(s_k+j) mod Cin,p]   (Section 4.2, output-centric forward)
//
// scc_mfma_fwd.hip gives every 32-filter tile its own wavefront, which fetches the tile's channel planes from
// L1/L2 and cuts every binary32 value into three bf16 pieces for itself.  When T tiles cover a channel, that is T
// fetches and T cuts of the same value; on such layers the kernel is bound by L2 -> L1 traffic and by the vector
// work of the cuts, not by HBM.  Here a workgroup of four wavefronts owns four consecutive tiles of scc_band.h's
// (window, filter) grid for the same 128 columns and walks the union of their channel spans in rounds of 32
// channels: the 256 lanes fetch a round (32 planes x 128 columns, one 16-byte load per lane and plane, 4 planes
// per lane), cut each value ONCE and park the bf16 pieces in LDS in the matrix instruction's operand layout
// (8 channels of one column = 16 bytes); every wavefront then takes its B operands from there with 16-byte LDS
// reads and no vector work.  A round a tile's own span does not reach is skipped by that wavefront.  Weights (A)
// are staged per wavefront as in scc_mfma_fwd.hip: coalesced reads of 32 consecutive weights per filter, cut once,
// zeros outside the filter's window, parked in a wavefront-private LDS block.  Two B buffers and two register
// sets: the loads of rounds r+1 and r+2 are in flight while round r is multiplied, one barrier per round.
//
// fp32 tensors, planes whose size is a multiple of 4 and 16-byte aligned tensors only (a lane owns 4 consecutive
// columns); the products are the six-of-nine bf16 partial products of scc_common.h, sums binary32.
#include <type_traits>

#include "scc_band.h"
#include "scc_common.h"

namespace scc {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWavesS = 4;                  // wavefronts (= tiles) per workgroup
constexpr int kColsS = 128;                 // columns per workgroup
constexpr int kRound = 32;                  // channels per round: two K groups of 16
constexpr int kBPiece = 2 * 2 * kColsS * 16;   // bytes of one bf16 piece of a round's B operands: [K group][half][column][8 ch]
constexpr int kBBuf = 3 * kBPiece;          // one B buffer
constexpr int kAHalf = 32 * 16 + 16;        // bytes of the 32 rows of one (K group, half-wave) of A, padded
constexpr int kAPiece = 4 * kAHalf;
constexpr int kABlock = 3 * kAPiece;        // a wavefront's A block
constexpr int kLdsS = 2 * kBBuf + kWavesS * kABlock;   // 73 KB: two workgroups per CU

struct SharedTiling {
    Band b;
    int TI, TM;    // tile = TM window starts x TI filters per start (32 rows)
    int IB, MB;    // tiles along the filter and the window axis; tile index = mb*IB + ib
    int U;         // channels a tile spans: L + g*(TM-1)
    int FG;        // workgroups per column tile: ceil(IB*MB / 4)
    int total;     // workgroups with work
    int chunk;     // consecutive workgroups given to one XCD
};

// AL4: g and L are multiples of 4, so a group of four consecutive weights is wholly inside or outside a window
template <bool AL4>
__global__ __launch_bounds__(kWavesS * 64, 2) void forward_shared32(const float* __restrict__ x,
                                                                 const float* __restrict__ w, float* __restrict__ y,
                                                                 Problem P, SharedTiling T)
{
    extern __shared__ __attribute__((aligned(16))) char lds_s[];
    char* const b_lds = lds_s;                   // two B buffers
    char* const a_lds = lds_s + 2 * kBBuf;       // then one A block per wavefront

    // workgroup -> (column tile, group of four tiles), group fastest; each XCD takes a contiguous run of that order
    const int bid = blockIdx.x;
    const int xcd = bid & 7, slot = bid >> 3;
    const int logical = xcd * T.chunk + slot;
    if (slot >= T.chunk || logical >= T.total) return;         // the whole workgroup leaves
    const int ct = logical / T.FG, fg = logical % T.FG;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int ntiles = T.IB * T.MB;
    const int tile = fg * kWavesS + wave;
    const bool tvalid = tile < ntiles;
    const int mb = (tvalid ? tile : ntiles - 1) / T.IB, ib = (tvalid ? tile : ntiles - 1) % T.IB;
    const int mb_first = (fg * kWavesS) / T.IB;
    const int last = fg * kWavesS + kWavesS - 1 < ntiles ? fg * kWavesS + kWavesS - 1 : ntiles - 1;
    const int mb_last = last / T.IB;
    const int span_step = T.b.g * T.TM;                        // channels between the spans of adjacent mb
    const int lo = span_step * mb_first;                       // first channel of the workgroup's walk (< Cin)
    const int walk = span_step * (mb_last - mb_first) + T.U;   // channels walked
    const int nround = (walk + kRound - 1) / kRound;
    const int d0 = span_step * (mb - mb_first);                // this tile's span is walk positions [d0, d0 + U)
    auto group_active = [&](int pos) { return tvalid && pos + 16 > d0 && pos < d0 + T.U; };
    auto round_active = [&](int r) { return tvalid && kRound * r + kRound > d0 && kRound * r < d0 + T.U; };

    const int lane = threadIdx.x & 63;
    const int f = lane & 31, h = lane >> 5;

    // ---- A side: the filter of tile row f --------------------------------------------------------------
    const int mi = f / T.TI, ii = f % T.TI;
    const int m = mb * T.TM + mi, i = ib * T.TI + ii;
    const int k = (int)(((uint32_t)m * (uint32_t)T.b.inv) % (uint32_t)T.b.P) + T.b.P * i;
    const bool fvalid = tvalid && (mi < T.TM) && (m < T.b.P) && (k < P.Cout);
    const int offv = fvalid ? d0 + T.b.g * mi : (1 << 30);     // walk position of the filter's first weight
    const int wrow = (fvalid ? k : 0) * P.L;
    char* A = a_lds + wave * kABlock;
    // staging lane (row 8*it + lane/8, group c = lane%8 of four weights): walk positions 32r + 4c .. +3, which
    // are K group c/4, half-wave (c/2)%2, values 4*(c%2) .. +3 of the operand
    const int sc = lane & 7;
    const int a_dst = ((sc >> 2) * 2 + ((sc >> 1) & 1)) * kAHalf + 8 * (sc & 1);
    int sro[4], srw[4];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        sro[it] = __shfl(offv, 8 * it + (lane >> 3), 64);
        srw[it] = __shfl(wrow, 8 * it + (lane >> 3), 64);
    }
    // two register sets: set (r & 1) takes the raw loads of round r, two rounds ahead of its use
    f32x4 ga[2][4];                                            // raw loaded weights; masked when parked
    uint32_t gam[2] = {0u, 0u};                                // bit 4*it + q: weight q of group `it` is inside the window
    auto issue_a = [&](auto SET, int r) {
        constexpr int set = decltype(SET)::value;
        gam[set] = 0;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int j0 = kRound * r + 4 * sc - sro[it];
            if (AL4) {
                const bool in = j0 >= 0 && j0 < P.L;
                ga[set][it] = *(const f32x4*)(w + (in ? srw[it] + j0 : 0));
                gam[set] |= in ? (0xfu << (4 * it)) : 0u;
            } else {
                // windows that start anywhere: the four weights are masked one by one, but still fetched with one
                // 16-byte load (4-byte aligned; what it reads beside the window belongs to the same or the next
                // filter's row) unless that load would leave the weight tensor, at its very first or last elements
                uint32_t m4 = 0;
#pragma unroll
                for (int q = 0; q < 4; ++q) m4 |= (j0 + q >= 0 && j0 + q < P.L) ? (1u << q) : 0u;
                const int e0 = srw[it] + j0;
                if (m4 == 0u || (e0 >= 0 && e0 + 4 <= P.Cout * P.L)) {
                    typedef float f32x4u __attribute__((ext_vector_type(4), aligned(4)));
                    ga[set][it] = *(const f32x4u*)(w + (m4 ? e0 : 0));
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q) ga[set][it][q] = w[(m4 >> q) & 1u ? e0 + q : 0];
                }
                gam[set] |= m4 << (4 * it);
            }
        }
    };
    auto commit_a = [&](auto SET) {
        constexpr int set = decltype(SET)::value;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            uint32_t hi[2], mid[2], lo3[2];
            const uint32_t m4 = gam[set] >> (4 * it);
            const float v[4] = {m4 & 1u ? ga[set][it][0] : 0.f, m4 & 2u ? ga[set][it][1] : 0.f,
                                m4 & 4u ? ga[set][it][2] : 0.f, m4 & 8u ? ga[set][it][3] : 0.f};
            split3<4>([&](int e) { return v[e]; }, hi, mid, lo3);
            char* dst = A + a_dst + (8 * it + (lane >> 3)) * 16;
            *(u32x2*)dst = u32x2{hi[0], hi[1]};
            *(u32x2*)(dst + kAPiece) = u32x2{mid[0], mid[1]};
            *(u32x2*)(dst + 2 * kAPiece) = u32x2{lo3[0], lo3[1]};
        }
    };

    // ---- B side, loading role: thread (u = tid/32, q = tid%32) fetches the 4 columns 4q..4q+3 of the 4 planes at
    // walk positions 32r + 4u + e: K group u/4, half-wave (u/2)%2, operand values 4*(u%2) + e
    const int tid = threadIdx.x;
    const int lq = tid & 31, lu = tid >> 5;
    const uint32_t plane = (uint32_t)P.HW * 4u, wrapb = (uint32_t)P.Cin * plane;
    uint32_t lcol;                                             // byte offset of this thread's 4 columns in plane 0 of their sample
    {
        const uint32_t q = (uint32_t)ct * kColsS + 4u * (uint32_t)lq;
        const uint32_t qq = q < (uint32_t)P.NQ ? q : 0u;       // columns past the end read column 0 and are never stored
        const uint32_t n = qq / (uint32_t)P.HW, p = qq % (uint32_t)P.HW;
        lcol = (n * (uint32_t)P.Cin * (uint32_t)P.HW + p) * 4u;
    }
    uint32_t lrow[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) lrow[e] = (uint32_t)((lo + 4 * lu + e) % P.Cin) * plane;
    const uint32_t round_b = (uint32_t)(kRound % P.Cin) * plane;   // a round further, modulo the channel count
    const int b_dst = (((lu >> 2) * 2 + ((lu >> 1) & 1)) * kColsS + lq) * 16 + 8 * (lu & 1);
    const char* xb = (const char*)x;
    f32x4 braw[2][4];
    auto issue_b = [&](auto SET) {                             // the next round of the walk (cyclic: always in bounds)
        constexpr int set = decltype(SET)::value;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            braw[set][e] = *(const f32x4*)(xb + (lcol + lrow[e]));
            lrow[e] += round_b;
            lrow[e] -= lrow[e] >= wrapb ? wrapb : 0u;
        }
    };
    auto commit_b = [&](auto SET) {                            // set s -> LDS buffer s
        constexpr int set = decltype(SET)::value;
        char* dst = b_lds + set * kBBuf + b_dst;
#pragma unroll
        for (int j = 0; j < 4; ++j) {                           // column 4q + j is operand column (j, q): LDS column 32j + q
            uint32_t hi[2], mid[2], lo3[2];
            split3<4>([&](int e) { return braw[set][e][j]; }, hi, mid, lo3);
            *(u32x2*)(dst + j * 32 * 16) = u32x2{hi[0], hi[1]};
            *(u32x2*)(dst + j * 32 * 16 + kBPiece) = u32x2{mid[0], mid[1]};
            *(u32x2*)(dst + j * 32 * 16 + 2 * kBPiece) = u32x2{lo3[0], lo3[1]};
        }
    };

    f32x16 acc[4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;

    // one K group (16 channels) of round r, B operands from LDS buffer `buf`
    auto compute = [&](int r, int s, int buf) {
        if (!group_active(kRound * r + 16 * s)) return;
        const char* bb = b_lds + buf * kBBuf + f * 16;
        uint32_t ap[3][4];
#pragma unroll
        for (int q = 0; q < 3; ++q) {
            const u32x4 t = *(const u32x4*)(A + q * kAPiece + (s * 2 + h) * kAHalf + f * 16);
#pragma unroll
            for (int z = 0; z < 4; ++z) ap[q][z] = t[z];
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            uint32_t bp[3][4];
#pragma unroll
            for (int q = 0; q < 3; ++q) {
                const u32x4 t = *(const u32x4*)(bb + q * kBPiece + ((s * 2 + h) * kColsS + c * 32) * 16);
#pragma unroll
                for (int z = 0; z < 4; ++z) bp[q][z] = t[z];
            }
            acc[c] = mfma_bf16<8>(ap[2], bp[0], acc[c]);
            acc[c] = mfma_bf16<8>(ap[0], bp[2], acc[c]);
            acc[c] = mfma_bf16<8>(ap[1], bp[1], acc[c]);
            acc[c] = mfma_bf16<8>(ap[1], bp[0], acc[c]);
            acc[c] = mfma_bf16<8>(ap[0], bp[1], acc[c]);
            acc[c] = mfma_bf16<8>(ap[0], bp[0], acc[c]);
        }
    };

    // Round r lives in register set r & 1 while in flight and in LDS buffer r & 1 once parked.  Rounds 0 and 1 are
    // requested up front; then, per round r: request round r+2 (into the set round r came from), multiply the first
    // K group, park round r+1's B operands (cut while the matrix pipe is busy; the barrier that ended round r-1
    // says every wavefront is done with that buffer), multiply the second K group, park round r+1's weights (the
    // wavefront's own block: its reads of round r are done), barrier.  No load is conditional inside the loop (a
    // wait behind a branch that may have issued loads has to assume it did not, and would wait for the newest
    // request as well): the loop body runs while a round r+3 exists and the last rounds are written out.
    typedef std::integral_constant<int, 0> Set0;
    typedef std::integral_constant<int, 1> Set1;
    auto body = [&](auto PAR, auto OTHER, int r, auto ISSUE, auto COMMIT) {
        if constexpr (decltype(ISSUE)::value) {
            issue_a(PAR, r + 2);
            issue_b(PAR);
        }
        compute(r, 0, decltype(PAR)::value);
        if constexpr (decltype(COMMIT)::value) commit_b(OTHER);
        compute(r, 1, decltype(PAR)::value);
        if constexpr (decltype(COMMIT)::value) {
            if (round_active(r + 1)) commit_a(OTHER);
        }
        __syncthreads();
    };
    const std::true_type yes;
    const std::false_type no;
    issue_a(Set0(), 0);
    issue_b(Set0());
    issue_a(Set1(), 1);                                        // harmless when the walk has a single round: in bounds, never parked
    issue_b(Set1());
    if (round_active(0)) commit_a(Set0());
    commit_b(Set0());
    __syncthreads();
    int r = 0;
    for (; r + 3 < nround; r += 2) {
        body(Set0(), Set1(), r, yes, yes);
        body(Set1(), Set0(), r + 1, yes, yes);
    }
    const int rem = nround - r;                                // 1, 2 or 3 rounds left; r is even
    if (rem == 3) {
        body(Set0(), Set1(), r, yes, yes);
        body(Set1(), Set0(), r + 1, no, yes);
        body(Set0(), Set1(), r + 2, no, no);
    } else if (rem == 2) {
        body(Set0(), Set1(), r, no, yes);
        body(Set1(), Set0(), r + 1, no, no);
    } else {
        body(Set0(), Set1(), r, no, no);
    }
    if (!tvalid) return;

    // ---- store: accumulator register v holds tile row 8*(v/4) + 4*h + v%4, columns 4f .. 4f+3 of the tile ----
    // (every lane stays for the shuffles: lane fr holds the filter of tile row fr)
    const uint32_t q = (uint32_t)ct * kColsS + 4u * (uint32_t)f;
    const bool qlive = q < (uint32_t)P.NQ;
    const uint32_t qq = qlive ? q : 0u;
    const uint32_t n = qq / (uint32_t)P.HW, p = qq % (uint32_t)P.HW;
    float* yb = y + (size_t)n * P.Cout * P.HW + p;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int fr = 8 * (v >> 2) + 4 * h + (v & 3);
        const int kr = __shfl(k, fr, 64);
        const bool rvalid = __shfl((int)fvalid, fr, 64) != 0;
        if (rvalid && qlive) {
            const f32x4 o = {acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
            __builtin_nontemporal_store(o, (f32x4*)(yb + (size_t)kr * P.HW));   // written once, never re-read here
        }
    }
}

int pow2_floor_s(int v)
{
    int p = 1;
    while (p * 2 <= v) p *= 2;
    return p;
}

SharedTiling make_shared_tiling(const Problem& p)
{
    SharedTiling t;
    t.b = make_band(p);
    t.TI = pow2_floor_s(t.b.F < 32 ? t.b.F : 32);
    t.TM = 32 / t.TI < t.b.P ? 32 / t.TI : t.b.P;
    t.IB = (t.b.F + t.TI - 1) / t.TI;
    t.MB = (t.b.P + t.TM - 1) / t.TM;
    t.U = p.L + t.b.g * (t.TM - 1);
    t.FG = (t.IB * t.MB + kWavesS - 1) / kWavesS;
    const long long nct = (p.NQ + kColsS - 1) / kColsS;
    t.total = (int)(nct * t.FG);
    t.chunk = (t.total + 7) / 8;
    return t;
}

}  // namespace

bool forward_shared_eligible(const float* x, const float* w, const float* y, const Problem& p)
{
    const uintptr_t addr = (uintptr_t)x | (uintptr_t)y | (uintptr_t)w;
    if (!forward_mfma_eligible(p) || p.HW % 4 != 0 || (addr & 15) != 0) return false;
    const SharedTiling t = make_shared_tiling(p);
    return (long long)((p.NQ + kColsS - 1) / kColsS) * t.FG < (1ll << 28);
}

// Channels fetched by the tiles of a layer when every tile fetches its own span, over the channels fetched when
// four consecutive tiles share their walk: what sharing saves in fetches and cuts.
double forward_shared_gain(const Problem& p)
{
    const SharedTiling t = make_shared_tiling(p);
    const int ntiles = t.IB * t.MB;
    long long own = 0, sharedc = 0;
    for (int fg = 0; fg < t.FG; ++fg) {
        const int first = fg * kWavesS, last = first + kWavesS - 1 < ntiles ? first + kWavesS - 1 : ntiles - 1;
        own += (long long)(last - first + 1) * ((t.U + 15) / 16 * 16);
        const int walk = t.b.g * t.TM * (last / t.IB - first / t.IB) + t.U;
        sharedc += (walk + kRound - 1) / kRound * kRound;
    }
    return (double)own / (double)sharedc;
}

// Measured: the shared walk wins where four consecutive tiles fetch at least three times the channels of their
// common walk (c4 channel-expanding layer 3.3x: 115 against 137-160 us; cg = 1 at the metric shape 4x: 39 against
// 45 us) and the grid still fills the chip (two workgroups per CU); at 2.7x and below (cg = 2, co = 0.25, the
// metric layer) and on the few-column layers of the stack the per-tile kernel is as fast or faster.
bool forward_shared_preferred(const float* x, const float* w, const float* y, const Problem& p)
{
#ifdef SCC_SHARED_ALWAYS
    return forward_shared_eligible(x, w, y, p);
#else
    if (!forward_shared_eligible(x, w, y, p)) return false;
    const SharedTiling t = make_shared_tiling(p);
    return t.total >= 512 && forward_shared_gain(p) >= 3.0;
#endif
}

hipError_t launch_forward_shared(const float* x, const float* w, float* y, const Problem& p, hipStream_t st)
{
    const SharedTiling t = make_shared_tiling(p);
    const bool al4 = (t.b.g % 4 == 0) && (p.L % 4 == 0);
    const dim3 grid((unsigned)(8 * t.chunk)), block(kWavesS * 64);
    static const hipError_t allowed[2] = {
        hipFuncSetAttribute((const void*)forward_shared32<false>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsS),
        hipFuncSetAttribute((const void*)forward_shared32<true>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsS)};
    if (allowed[al4] != hipSuccess) return allowed[al4];
    if (al4)
        forward_shared32<true><<<grid, block, kLdsS, st>>>(x, w, y, p, t);
    else
        forward_shared32<false><<<grid, block, kLdsS, st>>>(x, w, y, p, t);
    return hipGetLastError();
}

}  // namespace scc
