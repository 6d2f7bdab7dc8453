// Forward SCC on the gfx950 matrix cores.  bf16 tensors go through the bf16 matrix instruction directly
// (exact products, fp32 sums); fp32 tensors are split exactly into three bf16 pieces per value and take six
// bf16 matrix instructions per K group (error below 2^-23 of each product, fp32 sums), which costs 3/8 of
// the matrix time of v_mfma_f32_32x32x2_f32 and measures the same error against an fp64 reference.
//
// y[n,k,p] = sum_j w[k,j] * x[n,(s_k+j) mod Cin,p]   (Section 4.2, output-centric forward)
// is computed as banded GEMM tiles: a tile of 32 filters (TM adjacent window starts x TI
// filters per start, see scc_band.h) times a span of U = L + g*(TM-1) channels, for 32*CT
// columns (a column is one (sample, pixel) pair).  When TM == 1 the tile is dense.
//
// One wavefront owns one tile.  A matrix instruction contracts K values from both half-waves;
// half h walks the channels lo + h*Uh + t, t = 0..Uh-1 (a chunk of KC steps is one instruction), so that a
// lane's successive A values are CONSECUTIVE weights of one filter (staged through LDS, see the kernel)
// and its B values are one channel plane after another at a fixed column (each half-wave reads 32*CT
// contiguous values of the plane).  The cyclic wrap is a compare-and-subtract on the channel index;
// nothing is copied.
#include "scc_band.h"
#include "scc_common.h"

namespace scc {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct FwdTiling {
    Band b;
    int TI, TM;    // tile = TM starts x TI filters per start; TI*TM <= 32 (TM is capped by P)
    int IB, MB;    // tiles along i and m
    int Uh;        // K-steps per tile (multiple of the chunk length); each half-wave covers Uh channels
    int Us;        // K-steps of one wavefront when S wavefronts share a tile: ceil(Uh / S) rounded to rounds
    int FG;        // workgroups per column tile = ceil(IB*MB * S / wavefronts per workgroup)
    int total;     // workgroups with work: column tiles (of 32*CT columns) * FG, filter-tile group fastest
    int chunk;     // consecutive workgroups of that order given to one XCD: ceil(total / 8)
    int stagger;   // ticks of the 100 MHz clock the second half of an 8-wavefront workgroup waits after kernel start
};

// CT   column groups of 32 per wavefront (the tile is 32 filters x 32*CT columns)
// KC   K-steps per pipelined chunk of B loads
// AL4  g and L are multiples of 4: groups of four weights are wholly inside or outside a window
// VEC  H*W is a multiple of CT: a lane owns CT CONSECUTIVE columns (one CT*4-byte load per plane,
//      one CT*4-byte store per output row); otherwise a lane owns columns f, f+32, ...
// T    storage type of x, w, y (float or bf16_t); sums are binary32 either way, products go through the
//      bf16 matrix instruction (bf16 values as stored, fp32 values as three bf16 pieces each)
// S    wavefronts sharing one tile (1, 2 or 4), each taking a slice of the contraction; their partial
//      tiles are added through LDS in slice order.  For layers with few columns and long windows.
// WPB  wavefronts per workgroup: 4, or 8 for grids of exactly two wavefronts per SIMD.  With 8 the second
//      four (one per SIMD, like the first four) issue their first request kStaggerTicks after the kernel
//      started, about when the first four get their first operands: every wavefront of such a grid is
//      resident at once, and without the stagger all of them load, then all multiply, then all store; with
//      it one half's stores and arithmetic overlap the other half's loads (17 against 19-21 us at the metric
//      layer; used only where it wins, see launch_chunk).
template <typename T_, int CT, int KC, bool AL4, bool VEC, int S, int WPB>
__global__ __launch_bounds__(WPB * 64) void forward_mfma32(const T_* __restrict__ x, const T_* __restrict__ w,
                                                      T_* __restrict__ y, Problem P, FwdTiling T)
{
    typedef T_ bvec __attribute__((ext_vector_type(CT)));               // CT consecutive columns of one plane
    typedef T_ avec __attribute__((ext_vector_type(4), aligned(sizeof(T_))));  // 4 consecutive weights
    constexpr uint32_t ES = sizeof(T_);
    constexpr int KA = 2 * KC;   // K-steps per round: two chunks of B loads
    constexpr int kAB = 2 * KA;  // K-steps per staged block of A operands: two rounds

    // workgroup -> (column tile, filter-tile group).  blockIdx % 8 names the XCD; each XCD takes a
    // contiguous run of the (column tile, group) order, so the groups of a column tile, which re-read
    // the same channel planes, share one XCD and its L2 whenever there are enough column tiles.
    const uint64_t t_start = WPB == 8 ? __builtin_amdgcn_s_memrealtime() : 0;   // 100 MHz, independent of core clocks
    const int bid = blockIdx.x;
    const int xcd = bid & 7, slot = bid >> 3;
    const int logical = xcd * T.chunk + slot;
    if (slot >= T.chunk || logical >= T.total) return;
    const int ct = logical / T.FG;
    const int fg = logical % T.FG;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int tile = fg * (WPB / S) + wave / S, split = wave % S;
    const bool tvalid = tile < T.IB * T.MB;
    if (S == 1 && !tvalid) return;                   // with S > 1 every wavefront has to reach the barrier
    const int mb = tile / T.IB, ib = tile % T.IB;
    const int t0 = split * T.Us;                     // this wavefront's K-steps [t0, t1)
    const int t1 = !tvalid ? t0 : (t0 + T.Us < T.Uh ? t0 + T.Us : T.Uh);

    const int lane = threadIdx.x & 63;
    const int f = lane & 31, h = lane >> 5;

    // ---- A side: this lane's filter -------------------------------------------------------
    const int mi = f / T.TI, ii = f % T.TI;
    const int m = mb * T.TM + mi, i = ib * T.TI + ii;
    const int k = (int)(((uint32_t)m * (uint32_t)T.b.inv) % (uint32_t)T.b.P) + T.b.P * i;  // P < 65536
    const bool fvalid = tvalid && (mi < T.TM) && (m < T.b.P) && (k < P.Cout);
    const int off = T.b.g * mi;                      // this filter's window starts `off` channels into the span
    const int wrow = (fvalid ? k : 0) * P.L;         // first weight of this lane's filter
    const int lo = T.b.g * mb * T.TM;                // first channel of the span (< Cin)
    const char* wb = (const char*)w;
    const char* xb = (const char*)x;

    // ---- A operands: through LDS, once per block of kAB K-steps --------------------------------
    // Read straight into operand layout, every lane would touch its own cache line (64 lines per load
    // instruction, as much L1 tag traffic as all the activation loads, and the first thing every wavefront
    // of the chip asks for).  Instead 8 lanes read one filter's 32 consecutive weights (4 lines per 8 lanes),
    // the values are cut into their bf16 pieces ONCE (fp32: hi, mid, lo; bf16: as stored), zeros where the
    // window does not reach or the filter does not exist, and parked in a wavefront-private LDS block:
    // row (h*32 + f), kParts pieces of kAB bf16 each.  A 16-byte LDS read is then one lane's 8 K values of
    // one piece.  The wavefront is the only user of its block: no barrier.
    constexpr int kParts = ES == 2 ? 1 : 3;
    constexpr int kG = kAB / 4;                      // groups of 4 weights in a full block row (8 or 4)
    constexpr int kPartB = kAB * 2;                  // bytes of one piece of a row
    constexpr int kRowB = kParts * kPartB + 16;      // + 16 bytes of padding (bank spread, keeps 16-byte alignment)
    // a wavefront's block also holds its partial tile when S wavefronts share a tile (see the end of the K loop)
    constexpr int kBlockB = (S > 1 && CT * 16 * 64 * 4 > 64 * kRowB) ? CT * 16 * 64 * 4 : 64 * kRowB;
    __shared__ __attribute__((aligned(16))) char a_lds[WPB * kBlockB];
    char* A = a_lds + wave * kBlockB;
    const int offv = fvalid ? off : (1 << 30);       // rows without a filter: every position is outside
    avec ga[kG];                                     // raw loaded weights; zeroed per mask bit when committed
    uint32_t gam = 0;                                // bit 4*it + q: weight q of group `it` is inside the window
    // position of group `it` of a block of nb steps in the (row, group) grid: full blocks take rows f and
    // 32+f together (kG lanes per row, 64/kG rows per trip), short ones walk the rows in order
    auto group_pos = [&](int it, int nb, uint32_t& row, uint32_t& c) {
        if (nb == kAB) {
            row = (uint32_t)((it % (kG / 2)) * (64 / kG) + lane / kG + 32 * (it / (kG / 2)));
            c = (uint32_t)(lane % kG);
        } else {
            const uint32_t e = (uint32_t)nb >> 2, idx = (uint32_t)(it * 64 + lane);
            row = idx / e;
            c = idx - row * e;
        }
    };
    // global -> registers: the weights of K-steps [tb, tb+nb) of both half-waves (nb a multiple of KA, <= kAB)
    auto stage_issue = [&](int tb, int nb) {
        gam = 0;
#pragma unroll
        for (int it = 0; it < kG; ++it) {
            uint32_t row, c;
            group_pos(it, nb, row, c);
            const bool act = row < 64u;              // short blocks have fewer groups than lanes * kG
            const int fr = (int)(row & 31u);
            const int ro = __shfl(offv, fr, 64), rw = __shfl(wrow, fr, 64);
            const int j0 = (int)((row >> 5) & 1u) * T.Uh + tb + 4 * (int)c - ro;
            if (AL4) {
                const bool in = act && j0 >= 0 && j0 < P.L;
                ga[it] = *(const avec*)(wb + (uint32_t)(in ? rw + j0 : 0) * ES);
                gam |= in ? (0xfu << (4 * it)) : 0u;
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int j = j0 + q;
                    const bool in = act && j >= 0 && j < P.L;
                    ga[it][q] = *(const T_*)(wb + (uint32_t)(in ? rw + j : 0) * ES);
                    gam |= in ? (1u << (4 * it + q)) : 0u;
                }
            }
        }
    };
    // registers -> LDS
    auto stage_commit = [&](int nb) {
#pragma unroll
        for (int it = 0; it < kG; ++it) {
            uint32_t row, c;
            group_pos(it, nb, row, c);
            if (row < 64u) {
                char* dst = A + row * kRowB + 8 * c;
                const uint32_t m4 = gam >> (4 * it);
                if constexpr (ES == 2) {
                    const uint32_t v0 = (m4 & 1u ? (uint32_t)ga[it][0] : 0u) | ((m4 & 2u ? (uint32_t)ga[it][1] : 0u) << 16);
                    const uint32_t v1 = (m4 & 4u ? (uint32_t)ga[it][2] : 0u) | ((m4 & 8u ? (uint32_t)ga[it][3] : 0u) << 16);
                    *(u32x2*)dst = u32x2{v0, v1};
                } else {
                    const float v[4] = {m4 & 1u ? ga[it][0] : 0.f, m4 & 2u ? ga[it][1] : 0.f, m4 & 4u ? ga[it][2] : 0.f,
                                        m4 & 8u ? ga[it][3] : 0.f};
                    uint32_t hi[2], mid[2], lo3[2];
                    split3<4>([&](int e) { return v[e]; }, hi, mid, lo3);
                    *(u32x2*)dst = u32x2{hi[0], hi[1]};
                    *(u32x2*)(dst + kPartB) = u32x2{mid[0], mid[1]};
                    *(u32x2*)(dst + 2 * kPartB) = u32x2{lo3[0], lo3[1]};
                }
            }
        }
    };

    // The second half of the workgroup holds its first request back.  The clock runs on, so the wait ends; the
    // poll count bounds it anyway (64 polls of 256+ cycles each are well beyond the delay).
    if constexpr (WPB == 8) {
        if (wave >= 4)
            for (int poll = 0; poll < 64 && __builtin_amdgcn_s_memrealtime() - t_start < (uint64_t)T.stagger; ++poll)
                __builtin_amdgcn_s_sleep(4);
    }

    // The first block of weights is requested before anything else is computed or loaded.
    const int nb0 = t1 - t0 < kAB ? t1 - t0 : kAB;
    if (t0 < t1) stage_issue(t0, nb0);
    __builtin_amdgcn_sched_barrier(0);

    // ---- B side: this lane's columns (byte offsets from x; the launcher checked they fit 32 bits) ----
    uint32_t xcol[CT], ycol[CT];
    bool live[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) {
        const uint32_t q = (uint32_t)ct * (32 * CT) + (VEC ? f * CT + c : c * 32 + f);
        live[c] = q < (uint32_t)P.NQ;
        const uint32_t qq = live[c] ? q : 0u;
        const uint32_t n = qq / (uint32_t)P.HW, p = qq % (uint32_t)P.HW;
        xcol[c] = (n * (uint32_t)P.Cin * (uint32_t)P.HW + p) * ES;
        ycol[c] = n * (uint32_t)P.Cout * (uint32_t)P.HW + p;
    }
    const uint32_t plane = (uint32_t)P.HW * ES;                  // bytes between channel planes
    const uint32_t wrap = (uint32_t)P.Cin * plane;               // bytes of one sample's channels
    uint32_t rowofs = (uint32_t)((lo + h * T.Uh + t0) % P.Cin) * plane;  // plane this half-wave reads next

    f32x16 acc[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;

    auto load_b = [&](bvec (&bd)[KC]) {
#pragma unroll
        for (int s = 0; s < KC; ++s) {
            if (VEC) {
                bd[s] = *(const bvec*)(xb + (uint32_t)(xcol[0] + rowofs));
            } else {
#pragma unroll
                for (int c = 0; c < CT; ++c) bd[s][c] = *(const T_*)(xb + (uint32_t)(xcol[c] + rowofs));
            }
            rowofs += plane;
            rowofs = (rowofs == wrap) ? 0u : rowofs;             // cyclic wrap past channel Cin-1
        }
    };
    // The KC steps of a chunk are the K values of one bf16 matrix instruction per column group and pair of
    // pieces (a half-wave's KC values side by side in its lanes' registers; which K-slot a value takes does
    // not matter as long as A and B agree).  bf16 tensors: one instruction, exact products.  fp32 tensors:
    // B is cut into its three bf16 pieces here, and six of the nine partial products are taken (the dropped
    // mid*lo, lo*mid, lo*lo are below 2^-23 of the product).  Sums are fp32 either way.
    auto mma = [&](int tl, const bvec (&bs)[KC]) {   // tl: first K-step of the chunk inside the staged block
        uint32_t ap[kParts][KC / 2];
#pragma unroll
        for (int q = 0; q < kParts; ++q) {
            const char* src = A + (h * 32 + f) * kRowB + q * kPartB + 2 * tl;
            if constexpr (KC == 8) {
                const u32x4 t = *(const u32x4*)src;
#pragma unroll
                for (int z = 0; z < 4; ++z) ap[q][z] = t[z];
            } else {
                const u32x2 t = *(const u32x2*)src;
                ap[q][0] = t[0];
                ap[q][1] = t[1];
            }
        }
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            if constexpr (ES == 2) {
                uint32_t bp[KC / 2];
#pragma unroll
                for (int e = 0; e < KC / 2; ++e)
                    bp[e] = (uint32_t)(T_)bs[2 * e][c] | ((uint32_t)(T_)bs[2 * e + 1][c] << 16);
                acc[c] = mfma_bf16<KC>(ap[0], bp, acc[c]);
            } else {
                uint32_t bh[KC / 2], bm[KC / 2], bl[KC / 2];
                split3<KC>([&](int e) { return bs[e][c]; }, bh, bm, bl);
                acc[c] = mfma_bf16<KC>(ap[2], bh, acc[c]);
                acc[c] = mfma_bf16<KC>(ap[0], bl, acc[c]);
                acc[c] = mfma_bf16<KC>(ap[1], bm, acc[c]);
                acc[c] = mfma_bf16<KC>(ap[1], bh, acc[c]);
                acc[c] = mfma_bf16<KC>(ap[0], bm, acc[c]);
                acc[c] = mfma_bf16<KC>(ap[0], bh, acc[c]);
            }
        }
    };

    // K loop over rounds of KA = 2*KC steps (Uh and the slices are multiples of KA; a block is two rounds):
    // B loads run KC steps ahead of the matrix instructions.  The last round is peeled so that no load in the
    // loop is conditional: behind a branch that may or may not have issued loads, the wait for an operand
    // has to assume the fewest loads behind it and so also waits for the refill just requested.
    bvec b0[KC], b1[KC];
    if (t0 < t1) {
        load_b(b0);
        load_b(b1);
        stage_commit(nb0);
        const int nr = (t1 - t0) / KA;
        int tb = t0, tl = 0;                          // block start, offset of the round inside the block
        for (int r = 0; r + 1 < nr; ++r) {
            // contractions longer than a block: the next block's weights are requested when a block starts and
            // parked when its last operand has been read, so their latency hides behind the block's rounds
            if (tl == 0 && tb + kAB < t1) stage_issue(tb + kAB, t1 - tb - kAB < kAB ? t1 - tb - kAB : kAB);
            mma(tl, b0);
            load_b(b0);
            mma(tl + KC, b1);
            load_b(b1);
            tl += KA;
            if (tl == kAB) {
                tb += kAB;
                tl = 0;
                stage_commit(t1 - tb < kAB ? t1 - tb : kAB);
            }
        }
        mma(tl, b0);
        mma(tl + KC, b1);
    }

    if constexpr (S > 1) {
        // add the slices of each tile, in slice order, into the wavefront that took slice 0; a wavefront parks
        // its partial tile in its own (now idle) weight block
        float* mine = (float*)A + lane;
        if (split > 0) {
#pragma unroll
            for (int c = 0; c < CT; ++c)
#pragma unroll
                for (int v = 0; v < 16; ++v) mine[(c * 16 + v) * 64] = acc[c][v];
        }
        __syncthreads();
        if (split > 0 || !tvalid) return;
#pragma unroll
        for (int sp = 1; sp < S; ++sp) {
            const float* other = (const float*)(a_lds + (wave + sp) * kBlockB) + lane;
#pragma unroll
            for (int c = 0; c < CT; ++c)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[c][v] += other[(c * 16 + v) * 64];
        }
    }

    // ---- store: register v of the accumulator holds tile row 8*(v/4) + 4*h + v%4, column f ----
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int fr = 8 * (v >> 2) + 4 * h + (v & 3);
        const int kr = __shfl(k, fr, 64);            // filter of tile row fr lives in lane fr's registers
        const bool rvalid = __shfl((int)fvalid, fr, 64) != 0;
        if (rvalid) {
            if (VEC) {
                if (live[0]) {                        // CT divides H*W: the CT columns are live together
                    bvec o;
#pragma unroll
                    for (int c = 0; c < CT; ++c) o[c] = from_f32<T_>(acc[c][v]);
                    __builtin_nontemporal_store(o, (bvec*)(y + (size_t)ycol[0] + (size_t)kr * P.HW));  // written once, not re-read here
                }
            } else {
#pragma unroll
                for (int c = 0; c < CT; ++c)
                    if (live[c]) __builtin_nontemporal_store(from_f32<T_>(acc[c][v]), y + (size_t)ycol[c] + (size_t)kr * P.HW);
            }
        }
    }
}

int pow2_floor(int v)
{
    int p = 1;
    while (p * 2 <= v) p *= 2;
    return p;
}

constexpr int kEnoughWaves = 1024;  // one wavefront per SIMD of the chip
constexpr int kStaggerTicks = 250;  // 2.5 us: measured on grids of 2048 wavefronts, 2.3 and 2.8 us gain 2 us, 1.8 us nothing

// K-steps per pipelined chunk of B loads: 8, or 4 when rounding the contraction to rounds of 16 steps would
// pad it more than rounds of 8 do (banded tiles whose span is not a multiple of 32 channels)
int chunk_steps(int U)
{
    const int half = (U + 1) / 2;
    return (half + 7) / 8 * 8 < (half + 15) / 16 * 16 ? 4 : 8;
}

FwdTiling filter_tiling(const Problem& p)
{
    FwdTiling t;
    t.b = make_band(p);
    t.TI = pow2_floor(t.b.F < 32 ? t.b.F : 32);
    t.TM = 32 / t.TI < t.b.P ? 32 / t.TI : t.b.P;
    t.IB = (t.b.F + t.TI - 1) / t.TI;
    t.MB = (t.b.P + t.TM - 1) / t.TM;
    const int U = p.L + t.b.g * (t.TM - 1);
    const int kc = chunk_steps(U);
    t.Uh = (((U + 1) / 2) + 2 * kc - 1) / (2 * kc) * (2 * kc);
    t.Us = t.Uh;
    t.FG = (t.IB * t.MB + 3) / 4;
    t.total = t.chunk = 0;
    t.stagger = kStaggerTicks;
    return t;
}

template <typename T_, int CT, bool VEC, int S, int KC, int WPB>
void launch_wpb(const T_* x, const T_* w, T_* y, const Problem& p, hipStream_t st)
{
    FwdTiling t = filter_tiling(p);
    const long long nct = (p.NQ + 32 * CT - 1) / (32 * CT);
    t.Us = ((t.Uh + S - 1) / S + 2 * KC - 1) / (2 * KC) * (2 * KC);
    t.FG = (t.IB * t.MB * S + WPB - 1) / WPB;
    t.total = (int)(nct * t.FG);
    t.chunk = (t.total + 7) / 8;
    const long long blocks = (long long)8 * t.chunk;
    const bool al4 = (t.b.g % 4 == 0) && (p.L % 4 == 0);
    if (al4)
        forward_mfma32<T_, CT, KC, true, VEC, S, WPB><<<dim3((unsigned)blocks), dim3(WPB * 64), 0, st>>>(x, w, y, p, t);
    else
        forward_mfma32<T_, CT, KC, false, VEC, S, WPB><<<dim3((unsigned)blocks), dim3(WPB * 64), 0, st>>>(x, w, y, p, t);
}

template <typename T_, int CT, bool VEC, int S, int KC>
void launch_chunk(const T_* x, const T_* w, T_* y, const Problem& p, hipStream_t st)
{
    // Workgroups of 8 wavefronts with staggered halves: only for grids that fill the chip exactly once with two
    // wavefronts per SIMD (all resident together, hence in lockstep), dense fp32 tiles of at least two rounds,
    // and at most 16 flop per byte.  Measured on other shapes it loses: larger grids run in generations that are
    // out of phase anyway, bf16 and single-round tiles have too little arithmetic to overlap, and layers with
    // more arithmetic per byte are slowed by the followers' late start.
    if constexpr (sizeof(T_) == 4 && CT == 4 && VEC && KC == 8 && S == 1) {
        const FwdTiling t = filter_tiling(p);
        const long long nct = (p.NQ + 32 * CT - 1) / (32 * CT), waves = nct * t.IB * t.MB;
        const bool once = waves >= 2 * kEnoughWaves && waves < 2 * kEnoughWaves + kEnoughWaves / 4;
        const bool light = (long long)p.Cout * p.L <= 32ll * (p.Cin + p.Cout);
        if (t.TM == 1 && (t.IB * t.MB) % 8 == 0 && t.Uh >= 32 && once && light) {
            launch_wpb<T_, CT, VEC, S, KC, 8>(x, w, y, p, st);
            return;
        }
    }
    launch_wpb<T_, CT, VEC, S, KC, 4>(x, w, y, p, st);
}

template <typename T_, int CT, bool VEC, int S>
void launch_split(const T_* x, const T_* w, T_* y, const Problem& p, hipStream_t st)
{
    const Band b = make_band(p);
    const int ti = pow2_floor(b.F < 32 ? b.F : 32), tm = 32 / ti < b.P ? 32 / ti : b.P;
    if (chunk_steps(p.L + b.g * (tm - 1)) == 4)
        launch_chunk<T_, CT, VEC, S, 4>(x, w, y, p, st);
    else
        launch_chunk<T_, CT, VEC, S, 8>(x, w, y, p, st);
}

template <typename T_, int CT, bool VEC>
void launch_cfg(const T_* x, const T_* w, T_* y, const Problem& p, hipStream_t st, long long waves)
{
    // share a tile between 2 or 4 wavefronts while there are fewer than two wavefronts per SIMD and each
    // slice of the contraction keeps at least 32 K-steps
    const FwdTiling t = filter_tiling(p);
    int split = 1;
    while (split < 4 && waves * split < 2 * kEnoughWaves && t.Uh / (2 * split) >= 32) split *= 2;
    if (split == 1)
        launch_split<T_, CT, VEC, 1>(x, w, y, p, st);
    else if (split == 2)
        launch_split<T_, CT, VEC, 2>(x, w, y, p, st);
    else
        launch_split<T_, CT, VEC, 4>(x, w, y, p, st);
}

}  // namespace

// Whether the matrix-core forward takes this problem (otherwise the generic kernel does).
bool forward_mfma_eligible(const Problem& p)
{
    // enough contraction depth and columns for a 32x32 tile to pay, and byte offsets that fit 32 bits
    const long long rows = p.Cin > p.Cout ? p.Cin : p.Cout;
    return p.L >= 8 && p.NQ >= 64 && p.Cout >= 8 && p.Cin < 65536 && (long long)p.NQ * rows * 4 < (1ll << 32) &&
           (long long)p.Cout * p.L * 4 < (1ll << 31);
}

template <typename T_>
hipError_t launch_forward_mfma(const T_* x, const T_* w, T_* y, const Problem& p, hipStream_t st)
{
    // Columns per wavefront: 128 when that still gives every SIMD a wavefront, else 64 or 32 (layers with
    // few columns and many filters).  Vector plane accesses (CT consecutive columns per lane) need planes whose
    // size is a multiple of CT and tensors aligned to the vector; otherwise a lane owns strided single columns.
    if constexpr (sizeof(T_) == 4) {
        if (forward_shared_preferred((const float*)x, (const float*)w, (const float*)y, p))
            return launch_forward_shared((const float*)x, (const float*)w, (float*)y, p, st);
    }
    const FwdTiling ft = filter_tiling(p);
    const long long tiles = (long long)ft.IB * ft.MB;
    auto waves = [&](int ct) { return (p.NQ + 32 * ct - 1) / (32 * ct) * tiles; };
    const uintptr_t addr = (uintptr_t)x | (uintptr_t)y | (uintptr_t)w;
    auto vec_ok = [&](int ct) { return p.HW % ct == 0 && (addr & (ct * sizeof(T_) - 1)) == 0; };
    // a tile's contraction can be shared by up to 4 wavefronts (launch_cfg): wide tiles, whose loads move 16 bytes
    // per lane and instruction, are kept as long as that sharing still gives every SIMD a wavefront
    auto shared = [&](long long wv) {
        int sp = 1;
        while (sp < 4 && wv * sp < 2 * kEnoughWaves && ft.Uh / (2 * sp) >= 32) sp *= 2;
        return wv * sp;
    };
    if (vec_ok(4) && shared(waves(4)) >= kEnoughWaves)
        launch_cfg<T_, 4, true>(x, w, y, p, st, waves(4));
    else if (vec_ok(2) && shared(waves(2)) >= kEnoughWaves)
        launch_cfg<T_, 2, true>(x, w, y, p, st, waves(2));
    else if (waves(2) >= kEnoughWaves)
        launch_cfg<T_, 2, false>(x, w, y, p, st, waves(2));
    else
        launch_cfg<T_, 1, false>(x, w, y, p, st, waves(1));
    return hipGetLastError();
}

template hipError_t launch_forward_mfma<float>(const float*, const float*, float*, const Problem&, hipStream_t);
template hipError_t launch_forward_mfma<bf16_t>(const bf16_t*, const bf16_t*, bf16_t*, const Problem&, hipStream_t);

}  // namespace scc
