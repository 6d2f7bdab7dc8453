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
#pragma once
#include "scc_band.h"
#include "scc_common.h"

#include <type_traits>

namespace scc {

namespace bwi {

typedef float f32x16 __attribute__((ext_vector_type(16)));

struct BwiTiling {
    Band b;
    int CB;   // channel blocks of 32
    int FG;     // workgroups per column tile = ceil(CB / 4)
    int total;  // workgroups with work: column tiles * FG, channel-block group fastest
    int chunk;  // consecutive workgroups of that order given to one XCD: ceil(total / 8)
};

__device__ __forceinline__ int floor_div(int a, int b)  // b > 0
{
    const int q = a / b;
    return (a % b != 0 && a < 0) ? q - 1 : q;
}

// T_ is the storage type of dy, w, dx (float or bf16_t); arithmetic is binary32 either way.
// S wavefronts (1, 2 or 4) share one tile, each taking a slice of the (window, filter) slots; their partial
// tiles are added through LDS in slice order (layers with few columns and many covering filters).
// WPB wavefronts per workgroup: 4, or 8 (all channel blocks of a column tile on one CU, sharing its L1) for grids
// that fill the chip exactly once: see launch_split.
// Bytes of LDS in which the wavefronts that share a tile add their partial tiles (S > 1).
template <int CT, int S, int WPB>
constexpr size_t reduce_bytes() { return S > 1 ? (size_t)(WPB / S) * (S - 1) * CT * 16 * 64 * sizeof(float) : 0; }

// `shared_red`: LDS of at least reduce_bytes<CT, S, WPB>() that the caller provides for that sum (a kernel that
// holds dynamic LDS for other workgroups of its grid lends it); null: the body declares its own.
template <typename T_, int CT, int KC, bool VEC, int S, int WPB, bool LENT = false>
__device__ __forceinline__ void backward_input_body(const T_* __restrict__ dy, const T_* __restrict__ w,
                                                    T_* __restrict__ dx, const Problem& P, const BwiTiling& T,
                                                    const int bid, float* shared_red = nullptr)
{
    typedef T_ bvec __attribute__((ext_vector_type(CT)));
    constexpr uint32_t ES = sizeof(T_);
    // bid is the workgroup's index in a launch whose first workgroup is a multiple of 8: bid % 8 names the XCD; each XCD takes a contiguous run of the (column tile, group) order, so the
    // channel blocks of a column tile, which re-read the same dy planes, share an XCD and its L2
    const int xcd = bid & 7, slot = bid >> 3;
    const int logical = xcd * T.chunk + slot;
    if (slot >= T.chunk || logical >= T.total) return;
    const int ct = logical / T.FG;
    const int fg = logical % T.FG;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int cb = fg * (WPB / S) + wave / S, split = wave % S;
    const bool tvalid = cb < T.CB;
    if (S == 1 && !tvalid) return;              // with S > 1 every wavefront has to reach the barrier

    const int lane = threadIdx.x & 63;
    const int f = lane & 31, h = lane >> 5;
    const int c0 = cb * 32;
    const int c = c0 + f;                       // this lane's input channel (A row)
    const bool cvalid = tvalid && c < P.Cin;
    // unwrapped window index range: g*m in [c0-L+1, c0+31]
    const int mlo = -floor_div(P.L - 1 - c0, T.b.g);   // ceil((c0-L+1)/g)
    const int M = floor_div(c0 + 31, T.b.g) - mlo + 1;  // window starts this block can see (>= 1)
    // K-steps: each half-wave walks Uh (window, filter) slots; an even number of chunks
    const int Uh = ((M * T.b.F + 1) / 2 + 2 * KC - 1) / (2 * KC) * (2 * KC);
    const int Us = ((Uh + S - 1) / S + 2 * KC - 1) / (2 * KC) * (2 * KC);   // K-steps of one slice
    const int t0 = split * Us < Uh ? split * Us : Uh;                         // this wavefront's K-steps [t0, t1)
    const int t1 = !tvalid ? t0 : (t0 + Us < Uh ? t0 + Us : Uh);
    const char* wb = (const char*)w;
    const char* gb = (const char*)dy;

    uint32_t gcol[CT], dcol[CT];
    bool live[CT];
#pragma unroll
    for (int cc = 0; cc < CT; ++cc) {
        const uint32_t q = (uint32_t)ct * (32 * CT) + (VEC ? f * CT + cc : cc * 32 + f);
        live[cc] = q < (uint32_t)P.NQ;
        const uint32_t qq = live[cc] ? q : 0u;
        const uint32_t n = qq / (uint32_t)P.HW, p = qq % (uint32_t)P.HW;
        gcol[cc] = (n * (uint32_t)P.Cout * (uint32_t)P.HW + p) * ES;
        dcol[cc] = n * (uint32_t)P.Cin * (uint32_t)P.HW + p;
    }

    // K-slot state of this half-wave: slot u = h*Uh + t  <->  (mm, i) = (u / F, u % F)
    const int u0 = h * Uh + t0;
    int mm = u0 / T.b.F, i = u0 % T.b.F;
    int mw = (mlo + mm) % T.b.P;                 // window index on the circle
    if (mw < 0) mw += T.b.P;
    int r = (int)(((uint32_t)mw * (uint32_t)T.b.inv) % (uint32_t)T.b.P);   // residue class owning window mw
    int ju = c - T.b.g * (mlo + mm);             // position of channel c inside that window (unwrapped)
    const uint32_t plane = (uint32_t)P.HW * ES;

    f32x16 acc[CT];
#pragma unroll
    for (int cc = 0; cc < CT; ++cc)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[cc][v] = 0.f;

    auto load_chunk = [&](T_ (&ad)[KC], uint32_t& am, bvec (&bd)[KC]) {
        am = 0;
#pragma unroll
        for (int s = 0; s < KC; ++s) {
            const int k = r + T.b.P * i;
            const bool kvalid = (mm < M) && (k < P.Cout);
            const bool in = kvalid && cvalid && ju >= 0 && ju < P.L;
            ad[s] = *(const T_*)(wb + (uint32_t)(in ? (k * P.L + ju) : 0) * ES);
            am |= in ? (1u << s) : 0u;
            const uint32_t rowofs = (uint32_t)(kvalid ? k : 0) * plane;
            if (VEC) {
                bd[s] = *(const bvec*)(gb + (uint32_t)(gcol[0] + rowofs));
            } else {
#pragma unroll
                for (int cc = 0; cc < CT; ++cc) bd[s][cc] = *(const T_*)(gb + (uint32_t)(gcol[cc] + rowofs));
            }
            // next slot: next filter of this window, or the first filter of the next window
            ++i;
            const bool nextw = (i == T.b.F);
            i = nextw ? 0 : i;
            mm += nextw ? 1 : 0;
            ju -= nextw ? T.b.g : 0;
            int rn = r + T.b.inv;                // r(m+1) = r(m) + inv (mod P)
            rn = (rn >= T.b.P) ? rn - T.b.P : rn;
            r = nextw ? rn : r;
        }
    };
    auto mma_chunk = [&](const T_ (&as)[KC], uint32_t am, const bvec (&bs)[KC]) {
        if constexpr (ES == 2) {
            // bf16 storage: the KC slots of a chunk are the K values of ONE bf16 matrix instruction per column
            // group (which K-slot a value takes does not matter as long as A and B agree); exact products
            uint32_t ap[KC / 2];
#pragma unroll
            for (int e = 0; e < KC / 2; ++e) {
                const uint32_t lo = (am >> (2 * e)) & 1u ? (uint32_t)as[2 * e] : 0u;
                const uint32_t hi = (am >> (2 * e + 1)) & 1u ? (uint32_t)as[2 * e + 1] : 0u;
                ap[e] = lo | (hi << 16);
            }
#pragma unroll
            for (int cc = 0; cc < CT; ++cc) {
                uint32_t bp[KC / 2];
#pragma unroll
                for (int e = 0; e < KC / 2; ++e)
                    bp[e] = (uint32_t)(T_)bs[2 * e][cc] | ((uint32_t)(T_)bs[2 * e + 1][cc] << 16);
                acc[cc] = mfma_bf16<KC>(ap, bp, acc[cc]);
            }
        } else {
            // fp32 storage: exact three-way bf16 split of every operand, six of the nine partial products
            // (the dropped ones are below 2^-23 of the product), fp32 accumulation
            uint32_t ah[KC / 2], amd[KC / 2], al[KC / 2];
            split3<KC>([&](int e) { return (am >> e) & 1u ? as[e] : 0.f; }, ah, amd, al);
#pragma unroll
            for (int cc = 0; cc < CT; ++cc) {
                uint32_t bh[KC / 2], bm[KC / 2], bl[KC / 2];
                split3<KC>([&](int e) { return bs[e][cc]; }, bh, bm, bl);
                acc[cc] = mfma_bf16<KC>(al, bh, acc[cc]);
                acc[cc] = mfma_bf16<KC>(ah, bl, acc[cc]);
                acc[cc] = mfma_bf16<KC>(amd, bm, acc[cc]);
                acc[cc] = mfma_bf16<KC>(amd, bh, acc[cc]);
                acc[cc] = mfma_bf16<KC>(ah, bm, acc[cc]);
                acc[cc] = mfma_bf16<KC>(ah, bh, acc[cc]);
            }
        }
    };

    // software pipelined over an even number of chunks (Uh is a multiple of 2*KC)
    T_ a0[KC], a1[KC];
    bvec b0[KC], b1[KC];
    uint32_t m0, m1;
    const int nch = (t1 - t0) / KC;
    if (nch > 0) {
        load_chunk(a0, m0, b0);
        for (int cix = 0; cix + 2 < nch; cix += 2) {
            load_chunk(a1, m1, b1);
            mma_chunk(a0, m0, b0);
            load_chunk(a0, m0, b0);
            mma_chunk(a1, m1, b1);
        }
        load_chunk(a1, m1, b1);
        mma_chunk(a0, m0, b0);
        mma_chunk(a1, m1, b1);
    }

    if constexpr (S > 1) {   // add the slices of each tile, in slice order, into the wavefront that took slice 0
        float* red;
        if constexpr (LENT) {
            red = shared_red;
        } else {
            __shared__ float own[(S > 1 ? (WPB / S) * (S - 1) : 1) * CT * 16 * 64];
            red = own;
        }
        float* mine = red + ((wave / S) * (S - 1) + (split - 1)) * (CT * 16 * 64) + lane;
        if (split > 0) {
#pragma unroll
            for (int cc = 0; cc < CT; ++cc)
#pragma unroll
                for (int v = 0; v < 16; ++v) mine[(cc * 16 + v) * 64] = acc[cc][v];
        }
        __syncthreads();
        if (split > 0 || !tvalid) return;
#pragma unroll
        for (int sp = 1; sp < S; ++sp) {
            const float* other = red + ((wave / S) * (S - 1) + (sp - 1)) * (CT * 16 * 64) + lane;
#pragma unroll
            for (int cc = 0; cc < CT; ++cc)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[cc][v] += other[(cc * 16 + v) * 64];
        }
    }

    // accumulator register v holds tile row 8*(v/4) + 4*h + v%4 (= channel c0 + that), column f
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int cr = c0 + 8 * (v >> 2) + 4 * h + (v & 3);
        if (cr < P.Cin) {
            if (VEC) {
                if (live[0]) {
                    bvec o;
#pragma unroll
                    for (int cc = 0; cc < CT; ++cc) o[cc] = from_f32<T_>(acc[cc][v]);
                    __builtin_nontemporal_store(o, (bvec*)(dx + (size_t)dcol[0] + (size_t)cr * P.HW));  // written once, not re-read here
                }
            } else {
#pragma unroll
                for (int cc = 0; cc < CT; ++cc)
                    if (live[cc]) __builtin_nontemporal_store(from_f32<T_>(acc[cc][v]), dx + (size_t)dcol[cc] + (size_t)cr * P.HW);
            }
        }
    }
}


// ---- host side: which variant of the body a layer takes, and its tiling -----------------------------------

template <int CT, int S, int WPB>
inline BwiTiling make_tiling(const Problem& p, long long* blocks)
{
    BwiTiling t;
    t.b = make_band(p);
    t.CB = (p.Cin + 31) / 32;
    const long long nct = (p.NQ + 32 * CT - 1) / (32 * CT);
    t.FG = (t.CB * S + WPB - 1) / WPB;
    t.total = (int)(nct * t.FG);
    t.chunk = (t.total + 7) / 8;
    *blocks = (long long)8 * t.chunk;
    return t;
}

// Calls f(CT, VEC, S, WPB, tiling, blocks) with the first four as std::integral_constant / std::bool_constant
// values: the variant backward_input_body<T_, CT, 8, VEC, S, WPB> that the layer takes, and its launch shape
// (blocks workgroups of WPB * 64 threads).
template <typename T_, typename F>
void select_backward_input(const T_* dy, const T_* dx, const Problem& p, F&& f)
{
    using std::bool_constant;
    using std::integral_constant;
    // workgroups of 8 wavefronts (0.6 us faster at the metric layer; delaying half of them, which pays in the
    // forward, does not here): only for grids that fill the chip exactly once with two wavefronts per SIMD, fp32,
    // windows that start on multiples of 32 channels, and at most 16 flop per byte, the shapes it was measured on
    auto with_wpb = [&](auto ct, auto vec, auto s) {
        constexpr int CT = decltype(ct)::value, S = decltype(s)::value;
        constexpr bool VEC = decltype(vec)::value;
        long long blocks = 0;
        if constexpr (sizeof(T_) == 4 && CT == 4 && VEC && S == 1) {
            const Band b = make_band(p);
            const long long cbs = (p.Cin + 31) / 32, nct = (p.NQ + 32 * CT - 1) / (32 * CT), waves = nct * cbs;
            const bool once = waves >= 2048 && waves < 2048 + 256;
            const bool light = (long long)p.Cout * p.L <= 32ll * (p.Cin + p.Cout);
            if (b.g % 32 == 0 && p.Cin % 32 == 0 && cbs % 8 == 0 && once && light) {
                const BwiTiling t = make_tiling<CT, S, 8>(p, &blocks);
                f(ct, vec, s, integral_constant<int, 8>{}, t, blocks);
                return;
            }
        }
        const BwiTiling t = make_tiling<CT, S, 4>(p, &blocks);
        f(ct, vec, s, integral_constant<int, 4>{}, t, blocks);
    };
    // share a tile between 2 or 4 wavefronts while there are fewer than two wavefronts per SIMD and each slice
    // keeps at least 32 K-steps; a block of 32 channels sees about (L+31)/g windows of F filters each
    auto with_split = [&](auto ct, auto vec, long long waves) {
        constexpr int CT = decltype(ct)::value;
        const Band b = make_band(p);
        const long long slots = ((long long)(p.L + 31) / b.g + 1) * b.F;
        int split = 1;
        while (split < 4 && waves * split < 2048 && slots / (4 * split) >= 32) split *= 2;
        if (split == 1)
            with_wpb(ct, vec, integral_constant<int, 1>{});
        else if (split == 2)
            with_wpb(ct, vec, integral_constant<int, 2>{});
        else
            with_wpb(ct, vec, integral_constant<int, 4>{});
    };
    // columns per wavefront: 128 when that still gives every SIMD a wavefront, else 64 or 32; vector plane
    // accesses need planes whose size is a multiple of the vector and tensors aligned to it
    constexpr long long kEnoughWaves = 1024;
    const long long blocks32 = (p.Cin + 31) / 32;
    auto waves = [&](int ct) { return (p.NQ + 32 * ct - 1) / (32 * ct) * blocks32; };
    const uintptr_t addr = (uintptr_t)dy | (uintptr_t)dx;
    auto vec_ok = [&](int ct) { return p.HW % ct == 0 && (addr & (ct * sizeof(T_) - 1)) == 0; };
    // a tile's contraction can be shared by up to 4 wavefronts (with_split): wide tiles, whose loads move 16 bytes
    // per lane and instruction, are kept as long as that sharing still gives every SIMD a wavefront
    auto shared = [&](long long wv) {
        const Band b = make_band(p);
        const long long slots = ((long long)(p.L + 31) / b.g + 1) * b.F;
        int sp = 1;
        while (sp < 4 && wv * sp < 2048 && slots / (4 * sp) >= 32) sp *= 2;
        return wv * sp;
    };
    if (vec_ok(4) && shared(waves(4)) >= kEnoughWaves)
        with_split(integral_constant<int, 4>{}, bool_constant<true>{}, waves(4));
    else if (vec_ok(2) && shared(waves(2)) >= kEnoughWaves)
        with_split(integral_constant<int, 2>{}, bool_constant<true>{}, waves(2));
    else if (waves(2) >= kEnoughWaves)
        with_split(integral_constant<int, 2>{}, bool_constant<false>{}, waves(2));
    else
        with_split(integral_constant<int, 1>{}, bool_constant<false>{}, waves(1));
}

}  // namespace bwi

}  // namespace scc
