// Grad-input of SCC on the gfx950 matrix cores for layers in which many 32-channel blocks pull from the same
// filters (few, long windows: cg <= 2; windows that start on every channel, as in the channel-expanding layers):
// the dy operand goes through LDS once per workgroup.
//
// dx[n,c,p] = sum over filters k whose window covers c of w[k,(c-s_k) mod Cin] * dy[n,k,p]
// (Section 4.2, input-centric backward: every input-gradient element PULLS from the filters covering its
// channel, so nothing is accumulated with atomics).
//
// scc_mfma_bwi_kernel.h gives every block of 32 channels its own wavefront, which fetches the dy planes of all
// filters covering the block and cuts every binary32 value into three bf16 pieces for itself.  Neighbouring blocks
// are covered by nearly the same filters, so on such layers every dy value is fetched and cut 3-4 times, and the
// wavefronts of a workgroup, each walking its own filter range, drift so far apart that the re-reads miss the L2
// (the channel-expanding layer read dy 3x from HBM).  Here a workgroup of four wavefronts owns four consecutive
// channel blocks for the same 128 columns and walks the union of their filters ONCE, in rounds of 32 dy planes:
// the 256 lanes fetch a round (one 16-byte load per lane and plane, 4 planes per lane), cut each value once and
// park the bf16 pieces in LDS in the matrix instruction's operand layout (scc_fwd_shared.hip does the same for
// the forward); every wavefront takes its B operands from there.  A round none of a block's filters falls into
// is skipped by that block's wavefront.
//
// The walk: windows in the order of their starts (scc_band.h: start g*m, filters k = r(m) + P*i), from the first
// window that covers the workgroup's first channel to the last that covers its last channel, but at most all P
// windows once (then every window is in the walk and the order is a rotation of the circle); walk position
// pos <-> (window pos / F, filter pos % F of that window).  A table in LDS, built when the workgroup starts, maps
// a position to the filter's weight row, the window's start and the dy plane.  The A operand needs no staging:
// lane f of a half-wave is channel c0 + f, and consecutive channels read consecutive weights of a filter's row
// (one coalesced 128-byte read per half-wave and K value); weights outside the window are masked to zero.
//
// fp32 tensors, planes whose size is a multiple of 4 and 16-byte aligned dy/dx only; the products are the
// six-of-nine bf16 partial products of scc_common.h, sums binary32.
#include <type_traits>

#include "scc_band.h"
#include "scc_common.h"

namespace scc {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

constexpr int kWavesG = 4;                  // wavefronts (= channel blocks) per workgroup
constexpr int kColsG = 128;                 // columns per workgroup
constexpr int kRoundG = 32;                 // dy planes per round: two K groups of 16
constexpr int kGPiece = 2 * 2 * kColsG * 16;   // bytes of one bf16 piece of a round's B operands: [K group][half][column][8 planes]
constexpr int kGBuf = 3 * kGPiece;          // one B buffer
constexpr int kMaxPos = 1024;               // walk positions the table holds (a round of slack included)
constexpr int kLdsG = 2 * kGBuf + kMaxPos * 16;   // 64 KB: two workgroups per CU

struct BwiSharedTiling {
    Band b;
    int CB;        // channel blocks of 32
    int FG;        // workgroups per column tile: ceil(CB / 4)
    int total;     // workgroups with work
    int chunk;     // consecutive workgroups given to one XCD
};

__host__ __device__ inline int floor_div_g(int a, int b)  // b > 0
{
    const int q = a / b;
    return (a % b != 0 && a < 0) ? q - 1 : q;
}

// Windows (unwrapped indices m, start g*m) that cover any channel of [c_lo, c_hi]: g*m in [c_lo - L + 1, c_hi]
__host__ __device__ inline void covering_windows(int c_lo, int c_hi, int L, int g, int* mlo, int* mhi)
{
    *mlo = -floor_div_g(L - 1 - c_lo, g);   // ceil((c_lo - L + 1) / g)
    *mhi = floor_div_g(c_hi, g);
}

__global__ __launch_bounds__(kWavesG * 64, 2) void backward_input_shared32(const float* __restrict__ dy,
                                                                           const float* __restrict__ w,
                                                                           float* __restrict__ dx, Problem P,
                                                                           BwiSharedTiling T)
{
    extern __shared__ __attribute__((aligned(16))) char lds_g[];
    char* const b_lds = lds_g;                              // two B buffers
    i32x4* const table = (i32x4*)(lds_g + 2 * kGBuf);       // per walk position: {k*L or -1, window start, byte offset of dy plane k, 0}

    // workgroup -> (column tile, group of four channel blocks), group fastest; each XCD takes a contiguous run
    const int bid = blockIdx.x;
    const int xcd = bid & 7, slot = bid >> 3;
    const int logical = xcd * T.chunk + slot;
    if (slot >= T.chunk || logical >= T.total) return;      // the whole workgroup leaves
    const int ct = logical / T.FG, fg = logical % T.FG;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int f = lane & 31, h = lane >> 5;
    const int F = T.b.F, Pw = T.b.P, g = T.b.g;

    // ---- the workgroup's walk ---------------------------------------------------------------------------
    const int cb_first = fg * kWavesG;
    const int cb_last = cb_first + kWavesG - 1 < T.CB ? cb_first + kWavesG - 1 : T.CB - 1;
    const int c_end = 32 * cb_last + 31 < P.Cin ? 32 * cb_last + 31 : P.Cin - 1;
    int mlo_w, mhi_w;
    covering_windows(32 * cb_first, c_end, P.L, g, &mlo_w, &mhi_w);
    const int nwin = mhi_w - mlo_w + 1 < Pw ? mhi_w - mlo_w + 1 : Pw;   // every window at most once
    const int npos = nwin * F;                               // walk positions [0, npos)
    const int nround = npos > 0 ? (npos + kRoundG - 1) / kRoundG : 1;   // channels no window covers: one round without filters
    const uint32_t plane = (uint32_t)P.HW * 4u;
    for (int pos = tid; pos < (nround + 1) * kRoundG; pos += kWavesG * 64) {
        const int mm = pos / F, i = pos - mm * F;
        int mw = (mlo_w + mm) % Pw;
        mw += mw < 0 ? Pw : 0;
        const int k = (int)(((uint32_t)mw * (uint32_t)T.b.inv) % (uint32_t)Pw) + Pw * i;
        const bool valid = pos < npos && k < P.Cout;
        table[pos] = i32x4{valid ? k * P.L : -1, g * mw, valid ? (int)((uint32_t)k * plane) : 0, 0};
    }

    // ---- this wavefront's channel block -----------------------------------------------------------------
    const int cb = cb_first + wave;
    const bool tvalid = cb <= cb_last;
    const int c0 = 32 * cb;
    const int c = c0 + f;                                    // this lane's channel (A row)
    const bool cvalid = tvalid && c < P.Cin;
    // the block's filters are the walk positions [a0, a0 + alen), modulo npos when the walk is the whole circle
    int a0 = 0, alen = 0;
    if (tvalid) {
        int mlo_b, mhi_b;
        covering_windows(c0, c0 + 31 < P.Cin ? c0 + 31 : P.Cin - 1, P.L, g, &mlo_b, &mhi_b);
        const int cnt = mhi_b - mlo_b + 1 < Pw ? mhi_b - mlo_b + 1 : Pw;
        a0 = (mlo_b - mlo_w) * F;
        a0 -= a0 >= npos ? npos : 0;                         // only when the walk is the whole circle
        alen = cnt * F;
    }
    auto overlap = [](int p0, int p1, int q0, int q1) { return p0 < q1 && q0 < p1; };
    auto group_active = [&](int pos) {                      // any of positions [pos, pos+16) belongs to the block
        const int e1 = a0 + alen < npos ? a0 + alen : npos;
        return overlap(pos, pos + 16, a0, e1) || (a0 + alen > npos && overlap(pos, pos + 16, 0, a0 + alen - npos));
    };

    // ---- A side: weights straight into operand layout, two rounds ahead ----------------------------------
    // lane (f, h) holds, for K group s of a round, the weights that multiply walk positions 32r + 16s + 8h + e
    // into channel c: w[k][(c - start) mod Cin] where that is inside the window
    float araw[2][16];
    uint32_t amask[2] = {0u, 0u};
    auto issue_a = [&](auto SET, int r) {
        constexpr int set = decltype(SET)::value;
        uint32_t mk = 0;
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const u32x2 ent = *(const u32x2*)&table[kRoundG * r + 16 * s + 8 * h + e];
                const int kl = (int)ent[0];
                int ju = c - (int)ent[1];
                ju += ju < 0 ? P.Cin : 0;
                const bool in = cvalid && kl >= 0 && ju < P.L;
                araw[set][8 * s + e] = w[in ? kl + ju : 0];
                mk |= in ? (1u << (8 * s + e)) : 0u;
            }
        amask[set] = mk;
    };

    // ---- B side, loading role: thread (u = tid/32, q = tid%32) fetches the 4 columns 4q..4q+3 of the 4 dy planes
    // at walk positions 32r + 4u + e: K group u/4, half-wave (u/2)%2, operand values 4*(u%2) + e
    const int lq = tid & 31, lu = tid >> 5;
    uint32_t lcol;                                           // byte offset of this thread's 4 columns in plane 0 of their sample
    {
        const uint32_t q = (uint32_t)ct * kColsG + 4u * (uint32_t)lq;
        const uint32_t qq = q < (uint32_t)P.NQ ? q : 0u;     // columns past the end read column 0 and are never stored
        const uint32_t n = qq / (uint32_t)P.HW, p = qq % (uint32_t)P.HW;
        lcol = (n * (uint32_t)P.Cout * (uint32_t)P.HW + p) * 4u;
    }
    const int b_dst = (((lu >> 2) * 2 + ((lu >> 1) & 1)) * kColsG + lq) * 16 + 8 * (lu & 1);
    const char* gb = (const char*)dy;
    f32x4 braw[2][4];
    auto issue_b = [&](auto SET, int r) {
        constexpr int set = decltype(SET)::value;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t rowb = (uint32_t)table[kRoundG * r + 4 * lu + e][2];   // plane 0 for positions without a filter
            braw[set][e] = *(const f32x4*)(gb + (lcol + rowb));
        }
    };
    auto commit_b = [&](auto SET) {                          // set s -> LDS buffer s
        constexpr int set = decltype(SET)::value;
        char* dst = b_lds + set * kGBuf + b_dst;
#pragma unroll
        for (int j = 0; j < 4; ++j) {                         // column 4q + j is operand column (j, q): LDS column 32j + q
            uint32_t hi[2], mid[2], lo3[2];
            split3<4>([&](int e) { return braw[set][e][j]; }, hi, mid, lo3);
            *(u32x2*)(dst + j * 32 * 16) = u32x2{hi[0], hi[1]};
            *(u32x2*)(dst + j * 32 * 16 + kGPiece) = u32x2{mid[0], mid[1]};
            *(u32x2*)(dst + j * 32 * 16 + 2 * kGPiece) = u32x2{lo3[0], lo3[1]};
        }
    };

    f32x16 acc[4];
#pragma unroll
    for (int cc = 0; cc < 4; ++cc)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[cc][v] = 0.f;

    // one K group (16 walk positions) of round r: A from register set SET, B operands from LDS buffer SET
    auto compute = [&](auto SET, int r, int s) {
        constexpr int set = decltype(SET)::value;
        if (!group_active(kRoundG * r + 16 * s)) return;
        uint32_t ah[4], am[4], al[4];
        split3<8>([&](int e) { return (amask[set] >> (8 * s + e)) & 1u ? araw[set][8 * s + e] : 0.f; }, ah, am, al);
        const char* bb = b_lds + set * kGBuf + f * 16;
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            uint32_t bp[3][4];
#pragma unroll
            for (int q = 0; q < 3; ++q) {
                const u32x4 t = *(const u32x4*)(bb + q * kGPiece + ((s * 2 + h) * kColsG + cc * 32) * 16);
#pragma unroll
                for (int z = 0; z < 4; ++z) bp[q][z] = t[z];
            }
            acc[cc] = mfma_bf16<8>(al, bp[0], acc[cc]);
            acc[cc] = mfma_bf16<8>(ah, bp[2], acc[cc]);
            acc[cc] = mfma_bf16<8>(am, bp[1], acc[cc]);
            acc[cc] = mfma_bf16<8>(am, bp[0], acc[cc]);
            acc[cc] = mfma_bf16<8>(ah, bp[1], acc[cc]);
            acc[cc] = mfma_bf16<8>(ah, bp[0], acc[cc]);
        }
    };

    // Round r lives in register set r & 1 while in flight and (its B operands) in LDS buffer r & 1 once parked.
    // Rounds 0 and 1 are requested up front; then, per round r: request round r+2's dy planes, multiply the first K
    // group, park round r+1's B operands (the barrier that ended round r-1 says every wavefront is done with that
    // buffer), multiply the second K group, request round r+2's weights into the registers round r's just left,
    // barrier.  No load is conditional inside the
    // loop (a wait behind a branch that may have issued loads has to assume it did not): the loop body runs while
    // a round r+3 exists and the last rounds are written out.  The table holds a round of positions without filters
    // past the walk, so requesting the second round of a walk that has only one stays in bounds.
    typedef std::integral_constant<int, 0> Set0;
    typedef std::integral_constant<int, 1> Set1;
    auto body = [&](auto PAR, auto OTHER, int r, auto ISSUE, auto COMMIT) {
        if constexpr (decltype(ISSUE)::value) issue_b(PAR, r + 2);     // round r's B values were parked a round ago
        compute(PAR, r, 0);
        if constexpr (decltype(COMMIT)::value) commit_b(OTHER);
        compute(PAR, r, 1);
        if constexpr (decltype(ISSUE)::value) issue_a(PAR, r + 2);     // round r's weights have just been used
        __syncthreads();
    };
    const std::true_type yes;
    const std::false_type no;
    __syncthreads();                                         // the table is complete
    issue_a(Set0(), 0);
    issue_b(Set0(), 0);
    issue_a(Set1(), 1);
    issue_b(Set1(), 1);
    commit_b(Set0());
    __syncthreads();
    int r = 0;
    for (; r + 3 < nround; r += 2) {
        body(Set0(), Set1(), r, yes, yes);
        body(Set1(), Set0(), r + 1, yes, yes);
    }
    const int rem = nround - r;                              // 1, 2 or 3 rounds left (nround >= 1); r is even
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

    // ---- store: accumulator register v holds channel c0 + 8*(v/4) + 4*h + v%4, columns 4f .. 4f+3 of the tile ----
    const uint32_t q = (uint32_t)ct * kColsG + 4u * (uint32_t)f;
    if (q >= (uint32_t)P.NQ) return;
    const uint32_t n = q / (uint32_t)P.HW, p = q % (uint32_t)P.HW;
    float* db = dx + (size_t)n * P.Cin * P.HW + p;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int cr = c0 + 8 * (v >> 2) + 4 * h + (v & 3);
        if (cr < P.Cin) {
            const f32x4 o = {acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
            __builtin_nontemporal_store(o, (f32x4*)(db + (size_t)cr * P.HW));   // written once, never re-read here
        }
    }
}

BwiSharedTiling make_bwi_shared_tiling(const Problem& p)
{
    BwiSharedTiling t;
    t.b = make_band(p);
    t.CB = (p.Cin + 31) / 32;
    t.FG = (t.CB + kWavesG - 1) / kWavesG;
    const long long nct = (p.NQ + kColsG - 1) / kColsG;
    t.total = (int)(nct * t.FG);
    t.chunk = (t.total + 7) / 8;
    return t;
}

// walk positions of the longest walk of a layer, and (filters walked by the blocks on their own) / (by the groups)
void walk_stats(const Problem& p, const BwiSharedTiling& t, int* longest, double* gain)
{
    long long own = 0, sharedp = 0;
    *longest = 0;
    for (int fg = 0; fg < t.FG; ++fg) {
        const int first = fg * kWavesG, last = first + kWavesG - 1 < t.CB ? first + kWavesG - 1 : t.CB - 1;
        int mlo, mhi;
        covering_windows(32 * first, 32 * last + 31 < p.Cin ? 32 * last + 31 : p.Cin - 1, p.L, t.b.g, &mlo, &mhi);
        const int nwin = mhi - mlo + 1 < t.b.P ? mhi - mlo + 1 : t.b.P;
        const int npos = nwin * t.b.F;
        if (npos > *longest) *longest = npos;
        sharedp += (npos + kRoundG - 1) / kRoundG * kRoundG;
        for (int cb = first; cb <= last; ++cb) {
            covering_windows(32 * cb, 32 * cb + 31 < p.Cin ? 32 * cb + 31 : p.Cin - 1, p.L, t.b.g, &mlo, &mhi);
            const int cnt = mhi - mlo + 1 < t.b.P ? mhi - mlo + 1 : t.b.P;
            own += (cnt * t.b.F + 15) / 16 * 16;
        }
    }
    *gain = (double)own / (double)sharedp;
}

}  // namespace

bool backward_input_shared_eligible(const float* dy, const float* dx, const Problem& p)
{
    const uintptr_t addr = (uintptr_t)dy | (uintptr_t)dx;
    if (!backward_input_mfma_eligible(p) || p.HW % 4 != 0 || (addr & 15) != 0) return false;
    const BwiSharedTiling t = make_bwi_shared_tiling(p);
    int longest;
    double gain;
    walk_stats(p, t, &longest, &gain);
    // the table holds the walk and one more round; weight offsets k*L + j fit an int (checked by the caller's eligibility)
    return (longest + kRoundG - 1) / kRoundG * kRoundG + kRoundG <= kMaxPos &&
           (long long)((p.NQ + kColsG - 1) / kColsG) * t.FG < (1ll << 28);
}

// Measured: the shared walk wins where the per-block kernel loses the re-reads of dy to HBM, i.e. where windows
// start more densely than channel blocks (g < 32), so that the four blocks of a column tile walk filter ranges
// that are shifted against each other and never meet in the L2 (channel-expanding layer: dy read once instead of
// three times, 124 against 133 us), and where four blocks walk nearly the same filters (cg = 1 at the metric
// shape, 4x: 40 against 44 us); the grid has to fill the chip (two workgroups per CU).  With fewer shared filters
// or fewer columns the per-block kernel is faster (cg = 2: 27 against 30 us; the stack's layers).
bool backward_input_shared_preferred(const float* dy, const float* dx, const Problem& p)
{
#ifdef SCC_SHARED_ALWAYS
    return backward_input_shared_eligible(dy, dx, p);
#else
    if (!backward_input_shared_eligible(dy, dx, p)) return false;
    const BwiSharedTiling t = make_bwi_shared_tiling(p);
    int longest;
    double gain;
    walk_stats(p, t, &longest, &gain);
    return t.total >= 512 && (gain >= 3.5 || (gain >= 2.9 && t.b.g < 32));
#endif
}

hipError_t launch_backward_input_shared(const float* dy, const float* w, float* dx, const Problem& p, hipStream_t st)
{
    const BwiSharedTiling t = make_bwi_shared_tiling(p);
    static const hipError_t allowed =
        hipFuncSetAttribute((const void*)backward_input_shared32, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsG);
    if (allowed != hipSuccess) return allowed;
    backward_input_shared32<<<dim3((unsigned)(8 * t.chunk)), dim3(kWavesG * 64), kLdsG, st>>>(dy, w, dx, p, t);
    return hipGetLastError();
}

}  // namespace scc
