// Tiling of the SCC filter set for the matrix-core kernels.
//
// Filter k starts at s_k = (k*stride) mod Cin (Algorithm 1 in closed form).  With
// g = gcd(stride, Cin) the starts are exactly the multiples g*m, m in [0, P), P = Cin/g:
// the P distinct windows of the channel-cyclic pattern (Section 4.2).  Filters with
// k mod P == r share the start g*m_r, m_r = (r * stride/g) mod P; the map r <-> m is a
// bijection, inverted with inv = (stride/g)^-1 mod P.  So the filter set is a grid
//     (m, i)  <->  k = ((m*inv) mod P) + P*i,      m in [0,P), i in [0, ceil(Cout/P)),  k < Cout
// in which filters of one column m see the SAME window (a dense GEMM) and adjacent columns
// see windows shifted by g channels (a band).  A tile of TM columns x TI rows spans
// L + g*(TM-1) input channels, of which every filter uses L.
#pragma once
#include "scc_common.h"

namespace scc {

struct Band {
    int g;    // spacing of distinct window starts (Cin when every filter starts at 0)
    int P;    // number of distinct window starts over all k >= 0
    int inv;  // residue r = (m*inv) mod P owns start g*m
    int F;    // ceil(Cout / P): most filters sharing one start
};

inline long long band_gcd(long long a, long long b)
{
    while (b) {
        long long t = a % b;
        a = b;
        b = t;
    }
    return a;
}

inline Band make_band(const Problem& p)
{
    Band b;
    if (p.stride == 0) {
        b.g = p.Cin;
        b.P = 1;
        b.inv = 0;
    } else {
        b.g = (int)band_gcd(p.stride, p.Cin);
        b.P = p.Cin / b.g;
        const int q = (p.stride / b.g) % b.P;  // coprime to P
        // extended Euclid: q * inv == 1 (mod P)
        long long r0 = b.P, r1 = q, t0 = 0, t1 = 1;
        while (r1 != 0) {
            const long long d = r0 / r1;
            const long long r2 = r0 - d * r1, t2 = t0 - d * t1;
            r0 = r1;
            r1 = r2;
            t0 = t1;
            t1 = t2;
        }
        int inv = (int)(((t0 % b.P) + b.P) % b.P);  // P == 1: q == 0 and inv == 0
        b.inv = inv;
    }
    b.F = (p.Cout + b.P - 1) / b.P;
    return b;
}

}  // namespace scc
