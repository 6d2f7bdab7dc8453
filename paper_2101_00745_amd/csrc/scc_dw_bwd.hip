// Gradients of the depthwise 3x3 stage (Eq. 2 of the paper) that precedes the SCC in a DW + SCC block:
//
//   z[n,a,m,q]  = sum_{i,j<3} kdw[a,i,j] * x[n,a, s*m+i-1, s*q+j-1]          (forward, zero outside the map)
//   dx[n,a,r,c] = sum over (i,j,m,q) with s*m+i-1 = r, s*q+j-1 = c of kdw[a,i,j] * dz[n,a,m,q]
//   dk[a,i,j]   = sum_{n,m,q} dz[n,a,m,q] * x[n,a, s*m+i-1, s*q+j-1]
//
// (the paper trains DW + SCC blocks end to end and gives no formula for these; they are the derivatives of Eq. 2).
// At stride 1 the grad-input is the stage itself applied to dz with every filter turned by 180 degrees, and runs on
// the forward's kernels; other strides gather per input pixel.  The filter gradient is nine dot products per
// channel over all samples and pixels: workgroups take (channel, slice of the samples), every thread keeps nine
// sums, a workgroup adds its threads' sums through LDS in a fixed order and writes one partial per slice, and a
// second kernel adds the slices in order: no atomics, bitwise reproducible.
#include "scc_common.h"
#include "scc_dw_strip.h"

namespace scc {

namespace {

// ---- grad-input, any stride: one thread per input pixel pulls from the outputs whose taps reach it ---------------
template <typename T_>
__global__ __launch_bounds__(256) void depthwise3x3_backward_input_gather(const T_* __restrict__ dz,
                                                                          const T_* __restrict__ kdw,
                                                                          T_* __restrict__ dx, int C, DwGeom G,
                                                                          long long items)
{
    const long long HWo = (long long)G.Ho * G.Wo;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < items; e += (long long)gridDim.x * 256) {
        const int c = (int)(e % G.W);
        long long t = e / G.W;
        const int r = (int)(t % G.H);
        t /= G.H;                                  // t = n*C + a
        const int a = (int)(t % C);
        const T_* go = dz + t * HWo;
        float out = 0.f;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int rr = r + 1 - i;              // = s*m
            if (rr < 0 || rr % G.s != 0 || rr / G.s >= G.Ho) continue;
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const int cc = c + 1 - j;          // = s*q
                if (cc < 0 || cc % G.s != 0 || cc / G.s >= G.Wo) continue;
                out += to_f32(kdw[a * 9 + i * 3 + j]) * to_f32(go[(long long)(rr / G.s) * G.Wo + cc / G.s]);
            }
        }
        dx[e] = from_f32<T_>(out);
    }
}

// ---- grad-input at stride 2 on even maps (H = 2*Ho, W = 2*Wo, Wo even, tensors aligned to 4 values): the taps
// that reach input pixel (r, c) are fixed by the parities of r and c, so a thread writes the 2 x 4 input pixels
// under two neighbouring outputs (m, q0), (m, q0+1) from the 2 x 3 outputs around them:
//   dx[2m  ][2q  ] = k11*g[m][q]                      dx[2m  ][2q+1] = k10*g[m][q+1] + k12*g[m][q]
//   dx[2m+1][2q  ] = k01*g[m+1][q] + k21*g[m][q]      dx[2m+1][2q+1] = k00*g[m+1][q+1] + k02*g[m+1][q] + k20*g[m][q+1] + k22*g[m][q]
template <typename T_>
__global__ __launch_bounds__(256) void depthwise3x3_backward_input_s2(const T_* __restrict__ dz, const T_* __restrict__ kdw,
                                                                      T_* __restrict__ dx, int C, DwGeom G, uint32_t items)
{
    typedef T_ tvec __attribute__((ext_vector_type(4)));
    typedef T_ tvec2 __attribute__((ext_vector_type(2)));
    const uint32_t W2 = G.Wo / 2;
    const size_t HWi = (size_t)G.H * G.W, HWo = (size_t)G.Ho * G.Wo;
    for (uint32_t e = blockIdx.x * 256u + threadIdx.x; e < items; e += gridDim.x * 256u) {
        const int q0 = (int)(e % W2) * 2;
        uint32_t t = e / W2;
        const int m = (int)(t % (uint32_t)G.Ho);
        t /= (uint32_t)G.Ho;                        // t = n*C + a
        const int a = (int)(t % (uint32_t)C);
        float k[9];
        dw::load_taps(kdw, a, false, k);
        const T_* g0 = dz + t * HWo + (size_t)m * G.Wo + q0;
        const bool down = m + 1 < G.Ho, right = q0 + 2 < G.Wo;
        const T_* g1 = down ? g0 + G.Wo : g0;
        const tvec2 a01 = *(const tvec2*)g0, b01 = *(const tvec2*)g1;
        const float a2 = right ? to_f32(g0[2]) : 0.f, b2raw = to_f32(g1[right ? 2 : 0]);
        const float ga[3] = {to_f32(a01[0]), to_f32(a01[1]), a2};
        const float gb[3] = {down ? to_f32(b01[0]) : 0.f, down ? to_f32(b01[1]) : 0.f, (down && right) ? b2raw : 0.f};
        tvec r0, r1;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            r0[2 * j] = from_f32<T_>(k[4] * ga[j]);
            r0[2 * j + 1] = from_f32<T_>(k[3] * ga[j + 1] + k[5] * ga[j]);
            r1[2 * j] = from_f32<T_>(k[1] * gb[j] + k[7] * ga[j]);
            r1[2 * j + 1] = from_f32<T_>(k[0] * gb[j + 1] + k[2] * gb[j] + k[6] * ga[j + 1] + k[8] * ga[j]);
        }
        T_* o = dx + t * HWi + (size_t)(2 * m) * G.W + 2 * q0;
        __builtin_nontemporal_store(r0, (tvec*)o);
        __builtin_nontemporal_store(r1, (tvec*)(o + G.W));
    }
}

// ---- grad-filter ----------------------------------------------------------------------------------------------
constexpr int kDkThreads = 256;

// the workgroup's nine sums: threads -> LDS -> thread t < 9 adds them in thread order
__device__ __forceinline__ void reduce_nine(const float (&s)[9], float* out9)
{
    __shared__ float part[9][kDkThreads];
#pragma unroll
    for (int t = 0; t < 9; ++t) part[t][threadIdx.x] = s[t];
    __syncthreads();
    if (threadIdx.x < 9) {
        float acc = 0.f;
        for (int u = 0; u < kDkThreads; ++u) acc += part[threadIdx.x][u];
        out9[threadIdx.x] = acc;
    }
}

// On strips (stride S = 1 or 2, output rows of whole column quads, input maps of exactly S times the output size,
// RB dividing the output rows, tensors aligned to 4 values): a thread reads the strip's RB rows of dz and its
// S*(RB-1)+3 rows of x once (dw::strip_row) and adds their products to its nine sums.
// Workgroup (a, slice) walks the strips of channel a in samples [slice*per, slice*per + per).
template <typename T_, int S, int RB>
__global__ __launch_bounds__(kDkThreads) void depthwise3x3_backward_filter_strips(const T_* __restrict__ x,
                                                                                  const T_* __restrict__ dz,
                                                                                  float* __restrict__ part, int N, int C,
                                                                                  DwGeom G, int per)
{
    typedef T_ tvec __attribute__((ext_vector_type(4)));
    constexpr int NR = S * (RB - 1) + 3;
    const int a = blockIdx.x, slice = blockIdx.y;
    const int n0 = slice * per, n1 = n0 + per < N ? n0 + per : N;
    const uint32_t W4 = G.Wo / 4, SB = G.Ho / RB, spp = W4 * SB;             // strips per plane
    const uint32_t items = (uint32_t)(n1 > n0 ? n1 - n0 : 0) * spp;
    const size_t HWi = (size_t)G.H * G.W, HWo = (size_t)G.Ho * G.Wo;
    const uint32_t lane = threadIdx.x & 63;
    float s[9] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // all lanes of a wavefront run the same number of trips (strip_row shuffles between lanes); lanes past the end
    // read strip 0 again and add nothing
    for (uint32_t e0 = 0; e0 < items; e0 += kDkThreads) {
        const uint32_t ee = e0 + threadIdx.x;
        const bool live = ee < items;
        const uint32_t e = live ? ee : 0;
        const int cw = (int)(e % W4) * 4;
        uint32_t t = e / W4;
        const int r0 = (int)(t % SB) * RB;
        const size_t plane = (size_t)(n0 + t / SB) * C + a;
        const T_* xc = x + plane * HWi + (size_t)(S * r0) * G.W + S * cw;
        const T_* gz = dz + plane * HWo + (size_t)r0 * G.Wo + cw;
        float g[RB][4];
#pragma unroll
        for (int rr = 0; rr < RB; ++rr) {
            const tvec m = *(const tvec*)(gz + rr * G.Wo);
#pragma unroll
            for (int i = 0; i < 4; ++i) g[rr][i] = live ? to_f32(m[i]) : 0.f;
        }
        const uint32_t rowmask = dw::strip_rowmask<S, RB>(r0, G.Ho);
#pragma unroll
        for (int tr = 0; tr < NR; ++tr) {
            float v[4 * S + 2];
            dw::strip_row<S>(xc, G.W, tr, rowmask, cw > 0, cw + 4 < G.Wo, lane == 0, lane == 63 || ee + 1 >= items, v);
#pragma unroll
            for (int rr = 0; rr < RB; ++rr) {
                const int di = tr - S * rr;      // tap row that pairs this input row with output row rr
                if (di < 0 || di > 2) continue;
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 3; ++j) s[di * 3 + j] += g[rr][i] * v[S * i + j];
            }
        }
    }
    reduce_nine(s, part + ((size_t)slice * C + a) * 9);
}

// Any stride and map size: a thread takes output pixels one by one.
template <typename T_>
__global__ __launch_bounds__(kDkThreads) void depthwise3x3_backward_filter_generic(const T_* __restrict__ x,
                                                                                   const T_* __restrict__ dz,
                                                                                   float* __restrict__ part, int N, int C,
                                                                                   DwGeom G, int per)
{
    const int a = blockIdx.x, slice = blockIdx.y;
    const int n0 = slice * per, n1 = n0 + per < N ? n0 + per : N;
    const long long HWi = (long long)G.H * G.W, HWo = (long long)G.Ho * G.Wo;
    const long long items = (long long)(n1 > n0 ? n1 - n0 : 0) * HWo;
    float s[9] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (long long e = threadIdx.x; e < items; e += kDkThreads) {
        const int q = (int)(e % G.Wo);
        long long t = e / G.Wo;
        const int m = (int)(t % G.Ho);
        const long long plane = (long long)(n0 + t / G.Ho) * C + a;
        const float g = to_f32(dz[plane * HWo + (long long)m * G.Wo + q]);
        const T_* xc = x + plane * HWi;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const int rr = G.s * m + i - 1;
            if (rr < 0 || rr >= G.H) continue;
#pragma unroll
            for (int j = 0; j < 3; ++j) {
                const int cc = G.s * q + j - 1;
                if (cc < 0 || cc >= G.W) continue;
                s[i * 3 + j] += g * to_f32(xc[(long long)rr * G.W + cc]);
            }
        }
    }
    reduce_nine(s, part + ((size_t)slice * C + a) * 9);
}

// dk[e] = sum over slices of part[slice][e], in slice order
__global__ __launch_bounds__(256) void depthwise3x3_filter_reduce(const float* __restrict__ part, float* __restrict__ dk,
                                                                  int count, int slices)
{
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= count) return;
    float s = 0.f;
    for (int sl = 0; sl < slices; ++sl) s += part[(size_t)sl * count + e];
    dk[e] = s;
}

// slices of the samples per channel: about 1024 workgroups in all, at least one sample per slice, at most 65535
int filter_slices(int N, int C)
{
    int sl = (1024 + C - 1) / C;
    if (sl > N) sl = N;
    if (sl > 65535) sl = 65535;
    return sl < 1 ? 1 : sl;
}

template <typename T, int S>
void launch_filter_strips(const T* x, const T* dz, float* part, int N, int C, const DwGeom& g, int slices, int per,
                          hipStream_t st)
{
    const dim3 grid((unsigned)C, (unsigned)slices), block(kDkThreads);
    if (g.Ho % 4 == 0)
        depthwise3x3_backward_filter_strips<T, S, 4><<<grid, block, 0, st>>>(x, dz, part, N, C, g, per);
    else if (g.Ho % 2 == 0)
        depthwise3x3_backward_filter_strips<T, S, 2><<<grid, block, 0, st>>>(x, dz, part, N, C, g, per);
    else
        depthwise3x3_backward_filter_strips<T, S, 1><<<grid, block, 0, st>>>(x, dz, part, N, C, g, per);
}

}  // namespace

size_t depthwise3x3_backward_workspace(int N, int C, const DwGeom&)
{
    const int slices = filter_slices(N, C);
    return slices > 1 ? (size_t)slices * C * 9 * sizeof(float) : 0;
}

template <typename T>
hipError_t launch_depthwise3x3_backward(const T* x, const T* kdw, const T* dz, T* dx, float* dk, float* workspace, int N,
                                        int C, const DwGeom& g, hipStream_t st)
{
    if (dx) {
        if (g.s == 1) {
            // the stage applied to dz (an Ho x Wo = H x W map) with the filters turned by 180 degrees
            DwGeom gz = g;
            const hipError_t e = launch_depthwise3x3(dz, kdw, dx, N, C, gz, st, true);
            if (e != hipSuccess) return e;
        } else if (g.s == 2 && g.H == 2 * g.Ho && g.W == 2 * g.Wo && g.Wo % 2 == 0 &&
                   (((uintptr_t)dz | (uintptr_t)dx) & (4 * sizeof(T) - 1)) == 0 &&
                   (long long)N * C * g.Ho * (g.Wo / 2) < (1ll << 31)) {
            const long long items = (long long)N * C * g.Ho * (g.Wo / 2);
            long long blocks = (items + 255) / 256;
            if (blocks > (1ll << 20)) blocks = 1ll << 20;
            depthwise3x3_backward_input_s2<T><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(dz, kdw, dx, C, g, (uint32_t)items);
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        } else {
            const long long items = (long long)N * C * g.H * g.W;
            long long blocks = (items + 255) / 256;
            if (blocks > (1ll << 20)) blocks = 1ll << 20;   // the kernel strides over what is left
            depthwise3x3_backward_input_gather<T><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(dz, kdw, dx, C, g, items);
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    if (dk) {
        const int slices = filter_slices(N, C);
        const int per = (N + slices - 1) / slices;
        float* part = slices > 1 ? workspace : dk;
        const bool strips = (g.s == 1 || g.s == 2) && g.Wo % 4 == 0 && g.H == g.s * g.Ho && g.W == g.s * g.Wo &&
                            (((uintptr_t)x | (uintptr_t)dz) & (4 * sizeof(T) - 1)) == 0 &&
                            (long long)per * g.Ho * (g.Wo / 4) < (1ll << 31);
        if (strips && g.s == 1)
            launch_filter_strips<T, 1>(x, dz, part, N, C, g, slices, per, st);
        else if (strips)
            launch_filter_strips<T, 2>(x, dz, part, N, C, g, slices, per, st);
        else
            depthwise3x3_backward_filter_generic<T><<<dim3((unsigned)C, (unsigned)slices), dim3(kDkThreads), 0, st>>>(
                x, dz, part, N, C, g, per);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        if (slices > 1) {
            depthwise3x3_filter_reduce<<<dim3((unsigned)((C * 9 + 255) / 256)), dim3(256), 0, st>>>(part, dk, C * 9, slices);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

template hipError_t launch_depthwise3x3_backward<float>(const float*, const float*, const float*, float*, float*, float*,
                                                        int, int, const DwGeom&, hipStream_t);
template hipError_t launch_depthwise3x3_backward<bf16_t>(const bf16_t*, const bf16_t*, const bf16_t*, bf16_t*, float*,
                                                         float*, int, int, const DwGeom&, hipStream_t);

}  // namespace scc
