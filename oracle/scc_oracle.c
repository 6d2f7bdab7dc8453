/*
 * CPU oracle for the sliding-channel convolution (SCC) of DSXplore.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
 * library is checked against.  Only the test-suite, the smoke entry and the
 * benchmark's cpu_baseline leg may build or call it; the product library
 * neither links nor imports it, and the two share no code.
 *
 * Everything is fp64: inputs arrive already widened to double, every sum is
 * accumulated in double, outputs are double.  Loops follow the definition
 * directly: no blocking, no fusion, no reordering beyond "parallel over
 * independent outputs".
 *
 * Passages followed:
 *   window sequence   - Algorithm 1 ("Compute channel indexes of one cycle")
 *                       continued past one cycle the way Algorithm 2 does
 *                       (filter k uses entry k mod cyclic_dist, i.e. the same
 *                       sequence simply keeps going);
 *   forward           - Section 4.2 "Output-Centric Forward Pass": each output
 *                       pixel is a dot product of the filter's weights with the
 *                       pixels at the same (x, y) across the window's channels;
 *   grad-input        - Section 4.2 "Input-Centric Backward Pass": each input
 *                       gradient pixel pulls from the output gradients of all
 *                       filters whose window covers its channel;
 *   grad-weight       - Section 4.2 names the gradient of the trainable weights
 *                       without describing a kernel; it is the derivative of
 *                       the forward definition with respect to w.
 *   depthwise 3x3     - Eq. 2 (Section 2.2): channel a of the output is the
 *                       3x3 spatial filter of channel a applied to channel a of
 *                       the input, the tap (i, j) reading the pixel
 *                       (m + i - 1, n + j - 1); it is the stage whose output the
 *                       SCC consumes in a DW + SCC block (Section 3.1).
 *   depthwise grads   - the derivatives of Eq. 2 with respect to its input and
 *                       its filters (the paper trains DW + SCC blocks end to end,
 *                       Section 5, and gives no formula): every product
 *                       kdw[a,i,j] * x[n,a,r,c] of the forward sum that forms
 *                       z[n,a,m,q] sends dz[n,a,m,q] * kdw[a,i,j] to dx[n,a,r,c]
 *                       and dz[n,a,m,q] * x[n,a,r,c] to dkdw[a,i,j].
 *
 * Readings taken where the paper is silent:
 *   - overlap in channels is int(co * group_width) with C truncation of the
 *     double product, as Algorithm 1 writes it;
 *   - weight j of filter k multiplies the j-th channel of the window counted
 *     from the window start, wrapping past the last channel to channel 0;
 *   - Cin must be divisible by cg.
 *   - Eq. 2: the taps are i, j in {0, 1, 2}, so the filter is centred on the
 *     output pixel; pixels outside the feature map count as zero (the paper keeps
 *     the spatial size of feature maps across a layer); no flip of the filter
 *     (the equation multiplies tap (i, j) with the pixel offset by (i-1, j-1));
 *     a spatial stride s (the paper's CNNs halve the feature map in some
 *     depthwise stages, the equation has none) centres output pixel (m, n) on
 *     input pixel (s*m, s*n), which gives floor((H-1)/s)+1 output rows.
 *
 * Layout: x[N][Cin][HW], y[N][Cout][HW], w[Cout][L], depthwise filters
 * kdw[C][3][3], all dense row-major.
 *
 * Pinning status (tests/test_oracle_pins.py): every function here is pinned
 * against the paper's worked example, library convolutions for the special
 * cases, the channel-stack composition, dense brute force, invariants and
 * finite differences; the depthwise stage against a library grouped
 * convolution, one-tap filters (pure shifts), tap counts at the border and a
 * dense matrix built tap by tap; its two gradients against a library's
 * automatic differentiation of the grouped convolution, the transpose of that
 * dense matrix, the adjoint identity and central finite differences.  Nothing
 * in this file is "parity unpinned".
 */
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Number of host threads the parallel loops below will use. */
int scc_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Window length and the channel overlap of adjacent filters (Algorithm 1:
 * group_width = Cin // cg; the step between virtual starts is
 * group_width - int(overlap * group_width)).  Returns 0, or -1 when the
 * arguments do not describe an SCC layer. */
int scc_oracle_window(int Cin, int cg, double co, int *L_out, int *ov_out)
{
    if (Cin <= 0 || cg <= 0 || Cin % cg != 0) return -1;
    if (!(co >= 0.0 && co <= 1.0)) return -1;
    int L = Cin / cg;
    int ov = (int)(co * (double)L);
    *L_out = L;
    *ov_out = ov;
    return 0;
}

/* Window start of every filter.  Algorithm 1 places each filter's window
 * L - ov channels after the previous one along an unbounded channel axis and
 * folds positions into [0, Cin); its dictionary only detects when the folded
 * windows repeat, and Algorithm 2 indexes it with k mod cyclic_dist, which
 * gives filter k the k-th position of this same sequence. */
int scc_oracle_starts(int Cin, int Cout, int cg, double co, int *start)
{
    int L, ov;
    if (scc_oracle_window(Cin, cg, co, &L, &ov) != 0 || Cout <= 0) return -1;
    long long unfolded = 0;
    for (int k = 0; k < Cout; ++k) {
        start[k] = (int)(unfolded % Cin);
        unfolded += L - ov;
    }
    return 0;
}

/* y[n,k,p] = sum_j w[k,j] * x[n, (s_k + j) mod Cin, p] */
int scc_oracle_forward(const double *x, const double *w, double *y,
                       int N, int Cin, int Cout, int HW, int cg, double co)
{
    int L, ov;
    if (scc_oracle_window(Cin, cg, co, &L, &ov) != 0) return -1;
    int *s = (int *)malloc(sizeof(int) * (size_t)Cout);
    if (!s) return -2;
    scc_oracle_starts(Cin, Cout, cg, co, s);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < Cout; ++k) {
            double *yo = y + ((size_t)n * Cout + k) * HW;
            for (int p = 0; p < HW; ++p) yo[p] = 0.0;
            for (int j = 0; j < L; ++j) {
                int c = (s[k] + j) % Cin;
                const double *xi = x + ((size_t)n * Cin + c) * HW;
                double wkj = w[(size_t)k * L + j];
                for (int p = 0; p < HW; ++p) yo[p] += wkj * xi[p];
            }
        }
    }
    free(s);
    return 0;
}

/* dx[n,c,p] = sum over filters k whose window covers c of
 *             w[k, (c - s_k) mod Cin] * dy[n,k,p]                       */
int scc_oracle_backward_input(const double *dy, const double *w, double *dx,
                              int N, int Cin, int Cout, int HW, int cg, double co)
{
    int L, ov;
    if (scc_oracle_window(Cin, cg, co, &L, &ov) != 0) return -1;
    int *s = (int *)malloc(sizeof(int) * (size_t)Cout);
    if (!s) return -2;
    scc_oracle_starts(Cin, Cout, cg, co, s);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int c = 0; c < Cin; ++c) {
            double *di = dx + ((size_t)n * Cin + c) * HW;
            for (int p = 0; p < HW; ++p) di[p] = 0.0;
            for (int k = 0; k < Cout; ++k) {
                int j = ((c - s[k]) % Cin + Cin) % Cin; /* position of c in window k */
                if (j >= L) continue;                   /* window k does not cover c */
                const double *go = dy + ((size_t)n * Cout + k) * HW;
                double wkj = w[(size_t)k * L + j];
                for (int p = 0; p < HW; ++p) di[p] += wkj * go[p];
            }
        }
    }
    free(s);
    return 0;
}

/* dw[k,j] = sum_{n,p} dy[n,k,p] * x[n, (s_k + j) mod Cin, p] */
int scc_oracle_backward_weight(const double *x, const double *dy, double *dw,
                               int N, int Cin, int Cout, int HW, int cg, double co)
{
    int L, ov;
    if (scc_oracle_window(Cin, cg, co, &L, &ov) != 0) return -1;
    int *s = (int *)malloc(sizeof(int) * (size_t)Cout);
    if (!s) return -2;
    scc_oracle_starts(Cin, Cout, cg, co, s);
#pragma omp parallel for collapse(2) schedule(static)
    for (int k = 0; k < Cout; ++k) {
        for (int j = 0; j < L; ++j) {
            int c = (s[k] + j) % Cin;
            double acc = 0.0;
            for (int n = 0; n < N; ++n) {
                const double *go = dy + ((size_t)n * Cout + k) * HW;
                const double *xi = x + ((size_t)n * Cin + c) * HW;
                for (int p = 0; p < HW; ++p) acc += go[p] * xi[p];
            }
            dw[(size_t)k * L + j] = acc;
        }
    }
    free(s);
    return 0;
}

/* Output rows (or columns) of the depthwise stage for an input of `size` rows
 * and spatial stride `stride`. */
int scc_oracle_depthwise_out(int size, int stride)
{
    if (size <= 0 || stride <= 0) return -1;
    return (size - 1) / stride + 1;
}

/* z[n,a,m,q] = sum_{i,j in 0..2} kdw[a,i,j] * x[n,a, stride*m + i - 1, stride*q + j - 1],
 * pixels outside the H x W map counting as zero (Eq. 2). */
int scc_oracle_depthwise3x3(const double *x, const double *kdw, double *z,
                            int N, int C, int H, int W, int stride)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || stride <= 0) return -1;
    const int Ho = scc_oracle_depthwise_out(H, stride), Wo = scc_oracle_depthwise_out(W, stride);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int a = 0; a < C; ++a) {
            const double *xi = x + ((size_t)n * C + a) * H * W;
            const double *ka = kdw + (size_t)a * 9;
            double *zo = z + ((size_t)n * C + a) * Ho * Wo;
            for (int m = 0; m < Ho; ++m) {
                for (int q = 0; q < Wo; ++q) {
                    double acc = 0.0;
                    for (int i = 0; i < 3; ++i) {
                        for (int j = 0; j < 3; ++j) {
                            int r = stride * m + i - 1, c = stride * q + j - 1;
                            if (r < 0 || r >= H || c < 0 || c >= W) continue;
                            acc += ka[i * 3 + j] * xi[(size_t)r * W + c];
                        }
                    }
                    zo[(size_t)m * Wo + q] = acc;
                }
            }
        }
    }
    return 0;
}

/* dx[n,a,r,c] and dkdw[a,i,j]: the forward sum of Eq. 2 walked once more, every
 * product handing its share of dz to both of its factors' gradients.
 * dx: N*C*H*W, dkdw: C*9; both are overwritten. */
int scc_oracle_depthwise3x3_backward(const double *x, const double *kdw, const double *dz,
                                     double *dx, double *dkdw,
                                     int N, int C, int H, int W, int stride)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || stride <= 0) return -1;
    const int Ho = scc_oracle_depthwise_out(H, stride), Wo = scc_oracle_depthwise_out(W, stride);
#pragma omp parallel for schedule(static)
    for (int a = 0; a < C; ++a) {
        const double *ka = kdw + (size_t)a * 9;
        double dk[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
        for (int n = 0; n < N; ++n) {
            const double *xi = x + ((size_t)n * C + a) * H * W;
            const double *go = dz + ((size_t)n * C + a) * Ho * Wo;
            double *gi = dx + ((size_t)n * C + a) * H * W;
            for (int e = 0; e < H * W; ++e) gi[e] = 0.0;
            for (int m = 0; m < Ho; ++m) {
                for (int q = 0; q < Wo; ++q) {
                    for (int i = 0; i < 3; ++i) {
                        for (int j = 0; j < 3; ++j) {
                            int r = stride * m + i - 1, c = stride * q + j - 1;
                            if (r < 0 || r >= H || c < 0 || c >= W) continue;
                            gi[(size_t)r * W + c] += ka[i * 3 + j] * go[(size_t)m * Wo + q];
                            dk[i * 3 + j] += go[(size_t)m * Wo + q] * xi[(size_t)r * W + c];
                        }
                    }
                }
            }
        }
        for (int t = 0; t < 9; ++t) dkdw[(size_t)a * 9 + t] = dk[t];
    }
    return 0;
}
