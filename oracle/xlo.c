/*
 * xlo -- CPU oracle for cross-layer fused CNN blocks.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition of every layer the fused GPU path
 * computes.  It exists so that tests, the smoke check and the benchmark's
 * cpu_baseline leg have something independent to compare against.  Nothing in
 * the product path may call, link or import it, and it shares no code, header,
 * table or helper with the HIP library.
 *
 * What it follows.  Layer fusion changes where intermediates live (on-chip
 * instead of global memory: paper section 2.2, Fig. 3), never what is
 * computed, so the reference result of a fused block is the plain layer-by-layer
 * result with full intermediates.  The layer vocabulary is the paper's
 * (section 2.2: convolution, pooling, activation, element-wise add, concat);
 * tensor and filter notation follows section 4.1: tensors [C,H,W] per image,
 * filters [Cout, Cin/groups, KH, KW] / pad, stride, group.
 *
 * Readings where the paper is silent:
 *   - "convolution" is cross-correlation (no filter flip), the convention of
 *     the Caffe networks the paper takes as input (section 4).
 *   - zero padding for convolution (section 3.3, padding strategy: the margin
 *     holds extra data so the next layer needs no branches -- that data is 0);
 *     max pooling ignores out-of-image taps.
 *   - output size floor((H + 2p - k)/s) + 1.
 *   - folded batch-norm is a per-output-channel y*scale + shift applied to the
 *     bias-free convolution sum; a plain bias is scale = 1, shift = bias.
 *
 * Precision: every sum is accumulated in double and rounded to float once per
 * layer output, so each stored intermediate is a float, as it is in the fused
 * kernel's on-chip copy.
 *
 * Parallelism: OpenMP over (image, output channel) only.  No blocking, no
 * vector intrinsics, no reordering of the definition.
 *
 * Pins (tests/test_oracle_*.py): sliding-window brute force in NumPy, 1x1 conv
 * == matmul, delta/identity filters, all-ones closed forms (one and two stacked
 * layers), linearity, batch independence, torch CPU conv2d/max_pool2d in
 * float64, pooling pad equivalence on non-negative input, mean of constants.
 */
#include <float.h>
#include <stddef.h>
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Number of threads the parallel loops use (1 when built without OpenMP). */
int xlo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void xlo_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/*
 * y[n,o,i,j] = act( scale[o] * sum_{c,u,v} x[n, g*cg + c, i*s - p + u, j*s - p + v] * w[o,c,u,v] + shift[o] )
 * with g = o / (Cout/groups), cg = Cin/groups, x = 0 outside the image
 * (paper section 3.2: one output pixel depends on all input channels inside
 * the filter window; section 4.1 filter notation).
 * scale == NULL means 1, shift == NULL means 0.  Returns 0, or -1 on bad sizes.
 */
int xlo_conv2d(const float *x, int N, int C, int H, int W,
               const float *w, int O, int kh, int kw, int stride, int pad, int groups,
               const float *scale, const float *shift, int relu, float *y)
{
    if (N < 0 || C <= 0 || O <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0 || groups <= 0) return -1;
    if (C % groups || O % groups) return -1;
    if (H + 2 * pad < kh || W + 2 * pad < kw) return -1;
    const int Ho = (H + 2 * pad - kh) / stride + 1;
    const int Wo = (W + 2 * pad - kw) / stride + 1;
    const int cg = C / groups;
    const int og = O / groups;
    const long long NO = (long long)N * O;
#pragma omp parallel for schedule(static)
    for (long long no = 0; no < NO; ++no) {
        const int n = (int)(no / O);
        const int o = (int)(no % O);
        const int g = o / og;
        const double sc = scale ? (double)scale[o] : 1.0;
        const double sh = shift ? (double)shift[o] : 0.0;
        for (int i = 0; i < Ho; ++i) {
            for (int j = 0; j < Wo; ++j) {
                double acc = 0.0;
                for (int c = 0; c < cg; ++c) {
                    const float *xc = x + ((size_t)n * C + (size_t)g * cg + c) * H * W;
                    const float *wc = w + ((size_t)o * cg + c) * kh * kw;
                    for (int u = 0; u < kh; ++u) {
                        const int yy = i * stride - pad + u;
                        if (yy < 0 || yy >= H) continue;
                        for (int v = 0; v < kw; ++v) {
                            const int xx = j * stride - pad + v;
                            if (xx < 0 || xx >= W) continue;
                            acc += (double)xc[(size_t)yy * W + xx] * (double)wc[u * kw + v];
                        }
                    }
                }
                double z = acc * sc + sh;
                if (relu && z < 0.0) z = 0.0;
                y[(((size_t)n * O + o) * Ho + i) * Wo + j] = (float)z;
            }
        }
    }
    return 0;
}

/* Max over the in-image taps of a k x k window (out-of-image taps ignored). */
int xlo_maxpool2d(const float *x, int N, int C, int H, int W, int k, int stride, int pad, float *y)
{
    if (k <= 0 || stride <= 0 || pad < 0 || pad >= k || H + 2 * pad < k || W + 2 * pad < k) return -1;
    const int Ho = (H + 2 * pad - k) / stride + 1;
    const int Wo = (W + 2 * pad - k) / stride + 1;
    const long long NC = (long long)N * C;
#pragma omp parallel for schedule(static)
    for (long long nc = 0; nc < NC; ++nc) {
        const float *xc = x + (size_t)nc * H * W;
        float *yc = y + (size_t)nc * Ho * Wo;
        for (int i = 0; i < Ho; ++i) {
            for (int j = 0; j < Wo; ++j) {
                float m = -FLT_MAX;
                for (int u = 0; u < k; ++u) {
                    const int yy = i * stride - pad + u;
                    if (yy < 0 || yy >= H) continue;
                    for (int v = 0; v < k; ++v) {
                        const int xx = j * stride - pad + v;
                        if (xx < 0 || xx >= W) continue;
                        const float t = xc[(size_t)yy * W + xx];
                        if (t > m) m = t;
                    }
                }
                yc[(size_t)i * Wo + j] = m;
            }
        }
    }
    return 0;
}

/* y[n,c] = mean over H*W of x[n,c,:,:], summed in double. */
int xlo_global_avgpool(const float *x, int N, int C, int H, int W, float *y)
{
    if (H <= 0 || W <= 0) return -1;
    const long long NC = (long long)N * C;
    const size_t hw = (size_t)H * W;
#pragma omp parallel for schedule(static)
    for (long long nc = 0; nc < NC; ++nc) {
        double s = 0.0;
        const float *xc = x + (size_t)nc * hw;
        for (size_t t = 0; t < hw; ++t) s += (double)xc[t];
        y[nc] = (float)(s / (double)hw);
    }
    return 0;
}

/* y = act(a + b), element-wise (merge mode's add, paper section 3.1 Fig. 5b). */
int xlo_add(const float *a, const float *b, long long count, int relu, float *y)
{
#pragma omp parallel for schedule(static)
    for (long long t = 0; t < count; ++t) {
        double z = (double)a[t] + (double)b[t];
        if (relu && z < 0.0) z = 0.0;
        y[t] = (float)z;
    }
    return 0;
}

/* y[n, 0:Ca] = a[n], y[n, Ca:Ca+Cb] = b[n]  (split mode's channel concatenation). */
int xlo_concat_channels(const float *a, int Ca, const float *b, int Cb, int N, long long hw, float *y)
{
    for (int n = 0; n < N; ++n) {
        float *yn = y + (size_t)n * (Ca + Cb) * hw;
        const float *an = a + (size_t)n * Ca * hw;
        const float *bn = b + (size_t)n * Cb * hw;
        for (long long t = 0; t < (long long)Ca * hw; ++t) yn[t] = an[t];
        for (long long t = 0; t < (long long)Cb * hw; ++t) yn[(size_t)Ca * hw + t] = bn[t];
    }
    return 0;
}
