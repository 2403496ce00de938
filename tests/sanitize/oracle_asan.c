/* Runs every function of the CPU oracle (oracle/xlo.c, compiled into this program with
 * -fsanitize=address,undefined) on exactly-sized heap buffers, so that any read or write outside a
 * tensor, any signed overflow or misaligned access in the loop nests stops the run.  Shapes cover
 * padding, strides, groups, 1x1 / 3x3 / 5x5 windows, windows larger than the image interior, one-pixel
 * images and an empty batch.  Values are checked only loosely (all-ones closed forms); the pins of the
 * arithmetic are the Python tests. */
#include <stdio.h>
#include <stdlib.h>

int xlo_conv2d(const float *x, int N, int C, int H, int W, const float *w, int O, int kh, int kw, int stride, int pad,
               int groups, const float *scale, const float *shift, int relu, float *y);
int xlo_maxpool2d(const float *x, int N, int C, int H, int W, int k, int stride, int pad, float *y);
int xlo_global_avgpool(const float *x, int N, int C, int H, int W, float *y);
int xlo_add(const float *a, const float *b, long long count, int relu, float *y);
int xlo_concat_channels(const float *a, int Ca, const float *b, int Cb, int N, long long hw, float *y);

static float *ones(size_t n)
{
    float *p = (float *)malloc(n ? n * sizeof(float) : 1);
    for (size_t i = 0; i < n; ++i) p[i] = 1.0f;
    return p;
}

static int failures = 0;
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "line %d: %s\n", __LINE__, #c); ++failures; } } while (0)

static void conv_case(int N, int C, int H, int W, int O, int k, int s, int p, int g)
{
    const int Ho = (H + 2 * p - k) / s + 1, Wo = (W + 2 * p - k) / s + 1;
    float *x = ones((size_t)N * C * H * W), *w = ones((size_t)O * (C / g) * k * k), *sh = ones(O);
    float *y = ones((size_t)N * O * Ho * Wo);
    CHECK(xlo_conv2d(x, N, C, H, W, w, O, k, k, s, p, g, NULL, sh, 1, y) == 0);
    if (N > 0 && p == 0) CHECK(y[0] == (float)((C / g) * k * k + 1));      /* every tap inside the image, + shift */
    if (N > 0 && p > 0 && k == 2 * p + 1 && H > p && W > p)                 /* corner: (p+1)^2 taps inside */
        CHECK(y[0] == (float)((C / g) * (p + 1) * (p + 1) + 1));
    free(x); free(w); free(sh); free(y);
}

int main(void)
{
    conv_case(2, 3, 9, 11, 8, 3, 2, 0, 1);
    conv_case(1, 16, 7, 5, 4, 3, 1, 1, 1);
    conv_case(2, 6, 13, 10, 5, 5, 1, 2, 1);
    conv_case(1, 8, 6, 6, 8, 3, 1, 1, 8);       /* depthwise */
    conv_case(1, 8, 6, 6, 4, 3, 2, 1, 2);       /* grouped */
    conv_case(3, 5, 1, 1, 7, 1, 1, 0, 1);       /* one pixel */
    conv_case(1, 2, 2, 2, 3, 5, 1, 2, 1);       /* window wider than the image */
    conv_case(0, 4, 5, 5, 4, 3, 1, 1, 1);       /* empty batch */
    {
        float *x = ones(2 * 3 * 7 * 9), *y = ones(2 * 3 * 4 * 5);
        CHECK(xlo_maxpool2d(x, 2, 3, 7, 9, 3, 2, 1, y) == 0 && y[0] == 1.0f && y[2 * 3 * 4 * 5 - 1] == 1.0f);
        CHECK(xlo_maxpool2d(x, 2, 3, 7, 9, 3, 2, 3, y) == -1);
        free(x); free(y);
        x = ones(2 * 3 * 7 * 9); y = ones(2 * 3 * 3 * 4);
        CHECK(xlo_maxpool2d(x, 2, 3, 7, 9, 3, 2, 0, y) == 0);
        free(x); free(y);
    }
    {
        float *x = ones(2 * 5 * 13 * 13), *y = ones(10);
        CHECK(xlo_global_avgpool(x, 2, 5, 13, 13, y) == 0 && y[9] == 1.0f);
        free(x); free(y);
    }
    {
        float *a = ones(1001), *b = ones(1001), *y = ones(1001);
        CHECK(xlo_add(a, b, 1001, 1, y) == 0 && y[1000] == 2.0f);
        free(a); free(b); free(y);
    }
    {
        float *a = ones(2 * 3 * 35), *b = ones(2 * 5 * 35), *y = ones(2 * 8 * 35);
        CHECK(xlo_concat_channels(a, 3, b, 5, 2, 35, y) == 0 && y[2 * 8 * 35 - 1] == 1.0f);
        free(a); free(b); free(y);
    }
    printf("oracle sanitizer run: %d failures\n", failures);
    return failures ? 1 : 0;
}
