/*
 * CPU oracle for the masked-binary U-Net inference path (MBU-Net, Sec. 3.1.1 layer
 * definition, Sec. 3.2.2 / Algorithm 1 for the layer's steps, Sec. 4.1 for the
 * full-precision first and last layers).
 *
 * THIS IS TEST INFRASTRUCTURE, not the product.  It is the plain definition of each
 * operation written out on UNPACKED values (int8 activations in {-1,+1}, int8
 * weights in {-1,0,+1}), with direct loops, int32 accumulation, no bit tricks, no
 * blocking, no fusion.  It shares no code, headers, tables or helpers with the HIP
 * library; only tests, the smoke check and the benchmark's cpu_baseline leg use it.
 *
 * Layouts: activations NHWC, conv weights OHWI = [Cout][3][3][Cin], images and
 * logits NCHW (float).  The OpenMP pragma only spreads independent output rows over
 * host cores; it does not change any arithmetic.
 *
 * Every function here is pinned by tests/test_oracle_*.py against brute force,
 * closed forms, invariants and PyTorch-CPU float64 library routines; nothing is
 * "parity unpinned" except the architectural readings listed in the design notes
 * (concat order, decoder channel plan), which are definitions rather than results.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

/* Masked layer (Sec. 3.1.1): ternary weights, binary input features.  One output is
 * the plain dot product over the 3x3 window and all input channels; taps that fall
 * outside the image contribute nothing (zero padding in the value domain, i.e. a
 * padded tap behaves like a masked weight).  Cross-correlation orientation: tap
 * (ky,kx) reads input pixel (y+ky-1, x+kx-1).  This is the quantity R of
 * Algorithm 1 (C_neg - C_pos) before thresholding. */
static int32_t conv_point(const int8_t *a, int H, int W, int Cin,
                          const int8_t *w, int n, int y, int x, int o)
{
    int32_t acc = 0;
    for (int ky = 0; ky < 3; ++ky) {
        int yy = y + ky - 1;
        if (yy < 0 || yy >= H) continue;
        for (int kx = 0; kx < 3; ++kx) {
            int xx = x + kx - 1;
            if (xx < 0 || xx >= W) continue;
            const int8_t *ap = a + (((size_t)n * H + yy) * W + xx) * Cin;
            const int8_t *wp = w + (((size_t)o * 3 + ky) * 3 + kx) * Cin;
            for (int c = 0; c < Cin; ++c)
                acc += (int32_t)wp[c] * (int32_t)ap[c];
        }
    }
    return acc;
}

void orc_conv3x3(const int8_t *a, int N, int H, int W, int Cin,
                 const int8_t *w, int Cout, int32_t *acc)
{
    long rows = (long)N * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (long r = 0; r < rows; ++r) {
        int n = (int)(r / H), y = (int)(r % H);
        for (int x = 0; x < W; ++x)
            for (int o = 0; o < Cout; ++o)
                acc[(((size_t)n * H + y) * W + x) * Cout + o] =
                    conv_point(a, H, W, Cin, w, n, y, x, o);
    }
}

/* Same definition evaluated only at K listed outputs; pts = K rows of (n,y,x,o).
 * Used to check full-size GPU results on samples. */
void orc_conv3x3_points(const int8_t *a, int N, int H, int W, int Cin,
                        const int8_t *w, int Cout,
                        const int32_t *pts, long K, int32_t *acc)
{
    (void)N; (void)Cout;
#pragma omp parallel for schedule(static)
    for (long k = 0; k < K; ++k)
        acc[k] = conv_point(a, H, W, Cin, w, pts[4 * k], pts[4 * k + 1],
                            pts[4 * k + 2], pts[4 * k + 3]);
}

/* Masked transposed convolution, kernel 2x2, stride 2 (the decoder's up-sampling layer,
 * Sec. 2.1; Sec. 3.2.2 says it is "performed similarly" to the convolution).  With
 * kernel = stride every output pixel receives exactly one tap:
 *   acc[n, 2y+dy, 2x+dx, o] = sum_c w[o][dy][dx][c] * a[n, y, x, c].
 * a is NHWC [N][H][W][Cin], w is [Cout][2][2][Cin], acc is NHWC [N][2H][2W][Cout]. */
void orc_tconv2x2(const int8_t *a, int N, int H, int W, int Cin,
                  const int8_t *w, int Cout, int32_t *acc)
{
    long rows = (long)N * H;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        int n = (int)(r / H), y = (int)(r % H);
        for (int x = 0; x < W; ++x) {
            const int8_t *ap = a + (((size_t)n * H + y) * W + x) * Cin;
            for (int dy = 0; dy < 2; ++dy)
                for (int dx = 0; dx < 2; ++dx)
                    for (int o = 0; o < Cout; ++o) {
                        const int8_t *wp = w + (((size_t)o * 2 + dy) * 2 + dx) * Cin;
                        int32_t s = 0;
                        for (int c = 0; c < Cin; ++c) s += (int32_t)wp[c] * (int32_t)ap[c];
                        acc[(((size_t)n * 2 * H + 2 * y + dy) * 2 * W + 2 * x + dx) * Cout + o] = s;
                    }
        }
    }
}

/* Algorithm 1, threshold step: output is +1 where R >= theta, else -1 (a tie
 * binarises to +1).  total = N*H*W*C values, channel fastest. */
void orc_threshold(const int32_t *acc, const int32_t *theta, long pixels, int C,
                   int8_t *out)
{
#pragma omp parallel for schedule(static)
    for (long p = 0; p < pixels; ++p)
        for (int o = 0; o < C; ++o)
            out[p * C + o] = acc[p * C + o] >= theta[o] ? 1 : -1;
}

/* 2x2 stride-2 max pooling on +-1 values (Sec. 3.2.2 calls it trivial).  The output has
 * floor(H/2) x floor(W/2) pixels: the last row / column of an odd-sized input belongs to no
 * window and is dropped (the paper's Carvana frames are 959 pixels wide, Appendix A.3). */
void orc_maxpool2x2(const int8_t *in, int N, int H, int W, int C, int8_t *out)
{
    int Ho = H / 2, Wo = W / 2;
    for (int n = 0; n < N; ++n)
        for (int y = 0; y < Ho; ++y)
            for (int x = 0; x < Wo; ++x)
                for (int c = 0; c < C; ++c) {
                    int8_t m = -1;
                    for (int dy = 0; dy < 2; ++dy)
                        for (int dx = 0; dx < 2; ++dx) {
                            int8_t v = in[(((size_t)n * H + 2 * y + dy) * W + 2 * x + dx) * C + c];
                            if (v > m) m = v;
                        }
                    out[(((size_t)n * Ho + y) * Wo + x) * C + c] = m;
                }
}

/* 2x nearest-neighbour up-sampling: out[y][x] = in[y/2][x/2]. */
void orc_upsample2x(const int8_t *in, int N, int H, int W, int C, int8_t *out)
{
    int Ho = 2 * H, Wo = 2 * W;
    for (int n = 0; n < N; ++n)
        for (int y = 0; y < Ho; ++y)
            for (int x = 0; x < Wo; ++x)
                for (int c = 0; c < C; ++c)
                    out[(((size_t)n * Ho + y) * Wo + x) * C + c] =
                        in[(((size_t)n * H + y / 2) * W + x / 2) * C + c];
}

/* Zero padding of a feature map to a larger size (decoder of a U-Net on frames whose sizes
 * are not multiples of 2^levels, Appendix A.3: after floor pooling the up-sampled tensor is
 * smaller than the encoder feature it is concatenated with, and is padded to that size
 * first).  out[n][y+top][x+left][c] = in[n][y][x][c]; every other element of out is 0, a
 * value that contributes nothing to the layer that follows.  in is [N][H][W][C], out is
 * [N][Ho][Wo][C] with Ho >= top + H and Wo >= left + W. */
void orc_zero_pad(const int8_t *in, int N, int H, int W, int C, int top, int left,
                  int Ho, int Wo, int8_t *out)
{
    for (int n = 0; n < N; ++n)
        for (int y = 0; y < Ho; ++y)
            for (int x = 0; x < Wo; ++x) {
                int yi = y - top, xi = x - left;
                int inside = yi >= 0 && yi < H && xi >= 0 && xi < W;
                for (int c = 0; c < C; ++c)
                    out[(((size_t)n * Ho + y) * Wo + x) * C + c] =
                        inside ? in[(((size_t)n * H + yi) * W + xi) * C + c] : 0;
            }
}

/* Skip concatenation (Sec. 2.1): channels of a first, then channels of b. */
void orc_concat(const int8_t *a, int Ca, const int8_t *b, int Cb, long pixels,
                int8_t *out)
{
    for (long p = 0; p < pixels; ++p) {
        for (int c = 0; c < Ca; ++c) out[p * (Ca + Cb) + c] = a[p * Ca + c];
        for (int c = 0; c < Cb; ++c) out[p * (Ca + Cb) + Ca + c] = b[p * Cb + c];
    }
}

/* Full-precision first layer (Sec. 4.1): 3x3 convolution, zero padding, no bias,
 * float32.  The sum runs in the fixed order ky -> kx -> ci, starting from 0.0f,
 * one correctly rounded fused multiply-add per term, so that the sign that feeds
 * the binary layers is defined exactly.  img is NCHW [N][Ci][H][W]; w is
 * [Co][3][3][Ci]; pre is NHWC [N][H][W][Co]; sgn = +1 where pre >= 0, else -1. */
void orc_stem(const float *img, int N, int Ci, int H, int W,
              const float *w, int Co, float *pre, int8_t *sgn)
{
    long rows = (long)N * H;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        int n = (int)(r / H), y = (int)(r % H);
        for (int x = 0; x < W; ++x)
            for (int o = 0; o < Co; ++o) {
                float s = 0.0f;
                for (int ky = 0; ky < 3; ++ky) {
                    int yy = y + ky - 1;
                    for (int kx = 0; kx < 3; ++kx) {
                        int xx = x + kx - 1;
                        if (yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
                        for (int ci = 0; ci < Ci; ++ci)
                            s = fmaf(w[(((size_t)o * 3 + ky) * 3 + kx) * Ci + ci],
                                     img[(((size_t)n * Ci + ci) * H + yy) * W + xx], s);
                    }
                }
                size_t idx = (((size_t)n * H + y) * W + x) * Co + o;
                if (pre) pre[idx] = s;
                sgn[idx] = s >= 0.0f ? 1 : -1;
            }
    }
}

/* Full-precision last layer (Sec. 4.1): 1x1 convolution on +-1 features, float32,
 * logit = b[k] + sum_c w[k][c]*a[c], summed in channel order with one fused
 * multiply-add per term.  a is NHWC int8; out is NCHW [N][K][H][W]. */
void orc_classifier(const int8_t *a, int N, int H, int W, int C,
                    const float *w, const float *b, int K, float *out)
{
    long rows = (long)N * H;
#pragma omp parallel for schedule(static)
    for (long r = 0; r < rows; ++r) {
        int n = (int)(r / H), y = (int)(r % H);
        for (int x = 0; x < W; ++x) {
            const int8_t *ap = a + (((size_t)n * H + y) * W + x) * C;
            for (int k = 0; k < K; ++k) {
                float s = b[k];
                for (int c = 0; c < C; ++c)
                    s = fmaf(w[(size_t)k * C + c], (float)ap[c], s);
                out[(((size_t)n * K + k) * H + y) * W + x] = s;
            }
        }
    }
}
