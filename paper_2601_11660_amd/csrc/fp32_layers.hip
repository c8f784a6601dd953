// The two full-precision layers of the network (Sec. 4.1): the 3x3 stem that turns
// the float image into the first binary feature map, and the 1x1 classifier that
// turns the last binary feature map into float logits.
#include "mbu_internal.h"

namespace mbu {

// Stem: one thread per pixel, all output channels.  The sum over the 3x3xCi window
// runs in the fixed order ky -> kx -> ci from 0.0f with one fused multiply-add per
// term: the sign of the result feeds bit-exact layers, so the rounding sequence is
// part of the definition.  Padded taps read 0.0f, which leaves the running sum
// unchanged bit for bit.  Weights are staged once per block in LDS and read as
// wave-uniform broadcasts.  bit = (sum >= 0).
template <int CI>
__global__ __launch_bounds__(256) void stem_kernel(const float *__restrict__ img, int N, int H,
                                                   int W, const float *__restrict__ w, int Co,
                                                   uint32_t *__restrict__ out)
{
    extern __shared__ float ws[];  // [Co][9*CI]
    for (int i = threadIdx.x; i < Co * 9 * CI; i += 256) ws[i] = w[i];
    __syncthreads();
    long pix = (long)blockIdx.x * 256 + threadIdx.x;
    long total = (long)N * H * W;
    if (pix >= total) return;
    int x = (int)(pix % W);
    long q = pix / W;
    int y = (int)(q % H);
    long n = q / H;
    float in[9 * CI];
#pragma unroll
    for (int ky = 0; ky < 3; ++ky)
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) {
            int yy = y + ky - 1, xx = x + kx - 1;
            bool ok = yy >= 0 && yy < H && xx >= 0 && xx < W;
#pragma unroll
            for (int ci = 0; ci < CI; ++ci)
                in[(ky * 3 + kx) * CI + ci] =
                    ok ? img[((n * CI + ci) * H + yy) * W + xx] : 0.0f;
        }
    int Cow = Co >> 5;
    for (int k = 0; k < Cow; ++k) {
        uint32_t word = 0;
        for (int b = 0; b < 32; ++b) {
            const float *wo = ws + (k * 32 + b) * 9 * CI;
            float s = 0.0f;
#pragma unroll
            for (int t = 0; t < 9 * CI; ++t) s = __builtin_fmaf(wo[t], in[t], s);
            word |= (uint32_t)(s >= 0.0f) << b;
        }
        out[pix * Cow + k] = word;
    }
}

int launch_stem(const float *img, int N, int Ci, int H, int W, const float *w, int Co,
                uint32_t *out_bits, hipStream_t s)
{
    long total = (long)N * H * W;
    unsigned blocks = (unsigned)((total + 255) / 256);
    size_t shmem = (size_t)Co * 9 * Ci * sizeof(float);
    if (Ci == 3)
        MBU_LAUNCH(stem_kernel<3>, dim3(blocks), dim3(256), shmem, s, img, N, H, W, w, Co,
                           out_bits);
    else if (Ci == 1)
        MBU_LAUNCH(stem_kernel<1>, dim3(blocks), dim3(256), shmem, s, img, N, H, W, w, Co,
                           out_bits);
    else
        return fail(MBU_ERR_SHAPE, "stem supports 1 or 3 image channels, got %d", Ci);
    return check_launch("stem");
}

// Classifier: one thread per pixel; logit_k = b_k + sum_c w[k][c] * a_c with a_c = +-1
// taken from the packed bits, accumulated in channel order with fused multiply-adds.
// Output is NCHW, so consecutive threads (consecutive x) write consecutive floats of
// one class plane.  CW = packed words per pixel (C = 32*CW).
template <int CW>
__global__ __launch_bounds__(256) void classifier_kernel(const uint32_t *__restrict__ act, int N,
                                                         int H, int W, const float *__restrict__ w,
                                                         const float *__restrict__ b, int K,
                                                         float *__restrict__ out)
{
    extern __shared__ float ws[];  // [K][32*CW] then [K] bias
    const int C = 32 * CW;
    for (int i = threadIdx.x; i < K * C; i += 256) ws[i] = w[i];
    for (int i = threadIdx.x; i < K; i += 256) ws[K * C + i] = b[i];
    __syncthreads();
    long pix = (long)blockIdx.x * 256 + threadIdx.x;
    long HW = (long)H * W;
    long total = (long)N * HW;
    if (pix >= total) return;
    long n = pix / HW, rem = pix - n * HW;
    float a[32 * CW];
#pragma unroll
    for (int k = 0; k < CW; ++k) {
        uint32_t word = act[pix * CW + k];
#pragma unroll
        for (int i = 0; i < 32; ++i) a[k * 32 + i] = ((word >> i) & 1u) ? 1.0f : -1.0f;
    }
    for (int k = 0; k < K; ++k) {
        float s = ws[K * C + k];
        const float *wk = ws + k * C;
#pragma unroll
        for (int c = 0; c < C; ++c) s = __builtin_fmaf(wk[c], a[c], s);
        out[(n * K + k) * HW + rem] = s;
    }
}

int launch_classifier(const uint32_t *act, int N, int H, int W, int C, const float *w,
                      const float *b, int K, float *out, hipStream_t s)
{
    long total = (long)N * H * W;
    unsigned blocks = (unsigned)((total + 255) / 256);
    size_t shmem = ((size_t)K * C + K) * sizeof(float);
    if (shmem > 60000) return fail(MBU_ERR_SHAPE, "classifier weights do not fit in LDS");
    switch (C / 32) {
    case 1: MBU_LAUNCH(classifier_kernel<1>, dim3(blocks), dim3(256), shmem, s, act, N, H, W, w, b, K, out); break;
    case 2: MBU_LAUNCH(classifier_kernel<2>, dim3(blocks), dim3(256), shmem, s, act, N, H, W, w, b, K, out); break;
    case 4: MBU_LAUNCH(classifier_kernel<4>, dim3(blocks), dim3(256), shmem, s, act, N, H, W, w, b, K, out); break;
    default: return fail(MBU_ERR_SHAPE, "classifier supports 32, 64 or 128 input channels, got %d", C);
    }
    return check_launch("classifier");
}

}  // namespace mbu
