// The two full-precision layers of the network (Sec. 4.1): the 3x3 stem that turns
// the float image into the first binary feature map, and the 1x1 classifier that
// turns the last binary feature map into float logits.
#include "mbu_internal.h"

namespace mbu {

// ---------------------------------------------------------------------------------
// Stem.  The sum over the 3x3xCi window runs in the fixed order ky -> kx -> ci from
// 0.0f with one fused multiply-add per term: the sign of the result feeds bit-exact
// layers, so the rounding sequence is part of the definition and the kernel is bound
// by the fp32 vector ALU (27*Co fused multiply-adds per pixel), not by memory.
// Padded taps read 0.0f, which leaves the running sum unchanged bit for bit.
//
// One thread owns two horizontally adjacent pixels; the weight of a term is
// wave-uniform, arrives through the scalar cache and feeds both pixels' chains.
// The output bit is the comparison "sum >= 0" itself (false for a NaN sum), shifted into
// the word one channel at a time.
template <int CI, bool WRITE_PRE>
__global__ __launch_bounds__(256) void stem_kernel(const float *__restrict__ img, int N, int H,
                                                   int W, const float *__restrict__ w, int Co,
                                                   uint32_t *__restrict__ out, float *__restrict__ pre)
{
    const int PW = (W + 1) >> 1;
    const long total = (long)N * H * PW;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int xp = (int)(idx % PW);
    const long q = idx / PW;
    const int y = (int)(q % H);
    const long n = q / H;
    const int x = 2 * xp;
    float in[3][4][CI];
#pragma unroll
    for (int ky = 0; ky < 3; ++ky)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int yy = y + ky - 1, xx = x + c - 1;
            const bool ok = yy >= 0 && yy < H && xx >= 0 && xx < W;
#pragma unroll
            for (int ci = 0; ci < CI; ++ci)
                in[ky][c][ci] = ok ? img[((n * CI + ci) * H + yy) * W + xx] : 0.0f;
        }
    const int Cow = Co >> 5;
    const size_t pix = ((size_t)n * H + y) * W + x;
    for (int k = 0; k < Cow; ++k) {
        uint32_t s0 = 0, s1 = 0;
#pragma unroll 2
        for (int b = 31; b >= 0; --b) {
            const float *wo = w + (size_t)(k * 32 + b) * 9 * CI;
            float a0 = 0.0f, a1 = 0.0f;
#pragma unroll
            for (int ky = 0; ky < 3; ++ky)
#pragma unroll
                for (int kx = 0; kx < 3; ++kx)
#pragma unroll
                    for (int ci = 0; ci < CI; ++ci) {
                        const float wv = wo[(ky * 3 + kx) * CI + ci];
                        a0 = __builtin_fmaf(wv, in[ky][kx][ci], a0);
                        a1 = __builtin_fmaf(wv, in[ky][kx + 1][ci], a1);
                    }
            s0 = (s0 << 1) | (a0 >= 0.0f ? 0u : 1u);
            s1 = (s1 << 1) | (a1 >= 0.0f ? 0u : 1u);
            if (WRITE_PRE) {
                pre[pix * Co + k * 32 + b] = a0;
                if (x + 1 < W) pre[(pix + 1) * Co + k * 32 + b] = a1;
            }
        }
        out[pix * Cow + k] = ~s0;
        if (x + 1 < W) out[(pix + 1) * Cow + k] = ~s1;
    }
}

int launch_stem_valu(const float *img, int N, int Ci, int H, int W, const float *w, int Co,
                     uint32_t *out_bits, float *out_pre, hipStream_t s)
{
    long total = (long)N * H * ((W + 1) / 2);
    unsigned blocks = (unsigned)((total + 255) / 256);
#define MBU_STEM_LAUNCH(CI, PRE) \
    MBU_LAUNCH((stem_kernel<CI, PRE>), dim3(blocks), dim3(256), 0, s, img, N, H, W, w, Co, out_bits, out_pre)
    if (Ci == 3) {
        if (out_pre) MBU_STEM_LAUNCH(3, true); else MBU_STEM_LAUNCH(3, false);
    } else if (Ci == 1) {
        if (out_pre) MBU_STEM_LAUNCH(1, true); else MBU_STEM_LAUNCH(1, false);
    } else {
        return fail(MBU_ERR_SHAPE, "stem supports 1 or 3 image channels, got %d", Ci);
    }
#undef MBU_STEM_LAUNCH
    return check_launch("stem");
}

// ---------------------------------------------------------------------------------
// Classifier: logit[k] = b[k] + sum_c w[k][c] * a_c, a_c = +-1 from the packed bits.
// The result only has to be accurate (not bit-reproducible), so the 1x1 convolution
// runs on the matrix cores as a (classes x channels) x (channels x pixels) product in
// bf16 with fp32 accumulation: +-1 is exact in bf16 and every fp32 weight is split
// into three bf16 terms hi + mid + lo (24 mantissa bits in total), so the products are
// exact and the only rounding is the fp32 accumulation.  The kernel is then bound by
// the NCHW logits it has to write.
//
// v_mfma_f32_32x32x16_bf16: rows = classes (padded to 32), columns = 32 consecutive
// pixels, 16 channels per instruction, 8 per lane half.  The channel order inside an
// instruction is free; it is chosen so that the two bf16 of a dword are channels p and
// p+16 of a packed word: (word << (15-p)) & 0x80008000 | 0x3f803f80 is then the pair
// (-a_p, -a_{p+16}), and the weights are stored negated to cancel the sign.
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

__device__ inline v8bf as_bf8(uint4 v) { return __builtin_bit_cast(v8bf, v); }

template <int CW>
__global__ __launch_bounds__(256) void classifier_kernel(const uint32_t *__restrict__ act,
                                                         long pixels, long HW,
                                                         const float *__restrict__ w,
                                                         const float *__restrict__ b, int K,
                                                         float *__restrict__ out)
{
    constexpr int C = 32 * CW;
    const int lane = threadIdx.x & 63;
    const int col = lane & 31, half = lane >> 5;
    const int row = col;  // class index of this lane in the weight operand

    // weight operand: instruction t = 2*wd + tp covers, in lane half h, dword d:
    // low bf16 = channel 32*wd + 8*tp + 4*h + d, high bf16 = that + 16
    uint4 wa[2 * CW][3];
#pragma unroll
    for (int t = 0; t < 2 * CW; ++t) {
        uint32_t parts[3][4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int clo = 32 * (t >> 1) + 8 * (t & 1) + 4 * half + d;
            float v[2];
            v[0] = row < K ? -w[(size_t)row * C + clo] : 0.0f;
            v[1] = row < K ? -w[(size_t)row * C + clo + 16] : 0.0f;
            uint32_t sp[2][3];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                float r = v[e];
#pragma unroll
                for (int j = 0; j < 3; ++j) {
                    const uint32_t top = __float_as_uint(r) & 0xffff0000u;  // truncated bf16
                    sp[e][j] = top;
                    r = r - __uint_as_float(top);                           // exact
                }
            }
#pragma unroll
            for (int j = 0; j < 3; ++j) parts[j][d] = (sp[0][j] >> 16) | sp[1][j];
        }
#pragma unroll
        for (int j = 0; j < 3; ++j)
            wa[t][j] = make_uint4(parts[j][0], parts[j][1], parts[j][2], parts[j][3]);
    }
    // accumulator register r of lane half h is class 8*(r/4) + 4*h + r%4
    float bias[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int cls = 8 * (r >> 2) + 4 * half + (r & 3);
        bias[r] = cls < K ? b[cls] : 0.0f;
    }
    const int sh = 4 - 4 * half;
    const long groups = (pixels + 31) / 32;
    const long wave_id = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const long n_waves = (long)gridDim.x * 4;
    // the packed words of the wave's next pixel group are fetched while the current group is
    // multiplied and stored
    auto fetch = [&](long g, uint32_t (&wd)[CW]) {
        const long pix = g * 32 + col;
        const long pc = pix < pixels ? pix : pixels - 1;
#pragma unroll
        for (int k = 0; k < CW; ++k) wd[k] = act[pc * CW + k];
    };
    uint32_t words[CW], next[CW];
    if (wave_id < groups) fetch(wave_id, words);
    for (long g = wave_id; g < groups; g += n_waves) {
        const long gn = g + n_waves < groups ? g + n_waves : g;
        fetch(gn, next);
        const long pix = g * 32 + col;
        const bool live = pix < pixels;
        v16f acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = bias[r];
#pragma unroll
        for (int t = 0; t < 2 * CW; ++t) {
            const uint32_t yv = words[t >> 1] << sh;
            uint4 bv;
            const int base = 11 - 8 * (t & 1);
            bv.x = ((yv << base) & 0x80008000u) | 0x3f803f80u;
            bv.y = ((yv << (base - 1)) & 0x80008000u) | 0x3f803f80u;
            bv.z = ((yv << (base - 2)) & 0x80008000u) | 0x3f803f80u;
            bv.w = ((yv << (base - 3)) & 0x80008000u) | 0x3f803f80u;
#pragma unroll
            for (int j = 0; j < 3; ++j)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf8(wa[t][j]), as_bf8(bv), acc, 0, 0, 0);
        }
        if (live) {
            const long n = pix / HW, rem = pix - n * HW;
            float *o = out + (size_t)n * K * HW + rem;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int cls = 8 * (r >> 2) + 4 * half + (r & 3);
                // written once, never read by this library: keep it out of the caches
                if (cls < K) __builtin_nontemporal_store(acc[r], o + (size_t)cls * HW);
            }
        }
#pragma unroll
        for (int k = 0; k < CW; ++k) words[k] = next[k];
    }
}

int launch_classifier(const uint32_t *act, int N, int H, int W, int C, const float *w,
                      const float *b, int K, float *out, hipStream_t s)
{
    long HW = (long)H * W, pixels = (long)N * HW;
    if (K > 32) return fail(MBU_ERR_SHAPE, "classifier supports at most 32 classes, got %d", K);
    long groups = (pixels + 31) / 32;
    // enough waves to fill the chip, several pixel groups per wave to amortise the weights
    unsigned blocks = (unsigned)min((groups + 3) / 4, (long)2048);
    switch (C / 32) {
    case 1: MBU_LAUNCH(classifier_kernel<1>, dim3(blocks), dim3(256), 0, s, act, pixels, HW, w, b, K, out); break;
    case 2: MBU_LAUNCH(classifier_kernel<2>, dim3(blocks), dim3(256), 0, s, act, pixels, HW, w, b, K, out); break;
    case 4: MBU_LAUNCH(classifier_kernel<4>, dim3(blocks), dim3(256), 0, s, act, pixels, HW, w, b, K, out); break;
    default: return fail(MBU_ERR_SHAPE, "classifier supports 32, 64 or 128 input channels, got %d", C);
    }
    return check_launch("classifier");
}

}  // namespace mbu
