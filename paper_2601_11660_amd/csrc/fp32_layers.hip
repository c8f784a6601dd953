// The two full-precision layers of the network (Sec. 4.1): the 3x3 stem that turns
// the float image into the first binary feature map, and the 1x1 classifier that
// turns the last binary feature map into float logits.
#include "mbu_internal.h"
#include <algorithm>

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
// fp16 with fp32 accumulation: +-1 is exact in fp16; every class row of the weights is
// scaled by a power of two into [0.5, 1) and split into two fp16 terms hi + lo (22
// significand bits), so the products are exact and the only rounding is the fp32
// accumulation; the scale is undone, and the bias added, by one fused multiply-add per
// logit.  The kernel is then bound by the NCHW logits it has to write.
//
// v_mfma_f32_32x32x16_f16: rows = classes (padded to 32), columns = 32 consecutive
// pixels, 16 channels per instruction, 8 per lane half.  The channel order inside an
// instruction is free; it is chosen so that the two fp16 of a dword are channels p and
// p+16 of a packed word: (word << (15-p)) & 0x80008000 | 0x3c003c00 is then the pair
// (-a_p, -a_{p+16}), and the weights are stored negated to cancel the sign.
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

__device__ inline v8h as_h8(uint4 v) { return __builtin_bit_cast(v8h, v); }

__device__ inline uint32_t f16_pair(float lo, float hi)
{
    const _Float16 a = (_Float16)lo, b = (_Float16)hi;   // round to nearest even
    return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
}

template <int CW>
__global__ __launch_bounds__(256, CW == 4 ? 2 : 3) void classifier_kernel(const uint32_t *__restrict__ act,
                                                         long pixels, long HW,
                                                         const float *__restrict__ w,
                                                         const float *__restrict__ b, int K,
                                                         float *__restrict__ out)
{
    constexpr int C = 32 * CW;
    constexpr int G = 2;          // pixel groups per iteration: independent accumulator chains
    const int lane = threadIdx.x & 63;
    const int col = lane & 31, half = lane >> 5;
    const int row = col;  // class index of this lane in the weight operand
    const size_t rbase = (size_t)(row < K ? row : 0) * C;   // loads are unconditional (clamped row)

    // power-of-two scale of this lane's class row: largest |weight| into [0.5, 1)
    float mx = 0.0f;
#pragma unroll 8
    for (int c = 0; c < C; ++c) mx = fmaxf(mx, fabsf(w[rbase + c]));
    int e = 0;
    if (mx > 0.0f && mx < __builtin_inff()) (void)frexpf(mx, &e);
    const float scale = ldexpf(1.0f, -e);

    // weight operand: instruction t = 2*wd + tp covers, in lane half h, dword d:
    // low fp16 = channel 32*wd + 8*tp + 4*h + d, high fp16 = that + 16
    uint4 wa[2 * CW][2];
#pragma unroll
    for (int t = 0; t < 2 * CW; ++t) {
        uint32_t hi4[4], lo4[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            const int clo = 32 * (t >> 1) + 8 * (t & 1) + 4 * half + d;
            const float w0 = w[rbase + clo], w1 = w[rbase + clo + 16];
            const float v0 = row < K ? -w0 * scale : 0.0f;   // exact scaling
            const float v1 = row < K ? -w1 * scale : 0.0f;
            const _Float16 h0 = (_Float16)v0, h1 = (_Float16)v1;
            hi4[d] = f16_pair(v0, v1);
            lo4[d] = f16_pair(v0 - (float)h0, v1 - (float)h1);
        }
        wa[t][0] = make_uint4(hi4[0], hi4[1], hi4[2], hi4[3]);
        wa[t][1] = make_uint4(lo4[0], lo4[1], lo4[2], lo4[3]);
    }
    // accumulator register r of lane half h is class 8*(r/4) + 4*h + r%4: its 1/scale and
    // bias come from the lane that holds that class row
    float mul[16], bias[16];
    const float inv = ldexpf(1.0f, e);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int cls = 8 * (r >> 2) + 4 * half + (r & 3);
        const float bv = b[cls < K ? cls : 0];
        bias[r] = cls < K ? bv : 0.0f;
        mul[r] = __shfl(inv, cls);
    }
    const int sh = 4 - 4 * half;
    const long groups = (pixels + 31) / 32;
    const long wave_id = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const long n_waves = (long)gridDim.x * 4;
    const long stride = n_waves * G;
    // The packed words of the wave's pixel groups are fetched two iterations ahead of their
    // use, so that the loads fly during the matrix instructions and the stores of two others.
    auto fetch = [&](long g0, uint32_t (&wd)[G][CW]) {
#pragma unroll
        for (int u = 0; u < G; ++u) {
            const long pix = (g0 + u) * 32 + col;
            const long pc = pix < pixels ? pix : pixels - 1;
#pragma unroll
            for (int k = 0; k < CW; ++k) wd[u][k] = act[pc * CW + k];
        }
    };
    uint32_t cur[G][CW], nx1[G][CW], nx2[G][CW];
    const long first = wave_id * G;
    if (first < groups) {
        fetch(first, cur);
        fetch(first + stride < groups ? first + stride : first, nx1);
    }
    for (long g0 = first; g0 < groups; g0 += stride) {
        const long g2 = g0 + 2 * stride < groups ? g0 + 2 * stride : g0;
        fetch(g2, nx2);
        v16f acc[G];
#pragma unroll
        for (int u = 0; u < G; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[u][r] = 0.0f;
#pragma unroll
        for (int t = 0; t < 2 * CW; ++t) {
            const int base = 11 - 8 * (t & 1);
#pragma unroll
            for (int u = 0; u < G; ++u) {
                const uint32_t yv = cur[u][t >> 1] << sh;
                uint4 bv;
                bv.x = ((yv << base) & 0x80008000u) | 0x3c003c00u;
                bv.y = ((yv << (base - 1)) & 0x80008000u) | 0x3c003c00u;
                bv.z = ((yv << (base - 2)) & 0x80008000u) | 0x3c003c00u;
                bv.w = ((yv << (base - 3)) & 0x80008000u) | 0x3c003c00u;
                acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_h8(wa[t][1]), as_h8(bv), acc[u], 0, 0, 0);
                acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_h8(wa[t][0]), as_h8(bv), acc[u], 0, 0, 0);
            }
        }
#pragma unroll
        for (int u = 0; u < G; ++u) {
            // Addressing with one wave-uniform base per class and one 32-bit offset per lane:
            // the image of the group's first pixel gives the base (scalar arithmetic); a lane
            // whose pixel lies in a later image adds whole images to its offset.
            const long gp = (g0 + u) * 32;                         // first pixel of the group
            if (gp >= pixels) break;
            const long n0 = gp / HW;
            const long rem0 = gp - n0 * HW;
            long rel = rem0 + col;                                  // pixel relative to image n0
            long off = rel;
            if (rem0 + 31 >= HW) {                                  // the group crosses an image border
                const long dn = rel / HW;
                off = dn * K * HW + (rel - dn * HW);
            }
            const bool live = gp + col < pixels;
            float *base = out + (size_t)n0 * K * HW;               // uniform
            const uint32_t lane_off = (uint32_t)(off + (long)(4 * half) * HW);   // class 4*half folded in
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (live && 8 * q + 4 * half < K) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int r = 4 * q + j;
                        // written once, never read by this library: keep it out of the caches
                        if (8 * q + 4 * half + j < K)
                            __builtin_nontemporal_store(__builtin_fmaf(acc[u][r], mul[r], bias[r]),
                                                        base + (size_t)(8 * q + j) * HW + lane_off);
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < G; ++u)
#pragma unroll
            for (int k = 0; k < CW; ++k) {
                cur[u][k] = nx1[u][k];
                nx1[u][k] = nx2[u][k];
            }
    }
}

// ---------------------------------------------------------------------------------
// Classifier for up to four classes (binary segmentation, the paper's tasks, Sec. 4.1): with so
// few outputs per pixel the matrix-core kernel above spends its time turning bits into fp16
// operands.  Here the block builds, once, a table per byte position of the packed words:
//   table[j][v][k] = sum_{i < 8} (bit i of v ? +w : -w)[k][8 j + i]          (float32, KP per entry)
// and a thread sums C / 8 table entries per pixel: logit[k] = b[k] + sum_j table[j][byte j][k].
// The partial sums are formed in another order than the channel-by-channel definition; the
// difference is a few float32 roundings (1e-7 relative), far inside the layer's 1e-4.
template <int KP>
__global__ __launch_bounds__(256) void classifier_lut_kernel(const uint32_t *__restrict__ act, long pixels,
                                                             long HW, int CW, const float *__restrict__ w,
                                                             const float *__restrict__ b, int K,
                                                             float *__restrict__ out)
{
    __shared__ float lut[16 * 256 * KP];
    const int nb = 4 * CW;            // byte positions
    {
        const int v = threadIdx.x;
        for (int j = 0; j < nb; ++j)
#pragma unroll
            for (int k = 0; k < KP; ++k) {
                float sum = 0.0f;
                if (k < K) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const float wv = w[(size_t)k * (32 * CW) + 8 * j + i];
                        sum += ((v >> i) & 1) ? wv : -wv;
                    }
                }
                lut[(j * 256 + v) * KP + k] = sum;
            }
    }
    float bias[KP];
#pragma unroll
    for (int k = 0; k < KP; ++k) bias[k] = k < K ? b[k] : 0.0f;
    __syncthreads();

    const long stride = (long)gridDim.x * 256;
    long p = (long)blockIdx.x * 256 + threadIdx.x;
    // (image, pixel inside the image) of p, advanced by the stride without divisions
    long n = p / HW, rem = p - n * HW;
    const long dn = stride / HW, dr = stride - dn * HW;
    for (; p < pixels; p += stride) {
        float acc[KP];
#pragma unroll
        for (int k = 0; k < KP; ++k) acc[k] = bias[k];
        for (int q = 0; q < CW; ++q) {
            const uint32_t word = act[p * CW + q];
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const float *e = lut + ((q * 4 + jj) * 256 + ((word >> (8 * jj)) & 255u)) * KP;
#pragma unroll
                for (int k = 0; k < KP; ++k) acc[k] += e[k];
            }
        }
        float *o = out + (size_t)n * K * HW + rem;
#pragma unroll
        for (int k = 0; k < KP; ++k)
            if (k < K) __builtin_nontemporal_store(acc[k], o + (size_t)k * HW);
        n += dn;
        rem += dr;
        if (rem >= HW) { rem -= HW; ++n; }
    }
}

int launch_classifier(const uint32_t *act, int N, int H, int W, int C, const float *w,
                      const float *b, int K, float *out, hipStream_t s)
{
    long HW = (long)H * W, pixels = (long)N * HW;
    if (K > 32) return fail(MBU_ERR_SHAPE, "classifier supports at most 32 classes, got %d", K);
    // a lane's offset from its group's image base must fit 32 bits
    if ((double)(K + 5) * (double)HW * 4.0 >= 4294967296.0)
        return fail(MBU_ERR_SHAPE, "classifier: image too large (%ld pixels, %d classes)", HW, K);
    if (K <= 4 && (C == 32 || C == 64 || C == 128)) {
        // few classes: table look-up, many pixels per thread so that building the table is amortised
        const unsigned blocks = (unsigned)std::max(1L, std::min((pixels + 2047) / 2048, 1024L));
        const int CW = C / 32;
        if (K == 1) MBU_LAUNCH(classifier_lut_kernel<1>, dim3(blocks), dim3(256), 0, s, act, pixels, HW, CW, w, b, K, out);
        else if (K == 2) MBU_LAUNCH(classifier_lut_kernel<2>, dim3(blocks), dim3(256), 0, s, act, pixels, HW, CW, w, b, K, out);
        else MBU_LAUNCH(classifier_lut_kernel<4>, dim3(blocks), dim3(256), 0, s, act, pixels, HW, CW, w, b, K, out);
        return check_launch("classifier");
    }
    long groups = (pixels + 31) / 32;
    // all waves resident at once, many pixel groups per wave to amortise splitting the weights.
    // Two blocks per compute unit: the kernel is bound by writing the logits, and measured on
    // MI355X (1x19x1024x2048) fewer concurrent writers sustain more of the HBM rate - 33.3 us with
    // 512 blocks against 37.6 (768), 41.5 (1024), 40.1 (384) and 48.8 (256).
    unsigned blocks = (unsigned)min((groups + 7) / 8, 512L);
    switch (C / 32) {
    case 1: MBU_LAUNCH(classifier_kernel<1>, dim3(blocks), dim3(256), 0, s, act, pixels, HW, w, b, K, out); break;
    case 2: MBU_LAUNCH(classifier_kernel<2>, dim3(blocks), dim3(256), 0, s, act, pixels, HW, w, b, K, out); break;
    case 4: MBU_LAUNCH(classifier_kernel<4>, dim3(blocks), dim3(256), 0, s, act, pixels, HW, w, b, K, out); break;
    default: return fail(MBU_ERR_SHAPE, "classifier supports 32, 64 or 128 input channels, got %d", C);
    }
    return check_launch("classifier");
}

}  // namespace mbu
