// Bit-packing kernels: activations (Sec. 1 / Algorithm 1 fragments) and the
// subtractive two-plane weight encoding (Sec. 3.2.1, b = b_pos - b_neg).
#include "mbu_internal.h"

namespace mbu {

// One thread produces one output word from up to 32 consecutive channel values.
template <typename T>
__global__ __launch_bounds__(256) void pack_act_kernel(const T *__restrict__ src, long pixels,
                                                       int C, int Cw, uint32_t *__restrict__ dst)
{
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    long total = pixels * Cw;
    if (idx >= total) return;
    long p = idx / Cw;
    int k = (int)(idx - p * Cw);
    const T *s = src + p * C + (long)k * 32;
    int n = min(32, C - k * 32);
    uint32_t word = 0;
    if (n == 32 && sizeof(T) == 1 && (C & 15) == 0) {
        const uint4 *v = reinterpret_cast<const uint4 *>(s);
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            uint4 x = v[q];
            uint32_t d[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    int8_t val = (int8_t)((d[j] >> (8 * b)) & 0xff);
                    word |= (uint32_t)(val > 0) << (q * 16 + j * 4 + b);
                }
        }
    } else if (n == 32 && sizeof(T) == 4 && (C & 3) == 0) {
        const float4 *v = reinterpret_cast<const float4 *>(s);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            float4 x = v[q];
            word |= (uint32_t)(x.x >= 0.0f) << (4 * q);
            word |= (uint32_t)(x.y >= 0.0f) << (4 * q + 1);
            word |= (uint32_t)(x.z >= 0.0f) << (4 * q + 2);
            word |= (uint32_t)(x.w >= 0.0f) << (4 * q + 3);
        }
    } else {
        for (int i = 0; i < n; ++i) {
            bool plus = sizeof(T) == 1 ? ((float)s[i] > 0.0f) : ((float)s[i] >= 0.0f);
            word |= (uint32_t)plus << i;
        }
    }
    dst[idx] = word;
}

int launch_pack_act(const void *src, int dtype, long pixels, int C, uint32_t *dst, hipStream_t s)
{
    int Cw = ceil_div(C, 32);
    long total = pixels * Cw;
    if (total == 0) return MBU_OK;
    unsigned blocks = (unsigned)((total + 255) / 256);
    if (dtype == 0)
        MBU_LAUNCH(pack_act_kernel<int8_t>, dim3(blocks), dim3(256), 0, s,
                           (const int8_t *)src, pixels, C, Cw, dst);
    else
        MBU_LAUNCH(pack_act_kernel<float>, dim3(blocks), dim3(256), 0, s,
                           (const float *)src, pixels, C, Cw, dst);
    return check_launch("pack_act");
}

// ---------------------------------------------------------------------------------
// Weights.  Thread (o, tap, word k) reads up to 32 ternary values and writes
//   * bit k of the positive and negative planes (vector-ALU section), and
//   * the 16-byte matrix-core fragment: 32 four-bit codes.  Code nibble q of dword d
//     carries input channel 32k + 4q + d (so that activations can be expanded with one
//     shift and one and-or per dword).  The code is the E2M1 value of w: 0x0 for a
//     masked weight, 0x2 (+1.0) for w = +1, 0xA (-1.0) for w = -1.
// Channels beyond cin and output channels beyond cout are packed as masked.
__global__ __launch_bounds__(256) void pack_weights_kernel(const int8_t *__restrict__ w,
                                                           BlobLayout L, uint8_t *__restrict__ blob)
{
    int words_m = 2 * L.ksteps;  // words per tap in the matrix section (>= cin_words)
    long total = (long)L.cout_pad64 * 9 * words_m;
    long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    int k = (int)(idx % words_m);
    int tap = (int)((idx / words_m) % 9);
    int o = (int)(idx / (9L * words_m));
    uint32_t pos = 0, neg = 0;
    if (o < L.cout && k < L.cin_words) {
        const int8_t *src = w + ((long)o * 9 + tap) * L.cin + (long)k * 32;
        int n = min(32, L.cin - k * 32);
        for (int i = 0; i < n; ++i) {
            int v = src[i];
            pos |= (uint32_t)(v > 0) << i;
            neg |= (uint32_t)(v < 0) << i;
        }
    }
    if (k < L.cin_words && (L.sections & MBU_BLOB_BIT_PLANES)) {
        uint32_t *P = reinterpret_cast<uint32_t *>(blob + L.off_pos);
        uint32_t *G = reinterpret_cast<uint32_t *>(blob + L.off_neg);
        size_t at = ((size_t)tap * L.cin_words + k) * L.cout_pad64 + o;
        P[at] = pos;
        G[at] = neg;
    }
    if (o < L.cout_tiles32 * 32) {
        uint32_t d[4];
#pragma unroll
        for (int dd = 0; dd < 4; ++dd) {
            uint32_t v = 0;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                int bit = 4 * q + dd;
                uint32_t code = ((pos >> bit) & 1u) ? 0x2u : (((neg >> bit) & 1u) ? 0xAu : 0x0u);
                v |= code << (4 * q);
            }
            d[dd] = v;
        }
        int tile64 = o >> 6, m = (o >> 5) & 1;
        int row = tile_channel_to_row(o & 31);
        int kstep = k >> 1, half = k & 1;
        int lane = half * 32 + row;
        uint4 *F = reinterpret_cast<uint4 *>(blob + L.off_f4);
        size_t at = ((((size_t)tile64 * L.ksteps + kstep) * 9 + tap) * 2 + m) * 64 + lane;
        F[at] = make_uint4(d[0], d[1], d[2], d[3]);
    }
}

// Kept-weight counts per (tap, output channel), their total, and the sum of the weights of
// an output channel (row 10; the matrix path's activations are 0 / 1, see conv_mfma.hip).
// One wave per output channel: the lanes stride over the input channels of a tap.
__global__ __launch_bounds__(256) void count_kept_kernel(const int8_t *__restrict__ w, BlobLayout L,
                                                         uint8_t *__restrict__ blob)
{
    const int o = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (o >= L.cout_pad64) return;
    int32_t *cnt = reinterpret_cast<int32_t *>(blob + L.off_cnt);
    int total = 0, wsum = 0;
    for (int tap = 0; tap < 9; ++tap) {
        int c = 0, sgn = 0;
        if (o < L.cout) {
            const int8_t *src = w + ((long)o * 9 + tap) * L.cin;
            for (int i = lane; i < L.cin; i += 64) {
                const int v = src[i];
                c += v != 0;
                sgn += (v > 0) - (v < 0);
            }
        }
        for (int off = 32; off > 0; off >>= 1) {
            c += __shfl_xor(c, off);
            sgn += __shfl_xor(sgn, off);
        }
        wsum += sgn;
        if (lane == 0) cnt[(size_t)tap * L.cout_pad64 + o] = c;
        total += c;
    }
    if (lane != 0) return;
    cnt[(size_t)9 * L.cout_pad64 + o] = total;
    cnt[(size_t)10 * L.cout_pad64 + o] = wsum;
}

int launch_pack_weights(const int8_t *w, const BlobLayout &L, void *blob, hipStream_t s)
{
    long total = (long)L.cout_pad64 * 9 * 2 * L.ksteps;
    unsigned blocks = (unsigned)((total + 255) / 256);
    MBU_LAUNCH(pack_weights_kernel, dim3(blocks), dim3(256), 0, s, w, L, (uint8_t *)blob);
    int rc = check_launch("pack_weights");
    if (rc) return rc;
    MBU_LAUNCH(count_kept_kernel, dim3(ceil_div(L.cout_pad64, 4)), dim3(256), 0, s, w, L,
                       (uint8_t *)blob);
    rc = check_launch("count_kept");
    if (rc || !(L.sections & MBU_BLOB_SUMMED_TAPS)) return rc;
    return launch_pack_upcat(w, L, blob, s);
}

}  // namespace mbu
