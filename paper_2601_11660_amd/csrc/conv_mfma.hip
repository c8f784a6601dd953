// Masked-binary 3x3 convolution on the matrix cores.
//
// CDNA4 has no 1-bit matrix instruction, but its 4-bit floating-point format (E2M1)
// represents -1, 0 and +1 exactly, products of such values are exact, and sums of up
// to 9*Cin <= 2^24 of them are exact in the fp32 accumulator - so the contraction
// R = sum w*a of Algorithm 1 can run on v_mfma_f32_32x32x64_f8f6f4 and still be the
// exact integer.  Masked weights and padded (out-of-image) activations are the code
// 0, which contributes nothing: no border correction is needed on this path.
//
// GEMM view per image: D[cout][pixel] = sum_{tap, cin} Wt[cout][tap, cin] * Act[tap, cin][pixel].
//   A operand (32 rows x 64 k)  = weights of 32 output channels, one tap, 64 input channels,
//                                 pre-arranged per lane by mbu_pack_weights;
//   B operand (64 k x 32 cols)  = 32 consecutive pixels of one image row, same tap/channels:
//                                 lane (col j, half h) supplies the 32 channels of packed
//                                 word h of that pixel, expanded from bits to nibbles;
//   D (32 x 32 fp32)            = lane (col j, half h), register r -> output channel 16h + r
//                                 of the tile (row order chosen at packing time).
// The bit->nibble expansion happens once per staged halo pixel when the block copies
// its (TH+2) x 34 pixel window of the current 64-channel step into LDS; the nine taps
// then read shifted windows of that tile.
#include "mbu_internal.h"

namespace mbu {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

__device__ inline v16f mfma_f4(v4i a, v4i b, v16f c)
{
    // The builtin takes 8-dword operands for every format; E2M1 (format code 4) uses the
    // low 4 dwords.  Zero scale arguments select the unscaled instruction.
    v8i a8 = {a.x, a.y, a.z, a.w, 0, 0, 0, 0};
    v8i b8 = {b.x, b.y, b.z, b.w, 0, 0, 0, 0};
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c, 4, 4, 0, 0, 0, 0);
}

// bits of one packed word -> 32 E2M1 codes of the NEGATED activation (bit 1 -> 0xA = -1.0,
// bit 0 -> 0x2 = +1.0); nibble q of dword d carries channel 4q + d.
__device__ inline uint4 expand_word(uint32_t w)
{
    uint4 r;
    r.x = ((w << 3) & 0x88888888u) | 0x22222222u;
    r.y = ((w << 2) & 0x88888888u) | 0x22222222u;
    r.z = ((w << 1) & 0x88888888u) | 0x22222222u;
    r.w = (w & 0x88888888u) | 0x22222222u;
    return r;
}

constexpr int TW = 32;            // pixels per matrix column tile (one image-row segment)
constexpr int HALO_W = TW + 2;

// Block = 4 waves; wave v owns image rows (2v, 2v+1) of an 8 x 32 pixel tile and
// 64 output channels: 2 x 2 accumulator tiles.
template <bool WRITE_ACC>
__global__ __launch_bounds__(256) void conv_mfma_kernel(
    const uint32_t *__restrict__ act, int N, int H, int W, int Cw, int ksteps,
    const uint4 *__restrict__ wfrag, int Cout, const int32_t *__restrict__ thresh,
    uint32_t *__restrict__ out_bits, int32_t *__restrict__ out_acc)
{
    constexpr int TH = 8;
    __shared__ uint4 tile[(TH + 2) * HALO_W * 2];  // [row][col][half] 16-byte fragments

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int tiles_x = (W + TW - 1) / TW;
    const int tiles_y = (H + TH - 1) / TH;
    int bid = blockIdx.x;
    const int tx = bid % tiles_x;
    bid /= tiles_x;
    const int ty = bid % tiles_y;
    const int n = bid / tiles_y;
    const int x0 = tx * TW, y0 = ty * TH;
    const int ct = blockIdx.y;  // 64-channel output tile

    v16f acc[2][2];
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[m][r][i] = 0.0f;

    const uint4 *wf0 = wfrag + ((size_t)(2 * ct) * 9 * ksteps) * 64 + lane;
    const uint4 *wf1 = wfrag + ((size_t)(2 * ct + 1) * 9 * ksteps) * 64 + lane;

    for (int ks = 0; ks < ksteps; ++ks) {
        __syncthreads();
        for (int i = threadIdx.x; i < (TH + 2) * HALO_W * 2; i += 256) {
            int h = i & 1;
            int p = i >> 1;
            int c = p % HALO_W, r = p / HALO_W;
            int yy = y0 + r - 1, xx = x0 + c - 1;
            int k = 2 * ks + h;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (yy >= 0 && yy < H && xx >= 0 && xx < W && k < Cw)
                v = expand_word(act[(((size_t)n * H + yy) * W + xx) * Cw + k]);
            tile[i] = v;
        }
        __syncthreads();
#pragma unroll
        for (int ky = 0; ky < 3; ++ky)
#pragma unroll
            for (int kx = 0; kx < 3; ++kx) {
                const int tap = ky * 3 + kx;
                uint4 a0 = wf0[((size_t)tap * ksteps + ks) * 64];
                uint4 a1 = wf1[((size_t)tap * ksteps + ks) * 64];
                v4i A0 = {(int)a0.x, (int)a0.y, (int)a0.z, (int)a0.w};
                v4i A1 = {(int)a1.x, (int)a1.y, (int)a1.z, (int)a1.w};
#pragma unroll
                for (int r = 0; r < 2; ++r) {
                    uint4 b = tile[((2 * wave + r + ky) * HALO_W + (col + kx)) * 2 + half];
                    v4i B = {(int)b.x, (int)b.y, (int)b.z, (int)b.w};
                    acc[0][r] = mfma_f4(A0, B, acc[0][r]);
                    acc[1][r] = mfma_f4(A1, B, acc[1][r]);
                }
            }
    }

    // Epilogue: threshold, pack 16 channel bits per lane, merge the two lane halves.
    const int Cow = Cout >> 5;
    const int x = x0 + col;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int y = y0 + 2 * wave + r;
        const bool inside = (y < H) && (x < W);
        const size_t pix = ((size_t)n * H + y) * W + x;
        uint32_t word_mine = 0;
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const int cbase = ct * 64 + m * 32 + 16 * half;
            uint32_t bits = 0;
            int vals[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                vals[i] = (int)acc[m][r][i];
                int th = (cbase + i) < Cout ? thresh[cbase + i] : 0x7fffffff;
                bits |= (uint32_t)(vals[i] >= th) << i;
            }
            if (WRITE_ACC) {
                if (inside && cbase < Cout) {
                    int4 *dst = reinterpret_cast<int4 *>(out_acc + pix * Cout + cbase);
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        dst[q] = make_int4(vals[4 * q], vals[4 * q + 1], vals[4 * q + 2], vals[4 * q + 3]);
                }
            }
            uint32_t other = (uint32_t)__shfl_xor((int)bits, 32);
            uint32_t word = half == 0 ? (bits | (other << 16)) : (other | (bits << 16));
            if (m == half) word_mine = word;
        }
        // lanes of half 0 store the word of channels 0..31, half 1 the word of 32..63
        const int widx = ct * 2 + half;
        if (out_bits && inside && widx < Cow) out_bits[pix * Cow + widx] = word_mine;
    }
}

int launch_conv_mfma(const uint32_t *act, int N, int H, int W, const BlobLayout &L,
                     const void *blob, const int32_t *thresh, uint32_t *out_bits,
                     int32_t *out_acc, hipStream_t s)
{
    const int TH = 8;
    long tiles = (long)N * ceil_div(H, TH) * ceil_div(W, TW);
    if (tiles > 0x7fffffffL) return fail(MBU_ERR_SHAPE, "too many tiles for one launch");
    dim3 grid((unsigned)tiles, (unsigned)(L.cout_pad64 / 64));
    const uint4 *wfrag = (const uint4 *)((const uint8_t *)blob + L.off_f4);
    if (out_acc)
        MBU_LAUNCH(conv_mfma_kernel<true>, grid, dim3(256), 0, s, act, N, H, W,
                           L.cin_words, L.ksteps, wfrag, L.cout, thresh, out_bits, out_acc);
    else
        MBU_LAUNCH(conv_mfma_kernel<false>, grid, dim3(256), 0, s, act, N, H, W,
                           L.cin_words, L.ksteps, wfrag, L.cout, thresh, out_bits, out_acc);
    return check_launch("conv_mfma");
}

}  // namespace mbu
