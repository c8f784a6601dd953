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

// ---------------------------------------------------------------------------------
// Fast kernel (packed bits only).
//
// Block = 4 waves arranged WM x WN: WM groups of RW image rows, WN groups of 64 output
// channels; block tile = (RW*WM) rows x 32 pixels x (64*WN) channels.  A wave owns
// RW x 2 accumulator tiles (RW = 4: 128 registers).
//
// K loop over 64-channel steps ks; inside a step three "groups", one per kernel column
// kx.  A group needs the 3 x 2 weight fragments of taps (ky, kx) (24 registers) and
// RW+2 activation fragments (LDS rows rho = r + ky), each feeding every (r, ky) pair
// with r + ky = rho: 6*RW matrix instructions per RW+2 LDS reads.  All 18 fragments of
// a step stay in registers; as soon as a group has issued its matrix instructions its
// registers are refilled with the same group's fragments of step ks+1, so weights
// arrive a whole step (three groups) ahead of their use.
//
// The halo window of step ks+1 is fetched from global memory at the start of step ks,
// expanded and written to the other LDS buffer at its end; one barrier per step.  The
// loop body has no branches: halo pixels outside the image are loaded from a clamped
// address and expanded with zero masks, the last step refetches itself.
//
// Epilogue: accumulators start at -theta (exact in fp32 after clamping theta to
// +-2^22, which cannot change any comparison because |R| <= 9*Cin < 2^20), so the
// output bit is the complement of the accumulator's sign bit: one funnel shift per
// register collects 16 channel bits, one cross-half exchange completes the word.
template <int RW>
__device__ __forceinline__ void group_mma(v16f (&acc)[RW][2], const v4i (&Wg)[3][2],
                                          const uint4 *tb)
{
#pragma unroll
    for (int rho = 0; rho < RW + 2; ++rho) {
        const uint4 b = tb[rho * 2 * HALO_W];
        const v4i B = {(int)b.x, (int)b.y, (int)b.z, (int)b.w};
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) {
            const int r = rho - ky;
            if (r >= 0 && r < RW) {
                acc[r][0] = mfma_f4(Wg[ky][0], B, acc[r][0]);
                acc[r][1] = mfma_f4(Wg[ky][1], B, acc[r][1]);
            }
        }
    }
}

// fragments of taps (ky, kx), ky = 0..2, both 32-channel halves of the wave's 64 channels;
// wk points at [tap 0][m 0][lane] of one 64-channel step of this wave's channel tile
__device__ __forceinline__ void load_group(v4i (&Wg)[3][2], const uint4 *wk, int kx)
{
#pragma unroll
    for (int ky = 0; ky < 3; ++ky)
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const uint4 a = wk[((ky * 3 + kx) * 2 + m) * 64];
            Wg[ky][m] = (v4i){(int)a.x, (int)a.y, (int)a.z, (int)a.w};
        }
}

template <int RW, int WM, int WN, bool CW_EVEN>
__global__ __launch_bounds__(256, 2) void conv_mfma_bits_kernel(
    const uint32_t *__restrict__ act, int N, int H, int W, int Cw, int ksteps,
    const uint4 *__restrict__ wfrag, int Cout, int tiles64, const int32_t *__restrict__ thresh,
    uint32_t *__restrict__ out_bits)
{
    constexpr int TH = RW * WM;
    constexpr int HR = TH + 2;
    constexpr int NPIX = HR * HALO_W;            // halo pixels per step
    constexpr int NLD = (NPIX + 255) / 256;      // staged pixels per thread
    constexpr int TILE = HR * 2 * HALO_W;        // uint4 entries per buffer, [row][half][col]
    __shared__ uint4 tile[2][TILE];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave % WM, wn = wave / WM;
    const int col = lane & 31, half = lane >> 5;
    const int tiles_x = (W + TW - 1) / TW;
    const int tiles_y = (H + TH - 1) / TH;
    int bid = blockIdx.x;
    const int tx = bid % tiles_x;
    bid /= tiles_x;
    const int ty = bid % tiles_y;
    const int n = bid / tiles_y;
    const int x0 = tx * TW, y0 = ty * TH;
    const int ct_raw = blockIdx.y * WN + wn;      // 64-channel output tile of this wave
    const bool has_ct = ct_raw < tiles64;
    const int ct = has_ct ? ct_raw : tiles64 - 1;

    // ---- accumulators start at -theta
    v16f acc[RW][2];
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const int cbase = ct * 64 + m * 32 + 16 * half;   // 16 consecutive channels per lane
        int th[16];
        if (cbase < Cout) {                                // Cout % 32 == 0: all 16 or none
            const int4 *tp = reinterpret_cast<const int4 *>(thresh + cbase);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int4 t = tp[q];
                th[4 * q] = t.x; th[4 * q + 1] = t.y; th[4 * q + 2] = t.z; th[4 * q + 3] = t.w;
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) th[i] = 0;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int t = max(-(1 << 22), min(1 << 22, th[i]));
            const float init = 0.0f - (float)t;
#pragma unroll
            for (int r = 0; r < RW; ++r) acc[r][m][i] = init;
        }
    }

    // ---- staging plan of this thread: halo pixels p = tid + 256*j
    const uint32_t *src[NLD];     // first word of the (clamped) pixel
    uint32_t m8[NLD], m2[NLD];    // expansion masks, zero for pixels outside the image
    int dst[NLD];                 // LDS entry of (row, half 0, col)
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
        int p = threadIdx.x + 256 * j;
        p = p < NPIX ? p : 0;     // surplus threads duplicate pixel 0 (same data, same slot)
        const int r = p / HALO_W, c = p - r * HALO_W;
        const int yy = y0 + r - 1, xx = x0 + c - 1;
        const bool in = yy >= 0 && yy < H && xx >= 0 && xx < W;
        const int yc = min(max(yy, 0), H - 1), xc = min(max(xx, 0), W - 1);
        src[j] = act + (((size_t)n * H + yc) * W + xc) * Cw;
        m8[j] = in ? 0x88888888u : 0u;
        m2[j] = in ? 0x22222222u : 0u;
        dst[j] = (r * 2) * HALO_W + c;
    }
    uint2 gq[NLD];
    auto stage_issue = [&](int ks) {
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            if (CW_EVEN) {
                gq[j] = *reinterpret_cast<const uint2 *>(src[j] + 2 * ks);
            } else {
                gq[j].x = src[j][2 * ks];
                gq[j].y = src[j][min(2 * ks + 1, Cw - 1)];
            }
        }
    };
    auto stage_commit = [&](int ks, uint4 *buf) {
        const bool second = CW_EVEN || (2 * ks + 1 < Cw);
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            const uint32_t a = gq[j].x, b = gq[j].y;
            const uint32_t k8 = m8[j], k2 = m2[j];
            const uint32_t l8 = second ? k8 : 0u, l2 = second ? k2 : 0u;
            uint4 e0, e1;
            e0.x = ((a << 3) & k8) | k2; e0.y = ((a << 2) & k8) | k2;
            e0.z = ((a << 1) & k8) | k2; e0.w = (a & k8) | k2;
            e1.x = ((b << 3) & l8) | l2; e1.y = ((b << 2) & l8) | l2;
            e1.z = ((b << 1) & l8) | l2; e1.w = (b & l8) | l2;
            buf[dst[j]] = e0;
            buf[dst[j] + HALO_W] = e1;
        }
    };

    // ---- weight fragments: [tile64][kstep][tap][m][lane], 18 KB per step and tile
    const uint4 *wk = wfrag + (size_t)ct * ksteps * (18 * 64) + lane;
    v4i Wg[3][3][2];   // [kx][ky][m]
    stage_issue(0);
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) load_group(Wg[kx], wk, kx);
    stage_commit(0, tile[0]);
    __syncthreads();

    const int tb_off = (wm * RW * 2 + half) * HALO_W + col;
    for (int ks = 0; ks < ksteps; ++ks) {
        const int kn = min(ks + 1, ksteps - 1);
        const uint4 *wn_ptr = wk + (size_t)kn * (18 * 64);
        const uint4 *tb = tile[ks & 1] + tb_off;
        // The scheduling fences keep every fetch where it is written: issued as early as its
        // destination registers are free, a whole step ahead of its use.
        stage_issue(kn);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) {
            group_mma<RW>(acc, Wg[kx], tb + kx);
            __builtin_amdgcn_sched_barrier(0);
            load_group(Wg[kx], wn_ptr, kx);
            __builtin_amdgcn_sched_barrier(0);
        }
        stage_commit(kn, tile[(ks + 1) & 1]);
        __syncthreads();
    }

    // ---- epilogue
    const int Cow = Cout >> 5;
    const int x = x0 + col;
    const int widx = ct * 2 + half;
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        const int y = y0 + wm * RW + r;
        uint32_t s0 = 0, s1 = 0;
#pragma unroll
        for (int i = 15; i >= 0; --i) {
            s0 = __builtin_amdgcn_alignbit(s0, __float_as_uint(acc[r][0][i]), 31);
            s1 = __builtin_amdgcn_alignbit(s1, __float_as_uint(acc[r][1][i]), 31);
        }
        // s = sign bits (1 = below threshold) of channels 16*half + i
        const uint32_t mine = (~s0 & 0xffffu) | (~s1 << 16);
        const uint32_t other = (uint32_t)__shfl_xor((int)mine, 32);
        const uint32_t word = half == 0 ? ((mine & 0xffffu) | (other << 16))
                                        : ((other >> 16) | (mine & 0xffff0000u));
        if (has_ct && y < H && x < W && widx < Cow)
            out_bits[(((size_t)n * H + y) * W + x) * Cow + widx] = word;
    }
}

// ---------------------------------------------------------------------------------
// Reference-quality kernel that can also write the int32 accumulators (parity and
// debugging).  Block = 4 waves; wave v owns image rows (2v, 2v+1) of an 8 x 32 pixel
// tile and 64 output channels: 2 x 2 accumulator tiles.
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

    const uint4 *wf = wfrag + (size_t)ct * ksteps * (18 * 64) + lane;  // [tile64][kstep][tap][m][lane]

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
                uint4 a0 = wf[((size_t)ks * 18 + tap * 2) * 64];
                uint4 a1 = wf[((size_t)ks * 18 + tap * 2 + 1) * 64];
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

template <int RW, int WM, int WN, bool CW_EVEN>
static int launch_bits_t(const uint32_t *act, int N, int H, int W, const BlobLayout &L,
                       const uint4 *wfrag, const int32_t *thresh, uint32_t *out_bits, hipStream_t s)
{
    const int tiles64 = L.cout_pad64 / 64;
    long tiles = (long)N * ceil_div(H, RW * WM) * ceil_div(W, TW);
    if (tiles > 0x7fffffffL) return fail(MBU_ERR_SHAPE, "too many tiles for one launch");
    dim3 grid((unsigned)tiles, (unsigned)ceil_div(tiles64, WN));
    MBU_LAUNCH((conv_mfma_bits_kernel<RW, WM, WN, CW_EVEN>), grid, dim3(256), 0, s, act, N, H, W,
               L.cin_words, L.ksteps, wfrag, L.cout, tiles64, thresh, out_bits);
    return check_launch("conv_mfma_bits");
}

template <int RW, int WM, int WN>
static int launch_bits(const uint32_t *act, int N, int H, int W, const BlobLayout &L,
                       const uint4 *wfrag, const int32_t *thresh, uint32_t *out_bits, hipStream_t s)
{
    if (L.cin_words % 2 == 0)
        return launch_bits_t<RW, WM, WN, true>(act, N, H, W, L, wfrag, thresh, out_bits, s);
    return launch_bits_t<RW, WM, WN, false>(act, N, H, W, L, wfrag, thresh, out_bits, s);
}

int launch_conv_mfma(const uint32_t *act, int N, int H, int W, const BlobLayout &L,
                     const void *blob, const int32_t *thresh, uint32_t *out_bits,
                     int32_t *out_acc, hipStream_t s)
{
    const uint4 *wfrag = (const uint4 *)((const uint8_t *)blob + L.off_f4);
    if (out_acc) {
        const int TH = 8;
        long tiles = (long)N * ceil_div(H, TH) * ceil_div(W, TW);
        if (tiles > 0x7fffffffL) return fail(MBU_ERR_SHAPE, "too many tiles for one launch");
        dim3 grid((unsigned)tiles, (unsigned)(L.cout_pad64 / 64));
        MBU_LAUNCH(conv_mfma_kernel<true>, grid, dim3(256), 0, s, act, N, H, W, L.cin_words,
                   L.ksteps, wfrag, L.cout, thresh, out_bits, out_acc);
        return check_launch("conv_mfma_acc");
    }
    // Shape of the block: spread the four waves over output channels when there are
    // enough of them, over image rows otherwise; halve the rows per wave when the
    // launch would not give every SIMD two waves.
    const int tiles64 = L.cout_pad64 / 64;
    const int WN = (tiles64 % 4 == 0) ? 4 : (tiles64 % 2 == 0) ? 2 : 1;
    const int WM = 4 / WN;
    const long blocks4 = (long)N * ceil_div(H, 4 * WM) * ceil_div(W, TW) * ceil_div(tiles64, WN);
    const bool small = blocks4 < 2 * 256;
#define MBU_GO(RW_, WM_, WN_) return launch_bits<RW_, WM_, WN_>(act, N, H, W, L, wfrag, thresh, out_bits, s)
    if (WN == 4) { if (small) MBU_GO(2, 1, 4); else MBU_GO(4, 1, 4); }
    if (WN == 2) { if (small) MBU_GO(2, 2, 2); else MBU_GO(4, 2, 2); }
    if (small) MBU_GO(2, 4, 1);
    MBU_GO(4, 4, 1);
#undef MBU_GO
}

}  // namespace mbu
