// Masked-binary transposed convolution, kernel 2x2, stride 2, on the matrix cores: the
// up-sampling layer of the decoder (Sec. 2.1; Sec. 3.2.2: "performed similarly"), followed
// by the same threshold / sign / bit-pack epilogue as Algorithm 1 (the quantised network
// puts batch norm and a binary activation after it, Appendix A.1).
//
// With kernel = stride every output pixel (2y+dy, 2x+dx) receives exactly one tap, so the
// layer is four independent 1x1 contractions, one per position p = 2*dy + dx:
//   D_p[cout][pixel] = sum_c W[cout][p][c] * A[c][pixel].
// Same FP4 encoding and operand layout as the 3x3 layer (exact integers in fp32).  No halo
// and no reuse of activations between taps: the activation fragment of a lane is ONE packed
// word, loaded straight from global memory and expanded in registers (7 vector ops),
// and it feeds the two channel tiles of one position.  The four waves of a block are the four
// positions of the same 4 x 32 input pixels and 64 output channels (8 accumulator tiles =
// 128 registers per wave); weights of the next step are fetched while the current step
// multiplies.
#include "mbu_internal.h"
#include "mfma_common.h"

namespace mbu {

TconvLayout tconv_layout(int cout, int cin)
{
    TconvLayout L;
    L.cout = cout;
    L.cin = cin;
    L.cin_words = ceil_div(cin, 32);
    L.cout_pad64 = ceil_div(cout, 64) * 64;
    L.ksteps = ceil_div(cin, 64);
    L.off_f4 = 256;
    L.total = round_up(L.off_f4 + (size_t)(L.cout_pad64 / 64) * L.ksteps * 8 * 64 * 16, 256);
    return L;
}

// Thread (o, position p, word k) packs 32 weights into one 16-byte fragment:
// fragments are uint4 [cout_pad64/64][ksteps][4 positions][2][64 lanes]; nibble q of dword d
// carries input channel 32k + 4q + d as the E2M1 code of -w (the activation side is negated
// too); lane = 32*(k&1) + tile row of the output channel.
__global__ __launch_bounds__(256) void pack_tconv_kernel(const int8_t *__restrict__ w,
                                                         TconvLayout L, uint8_t *__restrict__ blob)
{
    const int words = 2 * L.ksteps;
    const long total = (long)L.cout_pad64 * 4 * words;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int k = (int)(idx % words);
    const int p = (int)((idx / words) % 4);
    const int o = (int)(idx / (4L * words));
    uint32_t d[4] = {0, 0, 0, 0};
    if (o < L.cout && k < L.cin_words) {
        const int8_t *src = w + ((long)o * 4 + p) * L.cin + (long)k * 32;
        const int n = min(32, L.cin - k * 32);
        for (int i = 0; i < n; ++i) {
            const int v = src[i];
            const uint32_t code = v > 0 ? 0xAu : (v < 0 ? 0x2u : 0x0u);
            d[i & 3] |= code << (4 * (i >> 2));
        }
    }
    const int tile64 = o >> 6, m = (o >> 5) & 1;
    const int row = tile_channel_to_row(o & 31);
    const int lane = (k & 1) * 32 + row;
    uint4 *F = reinterpret_cast<uint4 *>(blob + L.off_f4);
    const size_t at = ((((size_t)tile64 * L.ksteps + (k >> 1)) * 4 + p) * 2 + m) * 64 + lane;
    F[at] = make_uint4(d[0], d[1], d[2], d[3]);
}

int launch_pack_tconv(const int8_t *w, const TconvLayout &L, void *blob, hipStream_t s)
{
    const long total = (long)L.cout_pad64 * 4 * 2 * L.ksteps;
    MBU_LAUNCH(pack_tconv_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, w, L,
               (uint8_t *)blob);
    return check_launch("pack_tconv_weights");
}

// weight fragments of one 64-channel step of one position: [m]
__device__ __forceinline__ void load_step(v4i (&Wt)[2], const uint4 *wk)
{
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const uint4 a = wk[m * 64];
        Wt[m] = (v4i){(int)a.x, (int)a.y, (int)a.z, (int)a.w};
    }
}

// A wave owns ONE position p = 2*dy + dx, 64 output channels and RG = 4 consecutive image rows
// x 32 input pixels: 8 accumulator tiles, and every weight fragment it fetches feeds four
// matrix instructions (one per row).  The four positions of a pixel group are four waves of
// the same block, which read the same activation words (L1 hits).
constexpr int RG = 4;

template <bool WRITE_ACC>
__global__ __launch_bounds__(256, 2) void tconv_mfma_kernel(
    const uint32_t *__restrict__ act, int N, int H, int W, int Cw, int ksteps,
    const uint4 *__restrict__ wfrag, int Cout, long groups, int groups_x, int groups_y,
    const int32_t *__restrict__ thresh, uint32_t *__restrict__ out_bits,
    int32_t *__restrict__ out_acc)
{
    const int lane = threadIdx.x & 63;
    const int p = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // position of this wave
    const long g = blockIdx.x;                          // (n, row group, 32-pixel column group)
    const int ct = blockIdx.y;                          // 64-channel output tile
    const int col = lane & 31, half = lane >> 5;
    const int gx = (int)(g % groups_x);
    const long q = g / groups_x;
    const int gy = (int)(q % groups_y);
    const long n = q / groups_y;
    const int x = gx * 32 + col;
    const int y0 = gy * RG;
    const bool in_x = x < W;

    const uint32_t *src[RG];
    uint32_t k8[RG];
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        const bool in = in_x && y0 + r < H;
        const int yc = min(y0 + r, H - 1), xc = in_x ? x : W - 1;
        src[r] = act + (((size_t)n * H + yc) * W + xc) * Cw;
        k8[r] = in ? 0x88888888u : 0u;
    }

    v16f acc[RG][2];
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const int cbase = ct * 64 + m * 32 + 16 * half;
        float init[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) init[i] = 0.0f;
        if (!WRITE_ACC && cbase < Cout) {              // accumulators start at -theta
            const int4 *tp = reinterpret_cast<const int4 *>(thresh + cbase);
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
                const int4 t = tp[qq];
                init[4 * qq] = 0.0f - (float)max(-(1 << 22), min(1 << 22, t.x));
                init[4 * qq + 1] = 0.0f - (float)max(-(1 << 22), min(1 << 22, t.y));
                init[4 * qq + 2] = 0.0f - (float)max(-(1 << 22), min(1 << 22, t.z));
                init[4 * qq + 3] = 0.0f - (float)max(-(1 << 22), min(1 << 22, t.w));
            }
        }
#pragma unroll
        for (int r = 0; r < RG; ++r)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[r][m][i] = init[i];
    }

    // fragments: [tile64][kstep][position][m][lane]
    const uint4 *wk = wfrag + ((size_t)ct * ksteps * 8 + p * 2) * 64 + lane;
    auto fetch_words = [&](int ks, uint32_t (&wd)[RG]) {
        const int k = min(2 * ks + half, Cw - 1);
#pragma unroll
        for (int r = 0; r < RG; ++r) wd[r] = src[r][k];
    };
    auto step = [&](int ks, const uint32_t (&wd)[RG], const v4i (&Wt)[2]) {
        const bool live = 2 * ks + half < Cw;          // second word of an odd word count
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            const uint32_t m8 = live ? k8[r] : 0u, m2 = m8 >> 2;
            const uint32_t word = wd[r];
            const v4i B = {(int)(((word << 3) & m8) | m2), (int)(((word << 2) & m8) | m2),
                           (int)(((word << 1) & m8) | m2), (int)((word & m8) | m2)};
#pragma unroll
            for (int m = 0; m < 2; ++m) acc[r][m] = mfma_f4(Wt[m], B, acc[r][m]);
        }
    };

    v4i Wa[2], Wb[2];
    uint32_t wa[RG], wb[RG];
    load_step(Wa, wk);
    fetch_words(0, wa);
    for (int ks = 0; ks < ksteps; ks += 2) {
        const int k1 = min(ks + 1, ksteps - 1), k2n = min(ks + 2, ksteps - 1);
        load_step(Wb, wk + (size_t)k1 * (8 * 64));
        fetch_words(k1, wb);
        step(ks, wa, Wa);
        load_step(Wa, wk + (size_t)k2n * (8 * 64));
        fetch_words(k2n, wa);
        if (ks + 1 < ksteps) step(ks + 1, wb, Wb);
    }

    // ---- epilogue: input pixel (y, x) -> output pixel (2y+dy, 2x+dx)
    const int Cow = Cout >> 5;
    const int dy = p >> 1, dx = p & 1;
    const uint32_t psel = half ? 0x07060302u : 0x05040100u;
#pragma unroll
    for (int r = 0; r < RG; ++r) {
        const int y = y0 + r;
        const bool in = in_x && y < H;
        const size_t pix = ((size_t)n * 2 * H + 2 * y + dy) * 2 * W + 2 * x + dx;
        if (WRITE_ACC) {
            uint32_t bits[2] = {0, 0};
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const int cbase = ct * 64 + m * 32 + 16 * half;
                int vals[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    vals[i] = (int)acc[r][m][i];
                    const int th = cbase < Cout ? thresh[cbase + i] : 0x7fffffff;
                    bits[m] |= (uint32_t)(vals[i] < th) << i;       // 1 = below threshold
                }
                if (in && cbase < Cout && out_acc) {
                    int4 *dst = reinterpret_cast<int4 *>(out_acc + pix * Cout + cbase);
#pragma unroll
                    for (int qq = 0; qq < 4; ++qq)
                        dst[qq] = make_int4(vals[4 * qq], vals[4 * qq + 1], vals[4 * qq + 2], vals[4 * qq + 3]);
                }
            }
            const uint32_t word = finish_word64(bits[0], bits[1], psel);
            if (in && out_bits && ct * 2 + half < Cow) out_bits[pix * Cow + ct * 2 + half] = word;
        } else {
            uint32_t s0 = 0, s1 = 0;
#pragma unroll
            for (int i = 15; i >= 0; --i) {
                s0 = __builtin_amdgcn_alignbit(s0, __float_as_uint(acc[r][0][i]), 31);
                s1 = __builtin_amdgcn_alignbit(s1, __float_as_uint(acc[r][1][i]), 31);
            }
            const uint32_t word = finish_word64(s0, s1, psel);
            if (in && ct * 2 + half < Cow) out_bits[pix * Cow + ct * 2 + half] = word;
        }
    }
}

int launch_tconv_mfma(const uint32_t *act, int N, int H, int W, const TconvLayout &L,
                      const void *blob, const int32_t *thresh, uint32_t *out_bits, int32_t *out_acc,
                      hipStream_t s)
{
    const int groups_x = ceil_div(W, 32), groups_y = ceil_div(H, RG);
    const long groups = (long)N * groups_y * groups_x;
    if (groups > 0x7fffffffL) return fail(MBU_ERR_SHAPE, "too many pixel groups for one launch");
    const uint4 *wfrag = (const uint4 *)((const uint8_t *)blob + L.off_f4);
    dim3 grid((unsigned)groups, (unsigned)(L.cout_pad64 / 64));   // 4 waves = the 4 positions
    if (out_acc)
        MBU_LAUNCH(tconv_mfma_kernel<true>, grid, dim3(256), 0, s, act, N, H, W, L.cin_words,
                   L.ksteps, wfrag, L.cout, groups, groups_x, groups_y, thresh, out_bits, out_acc);
    else
        MBU_LAUNCH(tconv_mfma_kernel<false>, grid, dim3(256), 0, s, act, N, H, W, L.cin_words,
                   L.ksteps, wfrag, L.cout, groups, groups_x, groups_y, thresh, out_bits, out_acc);
    return check_launch("tconv2x2_masked_binary");
}

}  // namespace mbu
