// Masked-binary transposed convolution, kernel 2x2, stride 2, on the matrix cores: the
// up-sampling layer of the decoder (Sec. 2.1; Sec. 3.2.2: "performed similarly"), followed
// by the same threshold / sign / bit-pack epilogue as Algorithm 1 (the quantised network
// puts batch norm and a binary activation after it, Appendix A.1).
//
// With kernel = stride every output pixel (2y+dy, 2x+dx) receives exactly one tap, so the
// layer is four independent 1x1 contractions, one per position p = 2*dy + dx:
//   D_p[cout][pixel] = sum_c W[cout][p][c] * A[c][pixel].
// Same FP4 encoding and operand layout as the 3x3 layer (exact integers in fp32), activations as
// the packed bit itself (code 1.0 / 0): sum w a = 2 sum w a' - sum w, and the sum of the weights
// of (position, channel) goes into the accumulators' start value with the threshold
// (mfma_common.h) - there is no padding here, so no 0.5 code either.  No halo
// and no reuse of activations between taps: the activation fragment of a lane is ONE packed
// word, loaded straight from global memory and expanded in registers (7 vector ops),
// and it feeds the two channel tiles of one position.  The four waves of a block are the four
// positions of the same 4 x 32 input pixels and 64 output channels (8 accumulator tiles =
// 128 registers per wave); weights of the next step are fetched while the current step
// multiplies.
#include "mbu_internal.h"
#include "mfma_common.h"
#include <algorithm>

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
    L.off_sum = round_up(L.off_f4 + (size_t)(L.cout_pad64 / 64) * L.ksteps * 8 * 64 * 16, 256);
    L.total = round_up(L.off_sum + (size_t)4 * L.cout_pad64 * sizeof(int32_t), 256);
    return L;
}

// Thread (o, position p, word k) packs 32 weights into one 16-byte fragment:
// fragments are uint4 [cout_pad64/64][ksteps][4 positions][2][64 lanes]; nibble q of dword d
// carries input channel 32k + 4q + d as the E2M1 code of w; lane = 32*(k&1) + tile row of the
// output channel.
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
            const uint32_t code = v > 0 ? 0x2u : (v < 0 ? 0xAu : 0x0u);
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

// Sum of the weights of every (position, output channel): one wave per pair.
__global__ __launch_bounds__(256) void sum_tconv_kernel(const int8_t *__restrict__ w, TconvLayout L,
                                                        uint8_t *__restrict__ blob)
{
    const int idx = blockIdx.x * 4 + (threadIdx.x >> 6);    // p * cout_pad64 + o
    const int lane = threadIdx.x & 63;
    if (idx >= 4 * L.cout_pad64) return;
    const int p = idx / L.cout_pad64, o = idx - p * L.cout_pad64;
    int sum = 0;
    if (o < L.cout) {
        const int8_t *src = w + ((long)o * 4 + p) * L.cin;
        for (int i = lane; i < L.cin; i += 64) sum += (src[i] > 0) - (src[i] < 0);
    }
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    if (lane == 0) reinterpret_cast<int32_t *>(blob + L.off_sum)[idx] = sum;
}

int launch_pack_tconv(const int8_t *w, const TconvLayout &L, void *blob, hipStream_t s)
{
    const long total = (long)L.cout_pad64 * 4 * 2 * L.ksteps;
    MBU_LAUNCH(pack_tconv_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, w, L,
               (uint8_t *)blob);
    int rc = check_launch("pack_tconv_weights");
    if (rc) return rc;
    MBU_LAUNCH(sum_tconv_kernel, dim3((unsigned)L.cout_pad64), dim3(256), 0, s, w, L, (uint8_t *)blob);
    return check_launch("pack_tconv_sums");
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
    const int32_t *__restrict__ thresh, const int32_t *__restrict__ wsum, int cout_pad64,
    uint32_t *__restrict__ out_bits, int32_t *__restrict__ out_acc)
{
    const int lane = threadIdx.x & 63;
    const int p = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // position of this wave
    const int32_t *ws = wsum + (size_t)p * cout_pad64;               // sums of this position's weights
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
        k8[r] = in ? 0x22222222u : 0u;
    }

    v16f acc[RG][2];
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const int cbase = ct * 64 + m * 32 + 16 * half;
        float init[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) init[i] = 0.0f;
        if (!WRITE_ACC && cbase < Cout) {              // accumulators start at -(theta + sum w) / 2
            const int4 *tp = reinterpret_cast<const int4 *>(thresh + cbase);
            const int4 *sp = reinterpret_cast<const int4 *>(ws + cbase);
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) {
                const int4 t = tp[qq], u = sp[qq];
                init[4 * qq] = start_value(t.x, u.x);
                init[4 * qq + 1] = start_value(t.y, u.y);
                init[4 * qq + 2] = start_value(t.z, u.z);
                init[4 * qq + 3] = start_value(t.w, u.w);
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
            const uint32_t m2 = live ? k8[r] : 0u;
            const uint32_t word = wd[r];
            const v4i B = {(int)((word << 1) & m2), (int)(word & m2), (int)((word >> 1) & m2),
                           (int)((word >> 2) & m2)};
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
                    // the accumulator holds sum w a' (an integer): sum w a = 2 sum w a' - sum w
                    vals[i] = 2 * (int)acc[r][m][i] - (cbase < Cout ? ws[cbase + i] : 0);
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

// ---------------------------------------------------------------------------------
// Fast kernel (packed bits only): the same wave tile - one position, RG rows x 32 input
// pixels x 64 output channels - but persistent.  A block keeps its 64-channel tile and strides
// over the pixel groups; the work of a wave is the flat sequence of (group, 64-channel step),
// and during every step the words and the two weight fragments of the step after the next -
// possibly the next group's - are fetched through buffer resources (lane offsets in
// registers, step offsets in scalar registers) into the free one of three register sets.  A group's first step takes -theta as the addend of its matrix instructions
// (no accumulator initialisation); its last step is followed by the sign collection and the
// stores.  With one block per pixel group, as in the kernel above, every block paid the
// latency of a dependent chain of loads before its first matrix instruction: 35 us for
// 128 -> 64 channels at 512x1024, against 4 us of matrix work.
template <int RG>
struct TconvRegs {
    uint32_t wd[RG];   // packed word (lane half's own) of the RG pixels
    v4i W[2];          // weight fragments of the two 32-channel tiles
};

template <int RG>
__global__ __launch_bounds__(256, RG == 2 ? 4 : 2) void tconv_bits_kernel(
    const uint32_t *__restrict__ act, int N, int H, int W, int Cw, int ksteps,
    const uint4 *__restrict__ wfrag, int Cout, int groups, int groups_x, int groups_y,
    const int32_t *__restrict__ thresh, const int32_t *__restrict__ wsum, int cout_pad64,
    uint32_t *__restrict__ out_bits)
{
    constexpr uint32_t BAD = 0x40000000u;   // beyond any tensor this kernel accepts (< 2^30 bytes)
    const int lane = threadIdx.x & 63;
    const int p = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // position of this wave
    const int32_t *ws = wsum + (size_t)p * cout_pad64;
    const int ct = blockIdx.y;                                        // 64-channel output tile
    const int col = lane & 31, half = lane >> 5;
    const int Cow = Cout >> 5;
    const int dy = p >> 1, dx = p & 1;
    const uint32_t psel = half ? 0x07060302u : 0x05040100u;

    const __amdgpu_buffer_rsrc_t ars =
        __builtin_amdgcn_make_buffer_rsrc((void *)act, 0, N * H * W * Cw * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(wfrag + (size_t)ct * ksteps * 8 * 64), 0, ksteps * 8 * 1024, 0x00020000);
    const __amdgpu_buffer_rsrc_t ors =
        __builtin_amdgcn_make_buffer_rsrc((void *)out_bits, 0, N * H * W * 4 * Cow * 4, 0x00020000);
    const int wlane = lane * 16;
    // output word of this lane inside a row of output pixels, for pixel group column 0
    const uint32_t out_lane = (ct * 2 + half < Cow) ? (uint32_t)(((2 * col + dx) * Cow + ct * 2 + half) * 4) : BAD;

    // ---- -(theta + sum w) / 2 for the 2 x 16 channels of this lane
    v16f init[2];
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const int cbase = ct * 64 + m * 32 + 16 * half;
        int th[16], su[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) th[i] = su[i] = 0;
        if (cbase < Cout) {
            const int4 *tp = reinterpret_cast<const int4 *>(thresh + cbase);
            const int4 *sp = reinterpret_cast<const int4 *>(ws + cbase);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int4 t = tp[q], u = sp[q];
                th[4 * q] = t.x; th[4 * q + 1] = t.y; th[4 * q + 2] = t.z; th[4 * q + 3] = t.w;
                su[4 * q] = u.x; su[4 * q + 1] = u.y; su[4 * q + 2] = u.z; su[4 * q + 3] = u.w;
            }
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) init[m][i] = start_value(th[i], su[i]);
    }

    // ---- per-group plan: byte offset of the lane's word 0 of each of the RG pixels (clamped
    // to the image) and whether the pixel exists
    struct Plan { uint32_t off[RG]; uint32_t k8[RG]; int gx, gy, n; };
    auto plan = [&](int g) {
        Plan P;
        P.gx = g % groups_x;
        const int q = g / groups_x;
        P.gy = q % groups_y;
        P.n = q / groups_y;
        const int x = P.gx * 32 + col;
        const int xc = min(x, W - 1);
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            const int y = P.gy * RG + r;
            const int yc = min(y, H - 1);
            P.off[r] = (uint32_t)((((P.n * H + yc) * W + xc) * Cw + half) * 4);
            P.k8[r] = (x < W && y < H) ? 0x22222222u : 0u;
        }
        return P;
    };
    // a word index past the pixel's last word (odd word count) reads the next pixel's first
    // word, or 0 past the end of the tensor: it is expanded with a zero mask either way
    auto fetch = [&](const Plan &P, int ks, TconvRegs<RG> &R) {
#pragma unroll
        for (int r = 0; r < RG; ++r) R.wd[r] = __builtin_amdgcn_raw_buffer_load_b32(ars, P.off[r], ks * 8, 0);
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const auto w = __builtin_amdgcn_raw_buffer_load_b128(wrs, wlane, ((ks * 4 + p) * 2 + m) * 1024, 0);
            R.W[m] = (v4i){(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
        }
    };

    // compute cursor (g, ks, cur) and fetch cursor (gf, kf, pf), which runs two steps ahead:
    // with ksteps >= 2 it is one or (ksteps = 2, at a group's last step) two groups ahead;
    // `pp` is the plan of the group it left last
    const int stride = gridDim.x;
    int g = blockIdx.x;
    if (g >= groups) return;
    Plan cur = plan(g);
    Plan pf = cur, pp = cur;
    int gf = g, kf = 0;
    TconvRegs<RG> S0, S1, S2;
    auto fetch_next = [&](TconvRegs<RG> &R) {
        fetch(pf, kf, R);
        if (++kf == ksteps) {
            kf = 0;
            gf += stride;
            pp = pf;
            if (gf < groups) pf = plan(gf);     // past the last group: the same data again, unused
        }
    };
    fetch_next(S0);
    fetch_next(S1);
    v16f acc[RG][2];
    int ks = 0;

    // one step with the register set R; the data of the step after the next goes to Rf.
    // Returns false when the wave has finished its last group.
    auto step = [&](const TconvRegs<RG> &R, TconvRegs<RG> &Rf) -> bool {
        fetch_next(Rf);
        __builtin_amdgcn_sched_barrier(0);
        const bool live = 2 * ks + half < Cw;          // second word of an odd word count
        v4i B[RG];
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            const uint32_t m2 = live ? cur.k8[r] : 0u;
            const uint32_t word = R.wd[r];
            B[r] = (v4i){(int)((word << 1) & m2), (int)(word & m2), (int)((word >> 1) & m2),
                         (int)((word >> 2) & m2)};
        }
        if (ks == 0) {
#pragma unroll
            for (int r = 0; r < RG; ++r)
#pragma unroll
                for (int m = 0; m < 2; ++m) acc[r][m] = mfma_f4(R.W[m], B[r], init[m]);
        } else {
#pragma unroll
            for (int r = 0; r < RG; ++r)
#pragma unroll
                for (int m = 0; m < 2; ++m) acc[r][m] = mfma_f4(R.W[m], B[r], acc[r][m]);
        }
        if (++ks < ksteps) return true;
        // ---- epilogue: input pixel (y, x) -> output pixel (2y + dy, 2x + dx)
        const uint32_t lane_off = (cur.gx * 32 + col < W) ? out_lane + (uint32_t)(cur.gx * 64 * Cow * 4) : BAD;
#pragma unroll
        for (int r = 0; r < RG; ++r) {
            const int y = cur.gy * RG + r;
            uint32_t s0 = 0, s1 = 0;
#pragma unroll
            for (int i = 15; i >= 0; --i) {
                s0 = __builtin_amdgcn_alignbit(s0, __float_as_uint(acc[r][0][i]), 31);
                s1 = __builtin_amdgcn_alignbit(s1, __float_as_uint(acc[r][1][i]), 31);
            }
            const uint32_t word = finish_word64(s0, s1, psel);
            if (y < H) {
                const uint32_t row_off = (uint32_t)((((cur.n * 2 * H + 2 * y + dy) * 2 * W) * Cow) * 4);
                __builtin_amdgcn_raw_buffer_store_b32(word, ors, lane_off + row_off, 0, 0);
            }
        }
        ks = 0;
        g += stride;
        cur = gf == g ? pf : pp;
        return g < groups;
    };

#pragma unroll 1
    for (;;) {
        if (!step(S0, S2)) break;
        if (!step(S1, S0)) break;
        if (!step(S2, S1)) break;
    }
}

// Weights resident, activations through LDS.  The kernel above lets every lane fetch its own
// packed word of every step: 8 useful bytes per 32-byte sector and request, the same sectors
// again for every step and for each of the four position waves - the address and cache path
// of the compute unit is busy four times as long as the matrix cores, which ran at a sixth of
// their rate.  Here the block fetches the words of a pixel group once, coalesced (16 bytes per
// thread, a row of 32 pixels is contiguous), and passes them through LDS ([row][word][pixel]:
// a wave's reads are conflict-free); the fetch of the next group is in flight while the current
// one multiplies, one barrier per group.  With KS <= 16 input steps the weights of a wave's
// position and channel tile are only 8 KS registers: loaded once.  A group's first step takes
// -theta as the addend of its matrix instructions.  RGX rows of 32 pixels per group, so that a group is 1024 words (512 for KS = 2): one fetch per thread.
// Needs an even word count (Cin a multiple of 64).
template <int KS, int RGX>
__global__ __launch_bounds__(256, 2) void tconv_res_kernel(
    const uint32_t *__restrict__ act, int N, int H, int W, const uint4 *__restrict__ wfrag, int Cout,
    int groups, int groups_x, int groups_y, const int32_t *__restrict__ thresh,
    const int32_t *__restrict__ wsum, int cout_pad64, uint32_t *__restrict__ out_bits)
{
    constexpr uint32_t BAD = 0x40000000u;   // beyond any tensor this kernel accepts (< 2^30 bytes)
    constexpr int CW = 2 * KS;              // words per pixel
    constexpr int TILE = RGX * CW * 32;     // words per pixel group
    constexpr int PW = TILE / 256;          // words per thread and group: 4 (2 for KS = 2)
    static_assert(PW == 4 || PW == 2, "one 16- or 8-byte fetch per thread");
    __shared__ float4 init_tab[4][2][2][4]; // [position][half][m][4 x 4 channels]: -(theta + sum w) / 2
    __shared__ uint32_t words[2][TILE];     // [buffer][row][word][pixel]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int p = __builtin_amdgcn_readfirstlane(tid >> 6);           // position of this wave
    const int ct = blockIdx.y;                                        // 64-channel output tile
    const int col = lane & 31, half = lane >> 5;
    const int Cow = Cout >> 5;
    const int dy = p >> 1, dx = p & 1;
    const uint32_t psel = half ? 0x07060302u : 0x05040100u;

    if (tid < 64) {   // thread (position, h, m, q) writes one float4 of the table (visible after the first barrier)
        const int pp = tid >> 4, h = (tid >> 3) & 1, m = (tid >> 2) & 1, q = tid & 3;
        const int cbase = ct * 64 + m * 32 + 16 * h + 4 * q;
        int4 t = make_int4(0, 0, 0, 0), u = make_int4(0, 0, 0, 0);
        if (cbase < Cout) {
            t = *reinterpret_cast<const int4 *>(thresh + cbase);
            u = *reinterpret_cast<const int4 *>(wsum + (size_t)pp * cout_pad64 + cbase);
        }
        init_tab[pp][h][m][q] = make_float4(start_value(t.x, u.x), start_value(t.y, u.y),
                                            start_value(t.z, u.z), start_value(t.w, u.w));
    }

    const __amdgpu_buffer_rsrc_t ars =
        __builtin_amdgcn_make_buffer_rsrc((void *)act, 0, N * H * W * CW * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t ors =
        __builtin_amdgcn_make_buffer_rsrc((void *)out_bits, 0, N * H * W * 4 * Cow * 4, 0x00020000);
    const uint32_t out_lane = (ct * 2 + half < Cow) ? (uint32_t)(((2 * col + dx) * Cow + ct * 2 + half) * 4) : BAD;

    // ---- the weights of this wave: [tile64][step][position][m][lane]
    v4i Wt[KS][2];
    {
        const uint4 *wk = wfrag + (size_t)ct * KS * 8 * 64 + lane;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const uint4 a = wk[((ks * 4 + p) * 2 + m) * 64];
                Wt[ks][m] = (v4i){(int)a.x, (int)a.y, (int)a.z, (int)a.w};
            }
    }

    // ---- staging: thread tid fetches words k0 .. k0 + PW - 1 of pixel spx of row sr of the group
    constexpr int PIECES = CW / PW;                    // fetches per pixel
    const int sr = tid / (32 * PIECES);
    const int spx = (tid / PIECES) % 32;
    const int k0 = (tid % PIECES) * PW;
    uint32_t *const swr = &words[0][(sr * CW + k0) * 32 + spx];     // + buffer * TILE, + 32 per word
    // ---- this lane's reads: word 2 ks + half of pixel col of row r
    const uint32_t *const srd = &words[0][half * 32 + col];         // + (r * CW + 2 ks) * 32

    struct Plan { int gx, gy, n; };
    auto plan = [&](int g) {
        Plan P;
        P.gx = g % groups_x;
        const int q = g / groups_x;
        P.gy = q % groups_y;
        P.n = q / groups_y;
        return P;
    };
    // the fetched words of a group, two groups ahead of the one being multiplied (two register
    // sets alternate): a fetch has two group times to arrive
    auto fetch = [&](const Plan &P, uint32_t (&st)[PW]) {
        const int x = P.gx * 32 + spx, y = P.gy * RGX + sr;
        // a pixel outside the image: any offset beyond the tensor (reads 0; masked at expansion)
        const uint32_t off = (x < W && y < H) ? (uint32_t)((((P.n * H + y) * W + x) * CW + k0) * 4) : BAD;
        if (PW == 4) {
            const auto v = __builtin_amdgcn_raw_buffer_load_b128(ars, off, 0, 0);
#pragma unroll
            for (int i = 0; i < PW; ++i) st[i] = v[i];
        } else {
            const auto v = __builtin_amdgcn_raw_buffer_load_b64(ars, off, 0, 0);
#pragma unroll
            for (int i = 0; i < PW; ++i) st[i] = v[i];
        }
    };
    auto commit = [&](int buf, const uint32_t (&st)[PW]) {
#pragma unroll
        for (int i = 0; i < PW; ++i) swr[buf * TILE + i * 32] = st[i];
    };

    // every thread of the block walks over the same groups (and reaches the same barriers)
    const int stride = gridDim.x;
    int g = blockIdx.x;               // < groups: the grid is not larger
    Plan cur = plan(g);
    // a group index past the last one: the words of the block's first group again, unused
    auto plan_or_first = [&](int gi) { return plan(gi < groups ? gi : (int)blockIdx.x); };
    uint32_t sa[PW], sb[PW];
    fetch(cur, sa);
    Plan nxt = plan_or_first(g + stride);
    fetch(nxt, sb);
    commit(0, sa);
    __syncthreads();
    int buf = 0;

    // one group: fetch of group g + 2 stride into sf, matrix work of group g from LDS buffer
    // `buf`, words of group g + stride (in sc since the previous group) into the other buffer.
    // Returns false after the block's last group (the same decision in every thread).
    auto group = [&](const uint32_t (&sc)[PW], uint32_t (&sf)[PW]) -> bool {
        const Plan nn = plan_or_first(g + 2 * stride);
        fetch(nn, sf);
        v16f acc[RGX][2];
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 f = init_tab[p][half][m][q];
#pragma unroll
                for (int r = 0; r < RGX; ++r) {
                    acc[r][m][4 * q] = f.x; acc[r][m][4 * q + 1] = f.y;
                    acc[r][m][4 * q + 2] = f.z; acc[r][m][4 * q + 3] = f.w;
                }
            }
        uint32_t k8[RGX];
#pragma unroll
        for (int r = 0; r < RGX; ++r)
            k8[r] = (cur.gx * 32 + col < W && cur.gy * RGX + r < H) ? 0x22222222u : 0u;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            v4i B[RGX];
#pragma unroll
            for (int r = 0; r < RGX; ++r) {
                const uint32_t m2 = k8[r];
                const uint32_t word = srd[buf * TILE + (r * CW + 2 * ks) * 32];
                B[r] = (v4i){(int)((word << 1) & m2), (int)(word & m2), (int)((word >> 1) & m2),
                             (int)((word >> 2) & m2)};
            }
#pragma unroll
            for (int r = 0; r < RGX; ++r)
#pragma unroll
                for (int m = 0; m < 2; ++m) acc[r][m] = mfma_f4(Wt[ks][m], B[r], acc[r][m]);
        }
        // ---- epilogue: input pixel (y, x) -> output pixel (2y + dy, 2x + dx)
        const uint32_t lane_off = (cur.gx * 32 + col < W) ? out_lane + (uint32_t)(cur.gx * 64 * Cow * 4) : BAD;
#pragma unroll
        for (int r = 0; r < RGX; ++r) {
            const int y = cur.gy * RGX + r;
            uint32_t s0 = 0, s1 = 0;
#pragma unroll
            for (int i = 15; i >= 0; --i) {
                s0 = __builtin_amdgcn_alignbit(s0, __float_as_uint(acc[r][0][i]), 31);
                s1 = __builtin_amdgcn_alignbit(s1, __float_as_uint(acc[r][1][i]), 31);
            }
            const uint32_t word = finish_word64(s0, s1, psel);
            if (y < H) {
                const uint32_t row_off = (uint32_t)((((cur.n * 2 * H + 2 * y + dy) * 2 * W) * Cow) * 4);
                __builtin_amdgcn_raw_buffer_store_b32(word, ors, lane_off + row_off, 0, 0);
            }
        }
        g += stride;
        if (g >= groups) return false;
        buf ^= 1;
        commit(buf, sc);       // the buffer the block read one group ago: every wave has passed
        __syncthreads();       // the barrier since
        cur = nxt;
        nxt = nn;
        return true;
    };
#pragma unroll 1
    for (;;) {
        if (!group(sb, sa)) break;
        if (!group(sa, sb)) break;
    }
}

template <int KS, int RGX>
static int launch_tconv_res(const uint32_t *act, int N, int H, int W, const TconvLayout &L, const uint4 *wfrag,
                            const int32_t *thresh, uint32_t *out_bits, hipStream_t s)
{
    const int groups_x = ceil_div(W, 32), groups_y = ceil_div(H, RGX);
    const long groups = (long)N * groups_y * groups_x;
    if (groups > 0x7fffffffL) return fail(MBU_ERR_SHAPE, "too many pixel groups for one launch");
    const int tiles64 = L.cout_pad64 / 64;
    // two blocks per compute unit in total, spread over the 64-channel tiles
    const int per_tile = (int)std::min(groups, (long)std::max(1, 512 / tiles64));
    const int32_t *wsum = (const int32_t *)((const uint8_t *)wfrag - L.off_f4 + L.off_sum);
    MBU_LAUNCH((tconv_res_kernel<KS, RGX>), dim3((unsigned)per_tile, (unsigned)tiles64), dim3(256), 0, s, act, N, H,
               W, wfrag, L.cout, (int)groups, groups_x, groups_y, thresh, wsum, L.cout_pad64, out_bits);
    return check_launch("tconv2x2_masked_binary");
}

int launch_tconv_mfma(const uint32_t *act, int N, int H, int W, const TconvLayout &L,
                      const void *blob, const int32_t *thresh, uint32_t *out_bits, int32_t *out_acc,
                      hipStream_t s)
{
    const int groups_x = ceil_div(W, 32), groups_y = ceil_div(H, RG);
    const long groups = (long)N * groups_y * groups_x;
    if (groups > 0x7fffffffL) return fail(MBU_ERR_SHAPE, "too many pixel groups for one launch");
    const uint4 *wfrag = (const uint4 *)((const uint8_t *)blob + L.off_f4);
    const int32_t *wsum = (const int32_t *)((const uint8_t *)blob + L.off_sum);
    // packed bits only, at least two input steps, every tensor below 1 GiB: the persistent
    // kernel, two blocks per compute unit spread over the 64-channel tiles
    const int tiles64 = L.cout_pad64 / 64;
    const double GiB = 1073741824.0;
    const bool small = (double)N * H * W * L.cin_words * 4 < GiB && (double)N * H * W * 4 * (L.cout >> 5) * 4 < GiB;
    // 128, 256, 512 or 1024 input channels (an even word count): weights resident
    if (!out_acc && small && L.cin_words == 2 * L.ksteps) {
        if (L.ksteps == 2) return launch_tconv_res<2, 4>(act, N, H, W, L, wfrag, thresh, out_bits, s);
        if (L.ksteps == 4) return launch_tconv_res<4, 4>(act, N, H, W, L, wfrag, thresh, out_bits, s);
        if (L.ksteps == 8) return launch_tconv_res<8, 2>(act, N, H, W, L, wfrag, thresh, out_bits, s);
        if (L.ksteps == 16) return launch_tconv_res<16, 1>(act, N, H, W, L, wfrag, thresh, out_bits, s);
    }
    if (!out_acc && L.ksteps >= 2 && small && (double)L.ksteps * 8 * 1024 < GiB) {
        constexpr int RGF = RG;
        const int gy2 = ceil_div(H, RGF);
        const long groups2 = (long)N * gy2 * groups_x;
        if (groups2 > 0x7fffffffL) return fail(MBU_ERR_SHAPE, "too many pixel groups for one launch");
        const int per_tile = (int)std::min(groups2, (long)std::max(1, 512 / tiles64));
        MBU_LAUNCH(tconv_bits_kernel<RGF>, dim3((unsigned)per_tile, (unsigned)tiles64), dim3(256), 0, s, act, N, H,
                   W, L.cin_words, L.ksteps, wfrag, L.cout, (int)groups2, groups_x, gy2, thresh, wsum, L.cout_pad64,
                   out_bits);
        return check_launch("tconv2x2_masked_binary");
    }
    dim3 grid((unsigned)groups, (unsigned)(L.cout_pad64 / 64));   // 4 waves = the 4 positions
    if (out_acc)
        MBU_LAUNCH(tconv_mfma_kernel<true>, grid, dim3(256), 0, s, act, N, H, W, L.cin_words,
                   L.ksteps, wfrag, L.cout, groups, groups_x, groups_y, thresh, wsum, L.cout_pad64, out_bits, out_acc);
    else
        MBU_LAUNCH(tconv_mfma_kernel<false>, grid, dim3(256), 0, s, act, N, H, W, L.cin_words,
                   L.ksteps, wfrag, L.cout, groups, groups_x, groups_y, thresh, wsum, L.cout_pad64, out_bits, out_acc);
    return check_launch("tconv2x2_masked_binary");
}

}  // namespace mbu
