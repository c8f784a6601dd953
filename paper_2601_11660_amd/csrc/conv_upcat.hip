// Masked-binary 3x3 convolution over [skip | 2x nearest up-sampled low] (Sec. 2.1: the decoder
// concatenates encoder features with the up-sampled decoder features), with the up-sampled
// part contracted at LOW resolution.
//
// Output pixel (2Y + dy, 2X + dx) sees the up-sampled image through its 3x3 window, but the
// nine taps fall on only 2 x 2 low-resolution pixels: rows {Y - 1, Y, Y} for dy = 0 and
// {Y, Y, Y + 1} for dy = 1, columns alike.  Summing the weights of the taps that share a low
// pixel gives, per parity class (dy, dx), a 2x2 kernel with entries in -4 .. 4 over the low
// tensor; zero padding of the up-sampled image is zero padding of the low tensor.  The FP4
// format (E2M1) holds 0, 1, 2, 3, 4 exactly, products and sums stay exact integers in fp32,
// so the result is bit-identical to the layer on the materialised tensor while the up-sampled
// channels cost 4 instead of 9 matrix instructions per step: with twice as many low channels
// as skip channels, 17/27 of the work.
//
// The four waves of a block are the four parity classes of the same 4 x 32 low pixels
// (8 x 64 output pixels) and 64 output channels: a wave's 32 matrix columns are output pixels
// of one class, i.e. every second pixel of every second row, and its accumulator tile is
// 4 rows x 32 columns x 64 channels as in the other kernels.  Per 64-channel step of the skip
// tensor the block stages a 10 x 66 pixel window, columns split by parity so that a wave's
// stride-2 fragments are contiguous in LDS; per step of the low tensor a 6 x 34 window.
// Everything else - FP4 codes, -theta start, fragments rotating through three registers,
// fetches a step ahead through buffer resources, persistent blocks - is as in conv_mfma.hip.
#include "mbu_internal.h"
#include "mfma_common.h"
#include <algorithm>

namespace mbu {

constexpr int UC_RW = 4;                      // low rows per block tile = output rows per wave
constexpr int UC_A_ROWS = 2 * UC_RW + 2;      // skip window: 10 rows
constexpr int UC_A_COLS = 66;                 //              66 pixels, 33 per column parity
constexpr int UC_A_ROW = 2 * 2 * 33;          // uint4 per window row: [half][parity][33]
constexpr int UC_B_ROWS = UC_RW + 2;          // low window: 6 rows
constexpr int UC_B_COLS = 34;
constexpr int UC_B_ROW = 2 * 34;              // uint4 per window row: [half][34]
constexpr int UC_TILE = UC_A_ROWS * UC_A_ROW; // the larger of the two windows

__global__ __launch_bounds__(256, 2) void conv_mfma_upcat_kernel(
    const uint32_t *__restrict__ act, const uint32_t *__restrict__ low, int N, int H, int W, int ksA,
    int ksL, const uint4 *__restrict__ wfrag, const uint4 *__restrict__ wup, int Cout, int tiles64,
    int ptiles, TileStep tstep, const int32_t *__restrict__ thresh, uint32_t *__restrict__ out_bits)
{
    constexpr int RW = UC_RW;
    constexpr int NB = 3;                       // activation fragments in flight per wave
    constexpr int NLA = (UC_A_ROWS * UC_A_COLS + 255) / 256;   // 3 skip pixels per thread
    __shared__ uint4 tile[2][UC_TILE];
    __shared__ float4 init_tab[4][2][2][4];     // [wave][half][m][4 x 4 channels]: -theta

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tid = threadIdx.x;
    const int dy = wave >> 1, dx = wave & 1;     // parity class of this wave
    const int col = lane & 31, half = lane >> 5;
    const int Hl = H >> 1, Wl = W >> 1;
    const int Cwa = 2 * ksA, Cwb = 2 * ksL;
    const int steps = ksA + ksL;
    const int ct = blockIdx.y;                   // 64-channel output tile of the block

    if (col < 8) {   // lanes (half, col < 8) write float4 number col of their half
        const int m = col >> 2, q = col & 3;
        const int cbase = ct * 64 + m * 32 + 16 * half + 4 * q;
        int4 t = make_int4(0, 0, 0, 0);
        if (cbase < Cout) t = *reinterpret_cast<const int4 *>(thresh + cbase);
        float4 f;
        f.x = 0.0f - (float)max(-(1 << 22), min(1 << 22, t.x));
        f.y = 0.0f - (float)max(-(1 << 22), min(1 << 22, t.y));
        f.z = 0.0f - (float)max(-(1 << 22), min(1 << 22, t.z));
        f.w = 0.0f - (float)max(-(1 << 22), min(1 << 22, t.w));
        init_tab[wave][half][m][q] = f;
    }

    const __amdgpu_buffer_rsrc_t ars =
        __builtin_amdgcn_make_buffer_rsrc((void *)act, 0, N * H * W * Cwa * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t brs =
        __builtin_amdgcn_make_buffer_rsrc((void *)low, 0, N * Hl * Wl * Cwb * 4, 0x00020000);
    // 3x3 fragments [tile64][skip+low steps][tap][m][lane]; combined fragments
    // [tile64][skip+low steps][class][a][b][m][lane] (only the low steps of either are read)
    const __amdgpu_buffer_rsrc_t w3 = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(wfrag + (size_t)ct * steps * (18 * 64)), 0, steps * (18 * 1024), 0x00020000);
    const __amdgpu_buffer_rsrc_t wu = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(wup + (size_t)ct * steps * (32 * 64)), 0, steps * (32 * 1024), 0x00020000);
    const int wlane = lane * 16;

    // ---- staging plan.  Skip window: pixel p = tid + 256 j -> window row p / 66, column p % 66
    // (image pixel (2 Y0 - 1 + row, 2 X0 - 1 + column)), stored at [row][half][column parity]
    // [column / 2].  Low window: pixel tid -> row tid / 34, column tid % 34 (low pixel
    // (Y0 - 1 + row, X0 - 1 + column)), stored at [row][half][column].
    uint32_t offa[NLA], offb;     // byte offsets of the (clamped) pixels
    uint32_t inside = 0;          // bits 0..2: skip pixels inside the image; bit 3: low pixel
    auto plan = [&](const TilePos &tp) {
        const int Y0 = tp.ty * RW, X0 = tp.tx * 32, n = tp.n;
        inside = 0;
#pragma unroll
        for (int j = 0; j < NLA; ++j) {
            int p = tid + 256 * j;
            p = p < UC_A_ROWS * UC_A_COLS ? p : 0;
            const int r = p / UC_A_COLS, c = p - r * UC_A_COLS;
            const int yy = 2 * Y0 - 1 + r, xx = 2 * X0 - 1 + c;
            const bool in = yy >= 0 && yy < H && xx >= 0 && xx < W;
            const int yc = min(max(yy, 0), H - 1), xc = min(max(xx, 0), W - 1);
            offa[j] = (uint32_t)((((n * H + yc) * W + xc) * Cwa) * 4);
            inside |= (in ? 1u : 0u) << j;
        }
        {
            const int p = tid < UC_B_ROWS * UC_B_COLS ? tid : 0;
            const int r = p / UC_B_COLS, c = p - r * UC_B_COLS;
            const int yy = Y0 - 1 + r, xx = X0 - 1 + c;
            const bool in = yy >= 0 && yy < Hl && xx >= 0 && xx < Wl;
            const int yc = min(max(yy, 0), Hl - 1), xc = min(max(xx, 0), Wl - 1);
            offb = (uint32_t)((((n * Hl + yc) * Wl + xc) * Cwb) * 4);
            inside |= (in ? 1u : 0u) << 3;
        }
    };
    uint2 gq[NLA];
    auto stage_issue = [&](int s) {
        if (s < ksA) {
#pragma unroll
            for (int j = 0; j < NLA; ++j) {
                const auto v = __builtin_amdgcn_raw_buffer_load_b64(ars, offa[j], s * 8, 0);
                gq[j] = make_uint2(v[0], v[1]);
            }
        } else {
            const auto v = __builtin_amdgcn_raw_buffer_load_b64(brs, offb, (s - ksA) * 8, 0);
            gq[0] = make_uint2(v[0], v[1]);
        }
    };
    auto expand_store = [&](uint2 g, bool in, uint4 *d0, uint4 *d1) {
        const uint32_t k8 = in ? 0x88888888u : 0u, k2 = k8 >> 2;
        const uint32_t a = g.x, b = g.y;
        uint4 e0, e1;
        e0.x = ((a << 3) & k8) | k2; e0.y = ((a << 2) & k8) | k2;
        e0.z = ((a << 1) & k8) | k2; e0.w = (a & k8) | k2;
        e1.x = ((b << 3) & k8) | k2; e1.y = ((b << 2) & k8) | k2;
        e1.z = ((b << 1) & k8) | k2; e1.w = (b & k8) | k2;
        *d0 = e0;
        *d1 = e1;
    };
    auto commit_skip = [&](uint4 *buf) {
#pragma unroll
        for (int j = 0; j < NLA; ++j) {
            int p = tid + 256 * j;
            p = p < UC_A_ROWS * UC_A_COLS ? p : 0;      // surplus threads duplicate pixel 0
            const int r = p / UC_A_COLS, c = p - r * UC_A_COLS;
            uint4 *d = buf + r * UC_A_ROW + (c & 1) * 33 + (c >> 1);
            expand_store(gq[j], (inside >> j) & 1u, d, d + 2 * 33);
        }
    };
    auto commit_low = [&](uint4 *buf) {
        const int p = tid < UC_B_ROWS * UC_B_COLS ? tid : 0;
        const int r = p / UC_B_COLS, c = p - r * UC_B_COLS;
        uint4 *d = buf + r * UC_B_ROW + c;
        expand_store(gq[0], (inside >> 3) & 1u, d, d + 34);
    };
    auto stage_commit = [&](int s, uint4 *buf) {
        if (s < ksA) commit_skip(buf);
        else commit_low(buf);
    };

    // ---- weights of a step in registers: Wg[kx][ky][m] for a skip step; a low step uses the
    // four slots kx = b < 2, ky = a < 2 for the combined taps (a, b) of this wave's class
    v4i Wg[3][3][2];
    // fragments of step s into slot (kx, ky): the 3x3 tap (ky, kx), or - for a low step, slots
    // kx, ky < 2 only - the combined tap (a, b) = (ky, kx) of this wave's class.  One load
    // instruction either way: resource and offset are selected with scalar instructions.
    auto load_w = [&](int s, int kx, int ky) {
        const bool up = s >= ksA;
        if (kx < 2 && ky < 2) {
            const __amdgpu_buffer_rsrc_t rs = up ? wu : w3;
            const int off = up ? (s * 32 + ((wave * 2 + ky) * 2 + kx) * 2) * 1024 : (s * 18 + (ky * 3 + kx) * 2) * 1024;
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const auto w = __builtin_amdgcn_raw_buffer_load_b128(rs, wlane, off + m * 1024, 0);
                Wg[kx][ky][m] = (v4i){(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
            }
        } else {
            // a low step does not use this slot: it is loaded all the same (from the last skip step)
            const int s3 = min(s, ksA - 1);
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const auto w = __builtin_amdgcn_raw_buffer_load_b128(w3, wlane, (s3 * 18 + (ky * 3 + kx) * 2 + m) * 1024, 0);
                Wg[kx][ky][m] = (v4i){(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
            }
        }
    };

    const int stride = gridDim.x;
    TilePos cur = tile_pos(blockIdx.x, tstep.tiles_x, tstep.tiles_y);
    plan(cur);
    stage_issue(0);
#pragma unroll
    for (int kx = 0; kx < 3; ++kx)
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) load_w(0, kx, ky);
    stage_commit(0, tile[0]);
    __syncthreads();

    // fragment addresses of this lane (uint4 units from the start of a window buffer)
    int baseA[3], baseB[2];
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) {
        const int s = dx + kx;                  // window column = 2 * col + s
        baseA[kx] = dy * UC_A_ROW + half * 66 + (s & 1) * 33 + (s >> 1) + col;
    }
#pragma unroll
    for (int b = 0; b < 2; ++b) baseB[b] = dy * UC_B_ROW + half * 34 + dx + b + col;

    const int Cow = Cout >> 5;
    const int widx = ct * 2 + half;
    const uint32_t psel = half ? 0x07060302u : 0x05040100u;
    int buf = 0;
    for (int pt = blockIdx.x; pt < ptiles; pt += stride) {
        v16f acc[RW][2];
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 f = init_tab[wave][half][m][q];
#pragma unroll
                for (int r = 0; r < RW; ++r) {
                    acc[r][m][4 * q] = f.x; acc[r][m][4 * q + 1] = f.y;
                    acc[r][m][4 * q + 2] = f.z; acc[r][m][4 * q + 3] = f.w;
                }
            }

        // ---- skip steps: fragment (kx, t) is window row dy + t, t = 2 r + ky; 27 fragments
        for (int s = 0; s < ksA; ++s) {
            const int sn = s + 1;                   // a skip step or the first low step
            const uint4 *tb = tile[buf];
            stage_issue(sn);
            __builtin_amdgcn_sched_barrier(0);
            constexpr int NF = 27;
            v4i fr[NB];
            auto frag = [&](int j) {
                const uint4 b = tb[baseA[j / 9] + (j % 9) * UC_A_ROW];
                return (v4i){(int)b.x, (int)b.y, (int)b.z, (int)b.w};
            };
#pragma unroll
            for (int j = 0; j < NB; ++j) fr[j] = frag(j);
#pragma unroll
            for (int j = 0; j < NF; ++j) {
                const int kx = j / 9, t = j % 9;
#pragma unroll
                for (int ky = 0; ky < 3; ++ky) {
                    const int r2 = t - ky;
                    if (r2 >= 0 && (r2 & 1) == 0 && r2 / 2 < RW) {
#pragma unroll
                        for (int m = 0; m < 2; ++m)
                            acc[r2 / 2][m] = mfma_f4(Wg[kx][ky][m], fr[j % NB], acc[r2 / 2][m]);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                if (j + NB < NF) fr[j % NB] = frag(j + NB);
                // tap (ky, kx) is done after t = 2 (RW - 1) + ky
                if (t >= 2 * (RW - 1)) load_w(sn, kx, t - 2 * (RW - 1));
                __builtin_amdgcn_sched_barrier(0);
            }
            buf ^= 1;
            stage_commit(sn, tile[buf]);
            __syncthreads();
        }
        // ---- low steps: fragment (b, t) is window row dy + t, t = r + a; 10 fragments
        for (int s = ksA; s < steps; ++s) {
            const bool last = s + 1 == steps;
            const int sn = last ? 0 : s + 1;        // a low step, or the next tile's first skip step
            if (last) {
                TilePos nxt = cur;
                if (pt + stride < ptiles) nxt.advance(tstep);
                plan(nxt);
            }
            const uint4 *tb = tile[buf];
            stage_issue(sn);
            __builtin_amdgcn_sched_barrier(0);
            constexpr int NF = 10;
            v4i fr[NB];
            auto frag = [&](int j) {
                const uint4 b = tb[baseB[j / 5] + (j % 5) * UC_B_ROW];
                return (v4i){(int)b.x, (int)b.y, (int)b.z, (int)b.w};
            };
#pragma unroll
            for (int j = 0; j < NB; ++j) fr[j] = frag(j);
#pragma unroll
            for (int j = 0; j < NF; ++j) {
                const int b = j / 5, t = j % 5;
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    const int r = t - a;
                    if (r >= 0 && r < RW) {
#pragma unroll
                        for (int m = 0; m < 2; ++m) acc[r][m] = mfma_f4(Wg[b][a][m], fr[j % NB], acc[r][m]);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                if (j + NB < NF) fr[j % NB] = frag(j + NB);
                // combined tap (a, b) is done after t = RW - 1 + a; the slots a low step does
                // not use are refilled along the way when the next tile's skip step follows
                if (t >= RW - 1) load_w(sn, b, t - (RW - 1));
                if (last) {
                    if (t == 0) load_w(sn, b, 2);
                    if (b == 0 && t >= 1 && t <= 3) load_w(sn, 2, t - 1);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            buf ^= 1;
            stage_commit(sn, tile[buf]);
            __syncthreads();
        }

        // ---- epilogue: row r of the wave is output row 2 (Y0 + r) + dy, column col is output
        // column 2 (X0 + col) + dx
        const int n = cur.n;
        const int x = 2 * (cur.tx * 32 + col) + dx;
        const bool ok = x < W && widx < Cow;
        uint32_t sgn[RW][2];
#pragma unroll
        for (int i = 15; i >= 0; --i)
#pragma unroll
            for (int r = 0; r < RW; ++r)
#pragma unroll
                for (int m = 0; m < 2; ++m)
                    sgn[r][m] = __builtin_amdgcn_alignbit(i == 15 ? 0u : sgn[r][m],
                                                          __float_as_uint(acc[r][m][i]), 31);
#pragma unroll
        for (int r = 0; r < RW; ++r) {
            const uint32_t word = finish_word64(sgn[r][0], sgn[r][1], psel);
            const int y = 2 * (cur.ty * RW + r) + dy;
            if (ok && y < H) out_bits[(((size_t)n * H + y) * W + x) * Cow + widx] = word;
        }
        cur.advance(tstep);
    }
}

// Combined weights of the up-sampled channels.  Thread (o, class, a, b, word k) sums the taps
// of the 3x3 kernel that fall on low pixel (a, b) of class (dy, dx) for 32 input channels and
// stores the E2M1 codes of the NEGATED sums (the activation side is negated too) as one
// 16-byte fragment: uint4 [cout_pad64/64][ksteps][class][a][b][2][64 lanes], nibble q of dword d
// = input channel 32k + 4q + d, lane = 32 (k & 1) + tile row of the output channel.
__global__ __launch_bounds__(256) void pack_upcat_kernel(const int8_t *__restrict__ w, BlobLayout L,
                                                         uint8_t *__restrict__ blob)
{
    const int words = 2 * L.ksteps;
    const long total = (long)L.cout_pad64 * 16 * words;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total) return;
    const int k = (int)(idx % words);
    const int tab = (int)((idx / words) % 16);
    const int o = (int)(idx / (16L * words));
    const int cls = tab >> 2, a = (tab >> 1) & 1, b = tab & 1;
    const int dy = cls >> 1, dx = cls & 1;
    // rows of the 3x3 kernel on low row a: dy = 0: {0}, {1, 2};  dy = 1: {0, 1}, {2}
    const int ky0 = dy == 0 ? (a ? 1 : 0) : (a ? 2 : 0), ky1 = dy == 0 ? (a ? 2 : 0) : (a ? 2 : 1);
    const int kx0 = dx == 0 ? (b ? 1 : 0) : (b ? 2 : 0), kx1 = dx == 0 ? (b ? 2 : 0) : (b ? 2 : 1);
    uint32_t d[4] = {0, 0, 0, 0};
    if (o < L.cout && k < L.cin_words) {
        const int n = min(32, L.cin - k * 32);
        for (int i = 0; i < n; ++i) {
            int v = 0;
            for (int ky = ky0; ky <= ky1; ++ky)
                for (int kx = kx0; kx <= kx1; ++kx) v += w[((long)o * 9 + ky * 3 + kx) * L.cin + (long)k * 32 + i];
            const int mag = v < 0 ? -v : v;     // 0..4 -> E2M1 0, 1.0, 2.0, 3.0, 4.0
            const uint32_t code = (mag == 0 ? 0u : mag == 1 ? 2u : mag == 2 ? 4u : mag == 3 ? 5u : 6u) |
                                  (v > 0 ? 8u : 0u);
            d[i & 3] |= code << (4 * (i >> 2));
        }
    }
    const int tile64 = o >> 6, m = (o >> 5) & 1;
    const int row = tile_channel_to_row(o & 31);
    const int lane = (k & 1) * 32 + row;
    uint4 *F = reinterpret_cast<uint4 *>(blob + L.off_up);
    const size_t at = (((((size_t)tile64 * L.ksteps + (k >> 1)) * 4 + cls) * 4 + a * 2 + b) * 2 + m) * 64 + lane;
    F[at] = make_uint4(d[0], d[1], d[2], d[3]);
}

int launch_pack_upcat(const int8_t *w, const BlobLayout &L, void *blob, hipStream_t s)
{
    const long total = (long)L.cout_pad64 * 16 * 2 * L.ksteps;
    MBU_LAUNCH(pack_upcat_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, w, L, (uint8_t *)blob);
    return check_launch("pack_upcat_weights");
}

bool conv_upcat_supported(int Ca, int Clow, int N, int H, int W, const BlobLayout &L, const uint32_t *out_bits,
                          const uint32_t *out_pool)
{
    const double lim = 1073741824.0;   // byte offsets are computed in 32 bits
    return out_bits && !out_pool && Ca > 0 && Clow > 0 && Ca % 64 == 0 && Clow % 64 == 0 && !(H & 1) && !(W & 1) &&
           (double)N * H * W * (Ca / 32) * 4 < lim && (double)N * (H / 2) * (W / 2) * (Clow / 32) * 4 < lim &&
           (double)L.ksteps * 32 * 1024 < lim;
}

int launch_conv_mfma_upcat(const uint32_t *act, int Ca, const uint32_t *low, int Clow, int N, int H, int W,
                           const BlobLayout &L, const void *blob, const int32_t *thresh, uint32_t *out_bits,
                           hipStream_t s)
{
    const uint4 *wfrag = (const uint4 *)((const uint8_t *)blob + L.off_f4);
    const uint4 *wup = (const uint4 *)((const uint8_t *)blob + L.off_up);
    const int tiles64 = L.cout_pad64 / 64;
    const int tiles_x = ceil_div(W / 2, 32), tiles_y = ceil_div(H / 2, UC_RW);
    const long tiles = (long)N * tiles_y * tiles_x;
    if (tiles > 0x7fffffffL) return fail(MBU_ERR_SHAPE, "too many tiles for one launch");
    // persistent blocks: two per compute unit in total, spread over the 64-channel tiles
    const int gx = (int)std::min(tiles, (long)std::max(1, 512 / tiles64));
    const TileStep tstep = tile_step(gx, tiles_x, tiles_y);
    MBU_LAUNCH(conv_mfma_upcat_kernel, dim3((unsigned)gx, (unsigned)tiles64), dim3(256), 0, s, act, low, N, H, W,
               Ca / 64, Clow / 64, wfrag, wup, L.cout, tiles64, (int)tiles, tstep, thresh, out_bits);
    return check_launch("conv_mfma_upcat");
}

}  // namespace mbu
