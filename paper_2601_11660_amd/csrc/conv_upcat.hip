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
// stride-2 fragments are contiguous in LDS; per 128 channels of the low tensor (two steps: a
// low step is only 32 matrix instructions per wave, too few per barrier) a 6 x 34 window.
// Everything else - FP4 codes, 0 / 1 activations and the start value that goes with them (a low
// pixel outside the image is 0.5 like any other), fragments rotating through three registers,
// fetches a step ahead through buffer resources, persistent blocks - is as in conv_mfma.hip.
//
// The window of the NEXT unit is fetched into registers at the start of a unit and expanded and
// written to the other LDS buffer one word per slot between the matrix instructions of the
// unit's later fragments: vector work hides only behind matrix instructions of the same wave.
// The slots are chosen so that every wait is a compile-time count (the staged words are older
// than the weight fragments fetched in the slots before) and the unit bodies are instantiated
// per kind of the next unit, so that no slot contains a branch: with a run-time branch in the
// slots the compiler drains the vector-memory counter there and the kernel gets slower, not
// faster (measured: 47.2 -> 49.9 us with branches, 47.2 -> 44.3 us without, 1536 -> 512).
#include "mbu_internal.h"
#include "mfma_common.h"
#include <algorithm>
#include <type_traits>

namespace mbu {

constexpr int UC_RW = 4;                      // low rows per block tile = output rows per wave
constexpr int UC_A_ROWS = 2 * UC_RW + 2;      // skip window: 10 rows
constexpr int UC_A_COLS = 66;                 //              66 pixels, 33 per column parity
constexpr int UC_A_ROW = 2 * 2 * 33;          // uint4 per window row: [half][parity][33]
constexpr int UC_B_ROWS = UC_RW + 2;          // low window: 6 rows
constexpr int UC_B_COLS = 34;
constexpr int UC_B_ROW = 2 * 34;              // uint4 per window row: [half][34]
constexpr int UC_B_SLICE = UC_B_ROWS * UC_B_ROW;   // one 64-channel slice of the low window
constexpr int UC_TILE = UC_A_ROWS * UC_A_ROW; // the larger of the two windows (2 low slices: 816)

__global__ __launch_bounds__(256, 2) void conv_mfma_upcat_kernel(
    const uint32_t *__restrict__ act, const uint32_t *__restrict__ low, int N, int H, int W, int ksA,
    int ksL, const uint4 *__restrict__ wfrag, const uint4 *__restrict__ wup, int Cout, int tiles64,
    int ptiles, TileStep tstep, const int32_t *__restrict__ thresh, const int32_t *__restrict__ wsum,
    uint32_t *__restrict__ out_bits)
{
    constexpr int RW = UC_RW;
    constexpr int NB = 3;                       // activation fragments in flight per wave
    constexpr int NLA = (UC_A_ROWS * UC_A_COLS + 255) / 256;   // 3 skip pixels per thread
    __shared__ uint4 tile[2][UC_TILE];
    __shared__ float4 init_tab[4][2][2][4];     // [wave][half][m][4 x 4 channels]: start values

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tid = threadIdx.x;
    const int dy = wave >> 1, dx = wave & 1;     // parity class of this wave
    const int col = lane & 31, half = lane >> 5;
    const int Hl = H >> 1, Wl = W >> 1;
    const int Cwa = 2 * ksA, Cwb = 2 * ksL;
    // units of work per tile: ksA steps of 64 skip channels, then ksL / 2 steps of 128 low channels
    // (a low step is only 4 taps: two of them per barrier)
    const int units = ksA + (ksL >> 1);
    const int ct = blockIdx.y;                   // 64-channel output tile of the block

    if (col < 8) {   // lanes (half, col < 8) write float4 number col of their half
        const int m = col >> 2, q = col & 3;
        const int cbase = ct * 64 + m * 32 + 16 * half + 4 * q;
        int4 t = make_int4(0, 0, 0, 0), u = make_int4(0, 0, 0, 0);
        if (cbase < Cout) {
            t = *reinterpret_cast<const int4 *>(thresh + cbase);
            u = *reinterpret_cast<const int4 *>(wsum + cbase);
        }
        init_tab[wave][half][m][q] = make_float4(start_value(t.x, u.x), start_value(t.y, u.y),
                                                 start_value(t.z, u.z), start_value(t.w, u.w));
    }

    const __amdgpu_buffer_rsrc_t ars =
        __builtin_amdgcn_make_buffer_rsrc((void *)act, 0, N * H * W * Cwa * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t brs =
        __builtin_amdgcn_make_buffer_rsrc((void *)low, 0, N * Hl * Wl * Cwb * 4, 0x00020000);
    // 3x3 fragments [tile64][64-channel step][tap][m][lane]; combined fragments
    // [tile64][64-channel step][class][a][b][m][lane] (steps count skip and low channels alike)
    const int steps = ksA + ksL;
    const __amdgpu_buffer_rsrc_t w3 = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(wfrag + (size_t)ct * steps * (18 * 64)), 0, steps * (18 * 1024), 0x00020000);
    const __amdgpu_buffer_rsrc_t wu = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(wup + (size_t)ct * steps * (32 * 64)), 0, steps * (32 * 1024), 0x00020000);
    const int wlane = lane * 16;

    // ---- staging plan.  Skip window: pixel p = tid + 256 j -> window row p / 66, column p % 66
    // (image pixel (2 Y0 - 1 + row, 2 X0 - 1 + column)), stored at [row][half][column parity]
    // [column / 2].  Low window: pixel tid -> row tid / 34, column tid % 34 (low pixel
    // (Y0 - 1 + row, X0 - 1 + column)), stored at [64-channel slice][row][half][column].
    // The LDS positions do not depend on the tile: two registers hold the four of them.
    uint32_t dst01, dst2b;
    {
        int d[NLA];
#pragma unroll
        for (int j = 0; j < NLA; ++j) {
            int p = tid + 256 * j;
            p = p < UC_A_ROWS * UC_A_COLS ? p : 0;      // surplus threads duplicate pixel 0
            const int r = p / UC_A_COLS, c = p - r * UC_A_COLS;
            d[j] = r * UC_A_ROW + (c & 1) * 33 + (c >> 1);
        }
        const int p = tid < UC_B_ROWS * UC_B_COLS ? tid : 0;
        const int r = p / UC_B_COLS, c = p - r * UC_B_COLS;
        dst01 = (uint32_t)d[0] | ((uint32_t)d[1] << 16);
        dst2b = (uint32_t)d[2] | ((uint32_t)(r * UC_B_ROW + c) << 16);
    }
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
    auto stage_issue = [&](int u) {
        if (u < ksA) {
#pragma unroll
            for (int j = 0; j < NLA; ++j) {
                const auto v = __builtin_amdgcn_raw_buffer_load_b64(ars, offa[j], u * 8, 0);
                gq[j] = make_uint2(v[0], v[1]);
            }
        } else {   // four words: two 64-channel slices
            const auto v = __builtin_amdgcn_raw_buffer_load_b128(brs, offb, (u - ksA) * 16, 0);
            gq[0] = make_uint2(v[0], v[1]);
            gq[1] = make_uint2(v[2], v[3]);
        }
    };
    auto expand_store = [&](uint2 g, bool in, uint4 *d0, uint4 *d1) {
        const uint32_t m2 = in ? 0x22222222u : 0u, p1 = in ? 0u : 0x11111111u;
        *d0 = expand_word_masked(g.x, m2, p1);
        *d1 = expand_word_masked(g.y, m2, p1);
    };
    auto stage_commit = [&](int u, uint4 *buf) {
        if (u < ksA) {
#pragma unroll
            for (int j = 0; j < NLA; ++j) {
                const uint32_t at = j == 0 ? (dst01 & 0xffffu) : j == 1 ? (dst01 >> 16) : (dst2b & 0xffffu);
                expand_store(gq[j], (inside >> j) & 1u, buf + at, buf + at + 2 * 33);
            }
        } else {
            const uint32_t at = dst2b >> 16;
#pragma unroll
            for (int q = 0; q < 2; ++q)
                expand_store(gq[q], (inside >> 3) & 1u, buf + q * UC_B_SLICE + at, buf + q * UC_B_SLICE + at + 34);
        }
    };

    // One word of that commit: the staged words of the next unit are expanded and written one per
    // slot between the matrix instructions of the current unit (vector work hides only behind
    // matrix instructions of the same wave).  SKIP: the next unit is a skip step (six words:
    // word i & 1 of staged pixel i >> 1), else a low unit (four words: word i & 1 of slice
    // i >> 1).  Everything but the data is a compile-time constant: no branches in the slots.
    auto commit_word = [&](auto SKIP, uint4 *buf, int i) {
        if constexpr (decltype(SKIP)::value) {
            const int j = i >> 1;
            const uint32_t at = (j == 0 ? (dst01 & 0xffffu) : j == 1 ? (dst01 >> 16) : (dst2b & 0xffffu)) + (i & 1) * (2 * 33);
            const bool in = (inside >> j) & 1u;
            buf[at] = expand_word_masked((i & 1) ? gq[j].y : gq[j].x, in ? 0x22222222u : 0u, in ? 0u : 0x11111111u);
        } else if (i < 4) {
            const int q = i >> 1;
            const uint32_t at = q * UC_B_SLICE + (dst2b >> 16) + (i & 1) * 34;
            const bool in = (inside >> 3) & 1u;
            buf[at] = expand_word_masked((i & 1) ? gq[q].y : gq[q].x, in ? 0x22222222u : 0u, in ? 0u : 0x11111111u);
        }
    };

    // ---- weights of a unit in registers.  Skip step: Wg[kx][ky][m] = tap (ky, kx).  Low double
    // step: the combined taps (a, b) of this wave's class for slice 0 in slots (kx, ky) = (b, a),
    // for slice 1 in slots (2, a) [b = 0] and (a, 2) [b = 1]; slot (2, 2) is idle.
    v4i Wg[3][3][2];
    // One load instruction per fragment whatever the unit's kind: resource and offset are
    // selected with scalar instructions.
    auto load_w = [&](int u, int kx, int ky) {
        const bool up = u >= ksA;
        if (kx == 2 && ky == 2) {
            const int s3 = min(u, ksA - 1);     // idle in a low unit: loaded all the same
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const auto w = __builtin_amdgcn_raw_buffer_load_b128(w3, wlane, (s3 * 18 + 8 * 2 + m) * 1024, 0);
                Wg[2][2][m] = (v4i){(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
            }
            return;
        }
        const int q = (kx < 2 && ky < 2) ? 0 : 1;
        const int b = q == 0 ? kx : (kx == 2 ? 0 : 1);
        const int a = q == 0 ? ky : (kx == 2 ? ky : kx);
        const int sl = ksA + 2 * (u - ksA) + q;          // 64-channel step of the slice
        const __amdgpu_buffer_rsrc_t rs = up ? wu : w3;
        const int off = up ? (sl * 32 + ((wave * 2 + a) * 2 + b) * 2) * 1024 : (u * 18 + (ky * 3 + kx) * 2) * 1024;
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const auto w = __builtin_amdgcn_raw_buffer_load_b128(rs, wlane, off + m * 1024, 0);
            Wg[kx][ky][m] = (v4i){(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
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

    // fragment addresses of this lane (uint4 units from the start of a window buffer): window
    // column 2 col + dx + kx lies in parity plane (dx + kx) & 1 at index col + (dx + kx) / 2
    const int baseX = dy * UC_A_ROW + half * 66 + (dx & 1) * 33 + col;                        // kx = 0; kx = 2: + 1
    const int baseY = dy * UC_A_ROW + half * 66 + ((dx + 1) & 1) * 33 + ((dx + 1) >> 1) + col;  // kx = 1
    const int baseB = dy * UC_B_ROW + half * 34 + dx + col;                                   // + b

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
        auto skip_step = [&](int u, auto NEXT_SKIP) {
            const int un = u + 1;                   // a skip step or the first low unit
            const uint4 *tb = tile[buf];
            stage_issue(un);
            __builtin_amdgcn_sched_barrier(0);
            constexpr int NF = 27;
            v4i fr[NB];
            auto frag = [&](int j) {
                const int kx = j / 9, t = j % 9;
                const uint4 b = tb[(kx == 1 ? baseY : baseX) + (kx == 2 ? 1 : 0) + t * UC_A_ROW];
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
                if (t >= 2 * (RW - 1)) load_w(un, kx, t - 2 * (RW - 1));
                // the next unit's window (fetched at the start of this one): one word per slot of
                // the last tap column, before that column's weight fetches
                if (j >= 18 && j < 24) commit_word(NEXT_SKIP, tile[buf ^ 1], j - 18);
                __builtin_amdgcn_sched_barrier(0);
            }
            buf ^= 1;
            __syncthreads();
        };
        for (int u = 0; u + 1 < ksA; ++u) skip_step(u, std::true_type{});
        skip_step(ksA - 1, std::false_type{});
        // ---- low units: fragment (q, b, t) is slice q, window row dy + t, t = r + a; 20 fragments
        auto low_unit = [&](int u, auto LAST) {
            constexpr bool last = decltype(LAST)::value;
            const int un = last ? 0 : u + 1;        // a low unit, or the next tile's first skip step
            if (last) {
                TilePos nxt = cur;
                if (pt + stride < ptiles) nxt.advance(tstep);
                plan(nxt);
            }
            const uint4 *tb = tile[buf];
            stage_issue(un);
            __builtin_amdgcn_sched_barrier(0);
            constexpr int NF = 20;
            v4i fr[NB];
            auto frag = [&](int j) {
                const int q = j / 10, b = (j % 10) / 5, t = j % 5;
                const uint4 v = tb[q * UC_B_SLICE + baseB + b + t * UC_B_ROW];
                return (v4i){(int)v.x, (int)v.y, (int)v.z, (int)v.w};
            };
#pragma unroll
            for (int j = 0; j < NB; ++j) fr[j] = frag(j);
#pragma unroll
            for (int j = 0; j < NF; ++j) {
                const int q = j / 10, b = (j % 10) / 5, t = j % 5;
#pragma unroll
                for (int a = 0; a < 2; ++a) {
                    const int r = t - a;
                    // slot of the combined tap (a, b) of slice q
                    const int kx = q == 0 ? b : (b == 0 ? 2 : a), ky = q == 0 ? a : (b == 0 ? a : 2);
                    if (r >= 0 && r < RW) {
#pragma unroll
                        for (int m = 0; m < 2; ++m) acc[r][m] = mfma_f4(Wg[kx][ky][m], fr[j % NB], acc[r][m]);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                if (j + NB < NF) fr[j % NB] = frag(j + NB);
                // combined tap (a, b) is done after t = RW - 1 + a: its slot is refilled for the
                // next unit; the idle slot too when the next tile's skip step follows
                if (t >= RW - 1) {
                    const int a = t - (RW - 1);
                    load_w(un, q == 0 ? b : (b == 0 ? 2 : a), q == 0 ? a : (b == 0 ? a : 2));
                }
                if (j == 0 && last) load_w(un, 2, 2);
                // the next unit's window, one word per slot (slots t = 0 .. 2 of the second slice)
                if (j >= 10 && t < 3) commit_word(LAST, tile[buf ^ 1], (j >= 15 ? 3 : 0) + t);
                __builtin_amdgcn_sched_barrier(0);
            }
            buf ^= 1;
            __syncthreads();
        };
        for (int u = ksA; u + 1 < units; ++u) low_unit(u, std::false_type{});
        low_unit(units - 1, std::true_type{});

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
// stores the E2M1 codes of the sums as one
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
                                  (v < 0 ? 8u : 0u);
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
    return (L.sections & MBU_BLOB_SUMMED_TAPS) && out_bits && !out_pool && Ca > 0 && Clow > 0 && Ca % 64 == 0 && Clow % 128 == 0 && !(H & 1) && !(W & 1) &&
           (double)N * H * W * (Ca / 32) * 4 < lim && (double)N * (H / 2) * (W / 2) * (Clow / 32) * 4 < lim &&
           (double)L.ksteps * 32 * 1024 < lim;
}

int launch_conv_mfma_upcat(const uint32_t *act, int Ca, const uint32_t *low, int Clow, int N, int H, int W,
                           const BlobLayout &L, const void *blob, const int32_t *thresh, uint32_t *out_bits,
                           hipStream_t s)
{
    const uint4 *wfrag = (const uint4 *)((const uint8_t *)blob + L.off_f4);
    const uint4 *wup = (const uint4 *)((const uint8_t *)blob + L.off_up);
    // sums of the weights per output channel: row 10 of the count section
    const int32_t *wsum = (const int32_t *)((const uint8_t *)blob + L.off_cnt) + (size_t)10 * L.cout_pad64;
    const int tiles64 = L.cout_pad64 / 64;
    const int tiles_x = ceil_div(W / 2, 32), tiles_y = ceil_div(H / 2, UC_RW);
    const long tiles = (long)N * tiles_y * tiles_x;
    if (tiles > 0x7fffffffL) return fail(MBU_ERR_SHAPE, "too many tiles for one launch");
    // persistent blocks: two per compute unit in total, spread over the 64-channel tiles
    const int gx = (int)std::min(tiles, (long)std::max(1, 512 / tiles64));
    const TileStep tstep = tile_step(gx, tiles_x, tiles_y);
    MBU_LAUNCH(conv_mfma_upcat_kernel, dim3((unsigned)gx, (unsigned)tiles64), dim3(256), 0, s, act, low, N, H, W,
               Ca / 64, Clow / 64, wfrag, wup, L.cout, tiles64, (int)tiles, tstep, thresh, wsum, out_bits);
    return check_launch("conv_mfma_upcat");
}

}  // namespace mbu
