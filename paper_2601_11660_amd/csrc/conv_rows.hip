// Masked-binary 3x3 convolution on the matrix cores for layers with at most 64 input
// channels (one 64-channel step): row-streaming kernel.  A second kernel at the end of the file
// applies the scheme to layers with two steps.
//
// With a single input step the contraction of a tile is short (18 matrix instructions per
// image row of 32 pixels x 64 channels) and the vector work around it - expanding the staged
// bits to 4-bit codes, collecting the output signs - costs about 60 % of the matrix time when
// it runs as a separate phase: vector instructions only hide behind matrix instructions of the
// same wave.  This kernel therefore has no phases.  A wave owns a strip of 32 pixel columns
// and 64 output channels, keeps the 18 weight fragments of the layer in registers for its
// whole life and walks down the image one row at a time.  Every row is 18 matrix
// instructions with one small piece of vector work slotted behind each of them:
//   - the three activation rows a 3x3 window touches are held in registers as 9 fragments
//     (3 rows x 3 tap columns); the row that enters is read from LDS into the registers of
//     the row that left, right after the 6 instructions of that tap row, and the roles of the
//     three fragment rows rotate (the loop body is six rows long: 3 roles x 2 accumulator
//     sets; a remainder of 2 or 4 rows moves the window by register copies instead);
//   - the halo row that enters the window two rows later is expanded from bits to codes and
//     written to one of two row slots in LDS; its bits were fetched from global memory two
//     rows earlier;
//   - the signs of the PREVIOUS row's accumulators (two accumulator sets alternate) are
//     collected, completed to words and stored - and, for a layer followed by 2x2 max pooling
//     (Sec. 2.1: OR of the bits), every second row also stores the pooled words.
// Accumulators start at -(theta + sum w) / 2 (activations enter as 0 / 1, mfma_common.h) through
// the addend of the row's first instruction per tile.
// No barriers, nothing shared between waves.
#include "mbu_internal.h"
#include "mfma_common.h"
#include <algorithm>

namespace mbu {

constexpr int RS_HW = 34;               // halo pixels per staged row
constexpr int RS_ROW = 2 * RS_HW;       // uint4 entries per staged row: [half][pixel]
constexpr int RS_RING = 2;              // staged rows kept in LDS
constexpr uint32_t RS_BAD_LANE = 0x40000000u;   // byte offsets that no tensor of < 2^30 bytes reaches
constexpr uint32_t RS_BAD_ROW = 0x80000000u;

#define RS_FENCE() __builtin_amdgcn_sched_barrier(0)
#define RS_PIN(x) asm volatile("" : "+v"(x))

struct RowsCtx {
    __amdgpu_buffer_rsrc_t in, out, pool;
    uint32_t in_voff;      // byte offset of this lane's halo pixel inside an image row
    uint32_t mx2;          // 0x22222222 when that pixel's column lies inside the image
    uint32_t out_voff;     // byte offset of this lane's output word inside an image row
    uint32_t pool_voff;    // ... of its pooled word inside a pooled row
    uint32_t psel;
    uint4 *wr;             // LDS: this lane's staged pixel, ring slot 0, word 0
    const uint4 *rd;       // LDS: this lane's fragment of tap column 0, ring slot 0
    int H, y0;
    int in_row_bytes, out_row_bytes, pool_row_bytes;
    // second input of the two-source form of the two-step kernel: words 2 and 3 of a pixel come
    // from a tensor of Hb rows (it may cover less than the frame: zeros where it has no pixel)
    __amdgpu_buffer_rsrc_t in2;
    uint32_t in2_voff, mx2b;
    int Hb, in2_row_bytes;
};

// the two packed words of this lane's halo pixel in image row yy (clamped into the image)
__device__ __forceinline__ void fetch_row(const RowsCtx &c, int yy, uint2 &g, bool even)
{
    const int yc = min(max(yy, 0), c.H - 1);
    const int soff = yc * c.in_row_bytes;
    if (even) {
        const auto v = __builtin_amdgcn_raw_buffer_load_b64(c.in, c.in_voff, soff, 0);
        g.x = v[0];
        g.y = v[1];
    } else {
        g.x = __builtin_amdgcn_raw_buffer_load_b32(c.in, c.in_voff, soff, 0);
        g.y = 0u;
    }
}

// sign words of one finished row: stores the row's words and, on odd rows, the pooled words
template <bool POOL, bool ODD>
__device__ __forceinline__ void store_row(const RowsCtx &c, uint32_t s, int i_row, uint32_t &wkeep)
{
    // s: bit k = sign of channel k + 16 * half of tile k / 16 ... (see collection order below)
    const uint32_t mine = ~s;
    const auto sw = __builtin_amdgcn_permlane32_swap(mine, mine, false, false);
    const uint32_t word = __builtin_amdgcn_perm(sw[1], sw[0], c.psel);
    const uint32_t roff = i_row >= 0 ? (uint32_t)((c.y0 + i_row) * c.out_row_bytes) : RS_BAD_ROW;
    __builtin_amdgcn_raw_buffer_store_b32(word, c.out, c.out_voff + roff, 0, 0);
    if (POOL) {
        if (!ODD) {
            wkeep = word;
        } else {
            uint32_t v = wkeep | word;
            // neighbouring lane (quad permute [1,0,3,2]) holds the next pixel of the row
            v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, true);
            const uint32_t poff =
                i_row >= 0 ? (uint32_t)(((c.y0 + i_row) >> 1) * c.pool_row_bytes) : RS_BAD_ROW;
            __builtin_amdgcn_raw_buffer_store_b32(v, c.pool, c.pool_voff + poff, 0, 0);
        }
    }
}

// One image row; P = parity of the row index i: accumulator set, ring slots and fetch register.
// F[(R3 + k) % 3] holds the fragments of halo row i + k (image row y0 + i + k - 1).  With COPY
// the window moves down by register copies and R3 stays 0; without, the row that enters takes
// the registers of the row that left and the caller steps R3 (three steps bring it back).
template <bool CW_EVEN, bool POOL, int P, int R3, bool COPY>
__device__ __forceinline__ void rows_step(const RowsCtx &c, const int i,
                                          const v4i (&Wg)[3][3][2], const v16f (&init)[2],
                                          v16f (&acc)[2][2], v4i (&F)[3][3], uint2 (&gq)[2], uint32_t &wkeep)
{
    constexpr int CUR = P, PRV = P ^ 1;
    constexpr int RD = P ^ 1, WR = P;      // ring slot of halo row i + 3 / i + 4

    uint32_t a = 0, b = 0, m2 = 0, p1 = 0, l2 = 0, q1 = 0;   // masks of expand_word_masked()
    uint4 e0, e1;
    uint32_t s = 0;
#pragma unroll
    for (int t = 0; t < 18; ++t) {
        const int ky = t / 6, kx = (t % 6) >> 1, m = t & 1;
        acc[CUR][m] = mfma_f4(Wg[kx][ky][m], F[(R3 + ky) % 3][kx], ky == 0 && kx == 0 ? init[m] : acc[CUR][m]);
        RS_FENCE();
        // ---- staging of halo row i + 4 (image row y0 + i + 3): bits fetched two rows ago
        if (t == 0) {
            a = gq[P].x;
            b = gq[P].y;
            const bool rin = c.y0 + i + 3 < c.H;
            m2 = rin ? c.mx2 : 0u;
            p1 = (~m2 >> 1) & 0x11111111u;
            l2 = CW_EVEN ? m2 : 0u;
            q1 = CW_EVEN ? p1 : 0u;
            e0.x = ((a << 1) & m2) | p1;
            RS_PIN(e0.x);
        } else if (t == 1) {
            e0.y = (a & m2) | p1;
            e0.z = ((a >> 1) & m2) | p1;
            RS_PIN(e0.y); RS_PIN(e0.z);
        } else if (t == 2) {
            e0.w = ((a >> 2) & m2) | p1;
            e1.x = ((b << 1) & l2) | q1;
            RS_PIN(e0.w); RS_PIN(e1.x);
        } else if (t == 3) {
            e1.y = (b & l2) | q1;
            e1.z = ((b >> 1) & l2) | q1;
            RS_PIN(e1.y); RS_PIN(e1.z);
        } else if (t == 4) {
            e1.w = ((b >> 2) & l2) | q1;
            RS_PIN(e1.w);
            c.wr[WR * RS_ROW] = e0;
            c.wr[WR * RS_ROW + RS_HW] = e1;
            // halo row i + 6 into the register just consumed
            fetch_row(c, c.y0 + i + 5, gq[P], CW_EVEN);
        }
        // ---- the window moves down one row: a fragment row is overwritten as soon as its tap
        // row has been issued
        if (COPY && (t == 5 || t == 11)) {
            const int k = t / 6;   // F[k] <- F[k + 1]
#pragma unroll
            for (int x = 0; x < 3; ++x) {
                F[k][x] = F[k + 1][x];
                RS_PIN(F[k][x]);
            }
        }
        // the row that enters the window (staged one row ago): with copies into the last
        // fragment row once its instructions are issued, without into the first one
        if (COPY ? t == 17 : t == 5) {
#pragma unroll
            for (int x = 0; x < 3; ++x) {
                const uint4 f = c.rd[RD * RS_ROW + x];
                F[COPY ? 2 : R3 % 3][x] = (v4i){(int)f.x, (int)f.y, (int)f.z, (int)f.w};
            }
        }
        // ---- signs of the previous row: one chain over the 32 registers, second tile first, so
        // that bit k of the result is register k % 16 of tile k / 16
        if (t >= 6 && t < 17) {
            const int first = (t - 6) * 3, last = min(first + 3, 32);
#pragma unroll
            for (int e = first; e < last; ++e) {
                const int mm = 1 - e / 16, r = 15 - e % 16;
                s = __builtin_amdgcn_alignbit(s, __float_as_uint(acc[PRV][mm][r]), 31);
            }
            RS_PIN(s);
        }
        if (t == 17) {
            // row i - 1 is odd when i is even; it exists unless i = 0
            const bool valid = P == 1 || i > 0;
            store_row<POOL, P == 0>(c, s, valid ? i - 1 : -1, wkeep);
        }
        RS_FENCE();
    }
}

template <bool CW_EVEN, bool POOL, int WPS>
__global__ __launch_bounds__(256, WPS) void conv_mfma_rows_kernel(
    const uint32_t *__restrict__ act, int H, int W, int Cw, const uint4 *__restrict__ wfrag, int Cout,
    int ctiles, int strips, int nseg, int seg_rows, int units, const int32_t *__restrict__ thresh,
    const int32_t *__restrict__ wsum, uint32_t *__restrict__ out_bits, uint32_t *__restrict__ out_pool)
{
    __shared__ uint4 lds[4][RS_RING * RS_ROW];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int gw = blockIdx.x * 4 + wave;
    if (gw >= units) return;                  // whole wave leaves; nothing is shared
    int q = gw;
    const int ct = q % ctiles; q /= ctiles;   // 64-channel output tile
    const int sx = q % strips; q /= strips;   // strip of 32 pixel columns
    const int sg = q % nseg;                  // segment of seg_rows image rows
    const int n = q / nseg;
    const int col = lane & 31, half = lane >> 5;
    const int Cow = Cout >> 5;
    const int y0 = sg * seg_rows;
    const int rows = min(H, y0 + seg_rows) - y0;

    RowsCtx c;
    c.H = H;
    c.y0 = y0;
    c.in_row_bytes = W * Cw * 4;
    c.out_row_bytes = W * Cow * 4;
    c.pool_row_bytes = (W >> 1) * Cow * 4;
    c.in = __builtin_amdgcn_make_buffer_rsrc((void *)(act + (size_t)n * H * W * Cw), 0, H * c.in_row_bytes,
                                             0x00020000);
    c.out = __builtin_amdgcn_make_buffer_rsrc((void *)(out_bits + (size_t)n * H * W * Cow), 0,
                                              H * c.out_row_bytes, 0x00020000);
    c.pool = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(POOL ? out_pool + (size_t)n * (H >> 1) * (W >> 1) * Cow : out_bits), 0,
        POOL ? (H >> 1) * c.pool_row_bytes : 0, 0x00020000);
    {
        const int p = min(lane, RS_HW - 1);   // surplus lanes duplicate the last halo pixel
        const int xx = sx * 32 + p - 1;
        c.in_voff = (uint32_t)(min(max(xx, 0), W - 1) * Cw * 4);
        c.mx2 = (xx >= 0 && xx < W) ? 0x22222222u : 0u;
        c.wr = lds[wave] + p;
        c.rd = lds[wave] + half * RS_HW + col;
        const int x = sx * 32 + col;
        const int widx = ct * 2 + half;
        const bool ok = x < W && widx < Cow;
        c.out_voff = ok ? (uint32_t)((x * Cow + widx) * 4) : RS_BAD_LANE;
        // (an odd last column has no 2x2 window; an odd last row has no partner row to trigger a store)
        c.pool_voff = (ok && (col & 1) == 0 && (x >> 1) < (W >> 1)) ? (uint32_t)(((x >> 1) * Cow + widx) * 4) : RS_BAD_LANE;
        c.psel = half ? 0x07060302u : 0x05040100u;
    }

    // ---- start values for the 2 x 16 channels of this lane (exact in fp32 after clamping theta
    // to +-2^22, which cannot change a comparison because |R| <= 9*64)
    v16f init[2];
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const int cbase = (ct * 2 + m) * 32 + 16 * half;
        int th[16], ws[16];
        if (cbase < Cout) {
            const int4 *tp = reinterpret_cast<const int4 *>(thresh + cbase);
            const int4 *sp = reinterpret_cast<const int4 *>(wsum + cbase);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int4 t = tp[k], u = sp[k];
                th[4 * k] = t.x; th[4 * k + 1] = t.y; th[4 * k + 2] = t.z; th[4 * k + 3] = t.w;
                ws[4 * k] = u.x; ws[4 * k + 1] = u.y; ws[4 * k + 2] = u.z; ws[4 * k + 3] = u.w;
            }
        } else {
#pragma unroll
            for (int k = 0; k < 16; ++k) th[k] = ws[k] = 0;
        }
#pragma unroll
        for (int k = 0; k < 16; ++k) init[m][k] = start_value(th[k], ws[k]);
    }

    // ---- weights: [tile64][tap][m][lane], resident for the whole strip
    v4i Wg[3][3][2];   // [kx][ky][m]
    {
        const uint4 *wk = wfrag + (size_t)ct * (18 * 64) + lane;
#pragma unroll
        for (int kx = 0; kx < 3; ++kx)
#pragma unroll
            for (int ky = 0; ky < 3; ++ky)
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    const uint4 w = wk[((ky * 3 + kx) * 2 + m) * 64];
                    Wg[kx][ky][m] = (v4i){(int)w.x, (int)w.y, (int)w.z, (int)w.w};
                }
    }

    // ---- prologue: halo rows 0..3 through the two ring slots (row j in slot j mod 2), rows
    // 0..2 into the window, row 3 left in the ring, rows 4 and 5 in flight.  LDS instructions
    // of one wave execute in order, so a read sees the write before it.
    uint2 gq[2];
    v4i F[3][3];
    {
        uint2 g4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) fetch_row(c, y0 - 1 + j, g4[j], CW_EVEN);
#pragma unroll
        for (int j = 0; j < 2; ++j) fetch_row(c, y0 + 3 + j, gq[j], CW_EVEN);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int yy = y0 - 1 + j;
            const uint32_t m2 = (yy >= 0 && yy < H) ? c.mx2 : 0u, p1 = (~m2 >> 1) & 0x11111111u;
            c.wr[(j & 1) * RS_ROW] = expand_word_masked(g4[j].x, m2, p1);
            c.wr[(j & 1) * RS_ROW + RS_HW] =
                expand_word_masked(g4[j].y, CW_EVEN ? m2 : 0u, CW_EVEN ? p1 : 0u);
            __builtin_amdgcn_wave_barrier();
            if (j < 3) {
#pragma unroll
                for (int x = 0; x < 3; ++x) {
                    const uint4 f = c.rd[(j & 1) * RS_ROW + x];
                    F[j][x] = (v4i){(int)f.x, (int)f.y, (int)f.z, (int)f.w};
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }

    v16f acc[2][2];
    acc[1][0] = init[0];     // "previous row" of row 0: collected, never stored
    acc[1][1] = init[1];
    uint32_t wkeep = 0;

    // Everything fetched so far has to be complete before the loop: the compiler sizes the
    // waits inside the loop for the worse of its two entries, and with fetches still pending
    // here the steady state would wait for its two-rows-ahead fetches a row early.
#pragma unroll
    for (int kx = 0; kx < 3; ++kx)
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) {
            RS_PIN(Wg[kx][ky][0]);
            RS_PIN(Wg[kx][ky][1]);
        }
    RS_PIN(gq[0].x); RS_PIN(gq[0].y); RS_PIN(gq[1].x); RS_PIN(gq[1].y);

    // six rows per trip: the accumulator sets alternate and the three fragment rows rotate, so
    // nothing is copied; what is left (0, 2 or 4 rows, and the odd row's partner, which is
    // computed and dropped) goes two rows per trip with the window moved by register copies
    int i = 0;
#pragma unroll 1
    for (; i + 6 <= rows; i += 6) {
        rows_step<CW_EVEN, POOL, 0, 0, false>(c, i, Wg, init, acc, F, gq, wkeep);
        rows_step<CW_EVEN, POOL, 1, 1, false>(c, i + 1, Wg, init, acc, F, gq, wkeep);
        rows_step<CW_EVEN, POOL, 0, 2, false>(c, i + 2, Wg, init, acc, F, gq, wkeep);
        rows_step<CW_EVEN, POOL, 1, 0, false>(c, i + 3, Wg, init, acc, F, gq, wkeep);
        rows_step<CW_EVEN, POOL, 0, 1, false>(c, i + 4, Wg, init, acc, F, gq, wkeep);
        rows_step<CW_EVEN, POOL, 1, 2, false>(c, i + 5, Wg, init, acc, F, gq, wkeep);
    }
#pragma unroll 1
    for (; i < rows; i += 2) {
        rows_step<CW_EVEN, POOL, 0, 0, true>(c, i, Wg, init, acc, F, gq, wkeep);
        rows_step<CW_EVEN, POOL, 1, 0, true>(c, i + 1, Wg, init, acc, F, gq, wkeep);
    }

    // ---- the signs of the last odd row, still in accumulator set 1
    uint32_t s = 0;
#pragma unroll
    for (int e = 0; e < 32; ++e) {
        const int mm = 1 - e / 16, r = 15 - e % 16;
        s = __builtin_amdgcn_alignbit(s, __float_as_uint(acc[1][mm][r]), 31);
    }
    store_row<POOL, true>(c, s, i - 1 < rows ? i - 1 : -1, wkeep);
}

// ---------------------------------------------------------------------------------------
// The same scheme for layers with TWO 64-channel input steps (65..128 input channels): a wave
// owns a strip of 32 pixel columns and 32 output channels, so that the weights (2 steps x 9 taps
// = 18 fragments, as above) and the window (2 x 9 fragments) still fit in registers next to two
// accumulator sets.  A row is again 18 matrix instructions (tap row, tap column, input step),
// all on one accumulator tile; the staging expands four words per pixel, the sign collection
// covers 16 channels per lane, and the waves of the other channel tiles stage the same strip
// again (the price of keeping a wave self-contained).
constexpr int R2_ROW = 2 * RS_ROW;      // uint4 entries per staged row: [step][half][pixel]

struct Rows2Stream {
    v16f acc[2];
    v4i F[2][3][3];     // [step][window row][tap column]
    uint4 gq[2];
    uint32_t wkeep;
};
struct Rows2Tmp {
    uint32_t w[4], m2[4], p1[4];   // fetched words and the masks of expand_word_masked() per word
    uint4 e[4];
    uint32_t s;
};

// the (three or) four packed words of this lane's halo pixel in image row yy (clamped); TWO: two
// words from each of two tensors
template <bool TWO>
__device__ __forceinline__ void fetch_row4(const RowsCtx &c, int yy, uint4 &g, bool four)
{
    const int yc = min(max(yy, 0), c.H - 1);
    const int soff = yc * c.in_row_bytes;
    if (TWO) {
        const auto v = __builtin_amdgcn_raw_buffer_load_b64(c.in, c.in_voff, soff, 0);
        const int yb = min(max(yy, 0), c.Hb - 1);
        const auto u = __builtin_amdgcn_raw_buffer_load_b64(c.in2, c.in2_voff, yb * c.in2_row_bytes, 0);
        g = make_uint4(v[0], v[1], u[0], u[1]);
    } else if (four) {
        const auto v = __builtin_amdgcn_raw_buffer_load_b128(c.in, c.in_voff, soff, 0);
        g = make_uint4(v[0], v[1], v[2], v[3]);
    } else {
        const auto v = __builtin_amdgcn_raw_buffer_load_b96(c.in, c.in_voff, soff, 0);
        g = make_uint4(v[0], v[1], v[2], 0u);
    }
}

// sign word of one finished row (16 channels per lane, both halves complete it to 32)
template <bool POOL, bool ODD>
__device__ __forceinline__ void store_row32(const RowsCtx &c, uint32_t s, int i_row, uint32_t &wkeep)
{
    const uint32_t word = finish_word32(s);
    const uint32_t roff = i_row >= 0 ? (uint32_t)((c.y0 + i_row) * c.out_row_bytes) : RS_BAD_ROW;
    __builtin_amdgcn_raw_buffer_store_b32(word, c.out, c.out_voff + roff, 0, 0);
    if (POOL) {
        if (!ODD) {
            wkeep = word;
        } else {
            uint32_t v = wkeep | word;
            v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, true);
            const uint32_t poff =
                i_row >= 0 ? (uint32_t)(((c.y0 + i_row) >> 1) * c.pool_row_bytes) : RS_BAD_ROW;
            __builtin_amdgcn_raw_buffer_store_b32(v, c.pool, c.pool_voff + poff, 0, 0);
        }
    }
}

// Matrix instruction t (of 18) of one image row and the vector work behind it; P, R3, COPY as
// in rows_step above.
template <bool CW4, bool POOL, bool TWO, int P, int R3, bool COPY>
__device__ __forceinline__ void rows2_step(const RowsCtx &c, const int i, const v4i (&Wg)[2][3][3],
                                           const v16f &init, Rows2Stream &st)
{
    constexpr int CUR = P, PRV = P ^ 1;
    constexpr int RD = P ^ 1, WR = P;      // ring slot of halo row i + 3 / i + 4
    Rows2Tmp tm;
#pragma unroll
    for (int t = 0; t < 18; ++t) {
        const int ky = t / 6, kx = (t % 6) >> 1, ks = t & 1;
        st.acc[CUR] = mfma_f4(Wg[ks][kx][ky], st.F[ks][(R3 + ky) % 3][kx], t == 0 ? init : st.acc[CUR]);
        RS_FENCE();
        // ---- staging of halo row i + 4 (image row y0 + i + 3): bits fetched two rows ago;
        // dword d of word k in slot 1 + (4 k + d) / 2
        if (t == 0) {
            const bool rin = c.y0 + i + 3 < c.H;
            const uint32_t m2 = rin ? c.mx2 : 0u, p1 = (~m2 >> 1) & 0x11111111u;
            // words 2 and 3 of the two-source form: inside the frame but possibly outside the
            // second tensor, whose missing pixels are zeros like pixels outside the frame
            const uint32_t m2b = (TWO && rin && c.y0 + i + 3 < c.Hb) ? c.mx2b : 0u;
            const uint32_t p1b = rin ? ((~m2b >> 1) & 0x11111111u) : p1;
            tm.w[0] = st.gq[P].x; tm.w[1] = st.gq[P].y; tm.w[2] = st.gq[P].z; tm.w[3] = st.gq[P].w;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                tm.m2[k] = (TWO && k >= 2) ? m2b : (k < 3 || CW4) ? m2 : 0u;
                tm.p1[k] = (TWO && k >= 2) ? p1b : (k < 3 || CW4) ? p1 : 0u;
            }
            tm.s = 0;
        }
        if (t >= 1 && t <= 8) {
#pragma unroll
            for (int q = 2 * (t - 1); q < 2 * t; ++q) {
                const int k = q >> 2, d = q & 3;
                const uint32_t sh = d == 0 ? tm.w[k] << 1 : d == 1 ? tm.w[k] : tm.w[k] >> (d - 1);
                const uint32_t v = (sh & tm.m2[k]) | tm.p1[k];
                if (d == 0) tm.e[k].x = v; else if (d == 1) tm.e[k].y = v; else if (d == 2) tm.e[k].z = v; else tm.e[k].w = v;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) { RS_PIN(tm.e[k].x); RS_PIN(tm.e[k].y); RS_PIN(tm.e[k].z); RS_PIN(tm.e[k].w); }
        }
        if (t == 8) {
#pragma unroll
            for (int k = 0; k < 4; ++k) c.wr[WR * R2_ROW + (k >> 1) * RS_ROW + (k & 1) * RS_HW] = tm.e[k];
            // halo row i + 6 into the register just consumed
            fetch_row4<TWO>(c, c.y0 + i + 5, st.gq[P], CW4);
        }
        if (COPY && (t == 5 || t == 11)) {
            const int k = t / 6;   // F[.][k] <- F[.][k + 1]
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int x = 0; x < 3; ++x) {
                    st.F[u][k][x] = st.F[u][k + 1][x];
                    RS_PIN(st.F[u][k][x]);
                }
        }
        if (COPY ? t == 17 : t == 5) {
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int x = 0; x < 3; ++x) {
                    const uint4 f = c.rd[RD * R2_ROW + u * RS_ROW + x];
                    st.F[u][COPY ? 2 : R3 % 3][x] = (v4i){(int)f.x, (int)f.y, (int)f.z, (int)f.w};
                }
        }
        // ---- signs of the previous row, register 15 first: bit k of the result is register k
        if (t >= 9 && t < 17) {
#pragma unroll
            for (int e = 2 * (t - 9); e < 2 * (t - 8); ++e)
                tm.s = __builtin_amdgcn_alignbit(tm.s, __float_as_uint(st.acc[PRV][15 - e]), 31);
            RS_PIN(tm.s);
        }
        if (t == 17) {
            const bool valid = P == 1 || i > 0;
            store_row32<POOL, P == 0>(c, tm.s, valid ? i - 1 : -1, st.wkeep);
        }
        RS_FENCE();
    }
}

template <bool CW4, bool POOL, bool TWO = false>
__global__ __launch_bounds__(256, 2) void conv_mfma_rows2k_kernel(
    const uint32_t *__restrict__ act, const uint32_t *__restrict__ act2, int Hb, int Wb, int H, int W, int Cw,
    const uint4 *__restrict__ wfrag, int Cout,
    int ctiles, int strips, int nseg, int seg_rows, int units, const int32_t *__restrict__ thresh,
    const int32_t *__restrict__ wsum, uint32_t *__restrict__ out_bits, uint32_t *__restrict__ out_pool)
{
    __shared__ uint4 lds[4][RS_RING * R2_ROW];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int gw = blockIdx.x * 4 + wave;
    if (gw >= units) return;                  // whole wave leaves; nothing is shared
    int q = gw;
    const int ct = q % ctiles; q /= ctiles;   // 32-channel output tile
    const int sx = q % strips; q /= strips;   // strip of 32 pixel columns
    const int sg = q % nseg;                  // segment of seg_rows image rows
    const int n = q / nseg;
    const int col = lane & 31, half = lane >> 5;
    const int Cow = Cout >> 5;
    const int y0 = sg * seg_rows;
    const int rows = min(H, y0 + seg_rows) - y0;

    RowsCtx c;
    c.H = H;
    c.y0 = y0;
    // two-source form: Cw counts the words of the first tensor (2), the second has 2 as well
    c.in_row_bytes = W * Cw * 4;
    c.out_row_bytes = W * Cow * 4;
    c.pool_row_bytes = (W >> 1) * Cow * 4;
    c.in = __builtin_amdgcn_make_buffer_rsrc((void *)(act + (size_t)n * H * W * Cw), 0, H * c.in_row_bytes,
                                             0x00020000);
    c.Hb = TWO ? Hb : H;
    c.in2_row_bytes = TWO ? Wb * 2 * 4 : 0;
    c.in2 = __builtin_amdgcn_make_buffer_rsrc((void *)(TWO ? act2 + (size_t)n * Hb * Wb * 2 : act), 0,
                                              TWO ? Hb * c.in2_row_bytes : 0, 0x00020000);
    c.out = __builtin_amdgcn_make_buffer_rsrc((void *)(out_bits + (size_t)n * H * W * Cow), 0,
                                              H * c.out_row_bytes, 0x00020000);
    c.pool = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(POOL ? out_pool + (size_t)n * (H >> 1) * (W >> 1) * Cow : out_bits), 0,
        POOL ? (H >> 1) * c.pool_row_bytes : 0, 0x00020000);
    {
        const int p = min(lane, RS_HW - 1);   // surplus lanes duplicate the last halo pixel
        const int xx = sx * 32 + p - 1;
        c.in_voff = (uint32_t)(min(max(xx, 0), W - 1) * Cw * 4);
        c.mx2 = (xx >= 0 && xx < W) ? 0x22222222u : 0u;
        c.in2_voff = TWO ? (uint32_t)(min(max(xx, 0), Wb - 1) * 2 * 4) : 0u;
        c.mx2b = (TWO && xx >= 0 && xx < Wb) ? 0x22222222u : 0u;
        c.wr = lds[wave] + p;
        c.rd = lds[wave] + half * RS_HW + col;
        const int x = sx * 32 + col;
        const bool ok = x < W && half == 0;   // both halves hold the finished word: one stores it
        c.out_voff = ok ? (uint32_t)((x * Cow + ct) * 4) : RS_BAD_LANE;
        c.pool_voff = (ok && (col & 1) == 0 && (x >> 1) < (W >> 1)) ? (uint32_t)(((x >> 1) * Cow + ct) * 4) : RS_BAD_LANE;
        c.psel = 0;
    }

    // ---- start values of the 16 channels of this lane
    v16f init;
    {
        const int cbase = ct * 32 + 16 * half;   // < Cout: ct < Cout / 32
        const int4 *tp = reinterpret_cast<const int4 *>(thresh + cbase);
        const int4 *sp = reinterpret_cast<const int4 *>(wsum + cbase);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int4 t = tp[k], u = sp[k];
            init[4 * k] = start_value(t.x, u.x); init[4 * k + 1] = start_value(t.y, u.y);
            init[4 * k + 2] = start_value(t.z, u.z); init[4 * k + 3] = start_value(t.w, u.w);
        }
    }

    // ---- weights: [tile64][step][tap][m][lane], resident for the whole strip
    v4i Wg[2][3][3];   // [step][kx][ky]
    {
        const uint4 *wk = wfrag + (size_t)(ct >> 1) * (2 * 18 * 64) + (ct & 1) * 64 + lane;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int kx = 0; kx < 3; ++kx)
#pragma unroll
                for (int ky = 0; ky < 3; ++ky) {
                    const uint4 w = wk[(ks * 9 + ky * 3 + kx) * 128];
                    Wg[ks][kx][ky] = (v4i){(int)w.x, (int)w.y, (int)w.z, (int)w.w};
                }
    }

    // ---- prologue: halo rows 0..3 through the two ring slots, rows 0..2 into the window, row 3
    // left in the ring, rows 4 and 5 in flight
    Rows2Stream st;
    {
        uint4 g4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) fetch_row4<TWO>(c, y0 - 1 + j, g4[j], CW4);
#pragma unroll
        for (int j = 0; j < 2; ++j) fetch_row4<TWO>(c, y0 + 3 + j, st.gq[j], CW4);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int yy = y0 - 1 + j;
            const bool rin = yy >= 0 && yy < H;
            const uint32_t m2 = rin ? c.mx2 : 0u, p1 = (~m2 >> 1) & 0x11111111u;
            const uint32_t m2b = (TWO && rin && yy < c.Hb) ? c.mx2b : 0u;
            const uint32_t p1b = rin ? ((~m2b >> 1) & 0x11111111u) : p1;
            const uint32_t wv[4] = {g4[j].x, g4[j].y, g4[j].z, g4[j].w};
#pragma unroll
            for (int k = 0; k < 4; ++k)
                c.wr[(j & 1) * R2_ROW + (k >> 1) * RS_ROW + (k & 1) * RS_HW] =
                    expand_word_masked(wv[k], (TWO && k >= 2) ? m2b : (k < 3 || CW4) ? m2 : 0u,
                                       (TWO && k >= 2) ? p1b : (k < 3 || CW4) ? p1 : 0u);
            __builtin_amdgcn_wave_barrier();
            if (j < 3) {
#pragma unroll
                for (int u = 0; u < 2; ++u)
#pragma unroll
                    for (int x = 0; x < 3; ++x) {
                        const uint4 f = c.rd[(j & 1) * R2_ROW + u * RS_ROW + x];
                        st.F[u][j][x] = (v4i){(int)f.x, (int)f.y, (int)f.z, (int)f.w};
                    }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
    st.acc[1] = init;     // "previous row" of row 0: collected, never stored
    st.wkeep = 0;

    // (everything fetched so far complete before the loop, as in the kernel above)
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int kx = 0; kx < 3; ++kx)
#pragma unroll
            for (int ky = 0; ky < 3; ++ky) RS_PIN(Wg[ks][kx][ky]);
    RS_PIN(st.gq[0].x); RS_PIN(st.gq[0].y); RS_PIN(st.gq[0].z); RS_PIN(st.gq[0].w);
    RS_PIN(st.gq[1].x); RS_PIN(st.gq[1].y); RS_PIN(st.gq[1].z); RS_PIN(st.gq[1].w);

    int i = 0;
#pragma unroll 1
    for (; i + 6 <= rows; i += 6) {
        rows2_step<CW4, POOL, TWO, 0, 0, false>(c, i, Wg, init, st);
        rows2_step<CW4, POOL, TWO, 1, 1, false>(c, i + 1, Wg, init, st);
        rows2_step<CW4, POOL, TWO, 0, 2, false>(c, i + 2, Wg, init, st);
        rows2_step<CW4, POOL, TWO, 1, 0, false>(c, i + 3, Wg, init, st);
        rows2_step<CW4, POOL, TWO, 0, 1, false>(c, i + 4, Wg, init, st);
        rows2_step<CW4, POOL, TWO, 1, 2, false>(c, i + 5, Wg, init, st);
    }
#pragma unroll 1
    for (; i < rows; i += 2) {
        rows2_step<CW4, POOL, TWO, 0, 0, true>(c, i, Wg, init, st);
        rows2_step<CW4, POOL, TWO, 1, 0, true>(c, i + 1, Wg, init, st);
    }

    // ---- the signs of the last odd row, still in accumulator set 1
    uint32_t s = 0;
#pragma unroll
    for (int e = 0; e < 16; ++e) s = __builtin_amdgcn_alignbit(s, __float_as_uint(st.acc[1][15 - e]), 31);
    store_row32<POOL, true>(c, s, i - 1 < rows ? i - 1 : -1, st.wkeep);
}

template <bool POOL>
static int launch_rows2k_t(const uint32_t *act, const uint32_t *act2, int Hb, int Wb, int N, int H, int W,
                           const BlobLayout &L, const uint4 *wfrag, const int32_t *thresh, uint32_t *out_bits,
                           uint32_t *out_pool, hipStream_t s)
{
    const int32_t *wsum =
        (const int32_t *)((const uint8_t *)wfrag - L.off_f4 + L.off_cnt) + (size_t)10 * L.cout_pad64;
    const int ctiles = L.cout >> 5;           // 32-channel tiles (cout is a multiple of 32)
    const int strips = ceil_div(W, 32);
    const long base = (long)N * strips * ctiles;
    const long slots = 2L * 4 * 256;
    const int want = (int)std::max(1L, slots / base);
    int seg_rows = ceil_div(H, want);
    seg_rows = std::max(2, seg_rows + (seg_rows & 1));        // even: 2x2 windows stay inside a segment
    const int nseg = ceil_div(H, seg_rows);
    const long units = base * nseg;
    if (units > 0x7fffffffL) return fail(MBU_ERR_SHAPE, "too many tiles for one launch");
    const int grid = (int)((units + 3) / 4);
    if (act2)   // [64 channels | 64 channels] of two tensors
        MBU_LAUNCH((conv_mfma_rows2k_kernel<true, POOL, true>), dim3(grid), dim3(256), 0, s, act, act2, Hb, Wb, H, W,
                   2, wfrag, L.cout, ctiles, strips, nseg, seg_rows, (int)units, thresh, wsum, out_bits, out_pool);
    else if (L.cin_words == 4)
        MBU_LAUNCH((conv_mfma_rows2k_kernel<true, POOL>), dim3(grid), dim3(256), 0, s, act, act2, 0, 0, H, W,
                   L.cin_words, wfrag, L.cout, ctiles, strips, nseg, seg_rows, (int)units, thresh, wsum, out_bits,
                   out_pool);
    else
        MBU_LAUNCH((conv_mfma_rows2k_kernel<false, POOL>), dim3(grid), dim3(256), 0, s, act, act2, 0, 0, H, W,
                   L.cin_words, wfrag, L.cout, ctiles, strips, nseg, seg_rows, (int)units, thresh, wsum, out_bits,
                   out_pool);
    return check_launch("conv_mfma_rows2k");
}

template <bool POOL, int WPS>
static int launch_rows_t(const uint32_t *act, int N, int H, int W, const BlobLayout &L, const uint4 *wfrag,
                  const int32_t *thresh, uint32_t *out_bits, uint32_t *out_pool, hipStream_t s)
{
    // sums of the weights per output channel: row 10 of the count section of the blob
    const int32_t *wsum =
        (const int32_t *)((const uint8_t *)wfrag - L.off_f4 + L.off_cnt) + (size_t)10 * L.cout_pad64;
    const int ctiles = L.cout_pad64 / 64;
    const int strips = ceil_div(W, 32);
    const long base = (long)N * strips * ctiles;
    // as many row segments as it takes to give every wave slot of the chip one unit
    const long slots = (long)WPS * 4 * 256;
    const int want = (int)std::max(1L, slots / base);
    int seg_rows = ceil_div(H, want);
    seg_rows = std::max(2, seg_rows + (seg_rows & 1));        // even: 2x2 windows stay inside a segment
    const int nseg = ceil_div(H, seg_rows);
    const long units = base * nseg;
    if (units > 0x7fffffffL) return fail(MBU_ERR_SHAPE, "too many tiles for one launch");
    const int grid = (int)((units + 3) / 4);
    if (L.cin_words == 2)
        MBU_LAUNCH((conv_mfma_rows_kernel<true, POOL, WPS>), dim3(grid), dim3(256), 0, s, act, H, W,
                   L.cin_words, wfrag, L.cout, ctiles, strips, nseg, seg_rows, (int)units, thresh, wsum,
                   out_bits, out_pool);
    else
        MBU_LAUNCH((conv_mfma_rows_kernel<false, POOL, WPS>), dim3(grid), dim3(256), 0, s, act, H, W,
                   L.cin_words, wfrag, L.cout, ctiles, strips, nseg, seg_rows, (int)units, thresh, wsum,
                   out_bits, out_pool);
    return check_launch("conv_mfma_rows");
}

bool conv_rows_supported(int H, int W, const BlobLayout &L, bool wants_bits)
{
    // one input step, packed output wanted, every image below 2^30 bytes on both sides
    return L.ksteps == 1 && wants_bits && (double)H * W * L.cin_words * 4 < 1073741824.0 &&
           (double)H * W * (L.cout >> 5) * 4 < 1073741824.0;
}

bool conv_rows2k_supported(int H, int W, const BlobLayout &L, bool wants_bits)
{
    // two input steps (three or four words per pixel), otherwise as above
    return L.ksteps == 2 && L.cin_words >= 3 && wants_bits && (double)H * W * L.cin_words * 4 < 1073741824.0 &&
           (double)H * W * (L.cout >> 5) * 4 < 1073741824.0;
}

int launch_conv_mfma_rows2k(const uint32_t *act, const uint32_t *act2, int Hb, int Wb, int N, int H, int W,
                            const BlobLayout &L, const void *blob, const int32_t *thresh, uint32_t *out_bits,
                            uint32_t *out_pool, hipStream_t s)
{
    if (!conv_rows2k_supported(H, W, L, out_bits != nullptr))
        return fail(MBU_ERR_SHAPE, "row-streaming kernel for two input steps: layer not supported");
    if (act2 && (L.cin != 128 || Hb < 1 || Wb < 1 || Hb > H || Wb > W))
        return fail(MBU_ERR_SHAPE, "row-streaming kernel for two inputs: 64 + 64 channels, second input inside the frame");
    const uint4 *wfrag = (const uint4 *)((const uint8_t *)blob + L.off_f4);
    if (out_pool) return launch_rows2k_t<true>(act, act2, Hb, Wb, N, H, W, L, wfrag, thresh, out_bits, out_pool, s);
    return launch_rows2k_t<false>(act, act2, Hb, Wb, N, H, W, L, wfrag, thresh, out_bits, out_pool, s);
}

int launch_conv_mfma_rows(const uint32_t *act, int N, int H, int W, const BlobLayout &L, const void *blob,
                          const int32_t *thresh, uint32_t *out_bits, uint32_t *out_pool, int waves_per_simd,
                          hipStream_t s)
{
    if (!conv_rows_supported(H, W, L, out_bits != nullptr))
        return fail(MBU_ERR_SHAPE, "row-streaming kernel: layer not supported");
    const uint4 *wfrag = (const uint4 *)((const uint8_t *)blob + L.off_f4);
    if (waves_per_simd == 1) {
        if (out_pool) return launch_rows_t<true, 1>(act, N, H, W, L, wfrag, thresh, out_bits, out_pool, s);
        return launch_rows_t<false, 1>(act, N, H, W, L, wfrag, thresh, out_bits, out_pool, s);
    }
    if (out_pool) return launch_rows_t<true, 2>(act, N, H, W, L, wfrag, thresh, out_bits, out_pool, s);
    return launch_rows_t<false, 2>(act, N, H, W, L, wfrag, thresh, out_bits, out_pool, s);
}

}  // namespace mbu
