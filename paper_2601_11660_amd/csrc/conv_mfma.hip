// Masked-binary 3x3 convolution on the matrix cores.
//
// CDNA4 has no 1-bit matrix instruction, but its 4-bit floating-point format (E2M1)
// represents -1, 0 and +1 exactly, products of such values are exact, and sums of up
// to 9*Cin <= 2^24 of them are exact in the fp32 accumulator - so the contraction
// R = sum w*a of Algorithm 1 can run on v_mfma_f32_32x32x64_f8f6f4 and still be the
// exact integer.  Masked weights are the code 0 and contribute nothing.  Activations enter
// as the packed bit itself (1.0 / 0.0, and 0.5 for a pixel outside the image), the constant
// this adds is folded into the start value of the accumulators (mfma_common.h): no border
// correction is needed on this path.
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
#include "mfma_common.h"

namespace mbu {

constexpr int TW = 32;            // pixels per matrix column tile (one image-row segment)
constexpr int HALO_W = TW + 2;

// ---------------------------------------------------------------------------------
// Fast kernel (packed bits only).
//
// Every wave works alone: no barrier and no data shared between the waves of a block.
// A wave owns one 64-channel output tile for its whole life and walks over pixel tiles
// of RW image rows x 32 pixels (RW x 2 accumulator tiles, RW = 4: 128 registers).  Its
// work is the flat sequence of steps (pixel tile, 64-channel input step ks).
//
// Step = three "groups", one per kernel column kx.  A group needs the 3 x 2 weight
// fragments of taps (ky, kx) (24 registers) and RW+2 activation fragments (LDS rows
// rho = r + ky), each feeding every (r, ky) pair with r + ky = rho: 6*RW matrix
// instructions per RW+2 LDS reads.  All 18 weight fragments of a step stay in
// registers; as soon as a group has issued its matrix instructions its registers are
// refilled with the same group's fragments of the next step, so weights arrive a whole
// step ahead of their use (with a single input step they simply stay).
//
// The (RW+2) x 34 pixel halo window of the NEXT step - which may belong to the next
// pixel tile - is fetched from global memory at the start of a step, expanded from bits
// to nibbles and written to the wave's other LDS buffer at its end, so the matrix
// pipeline never waits for staging, also across tile boundaries.  The step body has no
// branches: halo pixels outside the image are loaded from a clamped address and
// expanded with zero masks; after its last step a wave re-stages its last window.
//
// Epilogue per tile: accumulators start at -theta (exact in fp32 after clamping theta
// to +-2^22, which cannot change any comparison because |R| <= 9*Cin < 2^20), so the
// output bit is the complement of the accumulator's sign bit: one funnel shift per
// register collects 16 channel bits, one cross-half exchange completes the word.
template <int RW, int MT>
__device__ __forceinline__ void group_mma(v16f (&acc)[RW][MT], const v4i (&Wg)[3][MT],
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
#pragma unroll
                for (int m = 0; m < MT; ++m) acc[r][m] = mfma_f4(Wg[ky][m], B, acc[r][m]);
            }
        }
    }
}

// First group of a pixel tile: the matrix instruction that opens an accumulator tile
// (tap row ky = 0 at LDS row rho = r) takes -theta as its addend, so the accumulators are
// never initialised by separate moves.
template <int RW, int MT>
__device__ __forceinline__ void group_mma_first(v16f (&acc)[RW][MT], const v16f (&init)[MT],
                                                const v4i (&Wg)[3][MT], const uint4 *tb)
{
#pragma unroll
    for (int rho = 0; rho < RW + 2; ++rho) {
        const uint4 b = tb[rho * 2 * HALO_W];
        const v4i B = {(int)b.x, (int)b.y, (int)b.z, (int)b.w};
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) {
            const int r = rho - ky;
            if (r >= 0 && r < RW) {
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    acc[r][m] = mfma_f4(Wg[ky][m], B, ky == 0 ? init[m] : acc[r][m]);
            }
        }
    }
}

// fragments of taps (ky, kx), ky = 0..2, of the wave's MT 32-channel tiles; wk points at
// [tap 0][this wave's first 32-channel tile][lane] of one 64-channel input step
template <int MT>
__device__ __forceinline__ void load_group(v4i (&Wg)[3][MT], const uint4 *wk, int kx)
{
#pragma unroll
    for (int ky = 0; ky < 3; ++ky)
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            const uint4 a = wk[((ky * 3 + kx) * 2 + m) * 64];
            Wg[ky][m] = (v4i){(int)a.x, (int)a.y, (int)a.z, (int)a.w};
        }
}

// RW image rows x 32 pixels x (32*MT) output channels per wave: (RW, MT) = (4, 2) or (8, 1)
// both give 128 accumulator registers; MT = 1 halves the weight registers and doubles
// the reuse of every weight fragment at the price of more activation reads.
template <int RW, int MT, bool CW_EVEN, bool ONE_STEP>
__global__ __launch_bounds__(256, 2) void conv_mfma_bits_kernel(
    const uint32_t *__restrict__ act, int N, int H, int W, int Cw, int ksteps,
    const uint4 *__restrict__ wfrag, int Cout, int ctiles, int slots, int ptiles, TileStep tstep,
    const int32_t *__restrict__ thresh, const int32_t *__restrict__ wsum, uint32_t *__restrict__ out_bits)
{
    constexpr int HR = RW + 2;
    constexpr int NPIX = HR * HALO_W;            // halo pixels per step
    constexpr int NLD = (NPIX + 63) / 64;        // staged pixels per lane
    constexpr int TILE = HR * 2 * HALO_W;        // uint4 entries per buffer, [row][half][col]
    __shared__ uint4 lds[4][2][TILE];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int gw = blockIdx.x * 4 + wave;
    if (gw >= slots * ctiles) return;             // whole wave leaves; nothing is shared
    const int ct = gw % ctiles;                   // (32*MT)-channel output tile, fixed for the wave
    const int slot = gw / ctiles;
    const int col = lane & 31, half = lane >> 5;
    uint4(*tile)[TILE] = lds[wave];

    // ---- -theta for the MT x 16 channels of this lane
    v16f init[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int cbase = (ct * MT + m) * 32 + 16 * half;  // 16 consecutive channels per lane
        int th[16], ws[16];
        if (cbase < Cout) {                                 // Cout % 32 == 0: all 16 or none
            const int4 *tp = reinterpret_cast<const int4 *>(thresh + cbase);
            const int4 *sp = reinterpret_cast<const int4 *>(wsum + cbase);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int4 t = tp[q], u = sp[q];
                th[4 * q] = t.x; th[4 * q + 1] = t.y; th[4 * q + 2] = t.z; th[4 * q + 3] = t.w;
                ws[4 * q] = u.x; ws[4 * q + 1] = u.y; ws[4 * q + 2] = u.z; ws[4 * q + 3] = u.w;
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) th[i] = ws[i] = 0;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) init[m][i] = start_value(th[i], ws[i]);
    }

    // ---- staging plan for the window of a pixel tile: lane handles halo pixels lane + 64*j
    uint32_t src[NLD];            // word offset of the (clamped) pixel from `act`
    uint32_t m8[NLD];             // all ones inside the image, 0 outside
    auto plan = [&](const TilePos &tp) {
        const int tx = tp.tx, ty = tp.ty, n = tp.n;
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            int p = lane + 64 * j;
            p = p < NPIX ? p : 0;     // surplus lanes duplicate pixel 0 (same data, same slot)
            const int r = p / HALO_W, c = p - r * HALO_W;
            const int yy = ty * RW + r - 1, xx = tx * TW + c - 1;
            const bool in = yy >= 0 && yy < H && xx >= 0 && xx < W;
            const int yc = min(max(yy, 0), H - 1), xc = min(max(xx, 0), W - 1);
            src[j] = (uint32_t)((((size_t)n * H + yc) * W + xc) * Cw);
            m8[j] = in ? 0xffffffffu : 0u;
        }
    };
    uint2 gq[NLD];
    auto stage_issue = [&](int ks) {
        const uint32_t *base = act + 2 * ks;
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            if (CW_EVEN) {
                gq[j] = *reinterpret_cast<const uint2 *>(base + src[j]);
            } else {
                gq[j].x = base[src[j]];
                gq[j].y = act[src[j] + min(2 * ks + 1, Cw - 1)];
            }
        }
    };
    auto stage_commit = [&](int ks, uint4 *buf) {
        const bool second = CW_EVEN || (2 * ks + 1 < Cw);
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            int p = lane + 64 * j;
            p = p < NPIX ? p : 0;
            const int r = p / HALO_W, c = p - r * HALO_W;
            uint4 *d = buf + (r * 2) * HALO_W + c;
            const uint32_t a = gq[j].x, b = gq[j].y;
            const uint32_t m2 = m8[j] & 0x22222222u, p1 = ~m8[j] & 0x11111111u;
            d[0] = expand_word_masked(a, m2, p1);
            d[HALO_W] = expand_word_masked(b, second ? m2 : 0u, second ? p1 : 0u);
        }
    };

    // ---- weight fragments: [tile64][kstep][tap][m][lane], 18 KB per step and 64 channels
    const int t64 = (ct * MT) >> 1, mfirst = (ct * MT) & 1;
    const uint4 *wk = wfrag + ((size_t)t64 * ksteps * 18 + mfirst) * 64 + lane;
    v4i Wg[3][3][MT];   // [kx][ky][m]
    TilePos cur = tile_pos(slot, tstep.tiles_x, tstep.tiles_y);   // the only divisions
    plan(cur);
    stage_issue(0);
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) load_group<MT>(Wg[kx], wk, kx);
    stage_commit(0, tile[0]);

    const int tb_off = half * HALO_W + col;
    const int Cow = Cout >> 5;
    const uint32_t psel = half ? 0x07060302u : 0x05040100u;
    int buf = 0;
    for (int pt = slot; pt < ptiles; pt += slots) {
        v16f acc[RW][MT];
        if (!ONE_STEP) {
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int r = 0; r < RW; ++r) acc[r][m] = init[m];
        }

        for (int ks = 0; ks < ksteps; ++ks) {
            // the step after this one: next input step of this tile, or step 0 of the wave's
            // next tile (its own last window again when there is none)
            const bool last = ks + 1 == ksteps;
            const int kn = last ? 0 : ks + 1;
            if (last) {
                TilePos nxt = cur;
                if (pt + slots < ptiles) nxt.advance(tstep);
                plan(nxt);
            }
            const uint4 *tb = tile[buf] + tb_off;
            // The scheduling fences keep every fetch where it is written: issued as early as
            // its destination registers are free, a whole step ahead of its use.
            stage_issue(kn);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int kx = 0; kx < 3; ++kx) {
                if (ONE_STEP && kx == 0) group_mma_first<RW, MT>(acc, init, Wg[kx], tb + kx);
                else group_mma<RW, MT>(acc, Wg[kx], tb + kx);
                if (!ONE_STEP) {
                    __builtin_amdgcn_sched_barrier(0);
                    load_group<MT>(Wg[kx], wk + (size_t)kn * (18 * 64), kx);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            buf ^= 1;
            stage_commit(kn, tile[buf]);
            // LDS instructions of one wave execute in order, so the fragment reads of the
            // next step see these writes; the fence only stops the compiler from moving them.
            __builtin_amdgcn_wave_barrier();
        }

        // ---- epilogue of this pixel tile
        const int x = cur.tx * TW + col;
        const int y0 = cur.ty * RW;
        uint32_t *orow = out_bits + (((size_t)cur.n * H + y0) * W + x) * Cow;
        const size_t row_stride = (size_t)W * Cow;
        // all sign collections first (RW*MT independent dependency chains in one basic block),
        // then the words, then the stores
        uint32_t sgn[RW][MT];
#pragma unroll
        for (int i = 15; i >= 0; --i)
#pragma unroll
            for (int r = 0; r < RW; ++r)
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    sgn[r][m] = __builtin_amdgcn_alignbit(i == 15 ? 0u : sgn[r][m],
                                                          __float_as_uint(acc[r][m][i]), 31);
        uint32_t word[RW];
#pragma unroll
        for (int r = 0; r < RW; ++r)
            word[r] = MT == 2 ? finish_word64(sgn[r][0], sgn[r][MT - 1], psel) : finish_word32(sgn[r][0]);
#pragma unroll
        for (int r = 0; r < RW; ++r) {
            // MT == 2: half 0 stores the first word, half 1 the second; MT == 1: the storing
            // half alternates per row
            const int widx = MT == 2 ? ct * 2 + half : ((half == (r & 1)) ? ct : Cow);
            if (widx < Cow && y0 + r < H && x < W) orow[r * row_stride + widx] = word[r];
        }
        cur.advance(tstep);
    }
}

// ---------------------------------------------------------------------------------
// Block-cooperative variant for layers with several input steps: the four waves of a
// block share one staged halo window ((RW*WM+2) x 34 pixels, double buffered, one
// barrier per step) and are arranged WM x WN over image rows x 64-channel output tiles.
// Less staging work per wave than the wave-private kernel above; used when the K loop
// is long enough to amortise the per-tile prologue and epilogue.
//
// Two fusions of the decoder / encoder glue (Sec. 2.1) live here, because they only touch
// the staging and the epilogue:
//  TWO_SRC  the input is the channel concatenation [act | low]: word k of a halo pixel (y, x)
//           comes from act[y][x][k] for k < Cwa and from the second tensor otherwise - at
//           low[y/2][x/2][k - Cwa] when it is half size (nearest up-sampling, low_shift = 1)
//           or at low[y][x][k - Cwa] (low_shift = 0); neither the skip concatenation nor
//           the up-sampling is ever materialised.  The second tensor has Hb x Wb pixels of its
//           own and may cover less than the image (decoder of a frame whose size is not a
//           multiple of 2^levels): where it has no pixel its channels are zeros, staged like
//           pixels outside the image;
//  POOL     besides its own output the layer writes the 2x2 OR-pooled output (max pooling
//           of +-1 values): rows pair up inside a lane, columns with the neighbouring lane.
template <int RW, int WM, int WN, bool CW_EVEN, bool TWO_SRC, bool POOL>
__global__ __launch_bounds__(256, 2) void conv_mfma_block_kernel(
    const uint32_t *__restrict__ act, const uint32_t *__restrict__ low, int N, int H, int W,
    int Cwa, int Cwb, int low_shift, int Hb, int Wb, int ksteps, const uint4 *__restrict__ wfrag, int Cout,
    int tiles64, int ptiles, TileStep tstep, const int32_t *__restrict__ thresh,
    const int32_t *__restrict__ wsum, uint32_t *__restrict__ out_bits, uint32_t *__restrict__ out_pool)
{
    static_assert(WM * WN == 4, "four waves per block");
    constexpr int NB = 3;                        // activation fragments in flight per wave
    static_assert(!POOL || (RW % 2 == 0), "pooling pairs rows inside a wave");
    constexpr int NT = 256;
    constexpr int TH = RW * WM;
    constexpr int HR = TH + 2;
    constexpr int NPIX = HR * HALO_W;            // halo pixels per step
    constexpr int NLD = (NPIX + NT - 1) / NT;    // staged pixels per thread
    constexpr int TILE = HR * 2 * HALO_W;        // uint4 entries per buffer, [row][half][col]
    __shared__ uint4 tile[2][TILE];
    __shared__ float4 init_tab[4][2][2][4];      // [wave][half][m][4 x 4 channels]: -theta

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int tid = threadIdx.x;
    const int wm = wave % WM, wn = wave / WM;
    const int col = lane & 31, half = lane >> 5;
    const int Cw = Cwa + (TWO_SRC ? Cwb : 0);     // words per pixel of the (virtual) input
    const int Hl = H >> 1, Wl = W >> 1;
    const int ct_raw = blockIdx.y * WN + wn;      // 64-channel output tile of this wave
    const bool has_ct = ct_raw < tiles64;
    const int ct = has_ct ? ct_raw : tiles64 - 1;

    // ---- -theta of this wave's 64 channels, kept in LDS and reloaded at every pixel tile
    // (exact in fp32 after clamping theta to +-2^22; see the epilogue)
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

    // ---- staging plan of this thread for one pixel tile: halo pixels p = tid + NT*j.
    // Both sources are read through buffer resources (tensors below 4 GiB): byte offset of the
    // pixel in a register, offset of the 64-channel step in a scalar register.
    const __amdgpu_buffer_rsrc_t ars =
        __builtin_amdgcn_make_buffer_rsrc((void *)act, 0, (int)((size_t)N * H * W * Cwa * 4), 0x00020000);
    const __amdgpu_buffer_rsrc_t brs = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(TWO_SRC ? low : act), 0,
        TWO_SRC ? (int)((size_t)N * Hb * Wb * Cwb * 4) : 0, 0x00020000);
    uint32_t offa[NLD];                  // byte offset of the (clamped) pixel in act
    uint32_t offb[TWO_SRC ? NLD : 1];    // ... of the pixel (y/2, x/2) or (y, x) in low
    uint32_t inside = 0;                 // bit j: pixel j lies inside the image
    uint32_t inside_b = 0;               // bit j: ... and the second tensor has a pixel for it
    auto plan = [&](const TilePos &tp) {
        const int tx = tp.tx, ty = tp.ty, n = tp.n;
        inside = 0;
        inside_b = 0;
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            int p = tid + NT * j;
            p = p < NPIX ? p : 0;     // surplus threads duplicate pixel 0 (same data, same slot)
            const int r = p / HALO_W, c = p - r * HALO_W;
            const int yy = ty * TH + r - 1, xx = tx * TW + c - 1;
            const bool in = yy >= 0 && yy < H && xx >= 0 && xx < W;
            const int yc = min(max(yy, 0), H - 1), xc = min(max(xx, 0), W - 1);
            offa[j] = (uint32_t)((((size_t)n * H + yc) * W + xc) * Cwa * 4);
            inside |= (in ? 1u : 0u) << j;
            if (TWO_SRC) {   // second source: same pixel, or pixel (y/2, x/2) of a half-size tensor
                const int yb = yc >> low_shift, xb = xc >> low_shift;
                inside_b |= ((in && yb < Hb && xb < Wb) ? 1u : 0u) << j;
                offb[j] = (uint32_t)((((size_t)n * Hb + min(yb, Hb - 1)) * Wb + min(xb, Wb - 1)) * Cwb * 4);
            }
        }
    };
    // word k (wave-uniform) of staged pixel j of the virtual input
    auto word = [&](int j, int k) -> uint32_t {
        if (TWO_SRC && k >= Cwa) return __builtin_amdgcn_raw_buffer_load_b32(brs, offb[j], (k - Cwa) * 4, 0);
        return __builtin_amdgcn_raw_buffer_load_b32(ars, offa[j], k * 4, 0);
    };
    uint2 gq[NLD];
    auto stage_issue = [&](int ks) {
        const int k0 = 2 * ks;
        if (CW_EVEN) {   // both sources have an even word count: one aligned 8-byte load
            if (TWO_SRC && k0 >= Cwa) {
#pragma unroll
                for (int j = 0; j < NLD; ++j) {
                    const auto v = __builtin_amdgcn_raw_buffer_load_b64(brs, offb[j], (k0 - Cwa) * 4, 0);
                    gq[j] = make_uint2(v[0], v[1]);
                }
            } else {
#pragma unroll
                for (int j = 0; j < NLD; ++j) {
                    const auto v = __builtin_amdgcn_raw_buffer_load_b64(ars, offa[j], k0 * 4, 0);
                    gq[j] = make_uint2(v[0], v[1]);
                }
            }
        } else {
            const int k1 = min(k0 + 1, Cw - 1);
#pragma unroll
            for (int j = 0; j < NLD; ++j) {
                gq[j].x = word(j, k0);
                gq[j].y = word(j, k1);
            }
        }
    };
    auto stage_commit = [&](int ks, uint4 *buf) {
        const bool second = CW_EVEN || (2 * ks + 1 < Cw);
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            int p = tid + NT * j;
            p = p < NPIX ? p : 0;
            const int r = p / HALO_W, c = p - r * HALO_W;
            uint4 *d = buf + (r * 2) * HALO_W + c;
            const uint32_t a = gq[j].x, b = gq[j].y;
            // each of the step's two words belongs to one source (wave-uniform choice)
            const bool in0 = ((TWO_SRC && 2 * ks >= Cwa ? inside_b : inside) >> j) & 1u;
            const bool in1 = ((TWO_SRC && 2 * ks + 1 >= Cwa ? inside_b : inside) >> j) & 1u;
            d[0] = expand_word_masked(a, in0 ? 0x22222222u : 0u, in0 ? 0u : 0x11111111u);
            d[HALO_W] = expand_word_masked(b, (second && in1) ? 0x22222222u : 0u,
                                           (second && !in1) ? 0x11111111u : 0u);
        }
    };

    // One word of that commit (word i & 1 of staged pixel i >> 1), slotted between the matrix
    // instructions of a step's last fragments: vector work hides only behind matrix instructions
    // of the same wave.  No branch: a slot with control flow makes the compiler drain the
    // vector-memory counter there.
    auto commit_word = [&](int ks, uint4 *buf, int i) {
        const int j = i >> 1;
        int p = tid + NT * j;
        p = p < NPIX ? p : 0;
        const int r = p / HALO_W, c = p - r * HALO_W;
        const int k = 2 * ks + (i & 1);
        const bool have = (i & 1) == 0 || CW_EVEN || (k < Cw);
        const bool in = ((TWO_SRC && k >= Cwa ? inside_b : inside) >> j) & 1u;
        buf[(r * 2 + (i & 1)) * HALO_W + c] =
            expand_word_masked((i & 1) ? gq[j].y : gq[j].x, (have && in) ? 0x22222222u : 0u,
                               (have && !in) ? 0x11111111u : 0u);
    };

    // ---- weight fragments: [tile64][kstep][tap][m][lane], 18 KB per step and tile
    const uint4 *wk = wfrag + (size_t)ct * ksteps * (18 * 64) + lane;
    // the same fragments through a buffer resource: lane offset in a register, step and tap
    // offsets in scalar registers, no address arithmetic on the vector ALU
    const __amdgpu_buffer_rsrc_t wrs = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(wfrag + (size_t)ct * ksteps * (18 * 64)), 0, ksteps * (18 * 1024), 0x00020000);
    const int wlane = lane * 16;
    v4i Wg[3][3][2];   // [kx][ky][m]
    const int stride = gridDim.x;
    TilePos cur = tile_pos(blockIdx.x, tstep.tiles_x, tstep.tiles_y);   // the only divisions
    plan(cur);
    stage_issue(0);
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) load_group<2>(Wg[kx], wk, kx);
    stage_commit(0, tile[0]);
    __syncthreads();

    const int tb_off = (wm * RW * 2 + half) * HALO_W + col;
    const int Cow = Cout >> 5;
    const int widx = ct * 2 + half;
    const uint32_t psel = half ? 0x07060302u : 0x05040100u;
    int buf = 0;
    // The block walks over its pixel tiles; the work is the flat sequence of steps
    // (tile, 64-channel input step).  During a step the window and the weights of the NEXT
    // step are fetched - at a tile's last step those of the next tile's first - so neither
    // the matrix pipeline nor a new tile waits for staging.
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

        for (int ks = 0; ks < ksteps; ++ks) {
            const bool last = ks + 1 == ksteps;
            const int kn = last ? 0 : ks + 1;
            if (last) {
                TilePos nxt = cur;
                if (pt + stride < ptiles) nxt.advance(tstep);
                plan(nxt);
            }
            const uint4 *tb = tile[buf] + tb_off;
            // The scheduling fences keep every fetch where it is written: issued as early as
            // its destination registers are free, a whole step ahead of its use.
            stage_issue(kn);
            __builtin_amdgcn_sched_barrier(0);
            // The 3 x (RW + 2) activation fragments of the step, in the order they are used
            // (tap column, then window row), rotate through NB registers: the read of fragment
            // j + NB is issued right after the matrix instructions of fragment j, so the LDS
            // latency hides behind the instructions of the NB - 1 fragments in between.
            constexpr int NF = 3 * (RW + 2);
            v4i fr[NB];
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const uint4 b = tb[(j / (RW + 2)) + (j % (RW + 2)) * 2 * HALO_W];
                fr[j] = (v4i){(int)b.x, (int)b.y, (int)b.z, (int)b.w};
            }
#pragma unroll
            for (int j = 0; j < NF; ++j) {
                const int kx = j / (RW + 2), rho = j % (RW + 2);
#pragma unroll
                for (int ky = 0; ky < 3; ++ky) {
                    const int r = rho - ky;
                    if (r >= 0 && r < RW) {
#pragma unroll
                        for (int m = 0; m < 2; ++m)
                            acc[r][m] = mfma_f4(Wg[kx][ky][m], fr[j % NB], acc[r][m]);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                if (j + NB < NF) {
                    const int jn = j + NB;
                    const uint4 b = tb[(jn / (RW + 2)) + (jn % (RW + 2)) * 2 * HALO_W];
                    fr[j % NB] = (v4i){(int)b.x, (int)b.y, (int)b.z, (int)b.w};
                }
                // One weight fragment is fetched per slot.  Fragment (kx, ky, m) is free after
                // window row RW - 1 + ky of column kx; in that order the 18 fragments of the NEXT
                // step go to slots 3 .. 17 and the last three - tap column 2, first used in slot
                // 13 - to slots 0 .. 2 of the step that uses them.
                {
                    const int i = j < 3 ? 15 + j : j - 3;
                    const int g = i / 6, ky = (i % 6) >> 1, m = i & 1;
                    const auto w = __builtin_amdgcn_raw_buffer_load_b128(
                        wrs, wlane, ((j < 3 ? ks : kn) * 18 + (ky * 3 + g) * 2 + m) * 1024, 0);
                    Wg[g][ky][m] = (v4i){(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
                }
                // the next step's window (fetched at the start of this one): one word per slot
                if (j >= NF - 1 - 2 * NLD && j < NF - 1) commit_word(kn, tile[buf ^ 1], j - (NF - 1 - 2 * NLD));
                __builtin_amdgcn_sched_barrier(0);
            }
            buf ^= 1;
            __syncthreads();
        }

        // ---- epilogue of this pixel tile
        const int n = cur.n;
        const int x = cur.tx * TW + col;
        const int yb = cur.ty * TH + wm * RW;
        const bool ok = has_ct && x < W && widx < Cow;
        uint32_t words[RW];
        uint32_t *orow = out_bits + (((size_t)n * H + yb) * W + x) * Cow + widx;
        const size_t row_stride = (size_t)W * Cow;
        // all sign collections first (2*RW independent dependency chains in one basic block),
        // then the words, then the stores
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
        for (int r = 0; r < RW; ++r) words[r] = finish_word64(sgn[r][0], sgn[r][1], psel);
#pragma unroll
        for (int r = 0; r < RW; ++r)
            if (ok && yb + r < H && out_bits) orow[r * row_stride] = words[r];
        if (POOL) {
            // the tile origin is even: every 2x2 window lies inside one wave's rows and inside
            // one lane pair; an odd last row / column of the image belongs to no window
#pragma unroll
            for (int r = 0; r < RW; r += 2) {
                const int y = yb + r;
                uint32_t v = words[r] | words[r + 1];
                // neighbouring lane (quad permute [1,0,3,2]) holds the next pixel of the row
                v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, true);
                if (ok && (y >> 1) < Hl && (x >> 1) < Wl && (col & 1) == 0)
                    out_pool[(((size_t)n * Hl + (y >> 1)) * Wl + (x >> 1)) * Cow + widx] = v;
            }
        }
        cur.advance(tstep);
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
    const int32_t *__restrict__ wsum, uint32_t *__restrict__ out_bits, int32_t *__restrict__ out_acc)
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
            // 0.5 for every channel of a pixel outside the image, 0 for a word that does not exist
            uint4 v = make_uint4(0, 0, 0, 0);
            if (k < Cw) {
                if (yy >= 0 && yy < H && xx >= 0 && xx < W)
                    v = expand_word(act[(((size_t)n * H + yy) * W + xx) * Cw + k]);
                else
                    v = make_uint4(0x11111111u, 0x11111111u, 0x11111111u, 0x11111111u);
            }
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
                // the accumulator holds sum w a' (a half-integer): sum w a = 2 sum w a' - sum w
                vals[i] = (int)(2.0f * acc[m][r][i]) - ((cbase + i) < Cout ? wsum[cbase + i] : 0);
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

// the sums of the weights per output channel (row 10 of the count section) of the blob whose
// matrix fragments start at `wfrag`
static const int32_t *weight_sums(const uint4 *wfrag, const BlobLayout &L)
{
    const uint8_t *blob = (const uint8_t *)wfrag - L.off_f4;
    return (const int32_t *)(blob + L.off_cnt) + (size_t)10 * L.cout_pad64;
}


// Layers with two input steps: the row-streaming kernel (32 output channels per wave) or the
// block-cooperative one?  Measured on MI355X: 128->128 at 512x1024 30.5 us against 33.1 us,
// 128->256 at 256x512 21.3 us against 19.2 us - every wave of another channel tile stages the
// strip again, and short row segments pay the prologue more often.  So: at most four channel
// tiles, and segments of 24 rows or more when every wave slot has one.
static bool use_rows2k(int N, int H, int W, const BlobLayout &L, bool wants_bits)
{
    if (!conv_rows2k_supported(H, W, L, wants_bits)) return false;
    if (t_cfg.tune_rw == 9) return true;
    if (t_cfg.tune_rw != 0) return false;
    const long wave_rows = (long)N * H * ceil_div(W, 32) * (L.cout >> 5);
    return L.cout <= 128 && wave_rows >= 24L * 2048;
}
static const int kPersistentBlocks = 512;   // resident blocks of the block-cooperative kernel (2 per CU)

// waves per SIMD of the row-streaming kernel for single-step layers, 0 = kernel not used
static int rows_kernel_waves()
{
    const int m = t_cfg.tune_rw;
    return (m == 0 || m == 7 || m == 9) ? 2 : m == 8 ? 1 : 0;
}

bool conv_writes_pooled(int H, int W, const BlobLayout &L)
{
    if (H < 2 || W < 2) return false;
    return L.ksteps > 1 || (rows_kernel_waves() && conv_rows_supported(H, W, L, true));
}

template <int RW, int MT, bool CW_EVEN, bool ONE_STEP>
static int launch_bits_t(const uint32_t *act, int N, int H, int W, const BlobLayout &L,
                         const uint4 *wfrag, const int32_t *thresh, uint32_t *out_bits,
                         hipStream_t s)
{
    const int32_t *wsum = weight_sums(wfrag, L);
    const int ctiles = L.cout_pad64 / (32 * MT);
    const long ptiles = (long)N * ceil_div(H, RW) * ceil_div(W, TW);
    if (ptiles > 0x7fffffffL) return fail(MBU_ERR_SHAPE, "too many tiles for one launch");
    // two waves per SIMD over the whole chip; every wave keeps one output-channel tile
    // and strides over the pixel tiles
    const int max_waves = 2 * 4 * 256;
    if (ctiles > max_waves) return fail(MBU_ERR_SHAPE, "too many output channels");
    const int slots = (int)min(ptiles, (long)(max_waves / ctiles));
    const int waves = slots * ctiles;
    const TileStep tstep = tile_step(slots, ceil_div(W, TW), ceil_div(H, RW));
    MBU_LAUNCH((conv_mfma_bits_kernel<RW, MT, CW_EVEN, ONE_STEP>), dim3(ceil_div(waves, 4)),
               dim3(256), 0, s, act, N, H, W, L.cin_words, L.ksteps, wfrag, L.cout, ctiles, slots,
               (int)ptiles, tstep, thresh, wsum, out_bits);
    return check_launch("conv_mfma_bits");
}

// what a matrix-path launch works on: plain input, or the virtual concatenation
// [act | up-sampled low]; optional pooled second output
struct ConvIO {
    const uint32_t *act;
    const uint32_t *low;     // NULL = single source
    int low_shift;           // 1: low is read 2x up-sampled, 0: pixel for pixel
    int hb, wb;              // pixels of low; its (up-sampled) extent may fall short of the image
    int cwa, cwb;            // words per pixel of act / low
    uint32_t *out_bits;      // may be NULL when out_pool is set
    uint32_t *out_pool;      // NULL = no pooled output
};

template <int RW, int WM, int WN, bool TWO_SRC, bool POOL>
static int launch_block_t(const ConvIO &io, int N, int H, int W, const BlobLayout &L,
                          const uint4 *wfrag, const int32_t *thresh, hipStream_t s)
{
    const int tiles64 = L.cout_pad64 / 64;
    long tiles = (long)N * ceil_div(H, RW * WM) * ceil_div(W, TW);
    if (tiles > 0x7fffffffL) return fail(MBU_ERR_SHAPE, "too many tiles for one launch");
    if ((double)N * H * W * io.cwa * 4 >= 2147483648.0 ||
        (TWO_SRC && (double)N * io.hb * io.wb * io.cwb * 4 >= 2147483648.0))
        return fail(MBU_ERR_SHAPE, "input tensor too large for one launch (2 GiB)");
    // persistent blocks: two per compute unit in total, spread over the output-channel
    // groups; each strides over the pixel tiles
    const int groups = ceil_div(tiles64, WN);
    const long per_group = max(1, kPersistentBlocks / groups);
    dim3 grid((unsigned)min(tiles, per_group), (unsigned)groups);
    const TileStep tstep = tile_step((int)grid.x, ceil_div(W, TW), ceil_div(H, RW * WM));
    const bool even = (io.cwa % 2 == 0) && (!TWO_SRC || io.cwb % 2 == 0);
    if (even)
        MBU_LAUNCH((conv_mfma_block_kernel<RW, WM, WN, true, TWO_SRC, POOL>), grid, dim3(256), 0, s,
                   io.act, io.low, N, H, W, io.cwa, io.cwb, io.low_shift, io.hb, io.wb, L.ksteps, wfrag, L.cout, tiles64,
                   (int)tiles, tstep, thresh, weight_sums(wfrag, L), io.out_bits, io.out_pool);
    else
        MBU_LAUNCH((conv_mfma_block_kernel<RW, WM, WN, false, TWO_SRC, POOL>), grid, dim3(256), 0, s,
                   io.act, io.low, N, H, W, io.cwa, io.cwb, io.low_shift, io.hb, io.wb, L.ksteps, wfrag, L.cout, tiles64,
                   (int)tiles, tstep, thresh, weight_sums(wfrag, L), io.out_bits, io.out_pool);
    return check_launch("conv_mfma_block");
}

template <int RW, int WM, int WN>
static int launch_block(const ConvIO &io, int N, int H, int W, const BlobLayout &L,
                        const uint4 *wfrag, const int32_t *thresh, hipStream_t s)
{
    if (io.low && io.out_pool) return launch_block_t<RW, WM, WN, true, true>(io, N, H, W, L, wfrag, thresh, s);
    if (io.low) return launch_block_t<RW, WM, WN, true, false>(io, N, H, W, L, wfrag, thresh, s);
    if (io.out_pool) return launch_block_t<RW, WM, WN, false, true>(io, N, H, W, L, wfrag, thresh, s);
    return launch_block_t<RW, WM, WN, false, false>(io, N, H, W, L, wfrag, thresh, s);
}

template <int RW, int MT>
static int launch_bits(const uint32_t *act, int N, int H, int W, const BlobLayout &L,
                       const uint4 *wfrag, const int32_t *thresh, uint32_t *out_bits, hipStream_t s)
{
    if (L.ksteps == 1) {
        if (L.cin_words % 2 == 0)
            return launch_bits_t<RW, MT, true, true>(act, N, H, W, L, wfrag, thresh, out_bits, s);
        return launch_bits_t<RW, MT, false, true>(act, N, H, W, L, wfrag, thresh, out_bits, s);
    }
    if (L.cin_words % 2 == 0)
        return launch_bits_t<RW, MT, true, false>(act, N, H, W, L, wfrag, thresh, out_bits, s);
    return launch_bits_t<RW, MT, false, false>(act, N, H, W, L, wfrag, thresh, out_bits, s);
}

static int launch_block_auto(const ConvIO &io, int N, int H, int W, const BlobLayout &L,
                             const uint4 *wfrag, const int32_t *thresh, hipStream_t s)
{
    // waves of a block over output-channel tiles when there are enough of them
    const int tiles64 = L.cout_pad64 / 64;
    if (tiles64 % 4 == 0) return launch_block<4, 1, 4>(io, N, H, W, L, wfrag, thresh, s);
    if (tiles64 % 2 == 0) return launch_block<4, 2, 2>(io, N, H, W, L, wfrag, thresh, s);
    return launch_block<4, 4, 1>(io, N, H, W, L, wfrag, thresh, s);
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
                   L.ksteps, wfrag, L.cout, thresh, weight_sums(wfrag, L), out_bits, out_acc);
        return check_launch("conv_mfma_acc");
    }
    // Kernel choice (measured on MI355X): with a single 64-channel input step the vector work
    // per tile (staging, sign collection) is more than half the matrix time and only the
    // row-streaming kernel hides it (64->64 at 1024x2048: 25 us against 31 us for the
    // wave-private tile kernel, which remains for shapes the streaming kernel does not take);
    // with several steps the block-cooperative kernel stages least per wave and wins.
    const int mode = t_cfg.tune_rw;   // 0 = automatic; see mbu_set_conv_tuning
    if (use_rows2k(N, H, W, L, out_bits != nullptr))
        return launch_conv_mfma_rows2k(act, nullptr, 0, 0, N, H, W, L, blob, thresh, out_bits, nullptr, s);
    const bool want_block = mode == 1 || ((mode == 0 || mode == 9) && L.ksteps > 1);
    if (want_block) {
        ConvIO io{act, nullptr, 0, 0, 0, L.cin_words, 0, out_bits, nullptr};
        return launch_block_auto(io, N, H, W, L, wfrag, thresh, s);
    }
    if (rows_kernel_waves() && conv_rows_supported(H, W, L, out_bits != nullptr))
        return launch_conv_mfma_rows(act, N, H, W, L, blob, thresh, out_bits, nullptr, rows_kernel_waves(), s);
    if (mode == 6) return launch_bits<6, 1>(act, N, H, W, L, wfrag, thresh, out_bits, s);
    return launch_bits<3, 2>(act, N, H, W, L, wfrag, thresh, out_bits, s);
}

// Fused form: input = [act (Ca channels) | low (Clow channels)] when low is given - Hb x Wb
// pixels, read up-sampled 2x when low_shift = 1, zeros where its extent falls short of H x W -
// plus an optional 2x2-pooled second output.  The low-resolution decoder kernel, the
// row-streaming kernels for a single source, else the block-cooperative kernel.
int launch_conv_mfma_two(const uint32_t *act, int Ca, const uint32_t *low, int Clow, int low_shift,
                         int Hb, int Wb, int N, int H, int W, const BlobLayout &L, const void *blob,
                         const int32_t *thresh, uint32_t *out_bits, uint32_t *out_pool, hipStream_t s)
{
    if (low && low_shift == 1 && 2 * Hb == H && 2 * Wb == W && t_cfg.tune_rw != 1 &&
        conv_upcat_supported(Ca, Clow, N, H, W, L, out_bits, out_pool))
        return launch_conv_mfma_upcat(act, Ca, low, Clow, N, H, W, L, blob, thresh, out_bits, s);
    if (!low && rows_kernel_waves() && conv_rows_supported(H, W, L, out_bits != nullptr))
        return launch_conv_mfma_rows(act, N, H, W, L, blob, thresh, out_bits, out_pool, rows_kernel_waves(), s);
    if (!low && use_rows2k(N, H, W, L, out_bits != nullptr))
        return launch_conv_mfma_rows2k(act, nullptr, 0, 0, N, H, W, L, blob, thresh, out_bits, out_pool, s);
    // [64 channels | 64 channels of a second tensor of the layer's resolution] (first layer of the
    // last decoder level behind a transposed layer): the two-source form of the same kernel
    if (low && low_shift == 0 && Ca == 64 && Clow == 64 && t_cfg.tune_rw != 1 && use_rows2k(N, H, W, L, out_bits != nullptr))
        return launch_conv_mfma_rows2k(act, low, Hb, Wb, N, H, W, L, blob, thresh, out_bits, out_pool, s);
    const uint4 *wfrag = (const uint4 *)((const uint8_t *)blob + L.off_f4);
    ConvIO io{act, low, low ? low_shift : 0, low ? Hb : 0, low ? Wb : 0, ceil_div(Ca, 32),
              low ? ceil_div(Clow, 32) : 0, out_bits, out_pool};
    return launch_block_auto(io, N, H, W, L, wfrag, thresh, s);
}

}  // namespace mbu
