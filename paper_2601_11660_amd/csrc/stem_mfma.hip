// Full-precision first layer (Sec. 4.1) on the matrix cores, with sign bits that are
// identical to those of the sequential float32 definition.
//
// Definition (what the output bits must equal): y = sum over (ky, kx, ci) in that order of
// w * x, started at 0.0f, one fused multiply-add per term, zero padding; bit = (y >= 0).
// Only the SIGN of y leaves this layer, and the sign of a sum is known without the exact
// rounding sequence whenever a cheaper estimate is further from zero than its own error:
//
//   scaling        the sign of y[o, p] does not change when the weights of output channel o and
//                  the patch of pixel p are each multiplied by a positive power of two, so
//                  every weight row and every patch is scaled (exactly) to a Euclidean norm
//                  in [2^12, 2^13): whatever the magnitudes of the inputs, fp16 then neither
//                  overflows (values < 2^13) nor loses more than 2^-25 absolute per value to
//                  its subnormal range (2^-37 of the norm; 2^-26 of it if subnormal inputs
//                  were flushed);
//   fast estimate  every scaled float is split into two fp16 terms v = vh + vl + r, both
//                  rounded to nearest, |r| <= 2^-22 |v|; yf = sum wh*xh + wh*xl + wl*xh on
//                  v_mfma_f32_32x32x16_f16 (fp16 products are exact in the fp32 accumulator);
//   error budget   |yf - y| <= kappa * ||w_o||_2 * ||x_patch||_2 (in scaled units), every term
//                  relative to S = sum |w||x| <= ||w||_2 ||x||_2 (see STEM_KAPPA below): the
//                  rounding of the sequential chain itself, the terms the split drops, and the
//                  additions inside the matrix instructions, bounded for ANY order of addition
//                  and for rounding to nearest or truncation to 24 bits alike;
//   decision       |yf| >  T = kappa * max_o ||w_o|| * ||x_patch||  ->  sign(y) = sign(yf);
//                  otherwise the output is recomputed by the sequential chain itself, on the
//                  unscaled float32 inputs.
//
// About 1 output in 10^5 takes the second route with normally distributed data, so the
// layer costs 12 matrix instructions per 32 pixels x 64 channels instead of 64 x 27 fused
// multiply-adds per pixel.  Non-finite inputs, and norms outside [2^-60, 2^60], make T
// infinite and send every affected output down the sequential route; an all-zero patch gives
// +0.0f without any arithmetic.
//
// GEMM view: D[channel][pixel] = sum_k Wt[channel][k] * X[k][pixel], k = (ky*3 + kx)*Ci + ci
// (the memory order of the weights), padded to KT*16.  A wave owns 64 output channels
// (two 32-row tiles, weights scaled and split once and kept in registers) and walks over
// tiles of 32 consecutive pixels of an image row.  Lane (column j, half h) gathers the patch
// values k = 16t + 8h + i of pixel x0 + j through a raw buffer resource - a border tap or a
// padded k gets an offset beyond the buffer and reads 0.0f.
#include "mbu_internal.h"
#include "mfma_common.h"
#include <algorithm>

namespace mbu {

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef float v2f __attribute__((ext_vector_type(2)));

// Error budget of the fast estimate relative to S = sum |w_k||x_k| <= ||w||_2 ||x||_2, worst
// case, no measured term:
//   sequential chain (the definition's own rounding): 27 fused multiply-adds, each within 2^-24
//     of a partial sum that is at most S in magnitude                       27 * 2^-24 = 1.61e-6
//   terms the split drops: wl*xl, rw*x, w*rx with |wl|, |xl| <= 2^-11, |rw|, |rx| <= 2^-22
//     of the value                                                        ~  3 * 2^-22 = 0.72e-6
//   additions inside the matrix instructions.  The products of two fp16 values are exact in
//     fp32; what is assumed of the hardware is only that every addition it performs - in
//     whatever order - is accurate to 2^-23 of its result (round to nearest gives 2^-24,
//     truncation to 24 bits 2^-23).  The two groups of small products (wl*xh, wh*xl; at most
//     2^-10 S in total) are accumulated FIRST, while the accumulator is below 2^-10 S, so
//     their 56 additions contribute below 1e-8; the 28 additions of the wh*xh group (27 terms
//     and the constant) happen on partial sums of at most S(1 + 2^-9)        28 * 2^-23 = 3.34e-6
//   total 5.68e-6 < kappa = 2^-17 = 7.63e-6.
constexpr float STEM_KAPPA = 0x1p-17f;
constexpr uint32_t OOB = 0x80000000u;   // byte offset beyond any accepted image

// (a, b) -> packed fp16 pairs hi and lo with v = hi + lo + r, |r| <= 2^-22 |v| (+ 2^-25):
// both conversions round to nearest and the remainder is computed without error
__device__ __forceinline__ void split_pair(float a, float b, uint32_t &hi, uint32_t &lo)
{
    const v2f f = {a, b};
    const v2h h = __builtin_convertvector(f, v2h);
    const v2f r = f - __builtin_convertvector(h, v2f);
    hi = __builtin_bit_cast(uint32_t, h);                                   // low half = a
    lo = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, v2h));
}

// the power of two that brings a norm in [2^-60, 2^60] into [2^12, 2^13)
__device__ __forceinline__ float norm_scale(float nrm)
{
    const uint32_t e = (__float_as_uint(nrm) >> 23) & 0xffu;               // nrm in [2^(e-127), 2^(e-126))
    return __uint_as_float((266u - e) << 23);                              // 2^(12 - (e - 127))
}

__device__ __forceinline__ v8h as_v8h(const uint4 &v) { return __builtin_bit_cast(v8h, v); }

__device__ __forceinline__ float swap_add(float v)
{
    const uint32_t u = __float_as_uint(v);
    const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
}

template <int CI, bool WRITE_PRE>
__global__ __launch_bounds__(256) void stem_mfma_kernel(
    const float *__restrict__ img, uint32_t img_bytes, int N, int H, int W,
    const float *__restrict__ w, int Co, int nchunks, int nslots, int ntiles, TileStep tstep,
    uint32_t *__restrict__ out, float *__restrict__ pre)
{
    constexpr int KV = 9 * CI;             // terms per output
    constexpr int KT = (KV + 15) / 16;     // 16-wide K blocks
    constexpr int NS = KT * 8;             // patch values per lane
    // k = KV is the first padded term; it lives in slot BIAS_SLOT of the lanes of half BIAS_HALF
    constexpr int BIAS_SLOT = 8 * (KV / 16) + (KV % 8), BIAS_HALF = (KV / 8) % 2;
    static_assert(KV < 16 * KT, "a padded k is needed for the constant term");

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int gw = blockIdx.x * 4 + wave;
    if (gw >= nchunks * nslots) return;    // whole wave leaves; nothing is shared
    const int chunk = gw % nchunks;        // 64 output channels, fixed for the wave
    const int slot = gw / nchunks;
    const int col = lane & 31, half = lane >> 5;
    const bool tile1 = chunk * 64 + 32 < Co;   // second 32-channel tile exists (Co % 32 == 0)

    // ---- weights of this wave: every row scaled to a norm in [2^12, 2^13), split once, kept
    // in registers.  The lane holds half of the K range of row `col` of both channel tiles.
    uint4 Wh[2][KT], Wl[2][KT];
    float row_unscale[2];   // 1 / scale of this lane's row (exact), for the diagnostic output
    uint32_t rb = 0;        // bit pattern of the largest scaled row norm (see below)
    bool w_sane = true;     // every row norm is finite and inside [2^-60, 2^60], or exactly 0
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const int ch = chunk * 64 + m * 32 + tile_row_to_channel(col);
        float v[NS];
        float part = 0.0f;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int k = 16 * (s >> 3) + 8 * half + (s & 7);
            const bool ok = ch < Co && k < KV;
            const float wv = w[ok ? (size_t)ch * KV + k : 0];   // unconditional load
            v[s] = ok ? wv : 0.0f;
            part = __builtin_fmaf(v[s], v[s], part);
        }
        const float nrm = __builtin_sqrtf(swap_add(part));      // both halves: ||w_row||_2
        const bool in_range = nrm >= 0x1p-60f && nrm <= 0x1p60f;
        if (!(in_range || nrm == 0.0f)) w_sane = false;
        const float sc = in_range ? norm_scale(nrm) : 1.0f;
        // A row of zeros gives y = +0 for every pixel (bit 1), but its estimate 0 would never
        // be decided.  Such a row gets a weight on the first padded k, where every pixel
        // supplies the constant 1 (see BIAS_PAIR below): its estimate is 2^13, far above T.
        if (nrm == 0.0f && ch < Co && KV == 16 * (BIAS_SLOT >> 3) + 8 * half + (BIAS_SLOT & 7))
            v[BIAS_SLOT] = 0x1p13f;
        row_unscale[m] = 1.0f / sc;
        rb = max(rb, __float_as_uint(nrm * sc));
#pragma unroll
        for (int t = 0; t < KT; ++t) {
            uint32_t h4[4], l4[4];
#pragma unroll
            for (int d = 0; d < 4; ++d)
                split_pair(v[8 * t + 2 * d] * sc, v[8 * t + 2 * d + 1] * sc, h4[d], l4[d]);
            Wh[m][t] = make_uint4(h4[0], h4[1], h4[2], h4[3]);
            Wl[m][t] = make_uint4(l4[0], l4[1], l4[2], l4[3]);
        }
    }
    // wave maximum of the scaled row norms (unsigned order of the bit patterns of non-negative
    // floats is their numeric order) and wave-wide sanity of the rows
#pragma unroll
    for (int o = 16; o >= 1; o >>= 1) rb = max(rb, (uint32_t)__shfl_xor((int)rb, o));
    const float Wn = __uint_as_float(rb);
    w_sane = __builtin_amdgcn_ballot_w64(!w_sane) == 0;

    // ---- per-lane table of the NS gathered patch values: byte offset from the pixel and
    // which border makes the tap fall outside the image
    uint32_t off4[NS];
    uint32_t m_up = 0, m_dn = 0, m_lf = 0, m_rt = 0;
#pragma unroll
    for (int s = 0; s < NS; ++s) {
        const int k = 16 * (s >> 3) + 8 * half + (s & 7);
        const int kk = k < KV ? k : 0;
        const int tap = kk / CI, ci = kk - tap * CI;
        const int ky = tap / 3, kx = tap - 3 * ky;
        off4[s] = k < KV ? (uint32_t)(((long)ci * H * W + (long)(ky - 1) * W + (kx - 1)) * 4) : OOB;
        if (k < KV) {
            m_up |= (ky == 0 ? 1u : 0u) << s;
            m_dn |= (ky == 2 ? 1u : 0u) << s;
            m_lf |= (kx == 0 ? 1u : 0u) << s;
            m_rt |= (kx == 2 ? 1u : 0u) << s;
        }
    }
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)img, 0, (int)img_bytes, 0x00020000);

    const int Cow = Co >> 5;
    const uint32_t psel = half ? 0x07060302u : 0x05040100u;
    const int widx = chunk * 2 + half;
    // geometry of a tile for this lane, and the gather of its patch values (0.0f outside the image)
    struct Geo { int y, n, x, xc; uint32_t pb; };
    auto geometry = [&](const TilePos &tp) {
        Geo g;
        g.y = tp.ty; g.n = tp.n;
        g.x = tp.tx * 32 + col;
        g.xc = min(g.x, W - 1);
        g.pb = (uint32_t)((((size_t)g.n * CI * H + g.y) * W + g.xc) * 4);
        return g;
    };
    auto gather = [&](const TilePos &tp, const Geo &g, float (&v)[NS]) {
        const bool interior = g.y > 0 && g.y < H - 1 && tp.tx > 0 && tp.tx * 32 + 32 < W;
        if (interior) {
#pragma unroll
            for (int s = 0; s < NS; ++s)
                v[s] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc, g.pb + off4[s], 0, 0));
        } else {
            const uint32_t inv = (g.y == 0 ? m_up : 0u) | (g.y == H - 1 ? m_dn : 0u) |
                                 (g.xc == 0 ? m_lf : 0u) | (g.xc == W - 1 ? m_rt : 0u);
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                const uint32_t o = ((inv >> s) & 1u) ? OOB : g.pb + off4[s];
                v[s] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc, o, 0, 0));
            }
        }
    };

    // The operand planes of a tile: its patch values scaled to norm [2^12, 2^13) and split;
    // nx = scaled norm of the pixel's patch (0 for an all-zero patch, +inf when there is no
    // bound: non-finite or extreme values).  Built in pieces (see `tile`).
    struct Planes { uint4 h[KT], l[KT]; float nx, sc; };
    struct SplitState { float n2; uint32_t orb; float sc; };
    constexpr int NPIECE = 4 + NS / 2;
    auto split_piece = [&](int p, const float (&v)[NS], SplitState &st, Planes &P, uint32_t (&sh)[NS / 2],
                           uint32_t (&sl)[NS / 2]) {
        if (p == 0) {                       // squared norm of this lane's share, first half
            st.n2 = 0.0f;
#pragma unroll
            for (int s = 0; s < NS / 2; ++s) st.n2 = __builtin_fmaf(v[s], v[s], st.n2);
            asm volatile("" : "+v"(st.n2));
        } else if (p == 1) {                // ... second half
#pragma unroll
            for (int s = NS / 2; s < NS; ++s) st.n2 = __builtin_fmaf(v[s], v[s], st.n2);
            asm volatile("" : "+v"(st.n2));
        } else if (p == 2) {                // OR of the bit patterns: exact test for an all-zero patch
            st.orb = 0;
#pragma unroll
            for (int s = 0; s < NS; ++s) st.orb |= __float_as_uint(v[s]);
            asm volatile("" : "+v"(st.orb));
        } else if (p == 3) {                // both halves of the patch; the patch's scale
            const float nrm = __builtin_sqrtf(swap_add(st.n2));
            const auto sw = __builtin_amdgcn_permlane32_swap(st.orb, st.orb, false, false);
            const bool zero = ((sw[0] | sw[1]) << 1) == 0;
            const bool in_range = nrm >= 0x1p-60f && nrm <= 0x1p60f;
            st.sc = in_range ? norm_scale(nrm) : 1.0f;
            P.nx = zero ? 0.0f : (in_range ? nrm * st.sc : __builtin_inff());
            P.sc = st.sc;
            asm volatile("" : "+v"(st.sc), "+v"(P.nx));
        } else {                            // one pair of values: scale, split
            const int q = p - 4;
            split_pair(v[2 * q] * st.sc, v[2 * q + 1] * st.sc, sh[q], sl[q]);
            asm volatile("" : "+v"(sh[q]), "+v"(sl[q]));
        }
    };
    // the constant 1.0 (fp16) at the padded term k = KV of every pixel: its slot reads 0.0f
    const uint32_t bias_or = half == BIAS_HALF ? (0x3c00u << (16 * (BIAS_SLOT & 1))) : 0u;
    auto finish_planes = [&](Planes &P, uint32_t (&sh)[NS / 2], const uint32_t (&sl)[NS / 2]) {
        sh[BIAS_SLOT / 2] |= bias_or;
#pragma unroll
        for (int t = 0; t < KT; ++t) {
            P.h[t] = make_uint4(sh[4 * t], sh[4 * t + 1], sh[4 * t + 2], sh[4 * t + 3]);
            P.l[t] = make_uint4(sl[4 * t], sl[4 * t + 1], sl[4 * t + 2], sl[4 * t + 3]);
        }
    };

    // One tile: issue the loads of the tile after next, run the matrix instructions of the
    // current tile (operand planes B) with the scaling and split of the next tile's values
    // (vs -> Bn) cut into pieces, one after each matrix instruction - vector work is hidden only
    // between matrix instructions of the same wave - then decide and store.  Two sets of load
    // registers and two sets of operand planes alternate.
    TilePos ahead = tile_pos(slot, tstep.tiles_x, tstep.tiles_y);   // (tile in row, row, image)
    int tl_ahead = slot;                                           // tile index `ahead` stands for
    auto advance_ahead = [&]() {                                   // a wave's last tiles fetch themselves again
        if (tl_ahead + nslots < ntiles) { ahead.advance(tstep); tl_ahead += nslots; }
    };
    auto tile = [&](const Planes &B, Planes &Bn, float (&vs)[NS], float (&vl)[NS], const TilePos &pcur) {
        advance_ahead();
        gather(ahead, geometry(ahead), vl);
        const Geo gcur = geometry(pcur);

        // (the empty statements pin the loaded values to this iteration and "use" each piece's
        // results, so that the pieces stay between the matrix instructions as written)
#pragma unroll
        for (int s = 0; s < NS; ++s) asm volatile("" : "+v"(vs[s]));
        v16f acc[2];
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[m][i] = 0.0f;
        SplitState st;
        uint32_t sh[NS / 2], sl[NS / 2];
        int piece = 0, issued = 0;
        auto mma = [&](const uint4 (&WP)[2][KT], const uint4 (&BP)[KT]) {
#pragma unroll
            for (int t = 0; t < KT; ++t)
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_v8h(WP[m][t]), as_v8h(BP[t]), acc[m], 0, 0, 0);
                    ++issued;
                    __builtin_amdgcn_sched_barrier(0);
                    // one piece per matrix instruction, two while more pieces than instructions are left
                    if (piece < NPIECE) split_piece(piece++, vs, st, Bn, sh, sl);
                    if (piece < NPIECE && NPIECE - piece > 6 * KT - issued) split_piece(piece++, vs, st, Bn, sh, sl);
                    __builtin_amdgcn_sched_barrier(0);
                }
        };
        // small terms first; the two channel tiles alternate, so consecutive matrix
        // instructions never depend on each other
        mma(Wl, B.h);
        mma(Wh, B.l);
        mma(Wh, B.h);
#pragma unroll
        for (; piece < NPIECE; ++piece) split_piece(piece, vs, st, Bn, sh, sl);
        finish_planes(Bn, sh, sl);

        // ---- decision threshold of this pixel (scaled units; nx = +inf: no bound)
        const int y = gcur.y, n = gcur.n, x = gcur.x, xc = gcur.xc;
        const bool zero = B.nx == 0.0f;               // every patch value is +-0
        const float T = w_sane ? STEM_KAPPA * Wn * B.nx : __builtin_inff();
        float mn = __builtin_fminf(__builtin_fabsf(acc[0][0]), __builtin_fabsf(acc[0][1]));
#pragma unroll
        for (int i = 2; i < 16; ++i) mn = __builtin_fminf(mn, __builtin_fabsf(acc[0][i]));
        if (tile1) {
#pragma unroll
            for (int i = 0; i < 16; ++i) mn = __builtin_fminf(mn, __builtin_fabsf(acc[1][i]));
        }
        // (non-finite estimates need no test of their own: they only arise from non-finite
        // or extreme inputs, which make T infinite)
        const bool flag = x < W && !zero && !(mn > T);

        // ---- sign bits (1 = negative) of the 2 x 16 channels of this lane
        uint32_t sg[2] = {0u, 0u};
#pragma unroll
        for (int i = 15; i >= 0; --i)
#pragma unroll
            for (int m = 0; m < 2; ++m)
                sg[m] = __builtin_amdgcn_alignbit(sg[m], __float_as_uint(acc[m][i]), 31);

        const size_t pix = ((size_t)n * H + y) * W + xc;
        if (WRITE_PRE) {
            // the estimates in the units of the inputs: undo the (exact) scales of pixel and rows
            // (the row scales live in other lanes: fetched with every lane active)
            const float ux = 1.0f / B.sc;
#pragma unroll
            for (int m = 0; m < 2; ++m) {
                const int cb = chunk * 64 + m * 32 + 16 * half;
                float o16[16];
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    o16[i] = acc[m][i] * ux * __shfl(row_unscale[m], tile_channel_to_row(16 * half + i));
                if (x < W && cb < Co) {
                    float4 *dst = reinterpret_cast<float4 *>(pre + pix * Co + cb);
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        dst[q] = zero ? make_float4(0.0f, 0.0f, 0.0f, 0.0f)
                                      : make_float4(o16[4 * q], o16[4 * q + 1], o16[4 * q + 2], o16[4 * q + 3]);
                }
            }
        }

        // ---- sequential route for the undecided outputs (rare)
        if (__builtin_amdgcn_ballot_w64(flag) != 0) {
            if (WRITE_PRE) __builtin_amdgcn_s_waitcnt(0);   // the estimates are stored before the corrections
            if (flag) {
                // which outputs are undecided
                uint32_t fl[2];
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    fl[m] = 0;
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        fl[m] |= (!(__builtin_fabsf(acc[m][i]) > T) ? 1u : 0u) << i;
                    if (chunk * 64 + m * 32 + 16 * half >= Co) fl[m] = 0;
                }
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    const int cb = chunk * 64 + m * 32 + 16 * half;
                    while (fl[m]) {
                        const int i = __builtin_ctz(fl[m]);
                        fl[m] &= fl[m] - 1;
                        const float *wp = w + (size_t)(cb + i) * KV;
                        // the sum in its defined order, one kernel row (3 * CI terms) at a time;
                        // a tap outside the image is skipped, as in the definition
                        float s = 0.0f;
#pragma unroll
                        for (int ky = 0; ky < 3; ++ky) {
                            float pv[3 * CI], wv[3 * CI];
                            uint32_t okm = 0;
#pragma unroll
                            for (int e = 0; e < 3 * CI; ++e) {
                                const int kx = e / CI, ci = e - kx * CI;
                                const bool ok = !((ky == 0 && y == 0) || (ky == 2 && y == H - 1) ||
                                                  (kx == 0 && xc == 0) || (kx == 2 && xc == W - 1));
                                const uint32_t o = gcur.pb + (uint32_t)(((long)ci * H * W + (long)(ky - 1) * W + (kx - 1)) * 4);
                                pv[e] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc, ok ? o : OOB, 0, 0));
                                wv[e] = wp[ky * 3 * CI + e];
                                okm |= (ok ? 1u : 0u) << e;
                            }
#pragma unroll
                            for (int e = 0; e < 3 * CI; ++e) {
                                const float f = __builtin_fmaf(wv[e], pv[e], s);
                                s = ((okm >> e) & 1u) ? f : s;
                            }
                        }
                        sg[m] = (sg[m] & ~(1u << i)) | ((s >= 0.0f ? 0u : 1u) << i);   // NaN -> bit 0
                        if (WRITE_PRE) pre[pix * Co + cb + i] = s;
                    }
                }
            }
        }
        if (zero) { sg[0] = 0u; sg[1] = 0u; }   // a chain of zero terms ends at +0.0f
        const uint32_t word = finish_word64(sg[0], sg[1], psel);
        if (x < W && widx < Cow) out[pix * Cow + widx] = word;
    };

    float va[NS], vb[NS];
    Planes B0, B1;
    TilePos p0 = ahead;
    gather(p0, geometry(p0), va);
    {
        SplitState st;
        uint32_t sh[NS / 2], sl[NS / 2];
#pragma unroll
        for (int p = 0; p < NPIECE; ++p) split_piece(p, va, st, B0, sh, sl);
        finish_planes(B0, sh, sl);
    }
    advance_ahead();
    TilePos p1 = ahead;
    gather(p1, geometry(p1), va);
    for (int tl = slot; tl < ntiles; tl += 2 * nslots) {
        tile(B0, B1, va, vb, p0);
        p0 = p1;
        p1 = ahead;
        if (tl + nslots >= ntiles) break;
        tile(B1, B0, vb, va, p0);
        p0 = p1;
        p1 = ahead;
    }
}

// ---------------------------------------------------------------------------------------
// Row-walking variant for three image channels.
//
// The kernel above gathers and splits all 27 values of every patch although a value belongs
// to nine patches.  Here a wave walks down a strip of 32 pixel columns; for every image row it
// keeps the three rows of the 3x3 window as raw floats (lane p = halo pixel p of the strip:
// 9 values), scales and splits them ONCE per tile and hands them to the 32 patches of the row
// through wave-private LDS.  Sharing the split values means sharing the scale: instead of one
// power of two per patch the whole window (3 rows x 34 pixels x 3 channels) is scaled by one
// power of two s that brings its largest magnitude into [2^13, 2^14).  The error budget of the
// estimate changes in one place: the remainder of the split is bounded by 2^-22 |v| + 2^-25
// (the second term is the spacing of fp16 subnormals), and with a patch that is small against
// its window the absolute term no longer vanishes against the patch norm.  It is therefore part
// of the decision threshold:
//     T = kappa * max_o ||w_o|| * ||s x_patch||  +  2^-9
// (sum_k |w_k| 2^-25 <= sqrt(27) 2^13 2^-25 = 1.3e-3 < 2^-9 for rows scaled to a norm below
// 2^13).  Outputs with |estimate| <= T take the sequential route as before, so the bits are
// those of the definition whatever the data; a window that holds values more than ~2^17
// apart merely sends more of its small patches down that route.  Windows with a non-finite
// value, or with a largest magnitude below 2^-111, get T = +inf.  The squared patch norm is the
// sum of three per-pixel column sums exchanged through LDS; a NaN in it makes T NaN and the
// comparison fail, which is the sequential route again.
//
// K order of the matrix instruction (32 terms = 16 dwords of two fp16 values; lane (j, h) of a
// B operand supplies dwords 8t + 4h + d of block t): the LDS arrays hold one dword per halo
// pixel p - P_r[p] = channels (0, 1) of window row r, R01[p] = channel 2 of rows (0, 1),
// R2[p] = (channel 2 of row 2, 0) - and pixel j reads entries j, j + 1, j + 2 (kx = 0, 1, 2):
//     h = 0:  P0[j] P0[j+1] P0[j+2] P1[j]  |  P1[j+1] P1[j+2] R01[j]   R01[j+1]
//     h = 1:  P2[j] P2[j+1] P2[j+2] R2[j]  |  R2[j+1] R2[j+2] R01[j+2] (1.0, 0)
// The last dword is the constant that gives an all-zero weight row a decidable estimate (see
// the kernel above).  The weights are loaded in the same order.
constexpr int SR_HW = 34;                    // halo pixels of a strip
constexpr int SR_ARR = 36;                   // dwords per LDS array (34 used)
constexpr int SR_PLANE = 5 * SR_ARR;         // arrays P0 P1 R01 P2 R2 of one plane (hi or lo)
constexpr int SR_CONST = SR_PLANE - 1;       // spare dword of R2: the constant entry
constexpr int SR_N = 2 * SR_PLANE;           // per halo pixel: squared column norm, OR of the bits
constexpr int SR_WAVE = SR_N + 2 * SR_ARR;   // dwords per wave
constexpr float SR_FLOOR = 0x1p-9f;

// index into the 27 weights of an output channel for half h, dword dh = 4t + d, fp16 value e;
// -1: no term (weight 0), -2: the constant term
__host__ __device__ constexpr int sr_term(int h, int dh, int e)
{
    if (h == 0) {
        if (dh < 3) return (0 * 3 + dh) * 3 + e;
        if (dh < 6) return (1 * 3 + (dh - 3)) * 3 + e;
        return (e * 3 + (dh - 6)) * 3 + 2;
    }
    if (dh < 3) return (2 * 3 + dh) * 3 + e;
    if (dh < 6) return e == 0 ? (2 * 3 + (dh - 3)) * 3 + 2 : -1;
    if (dh == 6) return (e * 3 + 2) * 3 + 2;
    return e == 0 ? -2 : -1;
}

// maximum over the wave of a value that is the same non-negative number in no particular lane
// order (0 is the identity): shifts inside rows of 16 lanes, then lane 15 of a row into the
// next row, lane 31 into the upper half; lane 63 holds the result
__device__ __forceinline__ uint32_t wave_umax(uint32_t x)
{
    x = max(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, true));   // row_shr:1
    x = max(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, true));   // row_shr:2
    x = max(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, true));   // row_shr:4
    x = max(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, true));   // row_shr:8
    x = max(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false));  // row_bcast:15
    x = max(x, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false));  // row_bcast:31
    return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}

__global__ __launch_bounds__(256, 3) void stem_rows_kernel(
    const float *__restrict__ img, uint32_t img_bytes, int H, int W, const float *__restrict__ w, int Co,
    int nchunks, int strips, int nseg, int seg_rows, int units, uint32_t *__restrict__ out)
{
    constexpr int KV = 27;
    __shared__ uint32_t lds[4][SR_WAVE];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int gw = blockIdx.x * 4 + wave;
    if (gw >= units) return;                   // whole wave leaves; nothing is shared
    int q = gw;
    const int chunk = q % nchunks; q /= nchunks;   // 64 output channels
    const int sx = q % strips; q /= strips;        // strip of 32 pixel columns
    const int sg = q % nseg;                       // segment of seg_rows image rows
    const int n = q / nseg;
    const int col = lane & 31, half = lane >> 5;
    const bool tile1 = chunk * 64 + 32 < Co;       // second 32-channel tile exists (Co % 32 == 0)
    const int y0 = sg * seg_rows;
    const int rows = min(H, y0 + seg_rows) - y0;
    const int x0 = sx * 32;

    // ---- weights: rows scaled to a norm in [2^12, 2^13), split once, in the K order above
    uint4 Wh[2][2], Wl[2][2];
    uint32_t rb = 0;
    bool w_sane = true;
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const int ch = chunk * 64 + m * 32 + tile_row_to_channel(col);
        float v[16];
        float part = 0.0f;
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            const int k0 = sr_term(0, s >> 1, s & 1), k1 = sr_term(1, s >> 1, s & 1);
            const int k = half ? k1 : k0;
            const bool ok = ch < Co && k >= 0;
            const float wv = w[ok ? (size_t)ch * KV + k : 0];   // unconditional load
            v[s] = ok ? wv : 0.0f;
            part = __builtin_fmaf(v[s], v[s], part);
        }
        const float nrm = __builtin_sqrtf(swap_add(part));
        const bool in_range = nrm >= 0x1p-60f && nrm <= 0x1p60f;
        if (!(in_range || nrm == 0.0f)) w_sane = false;
        const float sc = in_range ? norm_scale(nrm) : 1.0f;
        if (nrm == 0.0f && ch < Co && half == 1) v[14] = 0x1p13f;   // the constant term (dword 7)
        rb = max(rb, __float_as_uint(nrm * sc));
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            uint32_t h4[4], l4[4];
#pragma unroll
            for (int d = 0; d < 4; ++d)
                split_pair(v[8 * t + 2 * d] * sc, v[8 * t + 2 * d + 1] * sc, h4[d], l4[d]);
            Wh[m][t] = make_uint4(h4[0], h4[1], h4[2], h4[3]);
            Wl[m][t] = make_uint4(l4[0], l4[1], l4[2], l4[3]);
        }
    }
    rb = wave_umax(rb);
    const float KW = STEM_KAPPA * 1.002f * __uint_as_float(rb);   // margin: the patch norm is good to 2^-10
    w_sane = __builtin_amdgcn_ballot_w64(!w_sane) == 0;

    // ---- addresses.  Staging: lane p < 34 owns halo pixel p (image column x0 - 1 + p); the
    // other lanes repeat pixel 33.  Zero padding: a column or row outside the image gets an
    // offset beyond the buffer and reads 0.0f.
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)img, 0, (int)img_bytes, 0x00020000);
    const int p = min(lane, SR_HW - 1);
    const int xs = x0 - 1 + p;
    const uint32_t xoff = (xs >= 0 && xs < W) ? (uint32_t)xs * 4u : OOB;
    uint32_t *const ldsw = lds[wave];
    uint32_t *const wr = ldsw + p;
    const uint32_t *const q0 = ldsw + (half ? 3 * SR_ARR : 0) + col;            // P0 | P2, then P1 | R2
    const uint32_t *const q2 = ldsw + 2 * SR_ARR + col + (half ? 2 : 0);        // R01[j] | R01[j+2]
    const uint32_t *const q3 = ldsw + (half ? SR_CONST : 2 * SR_ARR + col + 1); // R01[j+1] | constant
    if (lane == 0) {
        ldsw[SR_CONST] = 0x3c00u;              // (1.0, 0) in the hi plane, 0 in the lo plane
        ldsw[SR_CONST + SR_PLANE] = 0u;
    }

    const int Cow = Co >> 5;
    const uint32_t psel = half ? 0x07060302u : 0x05040100u;
    const int widx = chunk * 2 + half;
    const int xo = x0 + col;                   // output pixel column of this lane
    // packed output of image n as a buffer: lane offset inside a row, row offset per tile
    const uint32_t out_row_bytes = (uint32_t)W * Cow * 4u;
    const __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(out + (size_t)n * H * W * Cow), 0, (int)(H * out_row_bytes), 0x00020000);
    // (validity goes into the row offset alone: two out-of-range marks would add up to 0)
    const uint32_t out_voff = (uint32_t)(xo * Cow + widx) * 4u;

    struct Planes { uint4 h[2], l[2]; float ns[3]; uint32_t ob[3]; bool ok; };

    // one image row of the strip: three floats per lane
    auto fetch = [&](int yy, float (&v)[3]) {
        const bool rin = yy >= 0 && yy < H;
        const int yc = min(max(yy, 0), H - 1);
        const uint32_t vo = rin ? xoff : OOB;
#pragma unroll
        for (int c = 0; c < 3; ++c)
            v[c] = __uint_as_float(
                __builtin_amdgcn_raw_buffer_load_b32(rsrc, vo, (int)((((size_t)n * 3 + c) * H + yc) * W * 4), 0));
    };
    // largest magnitude of a row over the wave, as the bit pattern of a non-negative float
    auto row_max = [&](const float (&v)[3]) {
        const uint32_t a = __float_as_uint(v[0]) & 0x7fffffffu, b = __float_as_uint(v[1]) & 0x7fffffffu,
                       c = __float_as_uint(v[2]) & 0x7fffffffu;
        return wave_umax(max(max(a, b), c));
    };

    // Staging of a window (rows a[0..2], their maxima rm[0..2]) in pieces; piece k of STAGE_PIECES.
    // The scaled values are kept as the pairs that are split together: channels (0, 1) of a
    // row, channel 2 of rows (0, 1), channel 2 of row 2.
    struct Stage { v2f pr[3], z01, z2; float s; uint32_t orb; bool ok; uint32_t sh[5], sl[5]; };
    auto split2 = [](v2f f, uint32_t &hi, uint32_t &lo) {
        hi = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, v2h));
        // f - hi (exact: the difference has at most 24 bits) with the fp16 operand converted by
        // the instruction itself: -1.0 * hi.lo + f[0], -1.0 * hi.hi + f[1]
        v2f r;
        asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel_hi:[1,0,0]" : "=v"(r[0]) : "v"(hi), "v"(f[0]));
        asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r[1]) : "v"(hi), "v"(f[1]));
        lo = __builtin_bit_cast(uint32_t, __builtin_convertvector(r, v2h));
    };
    constexpr int STAGE_PIECES = 12;
    auto stage_piece = [&](int slot, const float (&a)[3][3], const uint32_t (&rm)[3], Stage &st, Planes &Bn) {
        // order of the pieces: scale (0, 1), OR (3), splits (4..8), column norm (2), LDS (9..11)
        constexpr int ORDER[12] = {0, 1, 3, 4, 5, 6, 7, 8, 2, 9, 10, 11};
        const int k = ORDER[slot];
        if (k == 0) {
            uint32_t mb = max(rm[0], rm[1]);
            asm volatile("" : "+s"(mb));       // wave-uniform: keeps the scale arithmetic on the scalar unit
            mb = max(mb, rm[2]);
            const uint32_t e = mb >> 23;
            st.ok = e >= 16u && e <= 254u;
            st.s = st.ok ? __uint_as_float((267u - e) << 23) : 1.0f;
            st.pr[0] = (v2f){a[0][0] * st.s, a[0][1] * st.s};
            st.pr[1] = (v2f){a[1][0] * st.s, a[1][1] * st.s};
            asm volatile("" : "+v"(st.pr[0]), "+v"(st.pr[1]));
        } else if (k == 1) {
            st.pr[2] = (v2f){a[2][0] * st.s, a[2][1] * st.s};
            st.z01 = (v2f){a[0][2] * st.s, a[1][2] * st.s};
            st.z2 = (v2f){a[2][2] * st.s, 0.0f};
            asm volatile("" : "+v"(st.pr[2]), "+v"(st.z01), "+v"(st.z2));
        } else if (k == 3) {
            uint32_t o[3];
#pragma unroll
            for (int r = 0; r < 3; ++r)
                o[r] = __float_as_uint(a[r][0]) | __float_as_uint(a[r][1]) | __float_as_uint(a[r][2]);
            st.orb = o[0] | o[1] | o[2];
            asm volatile("" : "+v"(st.orb));
        } else if (k == 4) {
            split2(st.pr[0], st.sh[0], st.sl[0]);
            asm volatile("" : "+v"(st.sh[0]), "+v"(st.sl[0]));
        } else if (k == 5) {
            split2(st.pr[1], st.sh[1], st.sl[1]);
            asm volatile("" : "+v"(st.sh[1]), "+v"(st.sl[1]));
        } else if (k == 6) {
            split2(st.z01, st.sh[2], st.sl[2]);
            asm volatile("" : "+v"(st.sh[2]), "+v"(st.sl[2]));
        } else if (k == 7) {
            split2(st.pr[2], st.sh[3], st.sl[3]);
            asm volatile("" : "+v"(st.sh[3]), "+v"(st.sl[3]));
        } else if (k == 8) {
            split2(st.z2, st.sh[4], st.sl[4]);
            asm volatile("" : "+v"(st.sh[4]), "+v"(st.sl[4]));
        } else if (k == 2) {
            // squared norm of this pixel's column from the leading fp16 terms (2^-10 relative,
            // covered by the margin in KW; what rounds to zero there is below 2^-24 and covered
            // by the constant part of the threshold), and its OR, for the three patches the
            // column belongs to
            float n2 = 0.0f;
#pragma unroll
            for (int i = 0; i < 5; ++i) {
                const v2h h = __builtin_bit_cast(v2h, st.sh[i]);
                n2 = __builtin_amdgcn_fdot2(h, h, n2, false);
            }
            ldsw[SR_N + 2 * p] = __float_as_uint(n2);
            ldsw[SR_N + 2 * p + 1] = st.orb;
        } else if (k == 9) {
            // array order in LDS: P0 P1 R01 P2 R2
#pragma unroll
            for (int i = 0; i < 5; ++i) {
                wr[i * SR_ARR] = st.sh[i];
                wr[i * SR_ARR + SR_PLANE] = st.sl[i];
            }
            __builtin_amdgcn_wave_barrier();
        } else if (k == 10) {
            // LDS instructions of a wave execute in order: these reads see the writes above
            Bn.h[0] = make_uint4(q0[0], q0[1], q0[2], q0[SR_ARR]);
            Bn.h[1] = make_uint4(q0[SR_ARR + 1], q0[SR_ARR + 2], q2[0], q3[0]);
            Bn.l[0] = make_uint4(q0[SR_PLANE], q0[SR_PLANE + 1], q0[SR_PLANE + 2], q0[SR_PLANE + SR_ARR]);
            Bn.l[1] = make_uint4(q0[SR_PLANE + SR_ARR + 1], q0[SR_PLANE + SR_ARR + 2], q2[SR_PLANE], q3[SR_PLANE]);
        } else {
            // the three columns of this lane's patch; the threshold is formed where it is used
#pragma unroll
            for (int d = 0; d < 3; ++d) {
                Bn.ns[d] = __uint_as_float(ldsw[SR_N + 2 * (col + d)]);
                Bn.ob[d] = ldsw[SR_N + 2 * (col + d) + 1];
            }
            Bn.ok = st.ok;
            __builtin_amdgcn_wave_barrier();   // the next window is written after these reads
        }
    };

    // ---- decision and store of a finished row
    struct Done { float T; bool zero; int i; };
    struct Epi { float mn; uint32_t sg[2]; };
    constexpr int EPI_PIECES = 7;
    auto epi_piece = [&](int k, const v16f (&acc)[2], const Done &dn, Epi &ep) {
        if (k == 0) {
            float mn = __builtin_fminf(__builtin_fabsf(acc[0][0]), __builtin_fabsf(acc[0][1]));
#pragma unroll
            for (int e = 2; e < 16; ++e) mn = __builtin_fminf(mn, __builtin_fabsf(acc[0][e]));
            ep.mn = mn;
            ep.sg[0] = ep.sg[1] = 0u;
            asm volatile("" : "+v"(ep.mn));
        } else if (k == 1) {
            if (tile1) {
                float mn = ep.mn;
#pragma unroll
                for (int e = 0; e < 16; ++e) mn = __builtin_fminf(mn, __builtin_fabsf(acc[1][e]));
                ep.mn = mn;
            }
            asm volatile("" : "+v"(ep.mn));
        } else if (k < 6) {
            // sign bits (1 = negative) of the 2 x 16 channels of this lane, four per tile and piece
#pragma unroll
            for (int e = 15 - 4 * (k - 2); e > 11 - 4 * (k - 2); --e)
#pragma unroll
                for (int m = 0; m < 2; ++m)
                    ep.sg[m] = __builtin_amdgcn_alignbit(ep.sg[m], __float_as_uint(acc[m][e]), 31);
            asm volatile("" : "+v"(ep.sg[0]), "+v"(ep.sg[1]));
        } else {
            const int y = y0 + dn.i;
            const float T = dn.T;
            const bool live = xo < W && dn.i >= 0 && dn.i < rows;
            const bool flag = live && !dn.zero && !(ep.mn > T);
            // ---- sequential route for the undecided outputs (rare)
            if (__builtin_amdgcn_ballot_w64(flag) != 0) {
                if (flag) {
                    uint32_t fl[2];
#pragma unroll
                    for (int m = 0; m < 2; ++m) {
                        fl[m] = 0;
#pragma unroll
                        for (int e = 0; e < 16; ++e)
                            fl[m] |= (!(__builtin_fabsf(acc[m][e]) > T) ? 1u : 0u) << e;
                        if (chunk * 64 + m * 32 + 16 * half >= Co) fl[m] = 0;
                    }
                    const uint32_t pb = (uint32_t)((((size_t)n * 3 * H + y) * W + xo) * 4);
                    // the 27 patch values of this pixel, fetched once and in one batch (a tap
                    // outside the image is skipped in the chain below)
                    float pv[27];
                    uint32_t okm = 0;
#pragma unroll
                    for (int u = 0; u < 27; ++u) {
                        const int ky = u / 9, kx = (u % 9) / 3, ci = u % 3;
                        const bool ok = !((ky == 0 && y == 0) || (ky == 2 && y == H - 1) ||
                                          (kx == 0 && xo == 0) || (kx == 2 && xo == W - 1));
                        const uint32_t o = pb + (uint32_t)(((long)ci * H * W + (long)(ky - 1) * W + (kx - 1)) * 4);
                        pv[u] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsrc, ok ? o : OOB, 0, 0));
                        okm |= (ok ? 1u : 0u) << u;
                    }
#pragma unroll
                    for (int m = 0; m < 2; ++m) {
                        const int cb = chunk * 64 + m * 32 + 16 * half;
                        while (fl[m]) {
                            const int e = __builtin_ctz(fl[m]);
                            fl[m] &= fl[m] - 1;
                            const float *wp = w + (size_t)(cb + e) * KV;
                            float wv[27];
#pragma unroll
                            for (int u = 0; u < 27; ++u) wv[u] = wp[u];
                            // the sum in its defined order: ky, kx, ci
                            float sum = 0.0f;
#pragma unroll
                            for (int u = 0; u < 27; ++u) {
                                const float f = __builtin_fmaf(wv[u], pv[u], sum);
                                sum = ((okm >> u) & 1u) ? f : sum;
                            }
                            ep.sg[m] = (ep.sg[m] & ~(1u << e)) | ((sum >= 0.0f ? 0u : 1u) << e);   // NaN -> bit 0
                        }
                    }
                }
            }
            if (dn.zero) { ep.sg[0] = 0u; ep.sg[1] = 0u; }   // a chain of zero terms ends at +0.0f
            const uint32_t word = finish_word64(ep.sg[0], ep.sg[1], psel);
            const uint32_t roff = live && widx < Cow ? (uint32_t)y * out_row_bytes : OOB;
            __builtin_amdgcn_raw_buffer_store_b32(word, orsrc, out_voff + roff, 0, 0);
        }
    };

    // ---- one tile: matrix instructions of row y on planes B, between them the staging of row
    // y + 1 (rows a[1], a[2] and the row fetched two tiles ago); then decision and store.
    // (Running the decision of row y - 1 between the matrix instructions as well, with a second
    // set of accumulators, measured no faster: the kernel is bound by the vector instruction
    // count, and three waves per SIMD - which the smaller register count allows - hide more.)
    auto tile = [&](const int i, const Planes &B, Planes &Bn, float (&a)[3][3], uint32_t (&rm)[3],
                    float (&ld)[3]) {
        const int y = y0 + i;
        // the window moves down one row
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            a[0][c] = a[1][c];
            a[1][c] = a[2][c];
            a[2][c] = ld[c];
        }
        rm[0] = rm[1];
        rm[1] = rm[2];
        rm[2] = row_max(a[2]);
        fetch(y + 4, ld);

        v16f acc[2];
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[m][e] = 0.0f;
        Stage st;
        Epi ep;
        Done dn;
        int slot = 0;
        auto mma = [&](const uint4 (&WP)[2][2], const uint4 (&BP)[2]) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int m = 0; m < 2; ++m) {
                    acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_v8h(WP[m][t]), as_v8h(BP[t]), acc[m], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (slot < STAGE_PIECES) stage_piece(slot, a, rm, st, Bn);
                    ++slot;
                    __builtin_amdgcn_sched_barrier(0);
                }
        };
        mma(Wl, B.h);      // small terms first
        mma(Wh, B.l);
        mma(Wh, B.h);
        static_assert(STAGE_PIECES <= 12 && EPI_PIECES <= 12, "one piece of each kind per matrix instruction");

        dn.zero = ((B.ob[0] | B.ob[1] | B.ob[2]) << 1) == 0;          // every patch value is +-0
        // (the hardware square root is good to 1 ulp; KW carries the margin)
        dn.T = (B.ok && w_sane) ? __builtin_fmaf(KW, __builtin_amdgcn_sqrtf(B.ns[0] + B.ns[1] + B.ns[2]), SR_FLOOR)
                                : __builtin_inff();
        dn.i = i;
#pragma unroll
        for (int k = 0; k < EPI_PIECES; ++k) epi_piece(k, acc, dn, ep);
    };

    // ---- prologue: rows y0 - 1 .. y0 + 1 staged for the first tile, rows y0 + 2 and y0 + 3 in flight
    float a[3][3], ld0[3], ld1[3];
    uint32_t rm[3];
    Planes B0, B1;
#pragma unroll
    for (int r = 0; r < 3; ++r) fetch(y0 - 1 + r, a[r]);
    fetch(y0 + 2, ld0);
    fetch(y0 + 3, ld1);
#pragma unroll
    for (int r = 0; r < 3; ++r) rm[r] = row_max(a[r]);
    {
        Stage st;
#pragma unroll
        for (int k = 0; k < STAGE_PIECES; ++k) stage_piece(k, a, rm, st, B0);
    }
    // two rows per trip (operand planes and fetch registers alternate); with an odd row count the
    // second row of the last trip is computed and dropped
#pragma unroll 1
    for (int i = 0; i < rows; i += 2) {
        tile(i, B0, B1, a, rm, ld0);
        tile(i + 1, B1, B0, a, rm, ld1);
    }
}

static int launch_stem_rows(const float *img, uint32_t bytes, int N, int H, int W, const float *w, int Co,
                            uint32_t *out_bits, hipStream_t s)
{
    const int nchunks = ceil_div(Co, 64);
    const int strips = ceil_div(W, 32);
    const long base = (long)N * strips * nchunks;
    // as many row segments as it takes to give every wave slot of the chip (three per SIMD) one unit
    const long slots = 3L * 4 * 256;
    const int want = (int)std::max(1L, slots / base);
    int seg_rows = ceil_div(H, want);
    seg_rows = std::max(2, seg_rows + (seg_rows & 1));
    const int nseg = ceil_div(H, seg_rows);
    const long units = base * nseg;
    if (units > 0x7fffffffL) return fail(MBU_ERR_SHAPE, "stem: too many tiles for one launch");
    MBU_LAUNCH(stem_rows_kernel, dim3((unsigned)((units + 3) / 4)), dim3(256), 0, s, img, bytes, H, W, w, Co,
               nchunks, strips, nseg, seg_rows, (int)units, out_bits);
    return check_launch("stem_rows");
}


int launch_stem_mfma(const float *img, int N, int Ci, int H, int W, const float *w, int Co,
                     uint32_t *out_bits, float *out_pre, hipStream_t s)
{
    const double bytes = (double)N * Ci * H * W * 4.0;
    if (bytes >= 2147483648.0) return fail(MBU_ERR_SHAPE, "stem: image larger than 2 GiB");
    // (the row-walking kernel addresses the packed output of one image with 31-bit offsets)
    if (Ci == 3 && !out_pre && t_cfg.stem_path != MBU_STEM_MFMA_GATHER && (double)(H + 1) * (W + 32) * (Co / 32) * 4.0 < 2147483648.0)
        return launch_stem_rows(img, (uint32_t)bytes, N, H, W, w, Co, out_bits, s);
    const int tiles_x = ceil_div(W, 32);
    const long ntiles = (long)N * H * tiles_x;
    if (ntiles > 0x7fffffffL) return fail(MBU_ERR_SHAPE, "stem: too many tiles for one launch");
    const int nchunks = ceil_div(Co, 64);
    // two waves per SIMD over the whole chip (what the register budget allows), so all waves
    // are resident at once; every wave keeps one 64-channel chunk
    const int max_waves = 2 * 4 * 256;
    if (nchunks > max_waves) return fail(MBU_ERR_SHAPE, "stem: too many output channels");
    const int nslots = (int)min(ntiles, (long)(max_waves / nchunks));
    const int waves = nslots * nchunks;
    const TileStep tstep = tile_step(nslots, tiles_x, H);
    const dim3 grid(ceil_div(waves, 4)), block(256);
#define MBU_STEM_LAUNCH(CI, PRE)                                                                    \
    MBU_LAUNCH((stem_mfma_kernel<CI, PRE>), grid, block, 0, s, img, (uint32_t)bytes, N, H, W, w, Co, \
               nchunks, nslots, (int)ntiles, tstep, out_bits, out_pre)
    if (Ci == 3) {
        if (out_pre) MBU_STEM_LAUNCH(3, true); else MBU_STEM_LAUNCH(3, false);
    } else if (Ci == 1) {
        if (out_pre) MBU_STEM_LAUNCH(1, true); else MBU_STEM_LAUNCH(1, false);
    } else {
        return fail(MBU_ERR_SHAPE, "stem supports 1 or 3 image channels, got %d", Ci);
    }
#undef MBU_STEM_LAUNCH
    return check_launch("stem_mfma");
}

}  // namespace mbu
