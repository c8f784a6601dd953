// Device helpers shared by the matrix-core kernels (3x3 layer and transposed 2x2 layer):
// the FP4 matrix instruction wrapper, the bit -> E2M1 expansion of activations and the
// completion of packed output words.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

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

// Activations enter the matrix instructions as a' = (a + 1) / 2, i.e. the packed bit itself:
// code 0x2 (1.0) for bit 1, 0x0 for bit 0, and 0x1 (0.5) for a pixel outside the image, whose
// value 0 lies half way.  Then sum w a = 2 sum w a' - sum w over ALL taps and channels, borders
// included, so the constant goes into the threshold: the accumulators start at
// -(theta + sum w) / 2 and hold half-integers (exact).  Half of the activation nibbles are zero
// this way; measured on MI355X the multi-step layers run 2-3 % faster than with +-1 codes.
//
// bits of one packed word -> 32 E2M1 codes; nibble q of dword d carries channel 4q + d.
__device__ inline uint4 expand_word(uint32_t w)
{
    uint4 r;
    r.x = (w << 1) & 0x22222222u;
    r.y = w & 0x22222222u;
    r.z = (w >> 1) & 0x22222222u;
    r.w = (w >> 2) & 0x22222222u;
    return r;
}
// the same under masks: m2 = 0x22222222 and p1 = 0 inside the image, m2 = 0 and p1 = 0x11111111
// outside (m2 = p1 = 0 for a word the tensor does not have)
__device__ __forceinline__ uint4 expand_word_masked(uint32_t w, uint32_t m2, uint32_t p1)
{
    uint4 r;
    r.x = ((w << 1) & m2) | p1;
    r.y = (w & m2) | p1;
    r.z = ((w >> 1) & m2) | p1;
    r.w = ((w >> 2) & m2) | p1;
    return r;
}
// -(theta + sum w) / 2 with theta clamped to +-2^22 (which cannot change a comparison);
// never -0.0, whose sign bit would read as "below the threshold"
__device__ __forceinline__ float start_value(int theta, int wsum)
{
    return 0.0f - 0.5f * (float)(max(-(1 << 22), min(1 << 22, theta)) + wsum);
}

// Completes the packed output words of one image row from the per-lane sign collections.
// s0 / s1: 16 sign bits (1 = below threshold) of channels 16*half + i of the wave's first /
// second 32-channel tile.  The two lane halves of a pixel are brought together with one
// v_permlane32_swap (lo = value of the pixel's lower-half lane, hi = of its upper-half lane,
// in every lane) and one byte permute picks word 0 (channels 0..31) in the lower half and
// word 1 (channels 32..63) in the upper half.  psel = 0x05040100 for half 0, 0x07060302 for
// half 1.
__device__ __forceinline__ uint32_t finish_word64(uint32_t s0, uint32_t s1, uint32_t psel)
{
    const uint32_t mine = (~s0 & 0xffffu) | (~s1 << 16);
    const auto sw = __builtin_amdgcn_permlane32_swap(mine, mine, false, false);
    // sw[0] = lower-half lane's value, sw[1] = upper-half lane's value
    return __builtin_amdgcn_perm(sw[1], sw[0], psel);
}

// Same for a wave that owns a single 32-channel tile: the word is (lo & 0xffff) | (hi << 16)
// in both halves.
__device__ __forceinline__ uint32_t finish_word32(uint32_t s0)
{
    const uint32_t mine = ~s0 & 0xffffu;
    const auto sw = __builtin_amdgcn_permlane32_swap(mine, mine, false, false);
    return sw[0] | (sw[1] << 16);
}

// Position of a pixel tile, advanced by a fixed stride without divisions: the stride is
// split on the host into (dx, dy, dn) = stride mod tiles_x, (stride / tiles_x) mod tiles_y,
// stride / (tiles_x * tiles_y).
struct TileStep {
    int tiles_x, tiles_y, dx, dy, dn;
};
struct TilePos {
    int tx, ty, n;
    __device__ __forceinline__ void advance(const TileStep &st)
    {
        tx += st.dx;
        if (tx >= st.tiles_x) { tx -= st.tiles_x; ++ty; }
        ty += st.dy;
        if (ty >= st.tiles_y) { ty -= st.tiles_y; ++n; }
        n += st.dn;
    }
};
__host__ __device__ inline TilePos tile_pos(int pt, int tiles_x, int tiles_y)
{
    TilePos p;
    p.tx = pt % tiles_x;
    const int q = pt / tiles_x;
    p.ty = q % tiles_y;
    p.n = q / tiles_y;
    return p;
}
inline TileStep tile_step(int stride, int tiles_x, int tiles_y)
{
    TileStep st;
    st.tiles_x = tiles_x;
    st.tiles_y = tiles_y;
    st.dx = stride % tiles_x;
    st.dy = (stride / tiles_x) % tiles_y;
    st.dn = stride / (tiles_x * tiles_y);
    return st;
}

}  // namespace mbu
