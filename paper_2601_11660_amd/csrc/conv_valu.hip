// Masked-binary 3x3 convolution on the vector ALU (Algorithm 1 on packed words,
// without matrix instructions).
//
// Eq. 2 with planes P = b_pos, G = b_neg and activation word A:  the set of kept taps
// whose sign disagrees with the activation is (A & G) | (~A & P) - one bitfield
// insert - so   acc = kept_in_image - 2 * popcount(mismatches),
// two vector-ALU instructions (v_bfi_b32, accumulating v_bcnt_u32_b32) per 32 taps.
//
// Mapping: lane = output channel (64 per wave), the pixel is wave-uniform, so the
// activation word is a scalar operand, both weight planes sit in vector registers,
// and the threshold compare of the 64 lanes *is* the packed output word pair.
// A wave walks a strip of TX pixels of one image row; input channels are processed
// in chunks of WCH words with the chunk's 2*9*WCH plane words held in registers.
#include "mbu_internal.h"

namespace mbu {

template <int WCH, int TX>
__global__ __launch_bounds__(256) void conv_valu_kernel(
    const uint32_t *__restrict__ act, int N, int H, int W, int Cw, int chunks,
    const uint32_t *__restrict__ pos, const uint32_t *__restrict__ neg,
    const int32_t *__restrict__ cnt, int cout_pad, int Cout,
    const int32_t *__restrict__ thresh, uint32_t *__restrict__ out_bits,
    int32_t *__restrict__ out_acc)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int strips_per_row = (W + TX - 1) / TX;
    const long strips = (long)N * H * strips_per_row;
    const long strip = (long)blockIdx.x * 4 + wave;
    if (strip >= strips) return;
    const int sx = (int)(strip % strips_per_row);
    const long row = strip / strips_per_row;
    const int y = (int)(row % H);
    const int n = (int)(row / H);
    const int x0 = sx * TX;
    const int o = blockIdx.y * 64 + lane;  // < cout_pad by construction

    int mism[TX];
#pragma unroll
    for (int i = 0; i < TX; ++i) mism[i] = 0;

    for (int ch = 0; ch < chunks; ++ch) {
        uint32_t P[9][WCH], G[9][WCH];
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int j = 0; j < WCH; ++j) {
                int k = ch * WCH + j;
                bool in = k < Cw;
                size_t at = ((size_t)t * Cw + (in ? k : 0)) * cout_pad + o;
                P[t][j] = in ? pos[at] : 0u;
                G[t][j] = in ? neg[at] : 0u;
            }
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) {
            const int yy = y + ky - 1;
            if (yy < 0 || yy >= H) continue;  // wave-uniform
            const uint32_t *arow = act + ((size_t)n * H + yy) * W * Cw;
#pragma unroll
            for (int i = -1; i <= TX; ++i) {
                const int xx = x0 + i;
                if (xx < 0 || xx >= W) continue;  // wave-uniform
                uint32_t A[WCH];
#pragma unroll
                for (int j = 0; j < WCH; ++j) {
                    int k = ch * WCH + j;
                    A[j] = k < Cw ? arow[(size_t)xx * Cw + k] : 0u;
                }
#pragma unroll
                for (int kx = 0; kx < 3; ++kx) {
                    const int px = i - kx + 1;  // output pixel fed through tap (ky,kx)
                    if (px < 0 || px >= TX) continue;
#pragma unroll
                    for (int j = 0; j < WCH; ++j) {
                        uint32_t a = A[j];
                        uint32_t bad = (a & G[ky * 3 + kx][j]) | (~a & P[ky * 3 + kx][j]);
                        mism[px] += __popc(bad);
                    }
                }
            }
        }
    }

    // kept-weight counts of the taps that fall inside the image
    int kept_tap[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) kept_tap[t] = cnt[(size_t)t * cout_pad + o];
    const int th = o < Cout ? thresh[o] : 0x7fffffff;
    const int Cow = Cout >> 5;
#pragma unroll
    for (int px = 0; px < TX; ++px) {
        const int x = x0 + px;
        if (x >= W) break;  // wave-uniform
        int kept = 0;
#pragma unroll
        for (int ky = 0; ky < 3; ++ky)
#pragma unroll
            for (int kx = 0; kx < 3; ++kx) {
                const int yy = y + ky - 1, xx = x + kx - 1;
                if (yy >= 0 && yy < H && xx >= 0 && xx < W) kept += kept_tap[ky * 3 + kx];
            }
        const int acc = kept - 2 * mism[px];
        const size_t pix = ((size_t)n * H + y) * W + x;
        if (out_acc && o < Cout) out_acc[pix * Cout + o] = acc;
        if (out_bits) {
            const unsigned long long m = __ballot(acc >= th);
            const int word = blockIdx.y * 2 + lane;
            if (lane < 2 && word < Cow)
                out_bits[pix * Cow + word] = lane == 0 ? (uint32_t)m : (uint32_t)(m >> 32);
        }
    }
}

template <int WCH, int TX>
static int launch_t(const uint32_t *act, int N, int H, int W, const BlobLayout &L,
                    const void *blob, const int32_t *thresh, uint32_t *out_bits,
                    int32_t *out_acc, hipStream_t s)
{
    const uint8_t *b = (const uint8_t *)blob;
    long strips = (long)N * H * ceil_div(W, TX);
    dim3 grid((unsigned)((strips + 3) / 4), (unsigned)(L.cout_pad64 / 64));
    MBU_LAUNCH((conv_valu_kernel<WCH, TX>), grid, dim3(256), 0, s, act, N, H, W,
                       L.cin_words, ceil_div(L.cin_words, WCH),
                       (const uint32_t *)(b + L.off_pos), (const uint32_t *)(b + L.off_neg),
                       (const int32_t *)(b + L.off_cnt), L.cout_pad64, L.cout, thresh, out_bits,
                       out_acc);
    return check_launch("conv_valu");
}

int launch_conv_valu(const uint32_t *act, int N, int H, int W, const BlobLayout &L,
                     const void *blob, const int32_t *thresh, uint32_t *out_bits,
                     int32_t *out_acc, hipStream_t s)
{
    if (L.cin_words == 1)
        return launch_t<1, 8>(act, N, H, W, L, blob, thresh, out_bits, out_acc, s);
    if (L.cin_words == 2 || L.cin_words == 3 || L.cin_words == 6)
        return launch_t<2, 8>(act, N, H, W, L, blob, thresh, out_bits, out_acc, s);
    return launch_t<4, 8>(act, N, H, W, L, blob, thresh, out_bits, out_acc, s);
}

}  // namespace mbu
