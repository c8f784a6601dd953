// Internal declarations shared by the translation units of the HIP library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "mbu.h"

namespace mbu {

// Record a failure description for mbu_last_error() and return `code`.
int fail(int code, const char *fmt, ...);
// Turn the HIP error state after a launch into a status.
int check_launch(const char *what);

// Settings of one call.  The process-wide settings (mbu_set_conv_path, mbu_set_conv_tuning,
// mbu_set_stem_path) live in atomics; every entry point copies them ONCE into this
// thread-local snapshot (begin_call) and everything below the entry point reads the copy, so
// a setter that runs on another thread cannot change a call that has started.
struct CallCfg {
    int conv_path;      // mbu_conv_path
    int stem_path;      // mbu_stem_path
    int tune_rw;        // kernel variant of the matrix-path convolution, 0 = automatic
    bool dry_run;       // true: launchers choose their kernel and record its name, launch nothing
    const char *kernel; // source name of the last kernel chosen by a launcher on this thread
};
extern thread_local CallCfg t_cfg;
void begin_call(bool dry_run = false);

// Launch wrapper: records which kernel was chosen; unless the call is a dry run it drops any
// stale error left by earlier, unrelated runtime calls (so that check_launch() reports this
// launch only) and launches.
#define MBU_LAUNCH(KERNEL_, grid, block, shmem, stream, ...)                         \
    do {                                                                            \
        mbu::t_cfg.kernel = #KERNEL_;                                               \
        if (!mbu::t_cfg.dry_run) {                                                  \
            (void)hipGetLastError();                                                \
            hipLaunchKernelGGL(KERNEL_, grid, block, shmem, stream, __VA_ARGS__);    \
        }                                                                           \
    } while (0)

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline size_t round_up(size_t v, size_t m) { return (v + m - 1) / m * m; }

// ---- layout of the packed-weight blob (all offsets in bytes from the blob start) ----
// Section V (vector-ALU path, optional: MBU_BLOB_BIT_PLANES): two bit planes, each uint32
// [9][cin_words][cout_pad64] (tap-major, output channel fastest so 64 lanes read 64
// consecutive words).  Always present: the kept-weight counts int32 [11][cout_pad64]: rows
// 0..8 per tap, row 9 the total, row 10 the sum of the channel's weights.
// Section M (matrix-core path): 4-bit codes, uint4 [cout_pad64/64][ksteps][9 taps][2][64 lanes],
// one 16-byte fragment per lane and (32 output channels, tap, 64 input channels); the 18
// fragments one wave needs for a 64-channel step are contiguous (18 KB).
// Section U (matrix-core path, optional: MBU_BLOB_SUMMED_TAPS; input channels that arrive 2x
// up-sampled): the 3x3 kernel summed
// over the taps that share a low-resolution pixel, 4-bit codes of sums in -4..4,
// uint4 [cout_pad64/64][ksteps][4 parity classes][2][2][2][64 lanes].
struct BlobLayout {
    int cout, cin;
    int sections;      // MBU_BLOB_* bits: which optional sections the blob holds (absent = size 0)
    int cin_words;     // ceil(cin/32)
    int cout_pad64;    // cout rounded up to 64
    int ksteps;        // ceil(cin/64): 64-channel steps of the matrix path
    int cout_tiles32;  // cout/32
    size_t off_pos, off_neg, off_cnt, off_f4, off_up, total;
};
BlobLayout blob_layout(int cout, int cin, int sections = MBU_BLOB_ALL);

// ---- packed blob of the transposed 2x2 stride-2 layer: 4-bit codes,
// uint4 [cout_pad64/64][ksteps][4 positions][2][64 lanes] after 256 bytes of header room, then the
// sum of the weights of every (position, output channel) (activations enter as 0 / 1)
struct TconvLayout {
    int cout, cin, cin_words, cout_pad64, ksteps;
    size_t off_f4, off_sum, total;   // fragments; int32 [4 positions][cout_pad64] sums of the weights
};
TconvLayout tconv_layout(int cout, int cin);

// Row order of output channels inside one 32-channel matrix tile: tile row i holds
// output channel tile_row_to_channel(i) of the tile, chosen so that the sixteen
// accumulator registers of a lane map to sixteen consecutive output-channel bits.
__host__ __device__ inline int tile_row_to_channel(int i) {
    // accumulator register r of lane-half h holds tile row 8*(r/4) + 4*h + r%4
    int g = i >> 3, h = (i >> 2) & 1, j = i & 3;
    return 16 * h + 4 * g + j;
}
__host__ __device__ inline int tile_channel_to_row(int c) {
    int h = c >> 4, g = (c >> 2) & 3, j = c & 3;
    return 8 * g + 4 * h + j;
}


// ---- kernel launchers (arguments already validated) ----
int launch_pack_act(const void *src, int dtype, long pixels, int C, uint32_t *dst, hipStream_t s);
int launch_pack_weights(const int8_t *w, const BlobLayout &L, void *blob, hipStream_t s);
int launch_conv_valu(const uint32_t *act, int N, int H, int W, const BlobLayout &L,
                     const void *blob, const int32_t *thresh, uint32_t *out_bits,
                     int32_t *out_acc, hipStream_t s);
int launch_conv_mfma(const uint32_t *act, int N, int H, int W, const BlobLayout &L,
                     const void *blob, const int32_t *thresh, uint32_t *out_bits,
                     int32_t *out_acc, hipStream_t s);
// Input = [act | low]: low has Hb x Wb pixels of Clow channels, read 2x up-sampled when
// low_shift = 1 and pixel for pixel when 0; where its (up-sampled) extent falls short of H x W
// its channels are zeros.  low = NULL: single input.  out_pool: optional 2x2-pooled output.
int launch_conv_mfma_two(const uint32_t *act, int Ca, const uint32_t *low, int Clow, int low_shift,
                         int Hb, int Wb, int N, int H, int W, const BlobLayout &L, const void *blob,
                         const int32_t *thresh, uint32_t *out_bits, uint32_t *out_pool, hipStream_t s);
// row-streaming kernel for layers with a single 64-channel input step (optional 2x2-pooled
// second output); waves_per_simd = 1 or 2
bool conv_rows_supported(int H, int W, const BlobLayout &L, bool wants_bits);
// the same scheme for layers with two 64-channel input steps, 32 output channels per wave
bool conv_rows2k_supported(int H, int W, const BlobLayout &L, bool wants_bits);
// act2 != NULL: the input is [act (64 channels) | act2 (64 channels, Hb x Wb pixels, zeros beyond)]
int launch_conv_mfma_rows2k(const uint32_t *act, const uint32_t *act2, int Hb, int Wb, int N, int H, int W,
                            const BlobLayout &L, const void *blob, const int32_t *thresh, uint32_t *out_bits,
                            uint32_t *out_pool, hipStream_t s);
int launch_conv_mfma_rows(const uint32_t *act, int N, int H, int W, const BlobLayout &L, const void *blob,
                          const int32_t *thresh, uint32_t *out_bits, uint32_t *out_pool, int waves_per_simd,
                          hipStream_t s);
// does the matrix path write the 2x2-pooled output of this layer from its own epilogue?
// (layers with several input steps always; single-step layers when the row-streaming kernel runs)
bool conv_writes_pooled(int H, int W, const BlobLayout &L);
// [skip | 2x up-sampled low] with the up-sampled channels contracted at low resolution
int launch_pack_upcat(const int8_t *w, const BlobLayout &L, void *blob, hipStream_t s);
bool conv_upcat_supported(int Ca, int Clow, int N, int H, int W, const BlobLayout &L, const uint32_t *out_bits,
                          const uint32_t *out_pool);
int launch_conv_mfma_upcat(const uint32_t *act, int Ca, const uint32_t *low, int Clow, int N, int H, int W,
                           const BlobLayout &L, const void *blob, const int32_t *thresh, uint32_t *out_bits,
                           hipStream_t s);
int launch_pack_tconv(const int8_t *w, const TconvLayout &L, void *blob, hipStream_t s);
int launch_tconv_mfma(const uint32_t *act, int N, int H, int W, const TconvLayout &L,
                      const void *blob, const int32_t *thresh, uint32_t *out_bits, int32_t *out_acc,
                      hipStream_t s);
int launch_maxpool(const uint32_t *in, int N, int H, int W, int Cw, uint32_t *out, hipStream_t s);
int launch_upsample(const uint32_t *in, int N, int H, int W, int Cw, uint32_t *out, hipStream_t s);
int launch_concat(const uint32_t *a, int Caw, const uint32_t *b, int Cbw, long pixels,
                  uint32_t *out, hipStream_t s);
// out[n][y][x] = [ skip[n][y][x] | up[n][y/2][x/2] ]  (H, W are the output size)
int launch_upcat(const uint32_t *skip, int Csw, const uint32_t *low, int Clw,
                 int N, int H, int W, uint32_t *out, hipStream_t s);
// first layer: sequential float32 chain on the vector ALU / matrix-core estimate with the
// sequential chain for undecided signs; out_pre (NHWC float32) may be NULL
int launch_stem_valu(const float *img, int N, int Ci, int H, int W, const float *w, int Co,
                     uint32_t *out_bits, float *out_pre, hipStream_t s);
int launch_stem_mfma(const float *img, int N, int Ci, int H, int W, const float *w, int Co,
                     uint32_t *out_bits, float *out_pre, hipStream_t s);
int launch_classifier(const uint32_t *act, int N, int H, int W, int C, const float *w,
                      const float *b, int K, float *out, hipStream_t s);

}  // namespace mbu
