/*
 * mbu.h - C ABI of the MI355X (gfx950) masked-binary U-Net inference library.
 *
 * The library executes the inference path of MBU-Net: binary activations a in
 * {-1,+1} bit-packed along channels, ternary ("masked") weights w in {-1,0,+1}
 * held as two bit planes (subtractive encoding, Sec. 3.2.1, Eq. 2), a 3x3
 * convolution whose every output is an integer dot product, and a fused epilogue
 * that compares with a per-channel integer threshold and re-packs the result
 * (Sec. 3.2.2, Algorithm 1).  Around it: bitwise pooling / up-sampling / skip
 * concatenation (Sec. 2.1, Sec. 3.2.2) and full-precision first and last layers
 * (Sec. 4.1).
 *
 * Conventions, valid for every entry point unless stated otherwise
 *  - Return value: MBU_OK (0) or a negative mbu_status.  mbu_last_error() gives a
 *    thread-local description of the last failure.  Arguments are validated on
 *    the host BEFORE anything is launched; an invalid call launches nothing.
 *  - All data pointers are DEVICE pointers owned by the caller (hipMalloc or a
 *    framework allocator) unless the parameter is documented as a host pointer.
 *    The library never allocates, frees or synchronises device memory.
 *  - Device pointers must be 16-byte aligned (MBU_ERR_ALIGN otherwise).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls are asynchronous with respect to the host and ordered on `stream`.
 *  - Packed activations: tensor [N][H][W][Cw] of uint32, Cw = ceil(C/32);
 *    channel c lives in bit (c % 32) of word (c / 32); bit 1 means +1, bit 0
 *    means -1.  Bits of the last word beyond C are 0 on output and ignored on
 *    input (their weights are packed as masked).
 *  - Unpacked layouts: activations NHWC, conv weights OHWI = [Cout][3][3][Cin],
 *    images and logits NCHW float32.
 */
#ifndef MBU_H_
#define MBU_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum mbu_status {
    MBU_OK = 0,
    MBU_ERR_NULL = -1,       /* a required pointer is NULL                           */
    MBU_ERR_SHAPE = -2,      /* non-positive / unsupported / inconsistent dimensions */
    MBU_ERR_ALIGN = -3,      /* a device pointer is not 16-byte aligned              */
    MBU_ERR_WORKSPACE = -4,  /* workspace too small                                  */
    MBU_ERR_HIP = -5,        /* the HIP runtime reported a launch/runtime failure    */
    MBU_ERR_ARG = -6         /* bad enum value, aliasing outputs, malformed blob     */
} mbu_status;

/* Which implementation mbu_conv3x3_masked_binary (and the network) uses. */
typedef enum mbu_conv_path {
    MBU_PATH_AUTO = 0,   /* library picks per layer shape (default)                       */
    MBU_PATH_VALU = 1,   /* bit path: one bitfield-insert + one accumulating popcount per  */
                         /* 32 taps on the vector ALU (Eq. 2 on packed words)             */
    MBU_PATH_MFMA = 2    /* bits expanded on the fly to 4-bit {-1,0,+1} codes and         */
                         /* contracted on the matrix cores, fp32 accumulators (exact)     */
} mbu_conv_path;

/* Description of the last failure on this thread ("" if none).  Host pointer,
 * owned by the library, valid until the next failing call on the thread. */
const char *mbu_last_error(void);

/* Select the convolution implementation process-wide.  MBU_ERR_ARG on a bad value.
 * Thread safety of this and the other setters (mbu_set_conv_tuning, mbu_set_stem_path): the
 * settings are process-wide atomics; every other entry point reads them ONCE when it is
 * entered, so a call that has started is not affected by a setter that runs meanwhile, and
 * all other entry points may be called from several threads at once (on different streams).
 * A sequence of calls that must see the same setting - a forward pass and the
 * mbu_unet_step_launches / mbu_unet_step_kernel queries that describe it - must not be
 * interleaved with a setter on another thread; the library does not serialise that. */
int mbu_set_conv_path(int path);
int mbu_get_conv_path(void);

/* Benchmarking hook: force the kernel variant of the matrix-path convolution process-wide.
 * kernel 0 = let the library choose per layer (default); 1 = block-cooperative kernel
 * (four waves share a staged window, 4 rows x 64 channels per wave; also instead of the
 * low-resolution kernel of layers with a 2x up-sampled second input); 3 = persistent
 * wave-private kernel with 3 rows x 64 channels per wave; 6 = the same with 6 rows x 32
 * channels; 7 / 8 = row-streaming kernel for layers with at most 64 input channels, two /
 * one waves per SIMD (7 is what 0 picks for such layers; other layers are not affected);
 * 9 = the row-streaming kernel also for every layer with 65..128 input channels (0 picks it
 * for such layers only with at most 128 output channels on large frames).
 * `reserved` must be 0.  Results never depend on it.  MBU_ERR_ARG otherwise. */
int mbu_set_conv_tuning(int kernel, int reserved);

/* Bit-packing of activations (Sec. 1: many binary values are grouped into one word
 * so one instruction handles them; Algorithm 1 consumes such fragments).
 *   src       NHWC [N][H][W][C]; src_dtype 0: int8 values, bit = (v > 0);
 *             src_dtype 1: float32 values, bit = (v >= 0)
 *   dst       uint32 [N][H][W][ceil(C/32)], pad bits written as 0
 * Errors: NULL pointers, non-positive dims, bad dtype, misaligned pointers. */
int mbu_pack_act(const void *src, int src_dtype, int N, int H, int W, int C,
                 uint32_t *dst, void *stream);

/* Size in bytes of the opaque packed-weight blob for a Cout x 3 x 3 x Cin layer.
 * `bytes` is a host pointer.  Cout must be a multiple of 32 (packed outputs). */
int mbu_packed_weights_bytes(int Cout, int Cin, size_t *bytes);

/* Subtractive two-plane encoding of masked weights (Sec. 3.2.1: b = b_pos - b_neg).
 *   w_ohwi   device int8 [Cout][3][3][Cin], values in {-1,0,+1} (anything else is
 *            treated by sign: >0 as +1, <0 as -1)
 *   packed   device blob of mbu_packed_weights_bytes(Cout,Cin) bytes, 16-byte
 *            aligned, written completely; layout is private to the library and
 *            holds the bit planes in the orders the kernels read them plus the
 *            per-(channel, tap) kept-weight counts used at image borders.
 * Channel padding up to the next multiple of 32/64 is packed as masked (0). */
int mbu_pack_weights(const int8_t *w_ohwi, int Cout, int Cin, void *packed,
                     void *stream);

/* The same with only the blob sections that will be read (Sec. 3.2.1 stores masked weights as
 * two bit planes; the matrix path needs its 4-bit fragments instead, and the 2x2 kernels of
 * summed taps only for layers whose second input arrives 2x up-sampled):
 *   MBU_BLOB_MATRIX       the 4-bit fragments and per-channel sums (always written)
 *   MBU_BLOB_BIT_PLANES   the two bit planes: read by the vector-ALU path (MBU_PATH_VALU)
 *   MBU_BLOB_SUMMED_TAPS  read by mbu_conv3x3_masked_binary_fused / _two_inputs with an
 *                         up-sampled second input and by such decoder layers of the network;
 *                         without it those calls still work, at the 9-tap cost
 * mbu_pack_weights = MBU_BLOB_ALL.  A blob with fewer sections is smaller (the summed taps are
 * 1.8x the fragments) and is only valid where its `sections` value travels with it: the
 * single-layer entry points assume MBU_BLOB_ALL; the network takes it per layer in
 * mbu_conv_layer.  MBU_ERR_ARG on unknown bits. */
#define MBU_BLOB_BIT_PLANES 1
#define MBU_BLOB_SUMMED_TAPS 2
#define MBU_BLOB_MATRIX 4
#define MBU_BLOB_ALL 7
int mbu_packed_weights_bytes_sections(int Cout, int Cin, int sections, size_t *bytes);
int mbu_pack_weights_sections(const int8_t *w_ohwi, int Cout, int Cin, int sections, void *packed,
                              void *stream);

/* Masked-binary 3x3 convolution, stride 1, padding 1, with the fused threshold /
 * sign / bit-pack epilogue (Algorithm 1; layer definition in Sec. 3.1.1).
 *   acc[n,y,x,o] = sum_{ky,kx,c} w[o,ky,kx,c] * a[n,y+ky-1,x+kx-1,c]
 * where taps outside the image contribute 0 (they behave as masked weights), and
 *   bit[n,y,x,o] = (acc >= thresh[o])           (a tie gives +1).
 *   act       packed activations [N][H][W][ceil(Cin/32)]
 *   packed_w  blob from mbu_pack_weights for (Cout, Cin)
 *   thresh    int32 [Cout]
 *   out_bits  packed [N][H][W][Cout/32], or NULL
 *   out_acc   int32 NHWC [N][H][W][Cout], or NULL (debug/parity; costs bandwidth)
 * At least one output must be non-NULL; outputs must not alias `act`.  On the matrix path a
 * packed input tensor (each of the two of the fused forms) must stay below 2 GiB.
 * Errors: NULL/misaligned pointers, non-positive dims, Cout % 32 != 0, input too large; a blob that
 * was packed for other (Cout, Cin) is undefined behaviour (checked only by size
 * arguments, the header is device memory). */
int mbu_conv3x3_masked_binary(const uint32_t *act, int N, int H, int W, int Cin,
                              const void *packed_w, int Cout, const int32_t *thresh,
                              uint32_t *out_bits, int32_t *out_acc, void *stream);

/* The same layer with the U-Net glue around it fused in (matrix path only, whatever
 * mbu_set_conv_path says): the skip concatenation and the 2x up-sampling that feed a
 * decoder layer (Sec. 2.1) are read in place instead of being materialised, and the 2x2
 * pooling that follows an encoder layer (Sec. 3.2.2) is written as a second output.
 *   act       packed [N][H][W][Ca/32]; Ca % 32 == 0 when `low` is given
 *   low       packed [N][H/2][W/2][ceil(Clow/32)] (sizes rounded down) or NULL (then Clow must
 *             be 0); the layer's input is the channel concatenation [act | low up-sampled 2x
 *             nearest], i.e. input pixel (y, x) takes its last Clow channels from
 *             low[y/2][x/2]; for odd H / W the last row / column has no such pixel and its
 *             last Clow channels are the value 0 (they add nothing)
 *   packed_w  blob packed for (Cout, Cin = Ca + Clow)
 *   out_bits  packed [N][H][W][Cout/32], or NULL
 *   out_pool  packed [N][H/2][W/2][Cout/32] (sizes rounded down: an odd last row / column is in
 *             no window) = bitwise OR of each 2x2 window of the layer's output, or NULL
 * H, W >= 2 when `low` or `out_pool` is given; at least one output non-NULL.
 * Errors as for mbu_conv3x3_masked_binary. */
int mbu_conv3x3_masked_binary_fused(const uint32_t *act, int Ca, const uint32_t *low, int Clow,
                                    int N, int H, int W, const void *packed_w, int Cout,
                                    const int32_t *thresh, uint32_t *out_bits, uint32_t *out_pool,
                                    void *stream);

/* The 3x3 layer on the plain channel concatenation [a | b] of two tensors of the layer's own
 * size, read in place (skip connection after a transposed up-sampling layer, Sec. 2.1);
 * matrix path only.  a [N][H][W][Ca/32] with Ca % 32 == 0, b [N][H][W][ceil(Cb/32)],
 * packed_w packed for (Cout, Ca + Cb); outputs as for mbu_conv3x3_masked_binary_fused. */
int mbu_conv3x3_masked_binary_concat(const uint32_t *a, int Ca, const uint32_t *b, int Cb, int N,
                                     int H, int W, const void *packed_w, int Cout,
                                     const int32_t *thresh, uint32_t *out_bits, uint32_t *out_pool,
                                     void *stream);

/* General form of the two calls above, for decoder levels of frames whose size is not a multiple
 * of 2^levels (Appendix A.3 lists 959 x 640 frames; Sec. 2.1 for the decoder): pooling drops an
 * odd last row / column on the way down, so the up-sampled feature is smaller than the skip
 * feature and is zero-padded to its size before the concatenation.  The layer's input is
 * [a | b'] where b' is b (Hb x Wb pixels, Cb channels) - read 2x nearest-neighbour up-sampled when
 * upsample = 1 - placed at the top left of the H x W frame; where b' has no pixel its channels
 * are the value 0 and add nothing to the sums (like taps outside the image).  Matrix path only.
 *   a [N][H][W][Ca/32], Ca % 32 == 0;  b [N][Hb][Wb][ceil(Cb/32)], (Hb, Wb) << upsample <= (H, W)
 *   packed_w packed for (Cout, Ca + Cb); outputs as for mbu_conv3x3_masked_binary_fused. */
int mbu_conv3x3_masked_binary_two_inputs(const uint32_t *a, int Ca, const uint32_t *b, int Cb, int Hb,
                                         int Wb, int upsample, int N, int H, int W, const void *packed_w,
                                         int Cout, const int32_t *thresh, uint32_t *out_bits,
                                         uint32_t *out_pool, void *stream);

/* Masked-binary transposed convolution, kernel 2x2, stride 2, with the threshold / sign /
 * bit-pack epilogue: the decoder's up-sampling layer (Sec. 2.1; Sec. 3.2.2 notes it is
 * performed like the convolution; the quantised network follows it with batch norm and a
 * binary activation, Appendix A.1, which fold into the integer threshold as in Algorithm 1).
 *   acc[n, 2y+dy, 2x+dx, o] = sum_c w[o,dy,dx,c] * a[n,y,x,c],  bit = (acc >= thresh[o]).
 * Weights: device int8 [Cout][2][2][Cin] in {-1,0,+1}, packed once into a blob of
 * mbu_packed_tconv_weights_bytes(Cout, Cin) bytes (layout private; matrix path only).
 *   act       packed [N][H][W][ceil(Cin/32)]
 *   out_bits  packed [N][2H][2W][Cout/32], or NULL
 *   out_acc   int32 NHWC [N][2H][2W][Cout], or NULL (parity / debugging)
 * Errors as for mbu_conv3x3_masked_binary. */
int mbu_packed_tconv_weights_bytes(int Cout, int Cin, size_t *bytes);
int mbu_pack_tconv_weights(const int8_t *w, int Cout, int Cin, void *packed, void *stream);
int mbu_tconv2x2_masked_binary(const uint32_t *act, int N, int H, int W, int Cin,
                               const void *packed_w, int Cout, const int32_t *thresh,
                               uint32_t *out_bits, int32_t *out_acc, void *stream);

/* 2x2 stride-2 max pooling on +-1 values = bitwise OR of the four packed words
 * (Sec. 3.2.2 lists pooling as trivial).  H, W >= 2; H/2 and W/2 round down: an odd last
 * row / column belongs to no window and is dropped.
 *   in [N][H][W][Cw] -> out [N][H/2][W/2][Cw], Cw = ceil(C/32). */
int mbu_maxpool2x2_bits(const uint32_t *in, int N, int H, int W, int C,
                        uint32_t *out, void *stream);

/* 2x nearest-neighbour up-sampling of packed activations: out[y][x] = in[y/2][x/2].
 * Stands in the decoder where Sec. 2.1 describes a transposed convolution.
 *   in [N][H][W][Cw] -> out [N][2H][2W][Cw]. */
int mbu_upsample2x_bits(const uint32_t *in, int N, int H, int W, int C,
                        uint32_t *out, void *stream);

/* Skip concatenation along channels (Sec. 2.1): channels of `a` first, then `b`.
 * Ca must be a multiple of 32 so that the result stays word aligned.
 *   a [N][H][W][Ca/32], b [N][H][W][ceil(Cb/32)] -> out [N][H][W][Ca/32+ceil(Cb/32)] */
int mbu_concat_bits(const uint32_t *a, int Ca, const uint32_t *b, int Cb,
                    int N, int H, int W, uint32_t *out, void *stream);

/* Which implementation the float32 first layer uses (results are identical bit for bit). */
typedef enum mbu_stem_path {
    MBU_STEM_AUTO = 0,   /* matrix cores, unless out_pre is requested (default)            */
    MBU_STEM_VALU = 1,   /* the sequential fused-multiply-add chain for every output       */
    MBU_STEM_MFMA = 2,   /* split-fp16 estimate on the matrix cores; outputs whose sign    */
                         /* the estimate cannot decide are recomputed by the chain         */
    MBU_STEM_MFMA_GATHER = 3  /* the same with the per-pixel gather kernel also for three  */
                         /* image channels (otherwise a wave walks down a strip of the     */
                         /* image and shares the split values between patches)             */
} mbu_stem_path;
int mbu_set_stem_path(int path);
int mbu_get_stem_path(void);

/* Full-precision first layer (Sec. 4.1: the first convolution stays full precision; its
 * binary activation feeds the masked-binary layers): 3x3, stride 1, zero padding, no bias,
 *   y[n,y,x,o] = sum over ky, kx, ci (in that order, from 0.0f, one fused multiply-add per
 *                term) of w[o,ky,kx,ci] * image[n,ci,y+ky-1,x+kx-1],   bit = (y >= 0).
 * The order is part of the definition because the sign feeds bit-exact layers.
 *   image_nchw  float32 [N][Ci][H][W], Ci in {1, 3}, at most 2 GiB
 *   w           float32 [Co][3][3][Ci], Co a positive multiple of 32
 *   out_bits    packed [N][H][W][Co/32]
 *   out_pre     float32 NHWC [N][H][W][Co] or NULL (parity / debugging).  On the VALU path
 *               (and with MBU_STEM_AUTO) these are the chain's values y.  With MBU_STEM_MFMA
 *               they are the matrix-core estimates, within 2^-17 * ||w_o||_2 * ||patch||_2
 *               of y, except for the recomputed outputs, which are y itself.
 * Errors: NULL / misaligned pointers, bad shapes. */
int mbu_stem_fp32(const float *image_nchw, int N, int Ci, int H, int W, const float *w, int Co,
                  uint32_t *out_bits, float *out_pre, void *stream);

/* Full-precision last layer (Sec. 4.1; Sec. 3.2.2 lists 1x1 convolutions as trivial):
 *   logit[n,k,y,x] = b[k] + sum_c w[k][c] * a[n,y,x,c],  a = +-1 from the packed bits.
 *   act          packed [N][H][W][C/32], C in {32, 64, 128}
 *   w, b         float32 [K][C], [K], K <= 32
 *   logits_nchw  float32 [N][K][H][W]
 * Accurate to about 1e-6 relative (fp32 accumulation of exact products). */
int mbu_classifier_fp32(const uint32_t *act, int N, int H, int W, int C, const float *w,
                        const float *b, int K, float *logits_nchw, void *stream);

/* Folds batch norm, bias and the binary activation that follow a masked-binary layer into the
 * integer threshold of Algorithm 1 (Sec. 3.2.2: the threshold covers batch norm, bias and the
 * binary activation).  HOST function, all pointers are host arrays of C entries.
 *   bit = ( gamma[c] * (acc + bias[c] - mean[c]) / sqrt(var[c] + eps) + beta[c] >= 0 )
 * is rewritten as (acc' >= thresh[c]) with acc' = acc, or acc' = -acc where flip[c] = 1 (negative
 * gamma): the caller negates the weights of those output channels before mbu_pack_weights.
 *   bias     NULL = no bias;  fan_in = largest |acc| (9 * Cin for the 3x3 layer), <= 2^22
 *   thresh   int32 [C], clamped to +-(fan_in + 1) (a constant bit for gamma = 0);  flip int8 [C]
 * Errors: NULL arrays, non-positive C / fan_in, non-finite parameters, var + eps <= 0. */
int mbu_fold_batchnorm(const double *gamma, const double *beta, const double *mean,
                       const double *var, double eps, const double *bias, int C, int fan_in,
                       int32_t *thresh, int8_t *flip);

/* Cost-aware masking priority (Sec. 3.1.2): score[l] = w_op * ops^[l] + (1 - w_op) * params^[l],
 * both counts min-max normalised to [0, 1] over the L layers; `order` lists the layer indices by
 * ascending score (the order in which layers are switched from binary to masked weights; ties
 * keep the lower index first).  HOST function, host arrays.
 * Errors: NULL arrays, L <= 0, w_op outside [0, 1], negative or non-finite counts. */
int mbu_cost_rank(const double *n_ops, const double *n_params, int L, double w_op, double *score,
                  int *order);

/* One masked-binary layer of the network: host struct, device pointers inside. */
typedef struct mbu_conv_layer {
    const void *packed_w;    /* blob from mbu_pack_weights(cout, cin)  */
    const int32_t *thresh;   /* int32 [cout]                           */
    int cin;
    int cout;
    int sections;            /* MBU_BLOB_* bits the blob was packed with; 0 = all of them
                                (mbu_pack_weights).  Ignored for transposed layers.       */
} mbu_conv_layer;

/* Network descriptor (host struct).  The network is: float32 3x3 stem
 * in_channels -> base with zero threshold and binarisation (Sec. 4.1: first layer
 * full precision); `levels` encoder levels of two masked-binary 3x3 layers each,
 * followed by 2x2 pooling; a bottleneck of two layers; `levels` decoder levels of
 * [2x up-sampling, concatenation skip-then-up, two layers]; float32 1x1 classifier
 * base -> n_classes (last layer full precision).  `convs` lists the
 * 2*(2*levels+1) masked-binary layers in execution order and must be consistent
 * (each layer's cin equals what the walk produces), else MBU_ERR_SHAPE. */
typedef struct mbu_unet_desc {
    int levels;
    int base;                       /* channels after the stem; multiple of 32   */
    int in_channels;                /* image channels (3)                        */
    int n_classes;
    const float *stem_w;            /* device [base][3][3][in_channels]          */
    const mbu_conv_layer *convs;    /* host array, 2*(2*levels+1) entries        */
    const float *cls_w;             /* device [n_classes][base]                  */
    const float *cls_b;             /* device [n_classes]                        */
    void **step_events;             /* optional host array of mbu_unet_num_steps()+1
                                       hipEvent_t: event i is recorded on the stream
                                       before step i if that step launches a kernel
                                       (mbu_unet_step_launches), the last one after
                                       the final step.  NULL = no events.          */
    int fuse;                       /* 0: one kernel per step, every step's output is
                                       written to the workspace.  1: on the matrix path
                                       the "cat" steps are folded into the layer that
                                       reads them (their workspace region stays unwritten)
                                       and pooling is folded into the layer before it
                                       where that layer runs the block kernel; such
                                       steps then take no time of their own.        */
    const mbu_conv_layer *up_convs; /* NULL: the decoder up-samples 2x nearest neighbour.
                                       Otherwise a host array of `levels` transposed 2x2
                                       stride-2 layers, deepest first (packed_w from
                                       mbu_pack_tconv_weights, cin = channels below,
                                       cout = channels of the level): the decoder is
                                       [transposed layer, concatenation skip-then-up, two
                                       3x3 layers] per level, as in Sec. 2.1.          */
} mbu_unet_desc;

/* Number of steps the forward pass consists of (stem, each conv, pool, [transposed layer,]
 * concatenation, classifier) for this descriptor. */
int mbu_unet_num_steps(const mbu_unet_desc *d);

/* Describes step `step` (0-based): a short static name, where its packed output
 * lives inside the workspace (byte offset), and the output's shape.  The last step
 * (classifier) writes to the logits, its offset is reported as (size_t)-1.
 * All out-pointers are host pointers and may be NULL. */
int mbu_unet_step_info(const mbu_unet_desc *d, int N, int H, int W, int step,
                       const char **name, size_t *ws_offset, int *h, int *w, int *c);

/* 1 if step `step` launches a kernel of its own under the descriptor's `fuse` setting and the
 * current convolution path, 0 if it is folded into a neighbouring layer (then its event in
 * step_events is not recorded), negative status on error. */
int mbu_unet_step_launches(const mbu_unet_desc *d, int N, int H, int W, int step);

/* Name of the kernel that step `step` launches for this shape under the current settings
 * (the kernel's name in the library's sources, as a profiler shows it without template
 * arguments; "" for a step that launches none).  Nothing is launched and no device pointer of
 * the descriptor is read.  *kernel is a host string owned by the library, valid until the next
 * call of this function on the thread. */
int mbu_unet_step_kernel(const mbu_unet_desc *d, int N, int H, int W, int step, const char **kernel);

/* Workspace size (bytes) mbu_unet_forward needs for this shape. */
int mbu_unet_workspace_bytes(const mbu_unet_desc *d, int N, int H, int W, size_t *bytes);

/* Whole-network inference on one stream (Sec. 2.1 for the topology; Algorithm 1 for
 * every inner layer; Sec. 4.1 for the float32 ends).  All intermediate activations
 * stay bit-packed in `workspace`; every step's output keeps its own region so it
 * can be inspected afterwards through mbu_unet_step_info.
 *   image_nchw   float32 [N][in_channels][H][W]
 *   logits_nchw  float32 [N][n_classes][H][W]
 * H, W >= 2^levels.  Sizes that are not multiples of 2^levels (Appendix A.3: 959 x 640 frames)
 * follow the usual U-Net reading, on which the paper is silent: pooling rounds the size down
 * (an odd last row / column is dropped), and in the decoder the up-sampled feature, smaller by
 * that row / column, is zero-padded at the bottom / right to the skip feature's size before the
 * concatenation; the padded elements are the value 0.  Packed bits cannot hold a 0, so such a
 * concatenation is never written to the workspace (whatever `fuse` says): the layer after it
 * reads both tensors in place.  On the vector-ALU path such sizes give MBU_ERR_SHAPE. */
int mbu_unet_forward(const mbu_unet_desc *d, const float *image_nchw, int N, int H, int W,
                     float *logits_nchw, void *workspace, size_t workspace_bytes,
                     void *stream);

/* For callers that can neither allocate device memory nor bring a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): mbu_unet_forward with
 * the workspace inside the library - a fixed device array of MBU_STATIC_WORKSPACE_BYTES that
 * every GPU the library runs on holds until the process ends.  Allocates nothing, frees
 * nothing, synchronises nothing; the caller still owns image and logits.  The device that owns
 * `stream`, the image and the logits must be the current device.
 *   MBU_ERR_WORKSPACE  the shape needs more than MBU_STATIC_WORKSPACE_BYTES
 *                      (mbu_unet_workspace_bytes tells; 1 x 3 x 512 x 512 with base 64 and four
 *                      levels fits, the 1024 x 2048 frame does not)
 *   other errors       as for mbu_unet_forward
 * All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU
 * (different streams or threads) race and give wrong results; calls on one stream are safe.
 * Intermediate activations cannot be inspected (mbu_unet_step_info offsets refer to a caller
 * workspace); step events in the descriptor work as usual. */
#define MBU_STATIC_WORKSPACE_BYTES (32u << 20)
int mbu_unet_forward_static(const mbu_unet_desc *d, const float *image_nchw, int N, int H, int W,
                            float *logits_nchw, void *stream);

/* Thin helpers over HIP events so that a caller without HIP headers (the Python
 * binding) can time work on the stream the kernels were launched on.  Events are
 * host handles.  mbu_event_elapsed_ms synchronises on `stop`. */
int mbu_event_create(void **event);
int mbu_event_destroy(void *event);
int mbu_event_record(void *event, void *stream);
int mbu_event_elapsed_ms(void *start, void *stop, float *ms);

#ifdef __cplusplus
}
#endif
#endif /* MBU_H_ */
