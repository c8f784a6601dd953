// C-ABI entry points: argument validation, dispatch, and the network walk.
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>
#include "mbu_internal.h"

// Workspace of mbu_unet_forward_static: device memory that belongs to the loaded library, one
// copy per GPU, held until the process ends.  In host code this name only stands for the
// symbol; the device address is looked up once per device (static_workspace()).
static __device__ __align__(256) unsigned char scratch[MBU_STATIC_WORKSPACE_BYTES];

namespace mbu {

static thread_local char g_err[512] = "";
// process-wide settings; read only through begin_call()
static std::atomic<int> g_conv_path{MBU_PATH_AUTO};
static std::atomic<int> g_stem_path{MBU_STEM_AUTO};
static std::atomic<int> g_tune_rw{0};

thread_local CallCfg t_cfg = {MBU_PATH_AUTO, MBU_STEM_AUTO, 0, false, ""};

void begin_call(bool dry_run)
{
    t_cfg.conv_path = g_conv_path.load(std::memory_order_relaxed);
    t_cfg.stem_path = g_stem_path.load(std::memory_order_relaxed);
    t_cfg.tune_rw = g_tune_rw.load(std::memory_order_relaxed);
    t_cfg.dry_run = dry_run;
    t_cfg.kernel = "";
}

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int check_launch(const char *what)
{
    if (t_cfg.dry_run) return MBU_OK;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(MBU_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return MBU_OK;
}

BlobLayout blob_layout(int cout, int cin, int sections)
{
    BlobLayout L;
    L.cout = cout;
    L.cin = cin;
    L.sections = sections;
    L.cin_words = ceil_div(cin, 32);
    L.cout_pad64 = ceil_div(cout, 64) * 64;
    L.ksteps = ceil_div(cin, 64);
    L.cout_tiles32 = L.cout_pad64 / 32;
    size_t plane = (sections & MBU_BLOB_BIT_PLANES) ? (size_t)9 * L.cin_words * L.cout_pad64 * sizeof(uint32_t) : 0;
    size_t off = 256;  // reserved header room
    L.off_pos = off; off = round_up(off + plane, 256);
    L.off_neg = off; off = round_up(off + plane, 256);
    L.off_cnt = off; off = round_up(off + (size_t)11 * L.cout_pad64 * sizeof(int32_t), 256);
    L.off_f4 = off;  off = round_up(off + (size_t)L.cout_tiles32 * 9 * L.ksteps * 64 * 16, 256);
    L.off_up = off;
    if (sections & MBU_BLOB_SUMMED_TAPS) off = round_up(off + (size_t)(L.cout_pad64 / 64) * L.ksteps * 32 * 64 * 16, 256);
    L.total = off;
    return L;
}

static int check_dims4(const char *fn, int N, int H, int W, int C)
{
    if (N <= 0 || H <= 0 || W <= 0 || C <= 0)
        return fail(MBU_ERR_SHAPE, "%s: dimensions must be positive (N=%d H=%d W=%d C=%d)", fn, N, H, W, C);
    if ((double)N * H * W * ((C + 31) / 32) > 4.0e9)
        return fail(MBU_ERR_SHAPE, "%s: tensor too large", fn);
    return MBU_OK;
}

#define MBU_REQ_PTR(fn, p)                                                        \
    do {                                                                          \
        if ((p) == nullptr) return mbu::fail(MBU_ERR_NULL, "%s: %s is NULL", fn, #p); \
        if (!mbu::aligned16(p)) return mbu::fail(MBU_ERR_ALIGN, "%s: %s is not 16-byte aligned", fn, #p); \
    } while (0)

// layout of a network layer's blob: `sections` 0 means a blob from mbu_pack_weights (everything)
static BlobLayout layer_layout(const mbu_conv_layer &L)
{
    return blob_layout(L.cout, L.cin, L.sections ? L.sections : MBU_BLOB_ALL);
}

// ------------------------------------------------------------------ network plan
struct Step {
    enum Kind { STEM, CONV, POOL, UPCAT, TCONV, CAT, CLS } kind;
    const char *name;
    int conv;        // index into d->convs for CONV
    int in, in2;     // producing steps of the inputs (-1 = image); in2 = second input of UPCAT / CAT
                     // (conv = index into d->up_convs for TCONV)
    int h, w, c;     // output shape
    size_t off;      // workspace offset of the output
};

static const char *kConvNames[] = {"enc1a", "enc1b", "enc2a", "enc2b", "enc3a", "enc3b", "enc4a",
                                   "enc4b", "enc5a", "enc5b", "enc6a", "enc6b"};
static const char *kDecNames[] = {"dec1a", "dec1b", "dec2a", "dec2b", "dec3a", "dec3b", "dec4a",
                                  "dec4b", "dec5a", "dec5b", "dec6a", "dec6b"};
static const char *kPoolNames[] = {"pool1", "pool2", "pool3", "pool4", "pool5", "pool6"};
static const char *kUpNames[] = {"up1", "up2", "up3", "up4", "up5", "up6"};
static const char *kCatNames[] = {"cat1", "cat2", "cat3", "cat4", "cat5", "cat6"};

static int build_plan(const mbu_unet_desc *d, int N, int H, int W, std::vector<Step> &steps,
                      size_t *ws_bytes)
{
    const char *fn = "mbu_unet";
    if (!d) return fail(MBU_ERR_NULL, "%s: descriptor is NULL", fn);
    if (d->levels < 1 || d->levels > 6) return fail(MBU_ERR_SHAPE, "%s: levels must be 1..6", fn);
    if (d->base <= 0 || d->base % 32) return fail(MBU_ERR_SHAPE, "%s: base must be a positive multiple of 32", fn);
    if (d->in_channels != 1 && d->in_channels != 3) return fail(MBU_ERR_SHAPE, "%s: in_channels must be 1 or 3", fn);
    if (d->n_classes <= 0 || d->n_classes > 32) return fail(MBU_ERR_SHAPE, "%s: n_classes must be 1..32", fn);
    if (d->base != 32 && d->base != 64 && d->base != 128)
        return fail(MBU_ERR_SHAPE, "%s: base must be 32, 64 or 128 (classifier width)", fn);
    if (!d->convs) return fail(MBU_ERR_NULL, "%s: convs is NULL", fn);
    int rc = check_dims4(fn, N, H, W, d->base);
    if (rc) return rc;
    int m = 1 << d->levels;
    if (H < m || W < m) return fail(MBU_ERR_SHAPE, "%s: H and W must be at least %d", fn, m);

    size_t off = 0;
    auto push = [&](Step::Kind k, const char *name, int conv, int in, int in2, int h, int w, int c) {
        Step s{k, name, conv, in, in2, h, w, c, off};
        if (k != Step::CLS) off += round_up((size_t)N * h * w * (c / 32) * 4, 256);
        else s.off = (size_t)-1;
        steps.push_back(s);
        return (int)steps.size() - 1;
    };
    int ci = 0;
    auto conv = [&](const char *name, int in, int h, int w, int cin) -> int {
        const mbu_conv_layer &L = d->convs[ci];
        if (L.cin != cin) return -1 - ci;
        if (L.cout <= 0 || L.cout % 32) return -1 - ci;
        if (L.sections & ~MBU_BLOB_ALL) return -1 - ci;
        return push(Step::CONV, name, ci++, in, -1, h, w, L.cout);
    };
    int h = H, w = W;
    int cur = push(Step::STEM, "stem", -1, -1, -1, h, w, d->base);
    std::vector<int> skips;
    for (int l = 0; l < d->levels; ++l) {
        for (int j = 0; j < 2; ++j) {
            cur = conv(kConvNames[2 * l + j], cur, h, w, steps[cur].c);
            if (cur < 0) return fail(MBU_ERR_SHAPE, "%s: conv layer %d has inconsistent channels", fn, -1 - cur);
        }
        skips.push_back(cur);
        h /= 2; w /= 2;      // floor: an odd last row / column is dropped
        cur = push(Step::POOL, kPoolNames[l], -1, cur, -1, h, w, steps[cur].c);
    }
    for (int j = 0; j < 2; ++j) {
        cur = conv(j ? "midb" : "mida", cur, h, w, steps[cur].c);
        if (cur < 0) return fail(MBU_ERR_SHAPE, "%s: conv layer %d has inconsistent channels", fn, -1 - cur);
    }
    for (int l = d->levels - 1; l >= 0; --l) {
        int sk = skips[l];
        // the up-sampled feature has twice the size of the level below, which is the skip
        // feature's size less the row / column that pooling dropped; the concatenation has
        // the skip feature's size (the missing elements count as zeros)
        const int hu = 2 * h, wu = 2 * w;
        h = steps[sk].h; w = steps[sk].w;
        if (d->up_convs) {
            // transposed decoder: masked transposed layer 2x2 stride 2, then plain concatenation
            const mbu_conv_layer &U = d->up_convs[d->levels - 1 - l];
            if (U.cin != steps[cur].c || U.cout <= 0 || U.cout % 32)
                return fail(MBU_ERR_SHAPE, "%s: transposed layer %d has inconsistent channels", fn, d->levels - 1 - l);
            cur = push(Step::TCONV, kUpNames[l], d->levels - 1 - l, cur, -1, hu, wu, U.cout);
            cur = push(Step::CAT, kCatNames[l], -1, sk, cur, h, w, steps[sk].c + steps[cur].c);
        } else {
            cur = push(Step::UPCAT, kCatNames[l], -1, sk, cur, h, w, steps[sk].c + steps[cur].c);
        }
        for (int j = 0; j < 2; ++j) {
            cur = conv(kDecNames[2 * l + j], cur, h, w, steps[cur].c);
            if (cur < 0) return fail(MBU_ERR_SHAPE, "%s: conv layer %d has inconsistent channels", fn, -1 - cur);
        }
    }
    if (steps[cur].c != d->base)
        return fail(MBU_ERR_SHAPE, "%s: last layer must produce %d channels, got %d", fn, d->base, steps[cur].c);
    push(Step::CLS, "classifier", -1, cur, -1, h, w, d->n_classes);
    if (ws_bytes) *ws_bytes = off;
    return MBU_OK;
}

// Is the second input of this concatenation step smaller than the first (frame size not a
// multiple of 2^levels)?  Its missing elements are zeros, which packed bits cannot hold, so
// such a concatenation is never materialised: the layer after it reads both tensors in place.
static bool cat_needs_padding(const std::vector<Step> &steps, const Step &cat)
{
    const Step &a = steps[cat.in], &b = steps[cat.in2];
    const int sh = cat.kind == Step::UPCAT ? 1 : 0;
    return (b.h << sh) != a.h || (b.w << sh) != a.w;
}

// Does step i launch a kernel of its own under the descriptor's fusion setting?
static bool step_launches(const mbu_unet_desc *d, const std::vector<Step> &steps, size_t i)
{
    const bool matrix = t_cfg.conv_path != MBU_PATH_VALU;
    const bool fuse = d->fuse != 0 && matrix;
    const Step &st = steps[i];
    if (st.kind == Step::UPCAT || st.kind == Step::CAT)
        return !fuse && !(matrix && cat_needs_padding(steps, st));
    if (!fuse) return true;
    if (st.kind == Step::POOL) {
        const Step &in = steps[st.in];
        return !(in.kind == Step::CONV &&
                 conv_writes_pooled(in.h, in.w, layer_layout(d->convs[in.conv])));
    }
    return true;
}

// "(conv_mfma_block_kernel<RW, WM, WN, ...>)" as written at the launch site -> "conv_mfma_block_kernel"
static const char *kernel_base_name(const char *written)
{
    static thread_local char name[96];
    size_t n = 0;
    for (const char *p = written; *p && n + 1 < sizeof(name); ++p) {
        if (*p == '(' || *p == ' ') continue;
        if (*p == '<' || *p == ')') break;
        name[n++] = *p;
    }
    name[n] = 0;
    return name;
}

static int run_conv(const uint32_t *act, int N, int H, int W, const BlobLayout &L, const void *packed_w,
                    const int32_t *thresh, uint32_t *out_bits, int32_t *out_acc, hipStream_t s)
{
    int path = t_cfg.conv_path;
    if (path == MBU_PATH_AUTO) path = MBU_PATH_MFMA;
    if (path == MBU_PATH_VALU) {
        if (!(L.sections & MBU_BLOB_BIT_PLANES))
            return fail(MBU_ERR_ARG, "the vector-ALU path needs a blob packed with MBU_BLOB_BIT_PLANES");
        return launch_conv_valu(act, N, H, W, L, packed_w, thresh, out_bits, out_acc, s);
    }
    return launch_conv_mfma(act, N, H, W, L, packed_w, thresh, out_bits, out_acc, s);
}

static int run_stem(const float *img, int N, int Ci, int H, int W, const float *w, int Co,
                    uint32_t *out_bits, float *out_pre, hipStream_t s)
{
    const bool valu = t_cfg.stem_path == MBU_STEM_VALU || (t_cfg.stem_path == MBU_STEM_AUTO && out_pre);
    if (valu) return launch_stem_valu(img, N, Ci, H, W, w, Co, out_bits, out_pre, s);
    return launch_stem_mfma(img, N, Ci, H, W, w, Co, out_bits, out_pre, s);
}

}  // namespace mbu

using namespace mbu;

extern "C" {

const char *mbu_last_error(void) { return g_err; }

int mbu_set_conv_path(int path)
{
    if (path != MBU_PATH_AUTO && path != MBU_PATH_VALU && path != MBU_PATH_MFMA)
        return fail(MBU_ERR_ARG, "mbu_set_conv_path: unknown path %d", path);
    g_conv_path.store(path, std::memory_order_relaxed);
    return MBU_OK;
}

int mbu_get_conv_path(void) { return g_conv_path.load(std::memory_order_relaxed); }

int mbu_set_stem_path(int path)
{
    if (path != MBU_STEM_AUTO && path != MBU_STEM_VALU && path != MBU_STEM_MFMA && path != MBU_STEM_MFMA_GATHER)
        return fail(MBU_ERR_ARG, "mbu_set_stem_path: unknown path %d", path);
    g_stem_path.store(path, std::memory_order_relaxed);
    return MBU_OK;
}

int mbu_get_stem_path(void) { return g_stem_path.load(std::memory_order_relaxed); }

int mbu_stem_fp32(const float *image_nchw, int N, int Ci, int H, int W, const float *w, int Co,
                  uint32_t *out_bits, float *out_pre, void *stream)
{
    const char *fn = "mbu_stem_fp32";
    begin_call();
    MBU_REQ_PTR(fn, image_nchw);
    MBU_REQ_PTR(fn, w);
    MBU_REQ_PTR(fn, out_bits);
    if (out_pre && !aligned16(out_pre)) return fail(MBU_ERR_ALIGN, "%s: out_pre is not 16-byte aligned", fn);
    if (Ci != 1 && Ci != 3) return fail(MBU_ERR_SHAPE, "%s: Ci must be 1 or 3, got %d", fn, Ci);
    if (Co <= 0 || Co % 32 || Co > 65536) return fail(MBU_ERR_SHAPE, "%s: Co must be a positive multiple of 32, got %d", fn, Co);
    int rc = check_dims4(fn, N, H, W, Co);
    if (rc) return rc;
    if ((double)N * Ci * H * W * 4.0 >= 2147483648.0) return fail(MBU_ERR_SHAPE, "%s: image larger than 2 GiB", fn);
    if (out_pre && (double)N * H * W * Co * 4.0 > 16.0e9) return fail(MBU_ERR_SHAPE, "%s: out_pre too large", fn);
    return run_stem(image_nchw, N, Ci, H, W, w, Co, out_bits, out_pre, (hipStream_t)stream);
}

int mbu_classifier_fp32(const uint32_t *act, int N, int H, int W, int C, const float *w,
                        const float *b, int K, float *logits_nchw, void *stream)
{
    const char *fn = "mbu_classifier_fp32";
    begin_call();
    MBU_REQ_PTR(fn, act);
    MBU_REQ_PTR(fn, w);
    MBU_REQ_PTR(fn, b);
    MBU_REQ_PTR(fn, logits_nchw);
    int rc = check_dims4(fn, N, H, W, C);
    if (rc) return rc;
    if (C != 32 && C != 64 && C != 128) return fail(MBU_ERR_SHAPE, "%s: C must be 32, 64 or 128, got %d", fn, C);
    if (K <= 0 || K > 32) return fail(MBU_ERR_SHAPE, "%s: K must be 1..32, got %d", fn, K);
    return launch_classifier(act, N, H, W, C, w, b, K, logits_nchw, (hipStream_t)stream);
}

int mbu_set_conv_tuning(int rows_per_wave, int reserved)
{
    if ((rows_per_wave != 0 && rows_per_wave != 1 && rows_per_wave != 3 && rows_per_wave != 6 &&
         rows_per_wave != 7 && rows_per_wave != 8 && rows_per_wave != 9) || reserved != 0)
        return fail(MBU_ERR_ARG, "mbu_set_conv_tuning: kernel in {0,1,3,6,7,8,9}, second argument 0");
    g_tune_rw.store(rows_per_wave, std::memory_order_relaxed);
    return MBU_OK;
}

int mbu_pack_act(const void *src, int src_dtype, int N, int H, int W, int C, uint32_t *dst,
                 void *stream)
{
    const char *fn = "mbu_pack_act";
    begin_call();
    MBU_REQ_PTR(fn, src);
    MBU_REQ_PTR(fn, dst);
    if (src_dtype != 0 && src_dtype != 1) return fail(MBU_ERR_ARG, "%s: src_dtype must be 0 (int8) or 1 (float32)", fn);
    int rc = check_dims4(fn, N, H, W, C);
    if (rc) return rc;
    return launch_pack_act(src, src_dtype, (long)N * H * W, C, dst, (hipStream_t)stream);
}

int mbu_packed_weights_bytes(int Cout, int Cin, size_t *bytes)
{
    const char *fn = "mbu_packed_weights_bytes";
    if (!bytes) return fail(MBU_ERR_NULL, "%s: bytes is NULL", fn);
    if (Cout <= 0 || Cin <= 0 || Cout % 32) return fail(MBU_ERR_SHAPE, "%s: need Cin > 0 and Cout a positive multiple of 32 (Cout=%d Cin=%d)", fn, Cout, Cin);
    if (Cout > 65536 || Cin > 65536) return fail(MBU_ERR_SHAPE, "%s: channel count too large", fn);
    *bytes = blob_layout(Cout, Cin).total;
    return MBU_OK;
}

int mbu_pack_weights(const int8_t *w_ohwi, int Cout, int Cin, void *packed, void *stream)
{
    return mbu_pack_weights_sections(w_ohwi, Cout, Cin, MBU_BLOB_ALL, packed, stream);
}

int mbu_packed_weights_bytes_sections(int Cout, int Cin, int sections, size_t *bytes)
{
    const char *fn = "mbu_packed_weights_bytes_sections";
    if (sections & ~MBU_BLOB_ALL) return fail(MBU_ERR_ARG, "%s: unknown section bits 0x%x", fn, sections);
    int rc = mbu_packed_weights_bytes(Cout, Cin, bytes);
    if (rc) return rc;
    *bytes = blob_layout(Cout, Cin, sections | MBU_BLOB_MATRIX).total;
    return MBU_OK;
}

int mbu_pack_weights_sections(const int8_t *w_ohwi, int Cout, int Cin, int sections, void *packed,
                              void *stream)
{
    const char *fn = "mbu_pack_weights";
    begin_call();
    MBU_REQ_PTR(fn, w_ohwi);
    MBU_REQ_PTR(fn, packed);
    size_t bytes;
    int rc = mbu_packed_weights_bytes_sections(Cout, Cin, sections, &bytes);
    if (rc) return rc;
    return launch_pack_weights(w_ohwi, blob_layout(Cout, Cin, sections | MBU_BLOB_MATRIX), packed,
                               (hipStream_t)stream);
}

int mbu_conv3x3_masked_binary(const uint32_t *act, int N, int H, int W, int Cin,
                              const void *packed_w, int Cout, const int32_t *thresh,
                              uint32_t *out_bits, int32_t *out_acc, void *stream)
{
    const char *fn = "mbu_conv3x3_masked_binary";
    begin_call();
    MBU_REQ_PTR(fn, act);
    MBU_REQ_PTR(fn, packed_w);
    MBU_REQ_PTR(fn, thresh);
    if (!out_bits && !out_acc) return fail(MBU_ERR_NULL, "%s: out_bits and out_acc are both NULL", fn);
    if (out_bits && !aligned16(out_bits)) return fail(MBU_ERR_ALIGN, "%s: out_bits is not 16-byte aligned", fn);
    if (out_acc && !aligned16(out_acc)) return fail(MBU_ERR_ALIGN, "%s: out_acc is not 16-byte aligned", fn);
    if ((const void *)out_bits == (const void *)act || (const void *)out_acc == (const void *)act)
        return fail(MBU_ERR_ARG, "%s: outputs must not alias the input", fn);
    int rc = check_dims4(fn, N, H, W, Cin);
    if (rc) return rc;
    if (Cout <= 0 || Cout % 32) return fail(MBU_ERR_SHAPE, "%s: Cout must be a positive multiple of 32, got %d", fn, Cout);
    if (Cout > 65536 || Cin > 65536) return fail(MBU_ERR_SHAPE, "%s: channel count too large", fn);
    rc = check_dims4(fn, N, H, W, Cout);
    if (rc) return rc;
    return run_conv(act, N, H, W, blob_layout(Cout, Cin), packed_w, thresh, out_bits, out_acc, (hipStream_t)stream);
}

int mbu_conv3x3_masked_binary_fused(const uint32_t *act, int Ca, const uint32_t *low, int Clow,
                                    int N, int H, int W, const void *packed_w, int Cout,
                                    const int32_t *thresh, uint32_t *out_bits, uint32_t *out_pool,
                                    void *stream)
{
    const char *fn = "mbu_conv3x3_masked_binary_fused";
    begin_call();
    MBU_REQ_PTR(fn, act);
    MBU_REQ_PTR(fn, packed_w);
    MBU_REQ_PTR(fn, thresh);
    if (!out_bits && !out_pool) return fail(MBU_ERR_NULL, "%s: out_bits and out_pool are both NULL", fn);
    if (out_bits && !aligned16(out_bits)) return fail(MBU_ERR_ALIGN, "%s: out_bits is not 16-byte aligned", fn);
    if (out_pool && !aligned16(out_pool)) return fail(MBU_ERR_ALIGN, "%s: out_pool is not 16-byte aligned", fn);
    if (low && !aligned16(low)) return fail(MBU_ERR_ALIGN, "%s: low is not 16-byte aligned", fn);
    if ((const void *)out_bits == (const void *)act || (const void *)out_pool == (const void *)act ||
        (low && ((const void *)out_bits == (const void *)low || (const void *)out_pool == (const void *)low)))
        return fail(MBU_ERR_ARG, "%s: outputs must not alias an input", fn);
    int rc = check_dims4(fn, N, H, W, Ca);
    if (rc) return rc;
    if ((low != nullptr) != (Clow > 0) || Clow < 0)
        return fail(MBU_ERR_SHAPE, "%s: Clow must be positive exactly when low is given (Clow=%d)", fn, Clow);
    if (low && Ca % 32) return fail(MBU_ERR_SHAPE, "%s: Ca must be a multiple of 32 when low is given, got %d", fn, Ca);
    if (out_pool && (H < 2 || W < 2))
        return fail(MBU_ERR_SHAPE, "%s: H and W must be at least 2 with out_pool (H=%d W=%d)", fn, H, W);
    if (low && (H < 2 || W < 2))
        return fail(MBU_ERR_SHAPE, "%s: H and W must be at least 2 with low (H=%d W=%d)", fn, H, W);
    if (Cout <= 0 || Cout % 32) return fail(MBU_ERR_SHAPE, "%s: Cout must be a positive multiple of 32, got %d", fn, Cout);
    if (Cout > 65536 || Ca + Clow > 65536) return fail(MBU_ERR_SHAPE, "%s: channel count too large", fn);
    rc = check_dims4(fn, N, H, W, Cout);
    if (rc) return rc;
    rc = check_dims4(fn, N, H, W, Ca + Clow);
    if (rc) return rc;
    // the matrix-path blob stores whole 32-channel words of each source one after the other
    const int cin_blob = Ca + Clow;
    return launch_conv_mfma_two(act, Ca, low, Clow, 1, H / 2, W / 2, N, H, W, blob_layout(Cout, cin_blob),
                                packed_w, thresh, out_bits, out_pool, (hipStream_t)stream);
}

int mbu_conv3x3_masked_binary_concat(const uint32_t *a, int Ca, const uint32_t *b, int Cb, int N,
                                     int H, int W, const void *packed_w, int Cout,
                                     const int32_t *thresh, uint32_t *out_bits, uint32_t *out_pool,
                                     void *stream)
{
    const char *fn = "mbu_conv3x3_masked_binary_concat";
    begin_call();
    MBU_REQ_PTR(fn, a);
    MBU_REQ_PTR(fn, b);
    MBU_REQ_PTR(fn, packed_w);
    MBU_REQ_PTR(fn, thresh);
    if (!out_bits && !out_pool) return fail(MBU_ERR_NULL, "%s: out_bits and out_pool are both NULL", fn);
    if (out_bits && !aligned16(out_bits)) return fail(MBU_ERR_ALIGN, "%s: out_bits is not 16-byte aligned", fn);
    if (out_pool && !aligned16(out_pool)) return fail(MBU_ERR_ALIGN, "%s: out_pool is not 16-byte aligned", fn);
    if ((const void *)out_bits == (const void *)a || (const void *)out_bits == (const void *)b ||
        (const void *)out_pool == (const void *)a || (const void *)out_pool == (const void *)b)
        return fail(MBU_ERR_ARG, "%s: outputs must not alias an input", fn);
    int rc = check_dims4(fn, N, H, W, Ca);
    if (rc) return rc;
    if (Cb <= 0) return fail(MBU_ERR_SHAPE, "%s: Cb must be positive, got %d", fn, Cb);
    if (Ca % 32) return fail(MBU_ERR_SHAPE, "%s: Ca must be a multiple of 32, got %d", fn, Ca);
    if (out_pool && (H < 2 || W < 2))
        return fail(MBU_ERR_SHAPE, "%s: H and W must be at least 2 with out_pool (H=%d W=%d)", fn, H, W);
    if (Cout <= 0 || Cout % 32) return fail(MBU_ERR_SHAPE, "%s: Cout must be a positive multiple of 32, got %d", fn, Cout);
    if (Cout > 65536 || Ca + Cb > 65536) return fail(MBU_ERR_SHAPE, "%s: channel count too large", fn);
    rc = check_dims4(fn, N, H, W, Cout);
    if (rc) return rc;
    rc = check_dims4(fn, N, H, W, Ca + Cb);
    if (rc) return rc;
    return launch_conv_mfma_two(a, Ca, b, Cb, 0, H, W, N, H, W, blob_layout(Cout, Ca + Cb), packed_w, thresh,
                                out_bits, out_pool, (hipStream_t)stream);
}

int mbu_conv3x3_masked_binary_two_inputs(const uint32_t *a, int Ca, const uint32_t *b, int Cb, int Hb,
                                         int Wb, int upsample, int N, int H, int W, const void *packed_w,
                                         int Cout, const int32_t *thresh, uint32_t *out_bits,
                                         uint32_t *out_pool, void *stream)
{
    const char *fn = "mbu_conv3x3_masked_binary_two_inputs";
    begin_call();
    MBU_REQ_PTR(fn, a);
    MBU_REQ_PTR(fn, b);
    MBU_REQ_PTR(fn, packed_w);
    MBU_REQ_PTR(fn, thresh);
    if (!out_bits && !out_pool) return fail(MBU_ERR_NULL, "%s: out_bits and out_pool are both NULL", fn);
    if (out_bits && !aligned16(out_bits)) return fail(MBU_ERR_ALIGN, "%s: out_bits is not 16-byte aligned", fn);
    if (out_pool && !aligned16(out_pool)) return fail(MBU_ERR_ALIGN, "%s: out_pool is not 16-byte aligned", fn);
    if ((const void *)out_bits == (const void *)a || (const void *)out_bits == (const void *)b ||
        (const void *)out_pool == (const void *)a || (const void *)out_pool == (const void *)b)
        return fail(MBU_ERR_ARG, "%s: outputs must not alias an input", fn);
    if (upsample != 0 && upsample != 1) return fail(MBU_ERR_ARG, "%s: upsample must be 0 or 1", fn);
    int rc = check_dims4(fn, N, H, W, Ca);
    if (rc) return rc;
    if (Cb <= 0) return fail(MBU_ERR_SHAPE, "%s: Cb must be positive, got %d", fn, Cb);
    if (Ca % 32) return fail(MBU_ERR_SHAPE, "%s: Ca must be a multiple of 32, got %d", fn, Ca);
    if (Hb <= 0 || Wb <= 0 || (Hb << upsample) > H || (Wb << upsample) > W)
        return fail(MBU_ERR_SHAPE, "%s: the second input (%d x %d pixels%s) must be non-empty and fit into "
                    "%d x %d", fn, Hb, Wb, upsample ? ", read 2x up-sampled" : "", H, W);
    if (out_pool && (H < 2 || W < 2))
        return fail(MBU_ERR_SHAPE, "%s: H and W must be at least 2 with out_pool (H=%d W=%d)", fn, H, W);
    if (Cout <= 0 || Cout % 32) return fail(MBU_ERR_SHAPE, "%s: Cout must be a positive multiple of 32, got %d", fn, Cout);
    if (Cout > 65536 || Ca + Cb > 65536) return fail(MBU_ERR_SHAPE, "%s: channel count too large", fn);
    rc = check_dims4(fn, N, H, W, Cout);
    if (rc) return rc;
    rc = check_dims4(fn, N, H, W, Ca + Cb);
    if (rc) return rc;
    return launch_conv_mfma_two(a, Ca, b, Cb, upsample, Hb, Wb, N, H, W, blob_layout(Cout, Ca + Cb), packed_w,
                                thresh, out_bits, out_pool, (hipStream_t)stream);
}

int mbu_packed_tconv_weights_bytes(int Cout, int Cin, size_t *bytes)
{
    const char *fn = "mbu_packed_tconv_weights_bytes";
    if (!bytes) return fail(MBU_ERR_NULL, "%s: bytes is NULL", fn);
    if (Cout <= 0 || Cin <= 0 || Cout % 32) return fail(MBU_ERR_SHAPE, "%s: need Cin > 0 and Cout a positive multiple of 32 (Cout=%d Cin=%d)", fn, Cout, Cin);
    if (Cout > 65536 || Cin > 65536) return fail(MBU_ERR_SHAPE, "%s: channel count too large", fn);
    *bytes = tconv_layout(Cout, Cin).total;
    return MBU_OK;
}

int mbu_pack_tconv_weights(const int8_t *w, int Cout, int Cin, void *packed, void *stream)
{
    const char *fn = "mbu_pack_tconv_weights";
    begin_call();
    MBU_REQ_PTR(fn, w);
    MBU_REQ_PTR(fn, packed);
    size_t bytes;
    int rc = mbu_packed_tconv_weights_bytes(Cout, Cin, &bytes);
    if (rc) return rc;
    return launch_pack_tconv(w, tconv_layout(Cout, Cin), packed, (hipStream_t)stream);
}

int mbu_tconv2x2_masked_binary(const uint32_t *act, int N, int H, int W, int Cin,
                               const void *packed_w, int Cout, const int32_t *thresh,
                               uint32_t *out_bits, int32_t *out_acc, void *stream)
{
    const char *fn = "mbu_tconv2x2_masked_binary";
    begin_call();
    MBU_REQ_PTR(fn, act);
    MBU_REQ_PTR(fn, packed_w);
    MBU_REQ_PTR(fn, thresh);
    if (!out_bits && !out_acc) return fail(MBU_ERR_NULL, "%s: out_bits and out_acc are both NULL", fn);
    if (out_bits && !aligned16(out_bits)) return fail(MBU_ERR_ALIGN, "%s: out_bits is not 16-byte aligned", fn);
    if (out_acc && !aligned16(out_acc)) return fail(MBU_ERR_ALIGN, "%s: out_acc is not 16-byte aligned", fn);
    if ((const void *)out_bits == (const void *)act || (const void *)out_acc == (const void *)act)
        return fail(MBU_ERR_ARG, "%s: outputs must not alias the input", fn);
    int rc = check_dims4(fn, N, H, W, Cin);
    if (rc) return rc;
    if (Cout <= 0 || Cout % 32) return fail(MBU_ERR_SHAPE, "%s: Cout must be a positive multiple of 32, got %d", fn, Cout);
    if (Cout > 65536 || Cin > 65536) return fail(MBU_ERR_SHAPE, "%s: channel count too large", fn);
    if ((double)N * H * W * 4.0 * (Cout / 32) > 4.0e9) return fail(MBU_ERR_SHAPE, "%s: output too large", fn);
    return launch_tconv_mfma(act, N, H, W, tconv_layout(Cout, Cin), packed_w, thresh, out_bits, out_acc,
                             (hipStream_t)stream);
}

int mbu_maxpool2x2_bits(const uint32_t *in, int N, int H, int W, int C, uint32_t *out, void *stream)
{
    const char *fn = "mbu_maxpool2x2_bits";
    begin_call();
    MBU_REQ_PTR(fn, in);
    MBU_REQ_PTR(fn, out);
    int rc = check_dims4(fn, N, H, W, C);
    if (rc) return rc;
    if (H < 2 || W < 2) return fail(MBU_ERR_SHAPE, "%s: H and W must be at least 2 (H=%d W=%d)", fn, H, W);
    return launch_maxpool(in, N, H, W, ceil_div(C, 32), out, (hipStream_t)stream);
}

int mbu_upsample2x_bits(const uint32_t *in, int N, int H, int W, int C, uint32_t *out, void *stream)
{
    const char *fn = "mbu_upsample2x_bits";
    begin_call();
    MBU_REQ_PTR(fn, in);
    MBU_REQ_PTR(fn, out);
    int rc = check_dims4(fn, N, H, W, C);
    if (rc) return rc;
    if ((double)N * H * W * 4.0 * ((C + 31) / 32) > 4.0e9) return fail(MBU_ERR_SHAPE, "%s: output too large", fn);
    return launch_upsample(in, N, H, W, ceil_div(C, 32), out, (hipStream_t)stream);
}

int mbu_concat_bits(const uint32_t *a, int Ca, const uint32_t *b, int Cb, int N, int H, int W,
                    uint32_t *out, void *stream)
{
    const char *fn = "mbu_concat_bits";
    begin_call();
    MBU_REQ_PTR(fn, a);
    MBU_REQ_PTR(fn, b);
    MBU_REQ_PTR(fn, out);
    int rc = check_dims4(fn, N, H, W, Ca);
    if (rc) return rc;
    rc = check_dims4(fn, N, H, W, Cb);
    if (rc) return rc;
    if (Ca % 32) return fail(MBU_ERR_SHAPE, "%s: Ca must be a multiple of 32, got %d", fn, Ca);
    return launch_concat(a, Ca / 32, b, ceil_div(Cb, 32), (long)N * H * W, out, (hipStream_t)stream);
}

int mbu_unet_num_steps(const mbu_unet_desc *d)
{
    if (!d) return fail(MBU_ERR_NULL, "mbu_unet_num_steps: descriptor is NULL");
    if (d->levels < 1 || d->levels > 6) return fail(MBU_ERR_SHAPE, "mbu_unet_num_steps: levels must be 1..6");
    return 1 + 3 * d->levels + 2 + (d->up_convs ? 4 : 3) * d->levels + 1;
}

int mbu_unet_step_info(const mbu_unet_desc *d, int N, int H, int W, int step, const char **name,
                       size_t *ws_offset, int *h, int *w, int *c)
{
    std::vector<Step> steps;
    int rc = build_plan(d, N, H, W, steps, nullptr);
    if (rc) return rc;
    if (step < 0 || step >= (int)steps.size()) return fail(MBU_ERR_ARG, "mbu_unet_step_info: step %d out of range", step);
    const Step &s = steps[step];
    if (name) *name = s.name;
    if (ws_offset) *ws_offset = s.off;
    if (h) *h = s.h;
    if (w) *w = s.w;
    if (c) *c = s.c;
    return MBU_OK;
}

int mbu_unet_step_launches(const mbu_unet_desc *d, int N, int H, int W, int step)
{
    begin_call();
    std::vector<Step> steps;
    int rc = build_plan(d, N, H, W, steps, nullptr);
    if (rc) return rc;
    if (step < 0 || step >= (int)steps.size()) return fail(MBU_ERR_ARG, "mbu_unet_step_launches: step %d out of range", step);
    return step_launches(d, steps, (size_t)step) ? 1 : 0;
}

int mbu_unet_workspace_bytes(const mbu_unet_desc *d, int N, int H, int W, size_t *bytes)
{
    if (!bytes) return fail(MBU_ERR_NULL, "mbu_unet_workspace_bytes: bytes is NULL");
    std::vector<Step> steps;
    return build_plan(d, N, H, W, steps, bytes);
}

}  // extern "C"

namespace mbu {

// The network walk shared by mbu_unet_forward and mbu_unet_step_kernel.  With t_cfg.dry_run
// set nothing is launched and no event is recorded; the launchers still make their choices and
// leave the chosen kernel's name in t_cfg.kernel, which is copied to kernel_of_step[i] for every
// step that launches one ("" for a step folded into a neighbouring layer).
static int walk(const mbu_unet_desc *d, const std::vector<Step> &steps, const float *image_nchw,
                int N, int H, int W, float *logits_nchw, uint8_t *ws, hipStream_t s,
                const char **kernel_of_step)
{
    const char *fn = "mbu_unet_forward";
    const bool dry = t_cfg.dry_run;
    auto buf = [&](int step) { return (uint32_t *)(ws + steps[step].off); };
    const bool matrix = t_cfg.conv_path != MBU_PATH_VALU;
    const bool fuse = d->fuse != 0 && matrix;
    int rc = MBU_OK;
    for (size_t i = 0; i < steps.size(); ++i) {
        const Step &st = steps[i];
        if (!dry && d->step_events && step_launches(d, steps, i) &&
            hipEventRecord((hipEvent_t)d->step_events[i], s) != hipSuccess)
            return fail(MBU_ERR_HIP, "%s: hipEventRecord failed", fn);
        t_cfg.kernel = "";
        switch (st.kind) {
        case Step::STEM:
            rc = run_stem(image_nchw, N, d->in_channels, H, W, d->stem_w, d->base, buf((int)i), nullptr, s);
            break;
        case Step::CONV: {
            const mbu_conv_layer &L = d->convs[st.conv];
            const Step &in = steps[st.in];
            // fused forms: read [skip | up(low)] in place; write the pooled output as well
            const bool cat_in = in.kind == Step::UPCAT || in.kind == Step::CAT;
            const bool from_cat = cat_in && (fuse || cat_needs_padding(steps, in));
            const bool next_pool = fuse && i + 1 < steps.size() && steps[i + 1].kind == Step::POOL &&
                                   conv_writes_pooled(st.h, st.w, layer_layout(L));
            if (from_cat || next_pool) {
                const uint32_t *a = from_cat ? buf(in.in) : buf(st.in);
                const int ca = from_cat ? steps[in.in].c : L.cin;
                const uint32_t *lo = from_cat ? buf(in.in2) : nullptr;
                const int clo = from_cat ? steps[in.in2].c : 0;
                const int hb = from_cat ? steps[in.in2].h : 0, wb = from_cat ? steps[in.in2].w : 0;
                rc = launch_conv_mfma_two(a, ca, lo, clo, in.kind == Step::UPCAT ? 1 : 0, hb, wb, N, st.h, st.w,
                                          layer_layout(L), L.packed_w, L.thresh,
                                          buf((int)i), next_pool ? buf((int)i + 1) : nullptr, s);
            } else {
                rc = run_conv(buf(st.in), N, st.h, st.w, layer_layout(L), L.packed_w, L.thresh,
                              buf((int)i), nullptr, s);
            }
            break;
        }
        case Step::POOL:
            if (step_launches(d, steps, i))
                rc = launch_maxpool(buf(st.in), N, steps[st.in].h, steps[st.in].w, st.c / 32, buf((int)i), s);
            break;
        case Step::UPCAT:
            if (step_launches(d, steps, i))
                rc = launch_upcat(buf(st.in), steps[st.in].c / 32, buf(st.in2), steps[st.in2].c / 32,
                                  N, st.h, st.w, buf((int)i), s);
            break;
        case Step::TCONV: {
            const mbu_conv_layer &U = d->up_convs[st.conv];
            rc = launch_tconv_mfma(buf(st.in), N, st.h / 2, st.w / 2, tconv_layout(U.cout, U.cin),
                                   U.packed_w, U.thresh, buf((int)i), nullptr, s);
            break;
        }
        case Step::CAT:
            if (step_launches(d, steps, i))
                rc = launch_concat(buf(st.in), steps[st.in].c / 32, buf(st.in2), steps[st.in2].c / 32,
                                   (long)N * st.h * st.w, buf((int)i), s);
            break;
        case Step::CLS:
            rc = launch_classifier(buf(st.in), N, st.h, st.w, steps[st.in].c, d->cls_w, d->cls_b,
                                   d->n_classes, logits_nchw, s);
            break;
        }
        if (rc) return rc;
        if (kernel_of_step) kernel_of_step[i] = t_cfg.kernel;
    }
    if (!dry && d->step_events && hipEventRecord((hipEvent_t)d->step_events[steps.size()], s) != hipSuccess)
        return fail(MBU_ERR_HIP, "%s: hipEventRecord failed", fn);
    return MBU_OK;
}

// validation shared by the forward entry points; fills the plan
static int check_forward(const char *fn, const mbu_unet_desc *d, const float *image_nchw, int N, int H,
                         int W, float *logits_nchw, std::vector<Step> &steps, size_t *need)
{
    int rc = build_plan(d, N, H, W, steps, need);
    if (rc) return rc;
    MBU_REQ_PTR(fn, image_nchw);
    MBU_REQ_PTR(fn, logits_nchw);
    MBU_REQ_PTR(fn, d->stem_w);
    MBU_REQ_PTR(fn, d->cls_w);
    MBU_REQ_PTR(fn, d->cls_b);
    int nconv = 2 * (2 * d->levels + 1);
    for (int i = 0; i < nconv; ++i) {
        MBU_REQ_PTR(fn, d->convs[i].packed_w);
        MBU_REQ_PTR(fn, d->convs[i].thresh);
    }
    for (int i = 0; d->up_convs && i < d->levels; ++i) {
        MBU_REQ_PTR(fn, d->up_convs[i].packed_w);
        MBU_REQ_PTR(fn, d->up_convs[i].thresh);
    }
    if (t_cfg.conv_path == MBU_PATH_VALU)
        for (const Step &st : steps)
            if ((st.kind == Step::UPCAT || st.kind == Step::CAT) && cat_needs_padding(steps, st))
                return fail(MBU_ERR_SHAPE, "%s: H and W must be multiples of %d on the vector-ALU path "
                            "(a padded decoder feature is only read in place by the matrix path)", fn, 1 << d->levels);
    return MBU_OK;
}

// Device address of `scratch` on the current device, looked up on the first call per device
// (with that device current) and kept; every GPU has its own copy at its own address.
static int static_workspace(const char *fn, void **ptr)
{
    static std::atomic<void *> addr[64];
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(MBU_ERR_HIP, "%s: hipGetDevice: %s", fn, hipGetErrorString(e));
    if (dev < 0 || dev >= 64) return fail(MBU_ERR_HIP, "%s: device index %d not supported", fn, dev);
    void *p = addr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(MBU_ERR_HIP, "%s: hipGetSymbolAddress: %s", fn, hipGetErrorString(e));
        addr[dev].store(p, std::memory_order_release);   // racing threads store the same address
    }
    *ptr = p;
    return MBU_OK;
}

}  // namespace mbu

extern "C" {

int mbu_unet_forward_static(const mbu_unet_desc *d, const float *image_nchw, int N, int H, int W,
                            float *logits_nchw, void *stream)
{
    const char *fn = "mbu_unet_forward_static";
    begin_call();
    std::vector<Step> steps;
    size_t need = 0;
    int rc = check_forward(fn, d, image_nchw, N, H, W, logits_nchw, steps, &need);
    if (rc) return rc;
    if (need > (size_t)MBU_STATIC_WORKSPACE_BYTES)
        return fail(MBU_ERR_WORKSPACE, "%s: this shape needs %zu bytes of workspace, the library's own "
                    "holds %zu; use mbu_unet_forward with a caller workspace", fn, need,
                    (size_t)MBU_STATIC_WORKSPACE_BYTES);
    void *ws = nullptr;
    rc = static_workspace(fn, &ws);
    if (rc) return rc;
    // every region of the workspace is written by the step that owns it before a later step
    // reads it, so nothing has to be cleared between calls
    return walk(d, steps, image_nchw, N, H, W, logits_nchw, (uint8_t *)ws, (hipStream_t)stream, nullptr);
}

int mbu_unet_step_kernel(const mbu_unet_desc *d, int N, int H, int W, int step, const char **kernel)
{
    const char *fn = "mbu_unet_step_kernel";
    begin_call(true);
    if (!kernel) return fail(MBU_ERR_NULL, "%s: kernel is NULL", fn);
    std::vector<Step> steps;
    int rc = build_plan(d, N, H, W, steps, nullptr);
    if (rc) return rc;
    if (step < 0 || step >= (int)steps.size()) return fail(MBU_ERR_ARG, "%s: step %d out of range", fn, step);
    std::vector<const char *> names(steps.size(), "");
    // a dry run dereferences no device pointer; the workspace is only an address base
    rc = walk(d, steps, nullptr, N, H, W, nullptr, (uint8_t *)256, nullptr, names.data());
    t_cfg.dry_run = false;
    if (rc) return rc;
    *kernel = kernel_base_name(names[step]);
    return MBU_OK;
}

int mbu_unet_forward(const mbu_unet_desc *d, const float *image_nchw, int N, int H, int W,
                     float *logits_nchw, void *workspace, size_t workspace_bytes, void *stream)
{
    const char *fn = "mbu_unet_forward";
    begin_call();
    std::vector<Step> steps;
    size_t need = 0;
    int rc = check_forward(fn, d, image_nchw, N, H, W, logits_nchw, steps, &need);
    if (rc) return rc;
    MBU_REQ_PTR(fn, workspace);
    if (workspace_bytes < need)
        return fail(MBU_ERR_WORKSPACE, "%s: workspace has %zu bytes, %zu needed", fn, workspace_bytes, need);
    return walk(d, steps, image_nchw, N, H, W, logits_nchw, (uint8_t *)workspace, (hipStream_t)stream, nullptr);
}

int mbu_event_create(void **event)
{
    if (!event) return fail(MBU_ERR_NULL, "mbu_event_create: event is NULL");
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return fail(MBU_ERR_HIP, "hipEventCreate failed");
    *event = (void *)e;
    return MBU_OK;
}

int mbu_event_destroy(void *event)
{
    if (!event) return fail(MBU_ERR_NULL, "mbu_event_destroy: event is NULL");
    return hipEventDestroy((hipEvent_t)event) == hipSuccess ? MBU_OK : fail(MBU_ERR_HIP, "hipEventDestroy failed");
}

int mbu_event_record(void *event, void *stream)
{
    if (!event) return fail(MBU_ERR_NULL, "mbu_event_record: event is NULL");
    return hipEventRecord((hipEvent_t)event, (hipStream_t)stream) == hipSuccess
               ? MBU_OK : fail(MBU_ERR_HIP, "hipEventRecord failed");
}

int mbu_event_elapsed_ms(void *start, void *stop, float *ms)
{
    if (!start || !stop || !ms) return fail(MBU_ERR_NULL, "mbu_event_elapsed_ms: NULL argument");
    hipError_t e = hipEventSynchronize((hipEvent_t)stop);
    if (e != hipSuccess) return fail(MBU_ERR_HIP, "hipEventSynchronize: %s", hipGetErrorString(e));
    e = hipEventElapsedTime(ms, (hipEvent_t)start, (hipEvent_t)stop);
    if (e != hipSuccess) return fail(MBU_ERR_HIP, "hipEventElapsedTime: %s", hipGetErrorString(e));
    return MBU_OK;
}

}  // extern "C"
