// Bandwidth-bound glue on packed activations: 2x2 OR-pooling (max of +-1 values,
// Sec. 3.2.2), 2x nearest-neighbour up-sampling, channel concatenation of the skip
// path (Sec. 2.1), and the fused up-sample + concatenate step of the decoder.
// Every kernel moves V = uint32 / uint2 / uint4 units (widest that divides the
// per-pixel word count) with one unit per thread and consecutive threads on
// consecutive units of the OUTPUT, so stores are fully coalesced.
#include "mbu_internal.h"

namespace mbu {

__device__ inline uint32_t vor(uint32_t a, uint32_t b) { return a | b; }
__device__ inline uint2 vor(uint2 a, uint2 b) { return make_uint2(a.x | b.x, a.y | b.y); }
__device__ inline uint4 vor(uint4 a, uint4 b)
{
    return make_uint4(a.x | b.x, a.y | b.y, a.z | b.z, a.w | b.w);
}

// H x W input pixels, Ho = H / 2, Wo = W / 2 (floor: an odd last row / column is in no window)
template <typename V>
__global__ __launch_bounds__(256) void maxpool_kernel(const V *__restrict__ in, long total, int H, int W,
                                                      int Wo, int Ho, int Cv, V *__restrict__ out)
{
    long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    int c = (int)(idx % Cv);
    long p = idx / Cv;
    int x = (int)(p % Wo);
    long q = p / Wo;
    int y = (int)(q % Ho);
    long n = q / Ho;
    const V *r0 = in + (((n * H + 2 * y) * W) + 2 * x) * Cv + c;
    const V *r1 = r0 + (long)W * Cv;
    out[idx] = vor(vor(r0[0], r0[Cv]), vor(r1[0], r1[Cv]));
}

template <typename V>
__global__ __launch_bounds__(256) void upsample_kernel(const V *__restrict__ in, long total,
                                                       int Wo, int Ho, int Cv, V *__restrict__ out)
{
    long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    int c = (int)(idx % Cv);
    long p = idx / Cv;
    int x = (int)(p % Wo);
    long q = p / Wo;
    int y = (int)(q % Ho);
    long n = q / Ho;
    out[idx] = in[((n * (Ho / 2) + (y >> 1)) * (Wo / 2) + (x >> 1)) * Cv + c];
}

template <typename V>
__global__ __launch_bounds__(256) void concat_kernel(const V *__restrict__ a, int Cav,
                                                     const V *__restrict__ b, int Cbv, long total,
                                                     V *__restrict__ out)
{
    long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    int Cv = Cav + Cbv;
    int c = (int)(idx % Cv);
    long p = idx / Cv;
    out[idx] = c < Cav ? a[p * Cav + c] : b[p * Cbv + (c - Cav)];
}

template <typename V>
__global__ __launch_bounds__(256) void upcat_kernel(const V *__restrict__ skip, int Csv,
                                                    const V *__restrict__ low, int Clv, long total,
                                                    int Wo, int Ho, V *__restrict__ out)
{
    long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    int Cv = Csv + Clv;
    int c = (int)(idx % Cv);
    long p = idx / Cv;
    if (c < Csv) {
        out[idx] = skip[p * Csv + c];
    } else {
        int x = (int)(p % Wo);
        long q = p / Wo;
        int y = (int)(q % Ho);
        long n = q / Ho;
        out[idx] = low[((n * (Ho / 2) + (y >> 1)) * (Wo / 2) + (x >> 1)) * Clv + (c - Csv)];
    }
}

static int vec_words(int a, int b = 0)
{
    int g = a | b;
    return (g % 4 == 0) ? 4 : (g % 2 == 0) ? 2 : 1;
}

#define MBU_DISPATCH_V(v, CALL)                 \
    do {                                        \
        if ((v) == 4) { typedef uint4 V; CALL; } \
        else if ((v) == 2) { typedef uint2 V; CALL; } \
        else { typedef uint32_t V; CALL; }      \
    } while (0)

int launch_maxpool(const uint32_t *in, int N, int H, int W, int Cw, uint32_t *out, hipStream_t s)
{
    int v = vec_words(Cw), Cv = Cw / v, Ho = H / 2, Wo = W / 2;
    long total = (long)N * Ho * Wo * Cv;
    if (total == 0) return MBU_OK;
    unsigned blocks = (unsigned)((total + 255) / 256);
    MBU_DISPATCH_V(v, MBU_LAUNCH(maxpool_kernel<V>, dim3(blocks), dim3(256), 0, s,
                                         (const V *)in, total, H, W, Wo, Ho, Cv, (V *)out));
    return check_launch("maxpool2x2_bits");
}

int launch_upsample(const uint32_t *in, int N, int H, int W, int Cw, uint32_t *out, hipStream_t s)
{
    int v = vec_words(Cw), Cv = Cw / v, Ho = 2 * H, Wo = 2 * W;
    long total = (long)N * Ho * Wo * Cv;
    if (total == 0) return MBU_OK;
    unsigned blocks = (unsigned)((total + 255) / 256);
    MBU_DISPATCH_V(v, MBU_LAUNCH(upsample_kernel<V>, dim3(blocks), dim3(256), 0, s,
                                         (const V *)in, total, Wo, Ho, Cv, (V *)out));
    return check_launch("upsample2x_bits");
}

int launch_concat(const uint32_t *a, int Caw, const uint32_t *b, int Cbw, long pixels,
                  uint32_t *out, hipStream_t s)
{
    int v = vec_words(Caw, Cbw);
    long total = pixels * ((Caw + Cbw) / v);
    if (total == 0) return MBU_OK;
    unsigned blocks = (unsigned)((total + 255) / 256);
    MBU_DISPATCH_V(v, MBU_LAUNCH(concat_kernel<V>, dim3(blocks), dim3(256), 0, s,
                                         (const V *)a, Caw / v, (const V *)b, Cbw / v, total,
                                         (V *)out));
    return check_launch("concat_bits");
}

int launch_upcat(const uint32_t *skip, int Csw, const uint32_t *low, int Clw, int N, int H, int W,
                 uint32_t *out, hipStream_t s)
{
    int v = vec_words(Csw, Clw);
    long total = (long)N * H * W * ((Csw + Clw) / v);
    if (total == 0) return MBU_OK;
    unsigned blocks = (unsigned)((total + 255) / 256);
    MBU_DISPATCH_V(v, MBU_LAUNCH(upcat_kernel<V>, dim3(blocks), dim3(256), 0, s,
                                         (const V *)skip, Csw / v, (const V *)low, Clw / v, total,
                                         W, H, (V *)out));
    return check_launch("upsample_concat");
}

}  // namespace mbu
