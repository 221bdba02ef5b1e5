// Output update with fused bias + ReLU (Sec. III-A, "Output Updating"),
// change-based max-pooling (Sec. III-E, last paragraph), and the filter-matrix
// repacking done once at layer creation.
//
// Update: a lane owns one listed column n (coalesced reads along a row of Y'),
// a work item is 256 columns x a group of output channels (all of them when there are
// many columns, so the listed pixel is looked up once); the cached output is written
// only at the listed pixels, all other values keep their bits.
#include "cb_kernels.h"

namespace cb {

namespace {

__device__ __forceinline__ float ld_elem(const float* p) { return *p; }
__device__ __forceinline__ float ld_elem(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }
__device__ __forceinline__ void st_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_elem(uint16_t* p, float v)
{
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) { *p = (uint16_t)((u >> 16) | 0x40); return; }
    u += 0x7FFFu + ((u >> 16) & 1u);
    *p = (uint16_t)(u >> 16);
}

constexpr int OCH = 4;   // output channels per batch of loads (pooling: per work item)
constexpr int OB1 = 8;   // the same when Y' is a single slab (no k-split): more loads in flight per lane

// channel groups of the output update for `tiles_n` column tiles: about 2048 work items when there
// are few tiles, one group (the listed pixel is looked up once for all channels) when there are many
__host__ __device__ inline int update_groups(int O, int tiles_n)
{
    int groups = (2048 + tiles_n - 1) / tiles_n;
    const int maxg = (O + OCH - 1) / OCH;
    return groups > maxg ? maxg : groups;
}

template <typename T>
__global__ __launch_bounds__(256) void update_kernel(int O, int Opad, int R, int Po, const float* __restrict__ Y,
                                                     const float* __restrict__ bias,
                                                     const int32_t* __restrict__ idx,
                                                     const int* __restrict__ count, int col0, int cap, int relu,
                                                     T* __restrict__ OUT)
{
    int ncols = *count - col0;
    if (ncols > cap) ncols = cap;
    if (ncols <= 0) return;
    const int ld = (ncols + 255) & ~255;
    const int nsplit = gemm_nsplit(ncols, R, O, Opad, cap);
    const size_t slab = (size_t)O * ld;
    const int tiles_n = ld >> 8;
    int groups = update_groups(O, tiles_n);
    int cpg = (O + groups - 1) / groups;                 // channels per work item, a multiple of the batch
    cpg = (cpg + OCH - 1) / OCH * OCH;
    groups = (O + cpg - 1) / cpg;
    const long total = (long)tiles_n * groups;
    for (long t = blockIdx.x; t < total; t += gridDim.x) {
        const int gi = (int)(t / tiles_n);
        const int n = (int)(t - (long)gi * tiles_n) * 256 + threadIdx.x;
        if (n >= ncols) continue;
        const int q = idx[col0 + n];
        const int o1 = (gi + 1) * cpg < O ? (gi + 1) * cpg : O;
        const float* yn = Y + n;
        T* outq = OUT + q;
        if (nsplit == 1) {
            // one slab: batches of OB1 channels, all loads of a batch issued before its first store
            for (int o0 = gi * cpg; o0 < o1; o0 += OB1) {
                float v[OB1];
#pragma unroll
                for (int j = 0; j < OB1; ++j) v[j] = o0 + j < o1 ? yn[(size_t)(o0 + j) * ld] : 0.f;
#pragma unroll
                for (int j = 0; j < OB1; ++j) {
                    const int o = o0 + j;
                    if (o < o1) {
                        float r = v[j] + bias[o];
                        if (relu) r = r > 0.f ? r : 0.f;
                        st_elem(outq + (size_t)o * Po, r);
                    }
                }
            }
            continue;
        }
        // Y' is float32 for every dtype (one rounding, after bias and ReLU); the
        // k-split partial products are added in split order.  All loads of a batch
        // are issued before the first add.
        for (int o0 = gi * cpg; o0 < o1; o0 += OCH) {
            float part[OCH][8];
#pragma unroll
            for (int j = 0; j < OCH; ++j)
#pragma unroll
                for (int sp = 0; sp < 8; ++sp) {
                    const int o = o0 + j;
                    part[j][sp] = (o < o1 && sp < nsplit) ? yn[sp * slab + (size_t)o * ld] : 0.f;
                }
#pragma unroll
            for (int j = 0; j < OCH; ++j) {
                const int o = o0 + j;
                if (o >= o1) break;
                float v = part[j][0];
#pragma unroll
                for (int sp = 1; sp < 8; ++sp) v += part[j][sp];
                v += bias[o];
                if (relu) v = v > 0.f ? v : 0.f;
                st_elem(outq + (size_t)o * Po, v);
            }
        }
    }
}

// One lane per listed producer pixel: recompute the pooled cell that holds it.
// Up to w*w listed pixels share a cell and write the same value.
// idx == null: every producer pixel counts as listed (the whole pooled map is recomputed).
// POOL2: null, or a pixel-major copy of the pooled output (Hp*Wp x O) that receives the same values.
template <typename T>
__global__ __launch_bounds__(256) void pool_kernel(int O, int Ho, int Wo, int w, int Hp, int Wp,
                                                   const T* __restrict__ OUT, const int32_t* __restrict__ idx,
                                                   const int* __restrict__ count, T* __restrict__ POOL,
                                                   T* __restrict__ POOL2)
{
    const int N = idx ? *count : Ho * Wo;
    if (N <= 0) return;
    const int tiles_n = (N + 255) >> 8;
    const int och = (O + OCH - 1) / OCH;
    const long total = (long)tiles_n * och;
    for (long t = blockIdx.x; t < total; t += gridDim.x) {
        const int oc = (int)(t / tiles_n);
        const int n = (int)(t - (long)oc * tiles_n) * 256 + threadIdx.x;
        if (n >= N) continue;
        const int q = idx ? idx[n] : n;
        const int yo = q / Wo, xo = q - yo * Wo;
        const int yp = yo / w, xp = xo / w;
        const int y1 = (yp + 1) * w < Ho ? (yp + 1) * w : Ho;
        const int x1 = (xp + 1) * w < Wo ? (xp + 1) * w : Wo;
        const int o1 = (oc + 1) * OCH < O ? (oc + 1) * OCH : O;
        if (w == 2) {
            // the common window: all sixteen loads of the item (four channels x 2 x 2, clamped at the
            // border: a clamped tap repeats a value of the window) are issued before the first compare
            const int ya = yp * 2, yb = ya + 1 < Ho ? ya + 1 : ya;
            const int xa = xp * 2, xb = xa + 1 < Wo ? xa + 1 : xa;
            T v[OCH][4];
#pragma unroll
            for (int j = 0; j < OCH; ++j) {
                const int o = oc * OCH + j < o1 ? oc * OCH + j : o1 - 1;
                const T* src = OUT + (size_t)o * Ho * Wo;
                v[j][0] = src[(size_t)ya * Wo + xa];
                v[j][1] = src[(size_t)ya * Wo + xb];
                v[j][2] = src[(size_t)yb * Wo + xa];
                v[j][3] = src[(size_t)yb * Wo + xb];
            }
#pragma unroll
            for (int j = 0; j < OCH; ++j) {
                const int o = oc * OCH + j;
                if (o >= o1) break;
                // same scan order as the general form: the first of equal maxima wins
                T best = v[j][0];
                float bv = ld_elem(&best);
#pragma unroll
                for (int e = 1; e < 4; ++e) {
                    const float cv = ld_elem(&v[j][e]);
                    if (cv > bv) { bv = cv; best = v[j][e]; }
                }
                POOL[((size_t)o * Hp + yp) * Wp + xp] = best;
                if (POOL2) POOL2[((size_t)yp * Wp + xp) * O + o] = best;
            }
            continue;
        }
        for (int o = oc * OCH; o < o1; ++o) {
            const T* src = OUT + (size_t)o * Ho * Wo;
            // maximum taken on the stored bit patterns' values; the winner's bits are copied
            T best = src[(size_t)(yp * w) * Wo + xp * w];
            float bv = ld_elem(&best);
            for (int y = yp * w; y < y1; ++y)
                for (int x = xp * w; x < x1; ++x) {
                    T c = src[(size_t)y * Wo + x];
                    float cv = ld_elem(&c);
                    if (cv > bv) { bv = cv; best = c; }
                }
            POOL[((size_t)o * Hp + yp) * Wp + xp] = best;
            if (POOL2) POOL2[((size_t)yp * Wp + xp) * O + o] = best;
        }
    }
}

// K (O x R, row-major == the O x C x kh x kw filter tensor) -> KT (R x Opad), zero
// padded; bias -> float32 (zeros when absent).
template <typename T>
__global__ __launch_bounds__(256) void pack_weights_kernel(int O, int Opad, int R, const T* __restrict__ w,
                                                           const T* __restrict__ bias, T* __restrict__ KT,
                                                           float* __restrict__ bias_f)
{
    const long n = (long)R * Opad;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long)gridDim.x * 256) {
        const int r = (int)(e / Opad), o = (int)(e - (long)r * Opad);
        KT[e] = o < O ? w[(size_t)o * R + r] : (T)0;
    }
    if (blockIdx.x == 0)
        for (int o = threadIdx.x; o < Opad; o += 256) bias_f[o] = (bias && o < O) ? ld_elem(bias + o) : 0.f;
}

}  // namespace

hipError_t launch_update(const Geom& g, const void* Y, const float* bias, const int32_t* idx,
                         const int* count, int col0, int cap, int relu, void* OUT, hipStream_t st, Tm tm)
{
    const int tiles_max = (cap + 255) / 256;
    long max_items = (long)tiles_max * update_groups(g.O, tiles_max);
    if (max_items < (g.O + OCH - 1) / OCH) max_items = (g.O + OCH - 1) / OCH;   // few tiles: one item per channel batch
    unsigned grid = (unsigned)(max_items < 2048 ? max_items : 2048);
    if (grid == 0) grid = 1;
    if (g.bf16)
        CB_LAUNCH(update_kernel<uint16_t>, dim3(grid), dim3(256), st, tm, g.O, g.Opad, g.R, g.Po, (const float*)Y, bias,
                  idx, count, col0, cap, relu, (uint16_t*)OUT);
    else
        CB_LAUNCH(update_kernel<float>, dim3(grid), dim3(256), st, tm, g.O, g.Opad, g.R, g.Po, (const float*)Y, bias, idx,
                  count, col0, cap, relu, (float*)OUT);
    return hipGetLastError();
}

hipError_t launch_pool(int O, int Ho, int Wo, int w, int bf16, const void* OUT, const int32_t* idx,
                       const int* count, void* POOL, void* POOL2, hipStream_t st)
{
    const int Hp = (Ho + w - 1) / w, Wp = (Wo + w - 1) / w;
    long max_items = (long)(((long)Ho * Wo + 255) / 256) * ((O + OCH - 1) / OCH);
    unsigned grid = (unsigned)(max_items < 2048 ? max_items : 2048);
    if (grid == 0) grid = 1;
    if (bf16)
        hipLaunchKernelGGL(pool_kernel<uint16_t>, dim3(grid), dim3(256), 0, st, O, Ho, Wo, w, Hp, Wp,
                           (const uint16_t*)OUT, idx, count, (uint16_t*)POOL, (uint16_t*)POOL2);
    else
        hipLaunchKernelGGL(pool_kernel<float>, dim3(grid), dim3(256), 0, st, O, Ho, Wo, w, Hp, Wp, (const float*)OUT,
                           idx, count, (float*)POOL, (float*)POOL2);
    return hipGetLastError();
}

hipError_t launch_pack_weights(const Geom& g, const void* w, const void* bias, void* KT, float* bias_f,
                               hipStream_t st)
{
    long n = (long)g.R * g.Opad;
    unsigned grid = (unsigned)((n + 255) / 256);
    if (grid > 2048) grid = 2048;
    if (g.bf16)
        hipLaunchKernelGGL(pack_weights_kernel<uint16_t>, dim3(grid), dim3(256), 0, st, g.O, g.Opad, g.R,
                           (const uint16_t*)w, (const uint16_t*)bias, (uint16_t*)KT, bias_f);
    else
        hipLaunchKernelGGL(pack_weights_kernel<float>, dim3(grid), dim3(256), 0, st, g.O, g.Opad, g.R, (const float*)w,
                           (const float*)bias, (float*)KT, bias_f);
    return hipGetLastError();
}

}  // namespace cb
