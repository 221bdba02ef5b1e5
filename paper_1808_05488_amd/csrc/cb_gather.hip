// Matrix generation for the listed output pixels only (Sec. III-A, "Matrix
// Generation"): column n of X' is the receptive field of output pixel idx[n],
// row (c*kh + j)*kw + i as in the construction of X below Eq. 2, zero padding
// applied on the fly.  The source is the layer's input state.
//
// The paper uses one thread per (pixel, filter tap) copying all channels.  Here a
// lane owns one column n (so consecutive lanes write consecutive addresses of a
// row of X', and -- because the index list is sorted and changes are spatially
// clustered -- mostly read consecutive addresses of the state), and a work item
// is (256 columns) x (one input channel): kh*kw rows.  The grid is persistent
// and strides over the work items; the number of columns is read from device
// memory, so no host round trip is needed.
#include "cb_kernels.h"

namespace cb {

namespace {

template <typename T>
__global__ __launch_bounds__(256) void gather_kernel(Geom g, const T* __restrict__ src,
                                                     const int32_t* __restrict__ idx,
                                                     const int* __restrict__ count, int col0, int cap,
                                                     T* __restrict__ X, int* __restrict__ ctl)
{
    int ncols = *count - col0;
    if (ncols > cap) ncols = cap;
    if (ncols <= 0) {
        if (blockIdx.x == 0 && threadIdx.x == 0 && col0 == 0) { ctl[CTL_LD] = 0; ctl[CTL_NCOLS] = 0; }
        return;
    }
    const int ld = (ncols + 255) & ~255;
    if (blockIdx.x == 0 && threadIdx.x == 0) { ctl[CTL_LD] = ld; ctl[CTL_NCOLS] = ncols; }
    const int tiles_n = ld >> 8;
    const long total = (long)tiles_n * g.C;
    const int kk = g.kh * g.kw;
    for (long t = blockIdx.x; t < total; t += gridDim.x) {
        const int c = (int)(t / tiles_n);
        const int n = (int)(t - (long)c * tiles_n) * 256 + threadIdx.x;
        const T* sc = src + (size_t)c * g.P;
        T* xr = X + (size_t)c * kk * ld + n;
        if (n < ncols) {
            const int q = idx[col0 + n];
            const int yo = q / g.Wo, xo = q - yo * g.Wo;
            const int y0 = yo * g.s - g.p, x0 = xo * g.s - g.p;
            for (int j = 0; j < g.kh; ++j) {
                const int yi = y0 + j;
                const bool yin = yi >= 0 && yi < g.H;
                const T* row = sc + (size_t)(yin ? yi : 0) * g.W;
                for (int i = 0; i < g.kw; ++i) {
                    const int xi = x0 + i;
                    T v = 0;
                    if (yin && xi >= 0 && xi < g.W) v = row[xi];
                    xr[(size_t)(j * g.kw + i) * ld] = v;
                }
            }
        } else {
            for (int r = 0; r < kk; ++r) xr[(size_t)r * ld] = 0;   // padding columns read by the GEMM tiles
        }
    }
}

}  // namespace

hipError_t launch_gather(const Geom& g, const void* src, const int32_t* idx, const int* count,
                         int col0, int cap, void* X, int* ctl, hipStream_t st, Tm tm)
{
    long max_items = (long)((cap + 255) / 256) * g.C;
    unsigned grid = (unsigned)(max_items < 2048 ? max_items : 2048);
    if (grid == 0) grid = 1;
    if (g.bf16)
        CB_LAUNCH(gather_kernel<uint16_t>, dim3(grid), dim3(256), st, tm, g, (const uint16_t*)src, idx,
                  count, col0, cap, (uint16_t*)X, ctl);
    else
        CB_LAUNCH(gather_kernel<float>, dim3(grid), dim3(256), st, tm, g, (const float*)src, idx, count,
                  col0, cap, (float*)X, ctl);
    return hipGetLastError();
}

}  // namespace cb
