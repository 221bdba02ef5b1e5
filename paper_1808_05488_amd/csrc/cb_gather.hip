// Matrix generation for the listed output pixels only (Sec. III-A, "Matrix
// Generation"): column n of X' is the receptive field of output pixel idx[n],
// row (c*kh + j)*kw + i as in the construction of X below Eq. 2, zero padding
// applied on the fly.  The source is the layer's input state.
//
// The paper uses one thread per (pixel, filter tap) copying all channels.  Here a
// lane owns one column n (so consecutive lanes write consecutive addresses of a
// row of X', and -- because the index list is sorted and changes are spatially
// clustered -- mostly read consecutive addresses of the state).  A work item is
// 256 columns x a group of input channels: the pixel's coordinates and the
// in-image mask of its filter rows and columns are worked out once per item, and
// each row then costs one load and one store with incremented addresses.  The
// loads go through a buffer resource; padding elements get an out-of-range offset
// and the hardware returns 0 for them.  The grid is persistent and strides over
// the work items; the number of columns is read from device memory (no host
// round trip), and the channel-group size is chosen there so that a few thousand
// columns still give every compute unit work.
#include "cb_kernels.h"

namespace cb {

namespace {

template <typename T> struct Ld;
template <> struct Ld<float> {
    static __device__ __forceinline__ float get(__amdgpu_buffer_rsrc_t r, unsigned off)
    { return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 0)); }
};
template <> struct Ld<uint16_t> {
    static __device__ __forceinline__ uint16_t get(__amdgpu_buffer_rsrc_t r, unsigned off)
    { return __builtin_amdgcn_raw_buffer_load_b16(r, (int)off, 0, 0); }
};

constexpr int GB = 32;   // rows gathered per batch (registers per lane)

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
    // channel groups: about 1024 work items when there are few column tiles
    int groups = (1024 + tiles_n - 1) / tiles_n;
    if (groups > g.C) groups = g.C;
    const int cg = (g.C + groups - 1) / groups;
    groups = (g.C + cg - 1) / cg;
    const long total = (long)tiles_n * groups;
    const int kk = g.kh * g.kw;
    // 32-bit byte offsets into the state; out-of-range offsets read as 0
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(src), 0, (int)((unsigned)g.C * (unsigned)g.P * (unsigned)sizeof(T)),
                                          0x00020000);
    for (long t = blockIdx.x; t < total; t += gridDim.x) {
        const int gi = (int)(t / tiles_n);
        const int n = (int)(t - (long)gi * tiles_n) * 256 + threadIdx.x;
        const int c0 = gi * cg, c1 = c0 + cg < g.C ? c0 + cg : g.C;
        T* xr = X + (size_t)c0 * kk * ld + n;
        if (n < ncols) {
            const int q = idx[col0 + n];
            const int yo = q / g.Wo, xo = q - yo * g.Wo;
            const int y0 = yo * g.s - g.p, x0 = xo * g.s - g.p;
            unsigned rowmask = 0, colmask = 0;      // filter rows / columns that fall inside the image
            for (int j = 0; j < g.kh; ++j) rowmask |= ((unsigned)(y0 + j) < (unsigned)g.H ? 1u : 0u) << j;
            for (int i = 0; i < g.kw; ++i) colmask |= ((unsigned)(x0 + i) < (unsigned)g.W ? 1u : 0u) << i;
            // Rows of this item in batches of GB: all loads of a batch are issued before its
            // first store.  Loads and stores share one in-order counter only among themselves,
            // so a wavefront that keeps both in flight has to drain everything at every wait;
            // separate load and store phases keep GB loads outstanding per lane instead of one.
            const int nelem = (c1 - c0) * kk;
            int j = 0, i = 0;                                   // wave-uniform position inside the filter
            unsigned cbase = ((unsigned)c0 * (unsigned)g.P + (unsigned)(y0 * g.W + x0)) * (unsigned)sizeof(T);
            unsigned rbase = cbase;
            for (int e0 = 0; e0 < nelem; e0 += GB) {
                T v[GB];
#pragma unroll
                for (int u = 0; u < GB; ++u) {
                    if (e0 + u < nelem) {
                        const unsigned ok = (rowmask >> j) & (colmask >> i) & 1u;
                        const unsigned off = (rbase + (unsigned)i * (unsigned)sizeof(T)) | (ok - 1u);
                        v[u] = Ld<T>::get(rsrc, off);
                        if (++i == g.kw) {
                            i = 0;
                            rbase += (unsigned)g.W * (unsigned)sizeof(T);
                            if (++j == g.kh) {
                                j = 0;
                                cbase += (unsigned)g.P * (unsigned)sizeof(T);
                                rbase = cbase;
                            }
                        }
                    }
                }
#pragma unroll
                for (int u = 0; u < GB; ++u)
                    if (e0 + u < nelem) xr[(size_t)(e0 + u) * ld] = v[u];
            }
        } else {
            const int rows = (c1 - c0) * kk;
            for (int r = 0; r < rows; ++r) xr[(size_t)r * ld] = 0;   // padding columns read by the GEMM tiles
        }
    }
}

}  // namespace

hipError_t launch_gather(const Geom& g, const void* src, const int32_t* idx, const int* count,
                         int col0, int cap, void* X, int* ctl, hipStream_t st, Tm tm)
{
    const unsigned grid = 2048;
    if (g.bf16)
        CB_LAUNCH(gather_kernel<uint16_t>, dim3(grid), dim3(256), st, tm, g, (const uint16_t*)src, idx,
                  count, col0, cap, (uint16_t*)X, ctl);
    else
        CB_LAUNCH(gather_kernel<float>, dim3(grid), dim3(256), st, tm, g, (const float*)src, idx, count,
                  col0, cap, (float*)X, ctl);
    return hipGetLastError();
}

}  // namespace cb
