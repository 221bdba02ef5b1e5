// Matrix generation for the listed output pixels only (Sec. III-A, "Matrix
// Generation"): column n of X' is the receptive field of output pixel idx[n],
// row (c*kh + j)*kw + i as in the construction of X below Eq. 2, zero padding
// applied on the fly.  The source is the layer's input state.
//
// The paper uses one thread per (pixel, filter tap) copying all channels.  Here a
// lane owns one column n (so consecutive lanes write consecutive addresses of a
// row of X', and -- because the index list is sorted and changes are spatially
// clustered -- mostly read consecutive addresses of the state).  A work item is
// 256 columns x a group of input channels.  The rows of one channel and one
// filter row are kw consecutive elements of the state: a lane fetches them as
// runs of up to four (float32) / three (bfloat16) elements with ONE load each --
// the vector memory pipeline's cost is per load and cache line touched, not per
// byte -- masks the taps that fall into the padding, and writes each element to
// its own row of X'.  Loads go through a buffer resource that begins GUARD bytes
// ahead of the state (the run of channel 0, image row 0 starts before the state
// for pixels on the left border, and a load whose first byte is out of range
// returns nothing; components beyond the end read as 0).  All loads of a batch
// are issued before its first store: loads and stores share one in-order
// counter, so a wavefront that keeps both in flight has to drain everything at
// every wait.  The grid is persistent and strides over the work items; the
// number of columns is read from device memory (no host round trip), and the
// channel-group size is chosen there so that a few thousand columns still give
// every compute unit work.
#include "cb_kernels.h"

namespace cb {

namespace {

typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

constexpr int GUARD = 128;   // readable bytes ahead of the source: pad <= 31 elements of 4 bytes

// A run of up to LEN elements starting at byte offset `off` of the buffer.
template <typename T> struct Run;
template <> struct Run<float> {
    static constexpr int LEN = 4;
    uintx4 v;
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, unsigned off)
    { v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0); }
    __device__ __forceinline__ float get(int e, unsigned) const { return __uint_as_float(v[e]); }
};
template <> struct Run<uint16_t> {
    static constexpr int LEN = 3;
    uintx2 v;                                    // the two aligned 32-bit words that hold the three elements
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, unsigned off)
    { v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)(off & ~3u), 0, 0); }
    __device__ __forceinline__ uint16_t get(int e, unsigned off) const
    {
        const unsigned sh = (off & 2u) << 3;     // odd element: data starts 16 bits in
        const unsigned lo = __builtin_amdgcn_alignbit(v[1], v[0], sh), hi = v[1] >> sh;
        return (uint16_t)(e == 0 ? lo : e == 1 ? lo >> 16 : hi);
    }
};

constexpr int NB = 8;        // runs per batch (registers per lane: 32 / 16)

// Many columns (GATHER_WIDE_MIN and more): a lane owns FOUR consecutive columns, so that every tap
// of the run is written with one 16-byte (float32) / 8-byte (bfloat16) store, and a work item is
// 1024 columns x a group of channels.  Four times fewer store instructions, four times the bytes in
// flight per wavefront: 3.4 -> 4.1 TB/s at 256 000 columns of 1152 rows.  The stores are marked
// non-temporal: X' is read next by another kernel, from HBM, and should not push the rows of the
// state that neighbouring tiles are about to re-read out of the L2.
constexpr int GATHER_WIDE_MIN = 32768;
constexpr int NBW = 3;       // runs per batch of the wide form (registers per lane: 4 x 4 x NBW)

__device__ __forceinline__ void store4(float* p, float a, float b, float c, float d)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    __builtin_nontemporal_store(f4{a, b, c, d}, reinterpret_cast<f4*>(p));
}
__device__ __forceinline__ void store4(uint16_t* p, uint16_t a, uint16_t b, uint16_t c, uint16_t d)
{
    __builtin_nontemporal_store(uintx2{(unsigned)a | ((unsigned)b << 16), (unsigned)c | ((unsigned)d << 16)},
                                reinterpret_cast<uintx2*>(p));
}

// KW = 3: filters three taps wide (one run per filter row, compile-time length); KW = 0: any width
template <typename T, int KW>
__device__ __forceinline__ void gather_wide(const Geom& g, __amdgpu_buffer_rsrc_t rsrc,
                                            const int32_t* __restrict__ idx, int col0, int ncols, int ld,
                                            T* __restrict__ X)
{
    constexpr int LEN = Run<T>::LEN;
    const int tiles_n = (ld + 1023) >> 10;
    int groups = (1024 + tiles_n - 1) / tiles_n;
    if (groups > g.C) groups = g.C;
    const int cg = (g.C + groups - 1) / groups;
    groups = (g.C + cg - 1) / cg;
    const long total = (long)tiles_n * groups;
    const int kw = KW ? KW : g.kw;
    const int kk = g.kh * kw;
    const int npc = (kw + LEN - 1) / LEN;
    const unsigned esz = (unsigned)sizeof(T);
    for (long t = blockIdx.x; t < total; t += gridDim.x) {
        const int gi = (int)(t / tiles_n);
        const int n = (int)(t - (long)gi * tiles_n) * 1024 + (int)threadIdx.x * 4;
        if (n >= ld) continue;                   // ld is a multiple of 256: a lane's four columns are all inside or all outside
        const int c0 = gi * cg, c1 = c0 + cg < g.C ? c0 + cg : g.C;
        T* xr = X + (size_t)c0 * kk * ld + n;
        unsigned rowmask[4], colmask[4], cbl[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const bool colv = n + k < ncols;     // columns beyond the last one are written as zeros
            const int q = colv ? idx[col0 + n + k] : 0;
            const int yo = q / g.Wo, xo = q - yo * g.Wo;
            const int y0 = yo * g.s - g.p, x0 = xo * g.s - g.p;
            rowmask[k] = colmask[k] = 0;
            if (colv) {
                for (int j = 0; j < g.kh; ++j) rowmask[k] |= ((unsigned)(y0 + j) < (unsigned)g.H ? 1u : 0u) << j;
                for (int i = 0; i < kw; ++i) colmask[k] |= ((unsigned)(x0 + i) < (unsigned)g.W ? 1u : 0u) << i;
            }
            cbl[k] = ((unsigned)c0 * (unsigned)g.P + (unsigned)(y0 * g.W + x0)) * esz + (unsigned)GUARD;
        }
        const int nruns = (c1 - c0) * g.kh * npc;
        // wave-uniform position of the next run to load / to store: filter row, first tap; rel = byte
        // offset of the run being loaded relative to the top-left tap of channel c0
        int jl = 0, il = 0, js = 0, is = 0;
        unsigned crel = 0, rrel = 0;
        size_t rows = 0;
        for (int e0 = 0; e0 < nruns; e0 += NBW) {
            Run<T> v[NBW][4];
            unsigned offs[NBW][4];
#pragma unroll
            for (int u = 0; u < NBW; ++u) {
                if (e0 + u < nruns) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        offs[u][k] = cbl[k] + rrel + (unsigned)il * esz;
                        v[u][k].load(rsrc, offs[u][k]);
                    }
                    il += LEN;
                    if (il >= kw) {
                        il = 0;
                        rrel += (unsigned)g.W * esz;
                        if (++jl == g.kh) {
                            jl = 0;
                            crel += (unsigned)g.P * esz;
                            rrel = crel;
                        }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < NBW; ++u) {
                if (e0 + u < nruns) {
                    const int len = KW ? KW : (kw - is < LEN ? kw - is : LEN);
#pragma unroll
                    for (int e = 0; e < LEN; ++e) {
                        if (e < len) {
                            T o[4];
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                const bool ok = (((rowmask[k] >> js) & (colmask[k] >> (is + e))) & 1u) != 0u;
                                o[k] = ok ? v[u][k].get(e, offs[u][k]) : (T)0;
                            }
                            store4(xr + (rows + e) * ld, o[0], o[1], o[2], o[3]);
                        }
                    }
                    rows += len;
                    is += LEN;
                    if (is >= kw) {
                        is = 0;
                        if (++js == g.kh) js = 0;
                    }
                }
            }
        }
    }
}

template <typename T>
__global__ __launch_bounds__(256) void gather_kernel(Geom g, const T* __restrict__ src,
                                                     const int32_t* __restrict__ idx,
                                                     const int* __restrict__ count, int col0, int cap,
                                                     T* __restrict__ X, int* __restrict__ ctl)
{
    constexpr int LEN = Run<T>::LEN;
    int ncols = *count - col0;
    if (ncols > cap) ncols = cap;
    if (ncols <= 0) {
        if (blockIdx.x == 0 && threadIdx.x == 0 && col0 == 0) { ctl[CTL_LD] = 0; ctl[CTL_NCOLS] = 0; }
        return;
    }
    const int ld = (ncols + 255) & ~255;
    if (blockIdx.x == 0 && threadIdx.x == 0) { ctl[CTL_LD] = ld; ctl[CTL_NCOLS] = ncols; }
    const unsigned esz = (unsigned)sizeof(T);
    // (whole 32-bit words are fetched: an odd bfloat16 element count is rounded up, the source's
    // allocation is padded)
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        reinterpret_cast<char*>(const_cast<T*>(src)) - GUARD, 0,
        (int)((((unsigned)g.C * (unsigned)g.P * esz + 3u) & ~3u) + (unsigned)GUARD), 0x00020000);
    if (ncols >= GATHER_WIDE_MIN) {
        if (g.kw == 3) gather_wide<T, 3>(g, rsrc, idx, col0, ncols, ld, X);
        else gather_wide<T, 0>(g, rsrc, idx, col0, ncols, ld, X);
        return;
    }
    const int tiles_n = ld >> 8;
    // channel groups: about 1024 work items when there are few column tiles
    int groups = (1024 + tiles_n - 1) / tiles_n;
    if (groups > g.C) groups = g.C;
    const int cg = (g.C + groups - 1) / groups;
    groups = (g.C + cg - 1) / cg;
    const long total = (long)tiles_n * groups;
    const int kk = g.kh * g.kw;
    const int npc = (g.kw + LEN - 1) / LEN;      // runs per filter row
    // Workgroup b runs on XCD b mod 8; every XCD takes a contiguous range of work items, so that
    // tiles that are neighbours in the (sorted) index list, and therefore read the same rows of
    // the state, share one L2 (the grid is a multiple of 8)
    const long per_xcd = (total + 7) / 8;
    const long xbase = (long)(blockIdx.x & 7) * per_xcd;
    for (long tt = blockIdx.x >> 3; tt < per_xcd; tt += gridDim.x >> 3) {
        const long t = xbase + tt;
        if (t >= total) break;
        const int gi = (int)(t / tiles_n);
        const int n = (int)(t - (long)gi * tiles_n) * 256 + threadIdx.x;
        const int c0 = gi * cg, c1 = c0 + cg < g.C ? c0 + cg : g.C;
        T* xr = X + (size_t)c0 * kk * ld + n;
        // a lane beyond the last column still runs (it writes the zero padding columns that
        // the GEMM tiles read): all its taps count as padding
        const bool colv = n < ncols;
        const int q = colv ? idx[col0 + n] : 0;
        const int yo = q / g.Wo, xo = q - yo * g.Wo;
        const int y0 = yo * g.s - g.p, x0 = xo * g.s - g.p;
        unsigned rowmask = 0, colmask = 0;      // filter rows / columns that fall inside the image
        if (colv) {
            for (int j = 0; j < g.kh; ++j) rowmask |= ((unsigned)(y0 + j) < (unsigned)g.H ? 1u : 0u) << j;
            for (int i = 0; i < g.kw; ++i) colmask |= ((unsigned)(x0 + i) < (unsigned)g.W ? 1u : 0u) << i;
        }
        const int nruns = (c1 - c0) * g.kh * npc;
        // wave-uniform position of the next run to load / to store: channel, filter row, first tap
        int jl = 0, il = 0, js = 0, is = 0;
        unsigned cbl = ((unsigned)c0 * (unsigned)g.P + (unsigned)(y0 * g.W + x0)) * esz + (unsigned)GUARD;
        unsigned rbl = cbl;                      // byte offset of tap (j, 0) of the run being loaded
        size_t rows = 0;                         // row of X' (relative to c0*kk) of the run being stored
        for (int e0 = 0; e0 < nruns; e0 += NB) {
            Run<T> v[NB];
            unsigned offs[NB];
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                if (e0 + u < nruns) {
                    offs[u] = rbl + (unsigned)il * esz;
                    v[u].load(rsrc, offs[u]);
                    il += LEN;
                    if (il >= g.kw) {
                        il = 0;
                        rbl += (unsigned)g.W * esz;
                        if (++jl == g.kh) {
                            jl = 0;
                            cbl += (unsigned)g.P * esz;
                            rbl = cbl;
                        }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                if (e0 + u < nruns) {
                    const unsigned rowok = (rowmask >> js) & 1u;
                    const int len = g.kw - is < LEN ? g.kw - is : LEN;
#pragma unroll
                    for (int e = 0; e < LEN; ++e) {
                        if (e < len) {
                            const bool ok = (rowok & (colmask >> (is + e))) != 0u;
                            xr[(rows + e) * ld] = ok ? v[u].get(e, offs[u]) : (T)0;
                        }
                    }
                    rows += len;
                    is += LEN;
                    if (is >= g.kw) {
                        is = 0;
                        if (++js == g.kh) js = 0;
                    }
                }
            }
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
