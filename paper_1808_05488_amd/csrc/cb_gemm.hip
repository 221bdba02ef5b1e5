// The one dense contraction of the path: Y' = K X' (Eq. 2 restricted to the
// listed columns; Sec. III-A, "Matrix Generation & Matrix Multiplication"),
// K: O x R filter matrix, X': R x N, Y': O x N.
//
// The paper calls a vendor GEMM.  Here it is a hand-written MFMA kernel for
// gfx950: both operands are k-major in memory (the filter matrix is stored
// transposed, R x Opad, at layer creation; X' is R x ld), so a BK x BM and a
// BK x BN tile are staged through LDS with 16-byte loads and read back as
// MFMA fragments without bank conflicts (row pitch = 16 mod 32 words).
// float32 uses v_mfma_f32_16x16x4_f32 (inputs stay float32: the 1e-4 parity bound
// leaves no room for reduced-precision operands); bfloat16 uses
// v_mfma_f32_16x16x16_bf16 with float32 accumulation.  Y' is float32 in both cases.
//
// The grid is persistent: the column count N lives in device memory, workgroups
// stride over the (n-tile, m-tile, k-split) space.  N is usually a few thousand
// columns, far too few tiles for 256 compute units, so the K dimension is split
// (gemm_nsplit) and each split writes its own partial product; the output-update
// kernel adds the partials in a fixed order.  Tiles that share X' columns are
// given to workgroups of the same XCD (id mod 8) so that the columns are served
// from that XCD's L2.
#include "cb_kernels.h"

namespace cb {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef short shortx4 __attribute__((ext_vector_type(4)));

constexpr int BK = 32;

// Work decomposition shared by both element types.
struct Work {
    int ncols, ld, NT, MT, nsplit, kchunk;
    long total;
};

template <int BM, int BN>
__device__ __forceinline__ bool make_work(int O, int Opad, int R, const int* count, int col0, int cap, Work& w)
{
    int ncols = *count - col0;
    if (ncols > cap) ncols = cap;
    if (ncols <= 0) return false;
    w.ncols = ncols;
    w.ld = (ncols + 255) & ~255;
    w.NT = (ncols + BN - 1) / BN;
    w.MT = Opad / BM;
    w.nsplit = gemm_nsplit(ncols, R, O, Opad, cap);
    w.kchunk = ((R + w.nsplit - 1) / w.nsplit + BK - 1) / BK * BK;
    w.total = (long)((w.NT + 7) & ~7) * w.MT * w.nsplit;
    return true;
}

// item t -> (n-tile, m-tile, split): the 8 XCDs take consecutive n-tiles; within an
// XCD the m-tiles and splits of one n-tile are consecutive.
__device__ __forceinline__ bool decode(const Work& w, long t, int& nt, int& mt, int& sp)
{
    const int xcd = (int)(t & 7);
    long s = t >> 3;
    mt = (int)(s % w.MT); s /= w.MT;
    sp = (int)(s % w.nsplit); s /= w.nsplit;
    nt = (int)s * 8 + xcd;
    return nt < w.NT;
}

template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(256) void gemm_f32_kernel(int O, int Opad, int R, const float* __restrict__ KT,
                                                       const float* __restrict__ X, float* __restrict__ Y,
                                                       const int* __restrict__ count, int col0, int cap,
                                                       int* __restrict__ ctl)
{
    static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
    constexpr int WM = BM / WGM, WN = BN / WGN;       // wavefront tile
    constexpr int TM = WM / 16, TN = WN / 16;         // 16x16 MFMA tiles per wavefront
    constexpr int BMP = BM + (BM % 32 == 16 ? 0 : 16);
    constexpr int BNP = BN + (BN % 32 == 16 ? 0 : 16);
    constexpr int AV = (BK * BM / 4 + 255) / 256;     // float4 loads per thread for the A tile
    constexpr int BV = (BK * BN / 4 + 255) / 256;
    __shared__ float As[BK * BMP];
    __shared__ float Bs[BK * BNP];

    Work w;
    if (!make_work<BM, BN>(O, Opad, R, count, col0, cap, w)) return;
    if (blockIdx.x == 0 && threadIdx.x == 0) ctl[CTL_NSPLIT] = w.nsplit;
    const int ld = w.ld;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm0 = (wv / WGN) * WM, wn0 = (wv % WGN) * WN;
    const int l16 = lane & 15, lq = lane >> 4;

    for (long t = blockIdx.x; t < w.total; t += gridDim.x) {
        int nt, mt, sp;
        if (!decode(w, t, nt, mt, sp)) continue;
        const int m0 = mt * BM, n0 = nt * BN;
        const int kbeg = sp * w.kchunk;
        const int kend = kbeg + w.kchunk < R ? kbeg + w.kchunk : R;

        floatx4 acc[TM][TN];
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b) acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};

        float4 ra[AV], rb[BV];
        auto gload = [&](int k0) {
#pragma unroll
            for (int v = 0; v < AV; ++v) {
                const int e = (v * 256 + tid) * 4;
                const int k = e / BM, m = e % BM;
                ra[v] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (e < BK * BM && k0 + k < kend)
                    ra[v] = *reinterpret_cast<const float4*>(KT + (size_t)(k0 + k) * Opad + m0 + m);
            }
#pragma unroll
            for (int v = 0; v < BV; ++v) {
                const int e = (v * 256 + tid) * 4;
                const int k = e / BN, n = e % BN;
                rb[v] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (e < BK * BN && k0 + k < kend)
                    rb[v] = *reinterpret_cast<const float4*>(X + (size_t)(k0 + k) * ld + n0 + n);
            }
        };
        auto lstore = [&]() {
#pragma unroll
            for (int v = 0; v < AV; ++v) {
                const int e = (v * 256 + tid) * 4;
                if (e < BK * BM) *reinterpret_cast<float4*>(&As[(e / BM) * BMP + e % BM]) = ra[v];
            }
#pragma unroll
            for (int v = 0; v < BV; ++v) {
                const int e = (v * 256 + tid) * 4;
                if (e < BK * BN) *reinterpret_cast<float4*>(&Bs[(e / BN) * BNP + e % BN]) = rb[v];
            }
        };

        if (kbeg < kend) gload(kbeg);
        for (int k0 = kbeg; k0 < kend; k0 += BK) {
            __syncthreads();                 // previous tile's fragments have been read
            lstore();
            __syncthreads();
            if (k0 + BK < kend) gload(k0 + BK);   // next tile's global loads overlap the MFMAs
#pragma unroll
            for (int kk = 0; kk < BK / 4; ++kk) {
                float af[TM], bf[TN];
#pragma unroll
                for (int a = 0; a < TM; ++a) af[a] = As[(kk * 4 + lq) * BMP + wm0 + a * 16 + l16];
#pragma unroll
                for (int b = 0; b < TN; ++b) bf[b] = Bs[(kk * 4 + lq) * BNP + wn0 + b * 16 + l16];
#pragma unroll
                for (int a = 0; a < TM; ++a)
#pragma unroll
                    for (int b = 0; b < TN; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[a], bf[b], acc[a][b], 0, 0, 0);
            }
        }

        // D fragment: lane holds column l16, rows 4*lq + r; split sp writes its own O x ld slab
        float* Ys = Y + (size_t)sp * O * ld;
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = m0 + wm0 + a * 16 + lq * 4 + r;
                    const int n = n0 + wn0 + b * 16 + l16;
                    if (m < O) Ys[(size_t)m * ld + n] = acc[a][b][r];
                }
    }
}

// bfloat16 operands (bit patterns), float32 accumulation, Y' kept in float32 (the
// single rounding to bfloat16 happens in the output update).  Tiles are
// transposed on the way into LDS so that the four consecutive k of a fragment
// are one 8-byte read.
template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(int O, int Opad, int R, const uint16_t* __restrict__ KT,
                                                        const uint16_t* __restrict__ X, float* __restrict__ Y,
                                                        const int* __restrict__ count, int col0, int cap,
                                                        int* __restrict__ ctl)
{
    static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 16, TN = WN / 16;
    constexpr int KP = BK + 4;                        // LDS row pitch in elements (k contiguous)
    constexpr int AV = (BK * BM / 8 + 255) / 256;     // 16-byte loads per thread
    constexpr int BV = (BK * BN / 8 + 255) / 256;
    __shared__ uint16_t As[BM * KP];
    __shared__ uint16_t Bs[BN * KP];

    Work w;
    if (!make_work<BM, BN>(O, Opad, R, count, col0, cap, w)) return;
    if (blockIdx.x == 0 && threadIdx.x == 0) ctl[CTL_NSPLIT] = w.nsplit;
    const int ld = w.ld;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm0 = (wv / WGN) * WM, wn0 = (wv % WGN) * WN;
    const int l16 = lane & 15, lq = lane >> 4;

    for (long t = blockIdx.x; t < w.total; t += gridDim.x) {
        int nt, mt, sp;
        if (!decode(w, t, nt, mt, sp)) continue;
        const int m0 = mt * BM, n0 = nt * BN;
        const int kbeg = sp * w.kchunk;
        const int kend = kbeg + w.kchunk < R ? kbeg + w.kchunk : R;

        floatx4 acc[TM][TN];
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b) acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};

        uint4 ra[AV], rb[BV];
        auto gload = [&](int k0) {
#pragma unroll
            for (int v = 0; v < AV; ++v) {
                const int e = (v * 256 + tid) * 8;
                const int k = e / BM, m = e % BM;
                ra[v] = make_uint4(0, 0, 0, 0);
                if (e < BK * BM && k0 + k < kend)
                    ra[v] = *reinterpret_cast<const uint4*>(KT + (size_t)(k0 + k) * Opad + m0 + m);
            }
#pragma unroll
            for (int v = 0; v < BV; ++v) {
                const int e = (v * 256 + tid) * 8;
                const int k = e / BN, n = e % BN;
                rb[v] = make_uint4(0, 0, 0, 0);
                if (e < BK * BN && k0 + k < kend)
                    rb[v] = *reinterpret_cast<const uint4*>(X + (size_t)(k0 + k) * ld + n0 + n);
            }
        };
        auto lstore = [&]() {
#pragma unroll
            for (int v = 0; v < AV; ++v) {
                const int e = (v * 256 + tid) * 8;
                if (e < BK * BM) {
                    const int k = e / BM, m = e % BM;
                    const uint32_t wd[4] = {ra[v].x, ra[v].y, ra[v].z, ra[v].w};
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        As[(m + q) * KP + k] = (uint16_t)(wd[q >> 1] >> ((q & 1) * 16));
                }
            }
#pragma unroll
            for (int v = 0; v < BV; ++v) {
                const int e = (v * 256 + tid) * 8;
                if (e < BK * BN) {
                    const int k = e / BN, n = e % BN;
                    const uint32_t wd[4] = {rb[v].x, rb[v].y, rb[v].z, rb[v].w};
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        Bs[(n + q) * KP + k] = (uint16_t)(wd[q >> 1] >> ((q & 1) * 16));
                }
            }
        };

        if (kbeg < kend) gload(kbeg);
        for (int k0 = kbeg; k0 < kend; k0 += BK) {
            __syncthreads();
            lstore();
            __syncthreads();
            if (k0 + BK < kend) gload(k0 + BK);
#pragma unroll
            for (int kk = 0; kk < BK / 16; ++kk) {
                shortx4 af[TM], bf[TN];
#pragma unroll
                for (int a = 0; a < TM; ++a)
                    af[a] = *reinterpret_cast<const shortx4*>(&As[(wm0 + a * 16 + l16) * KP + kk * 16 + lq * 4]);
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    bf[b] = *reinterpret_cast<const shortx4*>(&Bs[(wn0 + b * 16 + l16) * KP + kk * 16 + lq * 4]);
#pragma unroll
                for (int a = 0; a < TM; ++a)
#pragma unroll
                    for (int b = 0; b < TN; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(af[a], bf[b], acc[a][b], 0, 0, 0);
            }
        }

        float* Ys = Y + (size_t)sp * O * ld;
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = m0 + wm0 + a * 16 + lq * 4 + r;
                    const int n = n0 + wn0 + b * 16 + l16;
                    if (m < O) Ys[(size_t)m * ld + n] = acc[a][b][r];
                }
    }
}

}  // namespace

hipError_t launch_gemm(const Geom& g, const void* KT, const void* X, void* Y, const int* count,
                       int col0, int cap, int* ctl, hipStream_t st, Tm tm)
{
    const int bm = gemm_bm(g.O);
    const dim3 grid(1024), block(256);   // grid: multiple of 8 (XCD mapping), a few workgroups per CU
    if (g.bf16) {
        const uint16_t* k = (const uint16_t*)KT; const uint16_t* x = (const uint16_t*)X; float* y = (float*)Y;
        if (bm == 16)      CB_LAUNCH((gemm_bf16_kernel<16, 256, 1, 4>), grid, block, st, tm, g.O, g.Opad, g.R, k, x, y, count, col0, cap, ctl);
        else if (bm == 32) CB_LAUNCH((gemm_bf16_kernel<32, 128, 1, 4>), grid, block, st, tm, g.O, g.Opad, g.R, k, x, y, count, col0, cap, ctl);
        else               CB_LAUNCH((gemm_bf16_kernel<64, 64, 2, 2>), grid, block, st, tm, g.O, g.Opad, g.R, k, x, y, count, col0, cap, ctl);
    } else {
        const float* k = (const float*)KT; const float* x = (const float*)X; float* y = (float*)Y;
        if (bm == 16)      CB_LAUNCH((gemm_f32_kernel<16, 256, 1, 4>), grid, block, st, tm, g.O, g.Opad, g.R, k, x, y, count, col0, cap, ctl);
        else if (bm == 32) CB_LAUNCH((gemm_f32_kernel<32, 128, 1, 4>), grid, block, st, tm, g.O, g.Opad, g.R, k, x, y, count, col0, cap, ctl);
        else               CB_LAUNCH((gemm_f32_kernel<64, 64, 2, 2>), grid, block, st, tm, g.O, g.Opad, g.R, k, x, y, count, col0, cap, ctl);
    }
    return hipGetLastError();
}

}  // namespace cb
