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
// stride over the (n-tile, m-tile) space.  Tiles that share X' columns are
// given to workgroups of the same XCD (id mod 8) so that the columns are served
// from that XCD's L2.
#include "cb_kernels.h"

namespace cb {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef short shortx4 __attribute__((ext_vector_type(4)));

constexpr int BK = 16;

template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(256) void gemm_f32_kernel(int O, int Opad, int R, const float* __restrict__ KT,
                                                       const float* __restrict__ X, float* __restrict__ Y,
                                                       const int* __restrict__ count, int col0, int cap)
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

    int ncols = *count - col0;
    if (ncols > cap) ncols = cap;
    if (ncols <= 0) return;
    const int ld = (ncols + 255) & ~255;
    const int NT = (ncols + BN - 1) / BN;             // n-tiles that hold real columns
    const int MT = Opad / BM;
    const int NT8 = (NT + 7) & ~7;
    const long total = (long)NT8 * MT;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm0 = (wv / WGN) * WM, wn0 = (wv % WGN) * WN;
    const int l16 = lane & 15, lq = lane >> 4;

    for (long t = blockIdx.x; t < total; t += gridDim.x) {
        const int xcd = (int)(t & 7);
        const long s = t >> 3;
        const int mt = (int)(s % MT);
        const int nt = (int)(s / MT) * 8 + xcd;
        if (nt >= NT) continue;
        const int m0 = mt * BM, n0 = nt * BN;

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
                if (e < BK * BM && k0 + k < R)
                    ra[v] = *reinterpret_cast<const float4*>(KT + (size_t)(k0 + k) * Opad + m0 + m);
            }
#pragma unroll
            for (int v = 0; v < BV; ++v) {
                const int e = (v * 256 + tid) * 4;
                const int k = e / BN, n = e % BN;
                rb[v] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (e < BK * BN && k0 + k < R)
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

        gload(0);
        for (int k0 = 0; k0 < R; k0 += BK) {
            __syncthreads();                 // previous tile's fragments have been read
            lstore();
            __syncthreads();
            if (k0 + BK < R) gload(k0 + BK); // next tile's global loads overlap the MFMAs
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

        // D fragment: lane holds column l16, rows 4*lq + r
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = m0 + wm0 + a * 16 + lq * 4 + r;
                    const int n = n0 + wn0 + b * 16 + l16;
                    if (m < O) Y[(size_t)m * ld + n] = acc[a][b][r];
                }
    }
}

// bfloat16 operands (bit patterns), float32 accumulation, Y' kept in float32 (the
// single rounding to bfloat16 happens in the output update).  Tiles are transposed on the way into LDS so that the four
// consecutive k of a fragment are one 8-byte read.
template <int BM, int BN, int WGM, int WGN>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(int O, int Opad, int R, const uint16_t* __restrict__ KT,
                                                        const uint16_t* __restrict__ X, float* __restrict__ Y,
                                                        const int* __restrict__ count, int col0, int cap)
{
    static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 16, TN = WN / 16;
    constexpr int KP = BK + 4;                        // LDS row pitch in elements (k contiguous)
    constexpr int AV = (BK * BM / 8 + 255) / 256;     // 16-byte loads per thread
    constexpr int BV = (BK * BN / 8 + 255) / 256;
    __shared__ uint16_t As[BM * KP];
    __shared__ uint16_t Bs[BN * KP];

    int ncols = *count - col0;
    if (ncols > cap) ncols = cap;
    if (ncols <= 0) return;
    const int ld = (ncols + 255) & ~255;
    const int NT = (ncols + BN - 1) / BN;
    const int MT = Opad / BM;
    const int NT8 = (NT + 7) & ~7;
    const long total = (long)NT8 * MT;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm0 = (wv / WGN) * WM, wn0 = (wv % WGN) * WN;
    const int l16 = lane & 15, lq = lane >> 4;

    for (long t = blockIdx.x; t < total; t += gridDim.x) {
        const int xcd = (int)(t & 7);
        const long s = t >> 3;
        const int mt = (int)(s % MT);
        const int nt = (int)(s / MT) * 8 + xcd;
        if (nt >= NT) continue;
        const int m0 = mt * BM, n0 = nt * BN;

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
                if (e < BK * BM && k0 + k < R)
                    ra[v] = *reinterpret_cast<const uint4*>(KT + (size_t)(k0 + k) * Opad + m0 + m);
            }
#pragma unroll
            for (int v = 0; v < BV; ++v) {
                const int e = (v * 256 + tid) * 8;
                const int k = e / BN, n = e % BN;
                rb[v] = make_uint4(0, 0, 0, 0);
                if (e < BK * BN && k0 + k < R)
                    rb[v] = *reinterpret_cast<const uint4*>(X + (size_t)(k0 + k) * ld + n0 + n);
            }
        };
        auto lstore = [&]() {
#pragma unroll
            for (int v = 0; v < AV; ++v) {
                const int e = (v * 256 + tid) * 8;
                if (e < BK * BM) {
                    const int k = e / BM, m = e % BM;
                    const uint32_t w[4] = {ra[v].x, ra[v].y, ra[v].z, ra[v].w};
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        As[(m + q) * KP + k] = (uint16_t)(w[q >> 1] >> ((q & 1) * 16));
                }
            }
#pragma unroll
            for (int v = 0; v < BV; ++v) {
                const int e = (v * 256 + tid) * 8;
                if (e < BK * BN) {
                    const int k = e / BN, n = e % BN;
                    const uint32_t w[4] = {rb[v].x, rb[v].y, rb[v].z, rb[v].w};
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        Bs[(n + q) * KP + k] = (uint16_t)(w[q >> 1] >> ((q & 1) * 16));
                }
            }
        };

        gload(0);
        for (int k0 = 0; k0 < R; k0 += BK) {
            __syncthreads();
            lstore();
            __syncthreads();
            if (k0 + BK < R) gload(k0 + BK);
            shortx4 af[TM], bf[TN];
#pragma unroll
            for (int a = 0; a < TM; ++a)
                af[a] = *reinterpret_cast<const shortx4*>(&As[(wm0 + a * 16 + l16) * KP + lq * 4]);
#pragma unroll
            for (int b = 0; b < TN; ++b)
                bf[b] = *reinterpret_cast<const shortx4*>(&Bs[(wn0 + b * 16 + l16) * KP + lq * 4]);
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(af[a], bf[b], acc[a][b], 0, 0, 0);
        }

#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = m0 + wm0 + a * 16 + lq * 4 + r;
                    const int n = n0 + wn0 + b * 16 + l16;
                    if (m < O) Y[(size_t)m * ld + n] = acc[a][b][r];
                }
    }
}

}  // namespace

// Row-tile height used for a layer with O output channels; the transposed filter
// matrix is padded to a multiple of it.
int gemm_bm(int O) { return O <= 16 ? 16 : (O <= 32 ? 32 : 64); }

hipError_t launch_gemm(const Geom& g, const void* KT, const void* X, void* Y, const int* count,
                       int col0, int cap, hipStream_t st)
{
    const int bm = gemm_bm(g.O);
    const unsigned grid = 1024;     // multiple of 8 (XCD mapping), a few workgroups per CU
    if (g.bf16) {
        const uint16_t* k = (const uint16_t*)KT; const uint16_t* x = (const uint16_t*)X; float* y = (float*)Y;
        if (bm == 16)      hipLaunchKernelGGL((gemm_bf16_kernel<16, 256, 1, 4>), dim3(grid), dim3(256), 0, st, g.O, g.Opad, g.R, k, x, y, count, col0, cap);
        else if (bm == 32) hipLaunchKernelGGL((gemm_bf16_kernel<32, 128, 1, 4>), dim3(grid), dim3(256), 0, st, g.O, g.Opad, g.R, k, x, y, count, col0, cap);
        else               hipLaunchKernelGGL((gemm_bf16_kernel<64, 64, 2, 2>), dim3(grid), dim3(256), 0, st, g.O, g.Opad, g.R, k, x, y, count, col0, cap);
    } else {
        const float* k = (const float*)KT; const float* x = (const float*)X; float* y = (float*)Y;
        if (bm == 16)      hipLaunchKernelGGL((gemm_f32_kernel<16, 256, 1, 4>), dim3(grid), dim3(256), 0, st, g.O, g.Opad, g.R, k, x, y, count, col0, cap);
        else if (bm == 32) hipLaunchKernelGGL((gemm_f32_kernel<32, 128, 1, 4>), dim3(grid), dim3(256), 0, st, g.O, g.Opad, g.R, k, x, y, count, col0, cap);
        else               hipLaunchKernelGGL((gemm_f32_kernel<64, 64, 2, 2>), dim3(grid), dim3(256), 0, st, g.O, g.Opad, g.R, k, x, y, count, col0, cap);
    }
    return hipGetLastError();
}

}  // namespace cb
