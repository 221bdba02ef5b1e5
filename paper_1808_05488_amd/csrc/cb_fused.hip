// Fused back end: matrix generation, matrix multiplication and output update
// (Sec. III-A, last three processing steps) in one kernel.  The columns of X'
// for a tile of listed pixels are gathered from the input state straight into
// LDS, multiplied with the filter matrix on the MFMA units, and the result is
// written with bias + ReLU into the cached output at the listed pixels.  X' and
// Y' never exist in HBM.
//
// Work item = BN listed columns x BM output channels x all of K.  A workgroup is
// four wavefronts arranged WGM x WGN; a wavefront owns a (16*TM) x (16*TN) block
// of 16x16 MFMA tiles.
//   B operand (gathered receptive fields): LDS tile [k][n] holding a stage of up
//     to GU units of KC = 64 rows (all of K when it fits), filled by all 256
//     threads (lane = column, so consecutive lanes read consecutive pixels of the
//     state).  All gather loads of a stage are issued together and stored behind
//     one barrier pair: with a few thousand listed pixels the kernel is bound by
//     latency, not throughput, so barriers and exposed latencies are what count.
//   A operand (filter matrix): pre-packed at layer creation in MFMA fragment
//     order, so a wavefront reads the fragments of 16 k-values of one 16-row tile
//     as one fully coalesced 16-byte-per-lane load straight into registers (it is
//     L2 resident); no LDS traffic for A.  Same rolling prefetch, PF stages deep.
// The grid is persistent; N is read from device memory.  Each XCD (workgroup id
// mod 8) takes a contiguous range of column tiles: the index list is sorted, so
// neighbouring tiles read neighbouring state rows, which then stay in that XCD's L2.
#include "cb_kernels.h"

namespace cb {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef short shortx4 __attribute__((ext_vector_type(4)));

constexpr int KC = 64;   // rows of K per LDS stage

__device__ __forceinline__ float ld_src(const float* p) { return *p; }
__device__ __forceinline__ void st_out(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_out(uint16_t* p, float v)
{
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) { *p = (uint16_t)((u >> 16) | 0x40); return; }
    u += 0x7FFFu + ((u >> 16) & 1u);
    *p = (uint16_t)(u >> 16);
}

// Per listed pixel, one bit per filter tap t = j*kw + i (at most 63 taps; bit 63 is the
// marker of the zero rows that pad K to a multiple of 64): set when the tap falls into the
// zero padding around the image, all set when the lane has no pixel.  Two 32-bit halves.
__device__ __forceinline__ void tap_padding(const Geom& g, bool colv, int y0, int x0, unsigned& lo, unsigned& hi)
{
    unsigned long long pad = ~0ull;
    if (colv) {
        unsigned colpad = 0;
        for (int i = 0; i < g.kw; ++i) colpad |= ((unsigned)(x0 + i) < (unsigned)g.W ? 0u : 1u) << i;
        const unsigned rowfull = (1u << g.kw) - 1u;
        pad = 1ull << 63;
        for (int j = 0; j < g.kh; ++j)
            pad |= (unsigned long long)((unsigned)(y0 + j) < (unsigned)g.H ? colpad : rowfull) << (j * g.kw);
    }
    lo = (unsigned)pad;
    hi = (unsigned)(pad >> 32);
}
// all ones when tap t is padding for this lane, else 0 (ORed into the load offset: the
// buffer hardware returns 0 for an out-of-range offset)
__device__ __forceinline__ unsigned pad_ones(unsigned lo, unsigned hi, int t)
{
    return (unsigned)__builtin_amdgcn_sbfe((int)((t & 32) ? hi : lo), (unsigned)t & 31u, 1u);
}

template <int WGM, int WGN, int TM, int TN>
__device__ __forceinline__ void fused_f32_body(const Geom& g, const float* __restrict__ S,
                                               const int32_t* __restrict__ idx, const int N,
                                               const float4* __restrict__ KF, const int2* __restrict__ rowtab,
                                               const float* __restrict__ bias, int relu,
                                               float* __restrict__ OUT, int GU)
{
    static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
    constexpr int BM = 16 * TM * WGM, BN = 16 * TN * WGN;
    constexpr int BNP = BN + (BN % 32 == 16 ? 0 : 16);
    constexpr int LV = KC * BN / 256;            // gathered elements per thread per 64-row unit
    constexpr int RSTEP = 256 / BN;              // rows covered by one pass of the 256 threads
    constexpr int GUMAX = 64 / LV;               // units per stage held in registers (64 VGPRs)
    constexpr int UNIT = KC * BNP;               // floats of one unit in LDS
    constexpr int PF = TM * TN >= 2 ? 2 : 4;     // units of filter fragments in flight (register budget)
    constexpr int KB = TN >= 4 ? 4 : (TN == 2 ? 8 : 16);   // k-steps whose B fragments are read ahead of their MFMAs
    __shared__ int qs[BN];
    extern __shared__ int2 dyn_lds[];            // row table (Rpad entries), then the B stage (GU units)

    const int Rpad = (g.R + KC - 1) / KC * KC;
    int2* rtab = dyn_lds;
    float* Bs = reinterpret_cast<float*>(dyn_lds + Rpad);
    // raw buffer over the input state: 32-bit byte offsets, out-of-range reads return 0
    const __amdgpu_buffer_rsrc_t srsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(S), 0, (int)((unsigned)g.C * (unsigned)g.P * 4u), 0x00020000);
    // the row table is read once per gathered element: keep it in LDS, so that no gather
    // load depends on an earlier global load
    for (int r = threadIdx.x; r < Rpad; r += 256) rtab[r] = rowtab[r];
    const int nunits = Rpad / KC;                // 64-row units of K
    const int nss = (nunits + GU - 1) / GU;      // stages of GU units
    const int KG = Rpad / 16;                    // 16-row groups of the packed filter matrix
    const int NT = (N + BN - 1) / BN;
    const int MT = (g.O + BM - 1) / BM;
    const int per_xcd = (NT + 7) / 8;
    const long total = (long)per_xcd * 8 * MT;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm = wv / WGN, wn = wv % WGN;
    const int l16 = lane & 15, lq = lane >> 4;
    const int gn = tid % BN, gr = tid / BN;      // this thread's column and first row in a unit

    for (long t = blockIdx.x; t < total; t += gridDim.x) {
        const int xcd = (int)(t & 7);
        const long u = t >> 3;
        const int mt = (int)(u % MT);
        const int nt = xcd * per_xcd + (int)(u / MT);
        if (nt >= NT) continue;
        const int n0 = nt * BN, m0 = mt * BM;

        // this thread's column: top-left corner of the receptive field
        const bool colv = n0 + gn < N;
        const int q = colv ? idx[n0 + gn] : 0;
        const int yo = q / g.Wo, xo = q - yo * g.Wo;
        const int y0 = yo * g.s - g.p, x0 = xo * g.s - g.p;
        __syncthreads();                          // previous tile's epilogue has read qs; rtab is filled
        if (tid < BN) qs[tid] = (n0 + tid < N) ? idx[n0 + tid] : -1;

        // Gather through a buffer resource over the state: the offset of a padding element
        // is forced out of range and the hardware returns 0 for it, so a gathered element
        // costs one LDS read of its row-table entry, three or four integer operations and one load.
        unsigned padlo, padhi;
        tap_padding(g, colv, y0, x0, padlo, padhi);
        const unsigned base4 = (unsigned)(y0 * g.W + x0) * 4u;

        // One stage = up to GU units of 64 rows: all its gather loads are issued together
        // (one memory latency per stage), parked in registers, and stored to LDS behind one
        // barrier pair; the MFMAs of the whole stage then run without further barriers.
        float breg[GUMAX][LV];
        auto gload_stage = [&](int ss) {
            const int u0 = ss * GU;
#pragma unroll
            for (int uu = 0; uu < GUMAX; ++uu) {
                if (uu < GU && u0 + uu < nunits) {
#pragma unroll
                    for (int v = 0; v < LV; ++v) {
                        const int2 rt = rtab[(u0 + uu) * KC + gr + v * RSTEP];   // {byte offset, filter tap}
                        const unsigned off = (base4 + (unsigned)rt.x) | pad_ones(padlo, padhi, rt.y);
                        breg[uu][v] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(srsrc, (int)off, 0, 0));
                    }
                }
            }
        };
        auto lds_store_stage = [&](int ss) {
            const int u0 = ss * GU;
#pragma unroll
            for (int uu = 0; uu < GUMAX; ++uu) {
                if (uu < GU && u0 + uu < nunits) {
#pragma unroll
                    for (int v = 0; v < LV; ++v) Bs[uu * UNIT + (gr + v * RSTEP) * BNP + gn] = breg[uu][v];
                }
            }
        };
        // filter fragments of unit c: 4 groups of 16 rows per 16-row output tile, one fully
        // coalesced 16-byte-per-lane load each; issued unconditionally (clamped unit index) so
        // that the rolling prefetch can be waited for with exact counts
        float4 areg[PF][TM][4];
        auto aload = [&](int c, float4 (&dst)[TM][4]) {
#pragma unroll
            for (int a = 0; a < TM; ++a) {
                const int mtile = (m0 >> 4) + wm * TM + a;
#pragma unroll
                for (int kg = 0; kg < 4; ++kg)
                    dst[a][kg] = KF[((size_t)mtile * KG + c * 4 + kg) * 64 + lane];
            }
        };

        // two accumulator chains (even / odd k-steps) so that consecutive MFMAs are independent
        floatx4 acc[TM][TN], acc1[TM][TN];
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b) { acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f}; acc1[a][b] = acc[a][b]; }

        // one unit = 16 k-steps; the B fragments of KB k-steps are read from LDS ahead of their MFMAs
        auto compute = [&](int uu, const float4 (&af)[TM][4]) {
            const float* Bu = Bs + uu * UNIT;
#pragma unroll
            for (int k0 = 0; k0 < 16; k0 += KB) {
                float bfr[KB][TN];
#pragma unroll
                for (int ks = 0; ks < KB; ++ks)
#pragma unroll
                    for (int b = 0; b < TN; ++b)
                        bfr[ks][b] = Bu[((k0 + ks) * 4 + lq) * BNP + (wn * TN + b) * 16 + l16];
#pragma unroll
                for (int ks = 0; ks < KB; ++ks) {
                    const int kg = (k0 + ks) >> 2, kk = (k0 + ks) & 3;
#pragma unroll
                    for (int a = 0; a < TM; ++a) {
                        const float av = kk == 0 ? af[a][kg].x : kk == 1 ? af[a][kg].y
                                       : kk == 2 ? af[a][kg].z : af[a][kg].w;
#pragma unroll
                        for (int b = 0; b < TN; ++b) {
                            if (kk & 1) acc1[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bfr[ks][b], acc1[a][b], 0, 0, 0);
                            else        acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bfr[ks][b], acc[a][b], 0, 0, 0);
                        }
                    }
                }
            }
        };

        gload_stage(0);
        for (int ss = 0; ss < nss; ++ss) {
            const int u0 = ss * GU;
            const int ucount = nunits - u0 < GU ? nunits - u0 : GU;
            const int ulast = u0 + ucount - 1;
            __syncthreads();                      // the previous stage's fragments have been read
            lds_store_stage(ss);
            __syncthreads();
#pragma unroll
            for (int p = 0; p < PF; ++p) aload(u0 + p < ulast ? u0 + p : ulast, areg[p]);
            if (ss + 1 < nss) gload_stage(ss + 1);   // in flight during this stage's MFMAs
            const int nfull = ucount / PF;
            for (int grp = 0; grp < nfull; ++grp) {
#pragma unroll
                for (int p = 0; p < PF; ++p) {
                    const int uu = grp * PF + p;
                    compute(uu, areg[p]);
                    aload(u0 + uu + PF < ulast ? u0 + uu + PF : ulast, areg[p]);
                }
            }
#pragma unroll
            for (int p = 0; p < PF - 1; ++p)
                if (nfull * PF + p < ucount) compute(nfull * PF + p, areg[p]);
        }

#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b) acc[a][b] += acc1[a][b];

        // output update: bias + ReLU, written at the listed pixels only
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            const int qn = qs[(wn * TN + b) * 16 + l16];
            if (qn < 0) continue;
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = m0 + (wm * TM + a) * 16 + lq * 4 + r;
                    if (m < g.O) {
                        float v = acc[a][b][r] + bias[m];
                        if (relu) v = v > 0.f ? v : 0.f;
                        OUT[(size_t)m * g.Po + qn] = v;
                    }
                }
        }
    }
}

// Columns per workgroup tile are chosen on the device from N: with few listed pixels small
// tiles (16*TNS columns per wavefront column) give every compute unit work and short
// per-tile latency; from FUSED_LARGE_N columns on, wide tiles (16*TNL) re-read the filter
// matrix four times less often, which is what bounds the kernel then.
constexpr int FUSED_LARGE_N = 16384;

template <int WGM, int WGN, int TM, int TNS, int TNL>
__global__ __launch_bounds__(256, 2) void fused_f32_kernel(Geom g, const float* __restrict__ S,
                                                        const int32_t* __restrict__ idx,
                                                        const int* __restrict__ count,
                                                        const float4* __restrict__ KF,
                                                        const int2* __restrict__ rowtab,
                                                        const float* __restrict__ bias, int relu,
                                                        float* __restrict__ OUT, int gu_small, int gu_large)
{
    const int N = *count;
    if (N <= 0) return;
    if (N < FUSED_LARGE_N) fused_f32_body<WGM, WGN, TM, TNS>(g, S, idx, N, KF, rowtab, bias, relu, OUT, gu_small);
    else                   fused_f32_body<WGM, WGN, TM, TNL>(g, S, idx, N, KF, rowtab, bias, relu, OUT, gu_large);
}

// Filter matrix in MFMA fragment order for the float32 kernel:
//   KF[((mtile*KG + kgroup)*64 + lane)].{x,y,z,w}[kk] = K(m = mtile*16 + lane%16, k = kgroup*16 + kk*4 + lane/16)
// zero outside O x R.  Row table: for row r = (c*kh + j)*kw + i of X', the byte offset
// (c*P + j*W + i)*4 into the state and the filter tap j*kw + i; rows beyond R carry tap 63.
__global__ __launch_bounds__(256) void pack_fused_f32_kernel(Geom g, int Mt16, int KG, const float* __restrict__ w,
                                                             float4* __restrict__ KF, int2* __restrict__ rowtab)
{
    const long n = (long)Mt16 * KG * 64;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long)gridDim.x * 256) {
        const int lane = (int)(e & 63);
        const long gk = e >> 6;
        const int kgroup = (int)(gk % KG), mtile = (int)(gk / KG);
        const int m = mtile * 16 + (lane & 15);
        float v[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int k = kgroup * 16 + kk * 4 + (lane >> 4);
            v[kk] = (m < g.O && k < g.R) ? w[(size_t)m * g.R + k] : 0.f;
        }
        KF[e] = make_float4(v[0], v[1], v[2], v[3]);
    }
    const int Rpad = KG * 16;
    for (int r = blockIdx.x * 256 + threadIdx.x; r < Rpad; r += gridDim.x * 256) {
        int2 rt = make_int2(0, 63);                      // padding row: tap 63 never exists
        if (r < g.R) {
            const int kk = g.kh * g.kw;
            const int c = r / kk, ji = r - c * kk, j = ji / g.kw, i = ji - j * g.kw;
            rt = make_int2((int)(((unsigned)c * (unsigned)g.P + (unsigned)(j * g.W + i)) * 4u), ji);
        }
        rowtab[r] = rt;
    }
}


// ---------------------------------------------------------------------------------------------
// bfloat16 variant.  Same structure; differences:
//   * MFMA v_mfma_f32_16x16x32_bf16: a lane supplies 8 consecutive k of one row (A) / one column
//     (B), so the B stage in LDS is [n][k] with k contiguous (row pitch KPB = 72 elements =
//     144 bytes: eight lanes reading 16 bytes each then cover all 32 banks), read with one
//     16-byte LDS load per fragment;
//   * a thread gathers PAIRS of consecutive k for its column (two 2-byte buffer loads) and
//     writes them as one 32-bit LDS store;
//   * the filter matrix is packed as 16 bytes (8 k) per lane per 32-row group;
//   * accumulation stays float32; the cached output is rounded once to bfloat16.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
constexpr int KPB = KC + 8;

template <int WGM, int WGN, int TM, int TN>
__device__ __forceinline__ void fused_bf16_body(const Geom& g, const uint16_t* __restrict__ S,
                                                const int32_t* __restrict__ idx, const int N,
                                                const uint4* __restrict__ KF, const int2* __restrict__ rowtab,
                                                const float* __restrict__ bias, int relu,
                                                uint16_t* __restrict__ OUT, int GU)
{
    static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
    constexpr int BM = 16 * TM * WGM, BN = 16 * TN * WGN;
    constexpr int LVP = KC * BN / 512;           // gathered k-pairs per thread per 64-row unit
    constexpr int RSTEP = 256 / BN;              // pair rows covered by one pass of the 256 threads
    constexpr int GUMAX = 32 / LVP;              // units per stage held in registers (64 VGPRs)
    constexpr int UNIT = BN * KPB;               // bf16 elements of one unit in LDS
    constexpr int PF = TM * TN >= 2 ? 2 : 4;     // units of filter fragments in flight
    __shared__ int qs[BN];
    extern __shared__ int2 dyn_lds[];            // row table (Rpad entries), then the B stage (GU units)

    const int Rpad = (g.R + KC - 1) / KC * KC;
    int2* rtab = dyn_lds;
    uint16_t* Bs = reinterpret_cast<uint16_t*>(dyn_lds + Rpad);
    const __amdgpu_buffer_rsrc_t srsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(S), 0, (int)((unsigned)g.C * (unsigned)g.P * 2u), 0x00020000);
    for (int r = threadIdx.x; r < Rpad; r += 256) rtab[r] = rowtab[r];
    const int nunits = Rpad / KC;
    const int nss = (nunits + GU - 1) / GU;
    const int KG = Rpad / 32;                    // 32-row groups of the packed filter matrix
    const int NT = (N + BN - 1) / BN;
    const int MT = (g.O + BM - 1) / BM;
    const int per_xcd = (NT + 7) / 8;
    const long total = (long)per_xcd * 8 * MT;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm = wv / WGN, wn = wv % WGN;
    const int l16 = lane & 15, lq = lane >> 4;
    const int gn = tid % BN, gr = tid / BN;      // this thread's column and first pair row in a unit

    for (long t = blockIdx.x; t < total; t += gridDim.x) {
        const int xcd = (int)(t & 7);
        const long u = t >> 3;
        const int mt = (int)(u % MT);
        const int nt = xcd * per_xcd + (int)(u / MT);
        if (nt >= NT) continue;
        const int n0 = nt * BN, m0 = mt * BM;

        const bool colv = n0 + gn < N;
        const int q = colv ? idx[n0 + gn] : 0;
        const int yo = q / g.Wo, xo = q - yo * g.Wo;
        const int y0 = yo * g.s - g.p, x0 = xo * g.s - g.p;
        __syncthreads();
        if (tid < BN) qs[tid] = (n0 + tid < N) ? idx[n0 + tid] : -1;

        unsigned padlo, padhi;
        tap_padding(g, colv, y0, x0, padlo, padhi);
        const unsigned base2 = (unsigned)(y0 * g.W + x0) * 2u;

        uint16_t breg[GUMAX][LVP][2];
        auto gload_stage = [&](int ss) {
            const int u0 = ss * GU;
#pragma unroll
            for (int uu = 0; uu < GUMAX; ++uu) {
                if (uu < GU && u0 + uu < nunits) {
#pragma unroll
                    for (int v = 0; v < LVP; ++v) {
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            const int2 rt = rtab[(u0 + uu) * KC + 2 * (gr + v * RSTEP) + h];
                            const unsigned off = (base2 + (unsigned)rt.x) | pad_ones(padlo, padhi, rt.y);
                            breg[uu][v][h] = __builtin_amdgcn_raw_buffer_load_b16(srsrc, (int)off, 0, 0);
                        }
                    }
                }
            }
        };
        auto lds_store_stage = [&](int ss) {
            const int u0 = ss * GU;
#pragma unroll
            for (int uu = 0; uu < GUMAX; ++uu) {
                if (uu < GU && u0 + uu < nunits) {
#pragma unroll
                    for (int v = 0; v < LVP; ++v)
                        *reinterpret_cast<uint32_t*>(&Bs[uu * UNIT + gn * KPB + 2 * (gr + v * RSTEP)]) =
                            (uint32_t)breg[uu][v][0] | ((uint32_t)breg[uu][v][1] << 16);
                }
            }
        };
        uint4 areg[PF][TM][2];
        auto aload = [&](int c, uint4 (&dst)[TM][2]) {
#pragma unroll
            for (int a = 0; a < TM; ++a) {
                const int mtile = (m0 >> 4) + wm * TM + a;
#pragma unroll
                for (int kg = 0; kg < 2; ++kg)
                    dst[a][kg] = KF[((size_t)mtile * KG + c * 2 + kg) * 64 + lane];
            }
        };

        floatx4 acc[TM][TN], acc1[TM][TN];
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b) { acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f}; acc1[a][b] = acc[a][b]; }

        auto compute = [&](int uu, const uint4 (&af)[TM][2]) {
            const uint16_t* Bu = Bs + uu * UNIT;
            uint4 bfr[2][TN];
#pragma unroll
            for (int kg = 0; kg < 2; ++kg)
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    bfr[kg][b] = *reinterpret_cast<const uint4*>(&Bu[((wn * TN + b) * 16 + l16) * KPB + kg * 32 + lq * 8]);
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b) {
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, af[a][0]),
                                                                        __builtin_bit_cast(bf16x8, bfr[0][b]), acc[a][b], 0, 0, 0);
                    acc1[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, af[a][1]),
                                                                         __builtin_bit_cast(bf16x8, bfr[1][b]), acc1[a][b], 0, 0, 0);
                }
        };

        gload_stage(0);
        for (int ss = 0; ss < nss; ++ss) {
            const int u0 = ss * GU;
            const int ucount = nunits - u0 < GU ? nunits - u0 : GU;
            const int ulast = u0 + ucount - 1;
            __syncthreads();
            lds_store_stage(ss);
            __syncthreads();
#pragma unroll
            for (int p = 0; p < PF; ++p) aload(u0 + p < ulast ? u0 + p : ulast, areg[p]);
            if (ss + 1 < nss) gload_stage(ss + 1);
            const int nfull = ucount / PF;
            for (int grp = 0; grp < nfull; ++grp) {
#pragma unroll
                for (int p = 0; p < PF; ++p) {
                    const int uu = grp * PF + p;
                    compute(uu, areg[p]);
                    aload(u0 + uu + PF < ulast ? u0 + uu + PF : ulast, areg[p]);
                }
            }
#pragma unroll
            for (int p = 0; p < PF - 1; ++p)
                if (nfull * PF + p < ucount) compute(nfull * PF + p, areg[p]);
        }

#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b) acc[a][b] += acc1[a][b];

#pragma unroll
        for (int b = 0; b < TN; ++b) {
            const int qn = qs[(wn * TN + b) * 16 + l16];
            if (qn < 0) continue;
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = m0 + (wm * TM + a) * 16 + lq * 4 + r;
                    if (m < g.O) {
                        float v = acc[a][b][r] + bias[m];
                        if (relu) v = v > 0.f ? v : 0.f;
                        st_out(OUT + (size_t)m * g.Po + qn, v);
                    }
                }
        }
    }
}

template <int WGM, int WGN, int TM, int TNS, int TNL>
__global__ __launch_bounds__(256, 2) void fused_bf16_kernel(Geom g, const uint16_t* __restrict__ S,
                                                           const int32_t* __restrict__ idx,
                                                           const int* __restrict__ count,
                                                           const uint4* __restrict__ KF,
                                                           const int2* __restrict__ rowtab,
                                                           const float* __restrict__ bias, int relu,
                                                           uint16_t* __restrict__ OUT, int gu_small, int gu_large)
{
    const int N = *count;
    if (N <= 0) return;
    if (N < FUSED_LARGE_N) fused_bf16_body<WGM, WGN, TM, TNS>(g, S, idx, N, KF, rowtab, bias, relu, OUT, gu_small);
    else                   fused_bf16_body<WGM, WGN, TM, TNL>(g, S, idx, N, KF, rowtab, bias, relu, OUT, gu_large);
}

// Filter matrix in fragment order for v_mfma_f32_16x16x32_bf16:
//   KF[(mtile*KG + kgroup)*64 + lane] = 8 bf16: K(m = mtile*16 + lane%16, k = kgroup*32 + 8*(lane/16) + 0..7)
// and the row table with 2-byte element offsets.
__global__ __launch_bounds__(256) void pack_fused_bf16_kernel(Geom g, int Mt16, int KG, const uint16_t* __restrict__ w,
                                                              uint4* __restrict__ KF, int2* __restrict__ rowtab)
{
    const long n = (long)Mt16 * KG * 64;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long)gridDim.x * 256) {
        const int lane = (int)(e & 63);
        const long gk = e >> 6;
        const int kgroup = (int)(gk % KG), mtile = (int)(gk / KG);
        const int m = mtile * 16 + (lane & 15);
        uint32_t v[4] = {0, 0, 0, 0};
#pragma unroll
        for (int qk = 0; qk < 8; ++qk) {
            const int k = kgroup * 32 + 8 * (lane >> 4) + qk;
            const uint32_t h = (m < g.O && k < g.R) ? w[(size_t)m * g.R + k] : 0u;
            v[qk >> 1] |= h << ((qk & 1) * 16);
        }
        KF[e] = make_uint4(v[0], v[1], v[2], v[3]);
    }
    const int Rpad = KG * 32;
    for (int r = blockIdx.x * 256 + threadIdx.x; r < Rpad; r += gridDim.x * 256) {
        int2 rt = make_int2(0, 63);
        if (r < g.R) {
            const int kk = g.kh * g.kw;
            const int c = r / kk, ji = r - c * kk, j = ji / g.kw, i = ji - j * g.kw;
            rt = make_int2((int)(((unsigned)c * (unsigned)g.P + (unsigned)(j * g.W + i)) * 2u), ji);
        }
        rowtab[r] = rt;
    }
}

}  // namespace

size_t fused_pack_bytes(const Geom& g)
{
    const size_t Rpad = (size_t)(g.R + KC - 1) / KC * KC;
    const size_t Mt16 = (size_t)(g.O + 127) / 128 * 8;     // 16-row tiles, padded to the largest row tile
    // 16 bytes per lane per k-group: 16 rows of float32, 32 rows of bfloat16
    return Mt16 * (Rpad / (g.bf16 ? 32 : 16)) * 64 * 16;
}
size_t fused_rowtab_bytes(const Geom& g) { return (size_t)(g.R + KC - 1) / KC * KC * 8; }
bool fused_supported(const Geom& g)
{
    // 32-bit byte offsets into the state; one padding bit per filter tap in a 64-bit word
    // whose top bit marks the rows that pad K; the row table must fit the dynamic LDS window
    return (long)g.C * g.P < (1L << 30) && g.kh * g.kw <= 63 && fused_rowtab_bytes(g) <= 40 * 1024;
}

hipError_t launch_pack_fused(const Geom& g, const void* w, void* KF, void* rowtab, hipStream_t st)
{
    const int KG = (g.R + KC - 1) / KC * KC / (g.bf16 ? 32 : 16);
    const int Mt16 = (g.O + 127) / 128 * 8;
    long n = (long)Mt16 * KG * 64;
    unsigned grid = (unsigned)((n + 255) / 256);
    if (grid > 2048) grid = 2048;
    if (g.bf16)
        hipLaunchKernelGGL(pack_fused_bf16_kernel, dim3(grid), dim3(256), 0, st, g, Mt16, KG, (const uint16_t*)w,
                           (uint4*)KF, (int2*)rowtab);
    else
        hipLaunchKernelGGL(pack_fused_f32_kernel, dim3(grid), dim3(256), 0, st, g, Mt16, KG, (const float*)w,
                           (float4*)KF, (int2*)rowtab);
    return hipGetLastError();
}

hipError_t launch_fused(const Geom& g, const void* src, const int32_t* idx, const int* count, const void* KF,
                        const void* rowtab, const float* bias, int relu, void* OUT, hipStream_t st, Tm tm)
{
    const dim3 grid(1024), block(256);
    const int2* rt = (const int2*)rowtab;
    // dynamic LDS: the row table, then as many 64-row units of the B stage as fit 64 KB
    // (never more than the registers of the gather hold, never more than K has), for the
    // small-N and the large-N tile shape
    const int nunits = (int)(fused_rowtab_bytes(g) / 8 / KC);
    auto unit_bytes = [&](int bn) {
        return g.bf16 ? (size_t)bn * KPB * 2 : (size_t)KC * (bn + (bn % 32 == 16 ? 0 : 16)) * 4;
    };
    auto stage_units = [&](int bn) {
        int gu = (int)((64 * 1024 - fused_rowtab_bytes(g)) / unit_bytes(bn));
        const int gumax = g.bf16 ? 32 / (KC * bn / 512) : 64 / (KC * bn / 256);
        if (gu > gumax) gu = gumax;
        if (gu > nunits) gu = nunits;
        return gu < 1 ? 1 : gu;
    };
    auto launch = [&](auto kernel, auto* s, auto* kf, auto* out, int bn_small, int bn_large) {
        const int gs = stage_units(bn_small), gl = stage_units(bn_large);
        const size_t a = gs * unit_bytes(bn_small), b = gl * unit_bytes(bn_large);
        const unsigned lds = (unsigned)(fused_rowtab_bytes(g) + (a > b ? a : b));
        hipExtLaunchKernelGGL(kernel, grid, block, lds, st, tm.start, tm.stop, 0, g, s, idx, count, kf, rt, bias, relu,
                              out, gs, gl);
    };
    // tile shapes (rows x columns): small N | large N
    if (g.bf16) {
        const uint16_t* s = (const uint16_t*)src;
        const uint4* kf = (const uint4*)KF;
        uint16_t* out = (uint16_t*)OUT;
#define CB_FUSED(wgm, wgn, tm_, tns, tnl) \
    launch(fused_bf16_kernel<wgm, wgn, tm_, tns, tnl>, s, kf, out, 16 * tns * wgn, 16 * tnl * wgn)
        if (g.O <= 16)      CB_FUSED(1, 4, 1, 1, 2);      // 16 x 64  |  16 x 128
        else if (g.O <= 32) CB_FUSED(2, 2, 1, 1, 2);      // 32 x 32  |  32 x 64
        else if (g.O <= 64) CB_FUSED(4, 1, 1, 1, 4);      // 64 x 16  |  64 x 64
        else                CB_FUSED(4, 1, 2, 1, 4);      // 128 x 16 | 128 x 64
#undef CB_FUSED
    } else {
        const float* s = (const float*)src;
        const float4* kf = (const float4*)KF;
        float* out = (float*)OUT;
#define CB_FUSED(wgm, wgn, tm_, tns, tnl) \
    launch(fused_f32_kernel<wgm, wgn, tm_, tns, tnl>, s, kf, out, 16 * tns * wgn, 16 * tnl * wgn)
        if (g.O <= 16)      CB_FUSED(1, 4, 1, 1, 2);
        else if (g.O <= 32) CB_FUSED(2, 2, 1, 1, 2);
        else if (g.O <= 64) CB_FUSED(4, 1, 1, 1, 4);
        else                CB_FUSED(4, 1, 2, 1, 4);
#undef CB_FUSED
    }
    return hipGetLastError();
}

}  // namespace cb
