// Fused back end, float32 and bfloat16, gathering from the channel-last shadow of the input
// state (Sec. III-A, last three processing steps in one kernel, like
// cb_fused_f32.hip).  The shadow holds the C values of a pixel side by side, so a
// filter tap of a listed pixel is C contiguous elements: sixteen lanes fetch 256
// contiguous bytes with one 16-byte load each -- fully coalesced, no chunk table,
// and one 16-byte LDS store per load.  (Written for float32; the bfloat16 form is
// the same kernel in bytes: a 256-byte unit of a column is 128 rows of K instead of
// 64, a 16-byte piece eight elements instead of four, and a lane's 16-byte B
// fragment feeds ONE v_mfma_f32_16x16x32_bf16 instead of four v_mfma_f32_16x16x4_f32.)
//
// K is walked tap-major: row k' = (j*kw + i)*C + c.  The order of the contraction is free as
// long as both operands agree; the filter matrix is packed in this order at layer creation
// (pack_fused_*_cl_kernel).  Requires C to be a power of two >= 16.
//
//   B operand: LDS tile [n][k'] (k' contiguous, row pitch LDK floats with LDK = 4 mod 32, so that
//     the 16-byte fragment reads of sixteen columns fall into different banks).  A lane reads
//     the four consecutive k' of its quarter of a 16-row k-group with ONE 16-byte LDS read and
//     uses them in four successive MFMAs: MFMA step kk of k-group kg contracts the rows
//     16*kg + 4*q + kk, q = 0..3 (q = lane / 16).
//   A operand, tile shapes, persistent grid, XCD-contiguous tile ranges, rolling prefetch of
//     the filter fragments, epilogue: as in cb_fused_f32.hip.
#include "cb_fused.h"

namespace cb {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <typename T, int WGM, int WGN, int TM, int TN>
__device__ __forceinline__ void fused_cl_body(const Geom& g, const T* __restrict__ S2,
                                                  const int32_t* __restrict__ idx, const int N,
                                                  const float4* __restrict__ KF, const float* __restrict__ bias,
                                                  int relu, T* __restrict__ OUT, T* __restrict__ OUT2, const int GUin)
{
    constexpr bool BF = sizeof(T) == 2;
    constexpr int UK = BF ? 128 : KC;            // rows of K in a 256-byte unit of a column
    constexpr int EPV = BF ? 8 : 4;              // elements per 16-byte piece
    constexpr unsigned ESZ = (unsigned)sizeof(T);
    static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
    constexpr int BM = 16 * TM * WGM, BN = 16 * TN * WGN;
    constexpr int NP = BN / 16;                  // columns per thread: column (tid / 16) + 16 * p
    constexpr int GUMAX = FUSED_CL_LOADS / NP;   // units per stage at most (register budget of the gather)
    constexpr int LDK = fused_cl_pitch(BN);      // floats per column of the B stage
    static_assert(GUMAX >= 1 && GUMAX * KC <= LDK, "a stage fits its LDS column");
    const int GU = GUin < 1 ? 1 : (GUin < GUMAX ? GUin : GUMAX);
    constexpr bool TWO = TM * TN < 4;            // second accumulator chain where a wavefront has few tiles
    constexpr int PF = TM * TN >= 2 ? 2 : 4;     // units of filter fragments in flight (register budget)
    __shared__ int qs[BN];
    extern __shared__ float4 dyn_lds4[];
    float* const Bs = reinterpret_cast<float*>(dyn_lds4);

    const int nunits = (g.R + UK - 1) / UK;      // 256-byte units of K
    const int lc = 31 - __builtin_clz((unsigned)g.C);          // C = 1 << lc
    const unsigned inv_kw = (65536u + (unsigned)g.kw - 1u) / (unsigned)g.kw;   // tap / kw = tap * inv_kw >> 16 for tap < 64
    // raw buffer over the shadow: 32-bit byte offsets; an offset beyond the end reads as 0
    const __amdgpu_buffer_rsrc_t srsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<T*>(S2), 0, (int)((unsigned)g.C * (unsigned)g.P * ESZ), 0x00020000);
    constexpr unsigned NOWHERE = 0xFFFFFFF0u;
    const int KG = nunits * 4;                   // 16-row groups of the packed filter matrix
    const __amdgpu_buffer_rsrc_t krsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float4*>(KF), 0, (int)((unsigned)((g.O + 127) / 128 * 8) * (unsigned)KG * 1024u), 0x00020000);
    const int NT = (N + BN - 1) / BN;
    const int MT = (g.O + BM - 1) / BM;
    const int per_xcd = (NT + 7) / 8;
    const long total = (long)per_xcd * 8 * MT;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm = wv / WGN, wn = wv % WGN;
    const int wm_s = __builtin_amdgcn_readfirstlane(wm);
    const int l16 = lane & 15, lq = lane >> 4;
    const int gc = tid >> 4, ch = tid & 15;      // first column of this thread, its 16-byte piece of a 64-row unit
    // a unit holds 64 / C taps when C < 64: this thread's piece lies in tap dt of the unit, channels cl .. cl + 3
    const int dt = (EPV * ch) >> lc, cl = (EPV * ch) & (g.C - 1);

    // the listed pixels of this thread's columns are requested one tile ahead
    int qnext[NP];
    auto fetch_q = [&](long tt, int (&q)[NP]) {
        const int ntt = (int)(tt & 7) * per_xcd + (int)((tt >> 3) / MT);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int n = ntt * BN + gc + 16 * p;
            q[p] = (tt < total && ntt < NT && n < N) ? idx[n] : -1;
        }
    };
    fetch_q(blockIdx.x, qnext);

    for (long t = blockIdx.x; t < total; t += gridDim.x) {
        const int xcd = (int)(t & 7);
        const long u = t >> 3;
        const int mt = (int)(u % MT);
        const int nt = xcd * per_xcd + (int)(u / MT);
        int q[NP];
#pragma unroll
        for (int p = 0; p < NP; ++p) q[p] = qnext[p];
        fetch_q(t + gridDim.x, qnext);
        if (nt >= NT) continue;
        const int m0 = mt * BM;
        const int uend = nunits;

        float4 areg[PF][TM][4];
        auto aload = [&](int c, float4 (&dst)[TM][4]) {
#pragma unroll
            for (int a = 0; a < TM; ++a) {
                const unsigned soff = (unsigned)(((m0 >> 4) + wm_s * TM + a) * KG + c * 4) * 1024u;
#pragma unroll
                for (int kg = 0; kg < 4; ++kg)
                    dst[a][kg] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(krsrc, lane * 16 + kg * 1024, (int)soff, 0));
            }
        };
        const bool ring = GU % PF == 0;
#pragma unroll
        for (int p = 0; p < PF; ++p) aload(p < uend - 1 ? p : uend - 1, areg[p]);

        // per column: which taps lie inside the image, and the byte offset of the top-left tap's
        // channel cl in the shadow (it may wrap below zero for pixels at the border: only taps
        // inside the image are fetched, and for those the sum is a valid offset again)
        unsigned long long ok[NP];
        unsigned base[NP];
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const bool colv = q[p] >= 0;
            const int qq = colv ? q[p] : 0;
            const int yo = qq / g.Wo, xo = qq - yo * g.Wo;
            const int y0 = yo * g.s - g.p, x0 = xo * g.s - g.p;
            ok[p] = taps_inside(g, colv, y0, x0);
            base[p] = (((unsigned)(y0 * g.W + x0) << lc) + (unsigned)cl) * ESZ;
        }
        __syncthreads();                          // the previous tile's epilogue has read qs
        if (ch == 0) {
#pragma unroll
            for (int p = 0; p < NP; ++p) qs[gc + 16 * p] = q[p];
        }

        // One stage = up to GU units: all its loads are issued together, parked in registers
        // and stored to LDS behind one barrier pair.  Unit u0 + r of column p: rows
        // (u0 + r)*64 + 4*ch .. + 3 of K, i.e. tap ((u0 + r)*64 >> lc) + dt, channels
        // ((u0 + r)*64 mod C) + cl .. + 3.  Taps outside the image, taps beyond the filter (the
        // rows that pad K to a multiple of 64) and columns without a pixel read as 0.
        float4 breg[GUMAX][NP];
        auto gload_stage = [&](int u0) {
            const int ucount = uend - u0 < GU ? uend - u0 : GU;
#pragma unroll
            for (int r = 0; r < GUMAX; ++r) {
                if (r < ucount) {
                    const unsigned kb = (unsigned)(u0 + r) * (unsigned)UK;
                    const unsigned tap = (kb >> lc) + (unsigned)dt;
                    const unsigned j = (tap * inv_kw) >> 16, i = tap - j * (unsigned)g.kw;
                    const unsigned toff = (((j * (unsigned)g.W + i) << lc) + (kb & (unsigned)(g.C - 1))) * ESZ;
#pragma unroll
                    for (int p = 0; p < NP; ++p) {
                        const bool in = ((ok[p] >> tap) & 1ull) != 0ull;     // tap < 64 always
                        breg[r][p] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(
                            srsrc, (int)(in ? base[p] + toff : NOWHERE), 0, 0));
                    }
                }
            }
        };
        auto lds_store_stage = [&](int u0) {
            const int ucount = uend - u0 < GU ? uend - u0 : GU;
            float* Bst = Bs + gc * LDK + 4 * ch;
#pragma unroll
            for (int r = 0; r < GUMAX; ++r) {
                if (r < ucount) {
#pragma unroll
                    for (int p = 0; p < NP; ++p)
                        *reinterpret_cast<float4*>(Bst + 16 * p * LDK + r * KC) = breg[r][p];
                }
            }
        };

        floatx4 acc[TM][TN], acc1[TWO ? TM : 1][TWO ? TN : 1];
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b) {
                acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};
                if (TWO) acc1[a][b] = acc[a][b];
            }

        // One unit = four k-groups of four MFMA steps.  The B fragments of the next k-group are
        // requested from LDS before the MFMAs of the current one are issued; the first k-group of
        // a unit is requested during the last k-group of the unit before it (same stage).
        // (wide tiles have no registers left for the carried fragments, and 128 MFMAs per k-group to hide
        // one exposed LDS read per unit behind)
        constexpr bool CARRY = TN < 4;
        float4 bcarry[CARRY ? TN : 1];
        auto compute = [&](int uu, const float4 (&af)[TM][4], bool first, bool more) {
            const float* Bu = Bs + (wn * TN * 16 + l16) * LDK + uu * KC + lq * 4;
            float4 bfr[2][TN];
            auto bload = [&](const float* base_, int kg, float4 (&dst)[TN]) {
#pragma unroll
                for (int b = 0; b < TN; ++b) dst[b] = *reinterpret_cast<const float4*>(base_ + b * 16 * LDK + kg * 16);
            };
            if (first || !CARRY) bload(Bu, 0, bfr[0]);
            else {
#pragma unroll
                for (int b = 0; b < TN; ++b) bfr[0][b] = bcarry[CARRY ? b : 0];
            }
#pragma unroll
            for (int kg = 0; kg < 4; ++kg) {
                if (kg + 1 < 4) bload(Bu, kg + 1, bfr[(kg + 1) & 1]);
                else if (CARRY && more) {
#pragma unroll
                    for (int b = 0; b < TN; ++b)
                        bcarry[CARRY ? b : 0] = *reinterpret_cast<const float4*>(Bu + KC + b * 16 * LDK);
                }
                if (TN >= 4) __builtin_amdgcn_sched_barrier(0);
                if constexpr (BF) {
#pragma unroll
                    for (int a = 0; a < TM; ++a)
#pragma unroll
                        for (int b = 0; b < TN; ++b) {
                            const bf16x8 av = __builtin_bit_cast(bf16x8, af[a][kg]), bv = __builtin_bit_cast(bf16x8, bfr[kg & 1][b]);
                            if (TWO && (kg & 1))
                                acc1[TWO ? a : 0][TWO ? b : 0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                    av, bv, acc1[TWO ? a : 0][TWO ? b : 0], 0, 0, 0);
                            else
                                acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bv, acc[a][b], 0, 0, 0);
                        }
                } else {
#pragma unroll
                    for (int k4 = 0; k4 < 4; ++k4) {
#pragma unroll
                        for (int a = 0; a < TM; ++a) {
                            const float av = k4 == 0 ? af[a][kg].x : k4 == 1 ? af[a][kg].y : k4 == 2 ? af[a][kg].z : af[a][kg].w;
#pragma unroll
                            for (int b = 0; b < TN; ++b) {
                                const float4& bq = bfr[kg & 1][b];
                                const float bv = k4 == 0 ? bq.x : k4 == 1 ? bq.y : k4 == 2 ? bq.z : bq.w;
                                if (TWO && (k4 & 1))
                                    acc1[TWO ? a : 0][TWO ? b : 0] = __builtin_amdgcn_mfma_f32_16x16x4f32(
                                        av, bv, acc1[TWO ? a : 0][TWO ? b : 0], 0, 0, 0);
                                else
                                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc[a][b], 0, 0, 0);
                            }
                        }
                    }
                }
                if (TN >= 4) __builtin_amdgcn_sched_barrier(0);
            }
        };

        gload_stage(0);
        for (int u0 = 0; u0 < uend; u0 += GU) {
            const int ucount = uend - u0 < GU ? uend - u0 : GU;
            const int ulast = u0 + ucount - 1;
            __syncthreads();                      // the previous stage's fragments have been read (first stage: qs is written)
            lds_store_stage(u0);
            __syncthreads();
            if (!ring && u0 != 0) {
#pragma unroll
                for (int p = 0; p < PF; ++p) aload(u0 + p < ulast ? u0 + p : ulast, areg[p]);
            }
            if (u0 + GU < uend) gload_stage(u0 + GU);   // in flight during this stage's MFMAs
            const int alast = ring ? uend - 1 : ulast;
            const int nfull = ucount / PF;
            for (int grp = 0; grp < nfull; ++grp) {
#pragma unroll
                for (int p = 0; p < PF; ++p) {
                    const int uu = grp * PF + p;
                    compute(uu, areg[p], uu == 0, uu + 1 < ucount);
                    aload(u0 + uu + PF < alast ? u0 + uu + PF : alast, areg[p]);
                }
            }
#pragma unroll
            for (int p = 0; p < PF - 1; ++p)
                if (nfull * PF + p < ucount) compute(nfull * PF + p, areg[p], nfull * PF + p == 0, nfull * PF + p + 1 < ucount);
        }

        if (TWO) {
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b) acc[a][b] += acc1[TWO ? a : 0][TWO ? b : 0];
        }
        // output update: bias + ReLU, written at the listed pixels only
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            const int qn = qs[(wn * TN + b) * 16 + l16];
            if (qn < 0) continue;
#pragma unroll
            for (int a = 0; a < TM; ++a) {
                const int mb = m0 + (wm * TM + a) * 16 + lq * 4;
                float v4[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = mb + r;
                    v4[r] = 0.f;
                    if (m < g.O) {
                        float v = acc[a][b][r] + bias[m];
                        if (relu) v = v > 0.f ? v : 0.f;
                        st_out(OUT + (size_t)m * g.Po + qn, v);
                        v4[r] = v;
                    }
                }
                // (a layer that keeps the pixel-major copy has a multiple of 16 output channels)
                if (OUT2 && mb < g.O) st_out4(OUT2 + (size_t)qn * g.O + mb, v4);
            }
        }
    }
}

// Wide tiles with a double-buffered B stage (layers with more than 64 output channels, from 16 384
// listed pixels on).  The workgroup tile is 128 x 128 (128 x 64 while the wider tiles would number
// fewer than the 512 workgroups that run at a time); a wavefront owns 32 rows x all columns, so every
// filter fragment is loaded by exactly one wavefront of the workgroup.  A stage is ONE 256-byte unit of
// every column, and two stage buffers alternate: the gathered unit u+1 is stored into the free buffer
// at the start of unit u and the loads of unit u+2 are issued right behind it, so that the only thing
// between the MFMAs of two units is one barrier.  The filter fragments run in a ring of four
// k-groups (one unit), each refilled for the next unit as soon as its MFMAs are issued.  No
// conditional loads in the unit loop: units beyond the end of K are gathered from nowhere (zeros) and
// never multiplied.  Per tile, everything with a memory round trip in it is requested at the start:
// the listed pixels (a tile ahead), the bias, and no integer division per column.
constexpr int FUSED_DB_PITCH = 272;               // bytes per column of a stage buffer: 256 + 16, i.e. 4 mod 32 banks
__host__ __device__ constexpr unsigned fused_db_lds(int bn) { return 2u * (unsigned)bn * FUSED_DB_PITCH; }

template <typename T, int WGM, int WGN, int TM, int TN>
__device__ __forceinline__ void fused_cl_db_body(const Geom& g, const T* __restrict__ S2,
                                                 const int32_t* __restrict__ idx, const int N,
                                                 const float4* __restrict__ KF, const float* __restrict__ bias,
                                                 int relu, T* __restrict__ OUT, T* __restrict__ OUT2)
{
    constexpr bool BF = sizeof(T) == 2;
    constexpr int UK = BF ? 128 : KC;            // rows of K in a 256-byte unit of a column
    constexpr int EPV = BF ? 8 : 4;              // elements per 16-byte piece
    constexpr unsigned ESZ = (unsigned)sizeof(T);
    static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
    constexpr int BM = 16 * TM * WGM, BN = 16 * TN * WGN;
    constexpr int NP = BN / 16;                  // columns per thread: column (tid / 16) + 16 * p
    constexpr int BUF = BN * FUSED_DB_PITCH;     // bytes of one stage buffer
    __shared__ int qs[BN];
    extern __shared__ float4 dyn_lds4[];
    char* const Bs = reinterpret_cast<char*>(dyn_lds4);

    const int nunits = (g.R + UK - 1) / UK;
    const int lc = 31 - __builtin_clz((unsigned)g.C);
    // q / Wo for 0 <= q < 2^30 without a division: floor(q * ceil(2^42 / Wo) / 2^42) is exact while
    // q * Wo < 2^42, and Wo < 2^12 here (the launcher checks)
    const unsigned long long inv_wo = ((1ull << 42) + (unsigned)g.Wo - 1ull) / (unsigned)g.Wo;
    const unsigned inv_kw = (65536u + (unsigned)g.kw - 1u) / (unsigned)g.kw;
    const __amdgpu_buffer_rsrc_t srsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<T*>(S2), 0, (int)((unsigned)g.C * (unsigned)g.P * ESZ), 0x00020000);
    constexpr unsigned NOWHERE = 0xFFFFFFF0u;
    const int KG = nunits * 4;
    const __amdgpu_buffer_rsrc_t krsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float4*>(KF), 0, (int)((unsigned)((g.O + 127) / 128 * 8) * (unsigned)KG * 1024u), 0x00020000);
    const int NT = (N + BN - 1) / BN;
    const int MT = (g.O + BM - 1) / BM;
    const int per_xcd = (NT + 7) / 8;
    const long total = (long)per_xcd * 8 * MT;

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int wm = wv / WGN, wn = wv % WGN;
    const int wm_s = __builtin_amdgcn_readfirstlane(wm);
    const int l16 = lane & 15, lq = lane >> 4;
    const int gc = tid >> 4, ch = tid & 15;
    const int dt = (EPV * ch) >> lc, cl = (EPV * ch) & (g.C - 1);

    int qnext[NP];
    auto fetch_q = [&](long tt, int (&q)[NP]) {
        const int ntt = (int)(tt & 7) * per_xcd + (int)((tt >> 3) / MT);
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const int n = ntt * BN + gc + 16 * p;
            q[p] = (tt < total && ntt < NT && n < N) ? idx[n] : -1;
        }
    };
    fetch_q(blockIdx.x, qnext);

    for (long t = blockIdx.x; t < total; t += gridDim.x) {
        const int xcd = (int)(t & 7);
        const long uq = t >> 3;
        const int mt = (int)(uq % MT);
        const int nt = xcd * per_xcd + (int)(uq / MT);
        int q[NP];
#pragma unroll
        for (int p = 0; p < NP; ++p) q[p] = qnext[p];
        fetch_q(t + gridDim.x, qnext);
        if (nt >= NT) continue;
        const int m0 = mt * BM;

        // ring of filter fragments: k-group kg of the unit being multiplied, TM row tiles
        float4 areg[4][TM];
        auto aload = [&](int u, int kg) {
            const int uc = u < nunits ? u : nunits - 1;
#pragma unroll
            for (int a = 0; a < TM; ++a) {
                const unsigned soff = (unsigned)(((m0 >> 4) + wm_s * TM + a) * KG + uc * 4 + kg) * 1024u;
                areg[kg][a] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(krsrc, lane * 16, (int)soff, 0));
            }
        };

        // per column: which filter rows (bits 0..15) and filter columns (bits 16..31) lie inside the
        // image (all clear for a column without a pixel), and the byte offset of the top-left tap's
        // channel cl in the shadow (may wrap below zero at the border: only taps inside are fetched)
        unsigned ok[NP];
        unsigned base[NP];
#pragma unroll
        for (int p = 0; p < NP; ++p) {
            const bool colv = q[p] >= 0;
            const int qq = colv ? q[p] : 0;
            const int yo = (int)(((unsigned long long)(unsigned)qq * inv_wo) >> 42), xo = qq - yo * g.Wo;
            const int y0 = yo * g.s - g.p, x0 = xo * g.s - g.p;
            unsigned m = 0;
            if (colv) {
                for (int j = 0; j < g.kh; ++j) m |= ((unsigned)(y0 + j) < (unsigned)g.H ? 1u : 0u) << j;
                for (int i = 0; i < g.kw; ++i) m |= ((unsigned)(x0 + i) < (unsigned)g.W ? 0x10000u : 0u) << i;
            }
            ok[p] = m;
            base[p] = (((unsigned)(y0 * g.W + x0) << lc) + (unsigned)cl) * ESZ;
        }

        float4 breg[NP];
        auto gload = [&](int u) {
            const unsigned kb = (unsigned)u * (unsigned)UK;
            const unsigned tap = (kb >> lc) + (unsigned)dt;
            const unsigned j = (tap * inv_kw) >> 16, i = tap - j * (unsigned)g.kw;
            const unsigned toff = (((j * (unsigned)g.W + i) << lc) + (kb & (unsigned)(g.C - 1))) * ESZ;
            // (rows that pad K to a whole unit have j >= kh: their bit is clear)
            const unsigned need = u < nunits && j < 16u ? (1u << j) | (0x10000u << i) : 0xFFFFFFFFu;
#pragma unroll
            for (int p = 0; p < NP; ++p) {
                const bool in = (ok[p] & need) == need;
                breg[p] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(
                    srsrc, (int)(in ? base[p] + toff : NOWHERE), 0, 0));
            }
        };
        auto lds_store = [&](int buf) {
            char* dst = Bs + buf * BUF + gc * FUSED_DB_PITCH + 16 * ch;
#pragma unroll
            for (int p = 0; p < NP; ++p) *reinterpret_cast<float4*>(dst + 16 * p * FUSED_DB_PITCH) = breg[p];
        };

        floatx4 acc[TM][TN];
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b) acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};

        // (the loads in flight at the loop's entry are the ones in flight at its back edge, in the same
        // order -- eight gathered pieces, then the filter fragments: where the two differ the compiler
        // waits for the longer of the two queues)
        gload(0);
        // bias of this wavefront's rows: requested now, used in the epilogue
        float bv[TM][4];
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = m0 + (wm * TM + a) * 16 + lq * 4 + r;
                bv[a][r] = bias[m < g.O ? m : g.O - 1];
            }
        __syncthreads();                          // the previous tile has read its last stage and its qs
        if (ch == 0) {
#pragma unroll
            for (int p = 0; p < NP; ++p) qs[gc + 16 * p] = q[p];
        }
        lds_store(0);
        gload(1);
#pragma unroll
        for (int kg = 0; kg < 4; ++kg) aload(0, kg);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();

        const char* const Bw = Bs + (wn * TN * 16 + l16) * FUSED_DB_PITCH + lq * 16;
        for (int u = 0; u < nunits; ++u) {
            const int cur = u & 1;
            // unit u+1 goes into the buffer that unit u-1 was read from; unit u+2 is requested
            lds_store(cur ^ 1);
            gload(u + 2);
            // (left to itself the compiler sinks these loads to the end of the unit, to re-use their
            // registers in between, and the next unit then starts by waiting for them)
            __builtin_amdgcn_sched_barrier(0);
            const char* const Bu = Bw + cur * BUF;
            // One set of B fragments: the MFMAs run column tile by column tile, and a column tile's
            // fragment of the next k-group is requested as soon as its TM MFMAs have been issued (the
            // other column tiles' MFMAs cover the LDS latency).
            float4 bfr[TN];
#pragma unroll
            for (int b = 0; b < TN; ++b) bfr[b] = *reinterpret_cast<const float4*>(Bu + b * 16 * FUSED_DB_PITCH);
#pragma unroll
            for (int kg = 0; kg < 4; ++kg) {
#pragma unroll
                for (int b = 0; b < TN; ++b) {
                    if constexpr (BF) {
                        const bf16x8 bv = __builtin_bit_cast(bf16x8, bfr[b]);
#pragma unroll
                        for (int a = 0; a < TM; ++a)
                            acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, areg[kg][a]), bv,
                                                                                acc[a][b], 0, 0, 0);
                    } else {
                        const float4 bq = bfr[b];
#pragma unroll
                        for (int k4 = 0; k4 < 4; ++k4) {
                            const float bv = k4 == 0 ? bq.x : k4 == 1 ? bq.y : k4 == 2 ? bq.z : bq.w;
#pragma unroll
                            for (int a = 0; a < TM; ++a) {
                                const float4& aq = areg[kg][a];
                                const float av = k4 == 0 ? aq.x : k4 == 1 ? aq.y : k4 == 2 ? aq.z : aq.w;
                                acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc[a][b], 0, 0, 0);
                            }
                        }
                    }
                    if (kg + 1 < 4)
                        bfr[b] = *reinterpret_cast<const float4*>(Bu + b * 16 * FUSED_DB_PITCH + (kg + 1) * 64);
                }
                aload(u + 1, kg);                 // the same k-group of the next unit
                __builtin_amdgcn_sched_barrier(0);
            }
            __syncthreads();
        }

        // output update: bias + ReLU, written at the listed pixels only
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            const int qn = qs[(wn * TN + b) * 16 + l16];
            if (qn < 0) continue;
#pragma unroll
            for (int a = 0; a < TM; ++a) {
                const int mb = m0 + (wm * TM + a) * 16 + lq * 4;
                float v4[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = mb + r;
                    float v = acc[a][b][r] + bv[a][r];
                    if (relu) v = v > 0.f ? v : 0.f;
                    if (m < g.O) st_out(OUT + (size_t)m * g.Po + qn, v);
                    v4[r] = v;
                }
                // (a layer that keeps the pixel-major copy has a multiple of 16 output channels)
                if (OUT2 && mb < g.O) st_out4(OUT2 + (size_t)qn * g.O + mb, v4);
            }
        }
    }
}

// tile shapes chosen from N on the device, as in the channel-first kernel
template <typename T, int WGM, int WGN, int TM, int TNS, int TNL, int TMH, int TNM, bool DB>
__global__ __launch_bounds__(256, 2) void fused_cl_kernel(Geom g, const T* __restrict__ S2,
                                                           const int32_t* __restrict__ idx,
                                                           const int* __restrict__ count,
                                                           const float4* __restrict__ KF,
                                                           const float* __restrict__ bias, int relu,
                                                           T* __restrict__ OUT, T* __restrict__ OUT2, int gu_small, int gu_large, int gu_mid)
{
    const int N = *count;
    if (N <= 0) return;
    // The 32-column tile halves what the MFMAs read of the filter matrix and costs about 1.75 narrow
    // tiles (bfloat16, where that traffic weighs more: about 1.25; 512 -> 512 at 3 645 listed pixels
    // 57.7 -> 36.6 us, 64 -> 64 at 13 480: 12.8 -> 9.4 us).  512 workgroups run at a time, and the kernel takes as many rounds as the busiest slot
    // has tiles: the wider tile is used where rounds x cost comes out lower (7 706 listed pixels,
    // 256 -> 256, K = 2304: 98 -> 93 us; 8 828 pixels, 64 -> 256, K = 3136, where 552 wide tiles are
    // two rounds: 160 us narrow, 173 us wide).
    const long tiles_m = (g.O + 16 * TM * WGM - 1) / (16 * TM * WGM);
    const long tiles_narrow = (long)((N + 16 * TNS * WGN - 1) / (16 * TNS * WGN)) * tiles_m;
    const long tiles_mid = TNM > 0 ? (long)((N + 16 * TNM * WGN - 1) / (16 * TNM * WGN)) * tiles_m : 0;
    if (TNM > 0 && gu_mid > 0 && N < FUSED_LARGE_N && tiles_narrow > FUSED_MID_TILES &&
        ((tiles_mid + 511) / 512) * (sizeof(T) == 2 ? 5 : 7) < ((tiles_narrow + 511) / 512) * 4) {
        if constexpr (DB) fused_cl_db_body<T, WGM, WGN, TM, (TNM > 0 ? TNM : TNS)>(g, S2, idx, N, KF, bias, relu, OUT, OUT2);
        else fused_cl_body<T, WGM, WGN, TM, (TNM > 0 ? TNM : TNS)>(g, S2, idx, N, KF, bias, relu, OUT, OUT2, gu_mid);
    } else if (N < FUSED_LARGE_N) {
        if (TMH > 0 && fused_half_rows(N, g.O, 16 * TNS * WGN, 16 * TM * WGM)) {
            if constexpr (DB) fused_cl_db_body<T, WGM, WGN, (TMH > 0 ? TMH : TM), TNS>(g, S2, idx, N, KF, bias, relu, OUT, OUT2);
            else fused_cl_body<T, WGM, WGN, (TMH > 0 ? TMH : TM), TNS>(g, S2, idx, N, KF, bias, relu, OUT, OUT2, gu_small);
        } else {
            if constexpr (DB) fused_cl_db_body<T, WGM, WGN, TM, TNS>(g, S2, idx, N, KF, bias, relu, OUT, OUT2);
            else fused_cl_body<T, WGM, WGN, TM, TNS>(g, S2, idx, N, KF, bias, relu, OUT, OUT2, gu_small);
        }
    } else if constexpr (DB) {
        // 128 x 128, double-buffered stage; 128 x 64 while the wider tiles would leave workgroup slots empty
        if ((long)((N + 127) / 128) * tiles_m < 512)
            fused_cl_db_body<T, WGM, WGN, TM, TNL>(g, S2, idx, N, KF, bias, relu, OUT, OUT2);
        else
            fused_cl_db_body<T, WGM, WGN, TM, 2 * TNL>(g, S2, idx, N, KF, bias, relu, OUT, OUT2);
    } else
        fused_cl_body<T, WGM, WGN, TM, TNL>(g, S2, idx, N, KF, bias, relu, OUT, OUT2, gu_large);
}

template <typename T>
hipError_t launch_fused_cl(const Geom& g, const FusedPlan& plan, const T* shadow, const int32_t* idx, const int* count,
                           const void* KF, const float* bias, int relu, T* OUT, T* OUT2, hipStream_t st, Tm tm)
{
    if (!plan.cl || (g.C & (g.C - 1)) != 0 || g.C < 16 || g.bf16 != (sizeof(T) == 2)) return hipErrorInvalidValue;
    const dim3 grid(1024), block(256);
    const float4* kf = (const float4*)KF;
#define CB_FUSED_CL(wgm, wgn, tm_, tns, tnl, tmh, tnm, db)                                                             \
    hipExtLaunchKernelGGL((fused_cl_kernel<T, wgm, wgn, tm_, tns, tnl, tmh, tnm, db>), grid, block, lds, st,           \
                          tm.start, tm.stop, 0, g, shadow, idx, count, kf, bias, relu, OUT, OUT2, plan.gu_small,       \
                          plan.gu_large, plan.gu_mid)
    unsigned lds = plan.lds_bytes;
    const bool db_ok = g.kh <= 16 && g.kw <= 16 && g.Wo < 4096;      // what the double-buffered body's tap masks and reciprocal hold
    // tile shapes (rows x columns): narrow | wide
    if (g.O <= 32 && db_ok && fused_db_lds(256) > lds) lds = fused_db_lds(256);
    if (g.O <= 16 && !db_ok)      CB_FUSED_CL(1, 4, 1, 1, 2, 0, 0, false);      // 16 x 64  |  16 x 128
    else if (g.O <= 16)           CB_FUSED_CL(1, 4, 1, 1, 2, 0, 0, true);       //   ... / 16 x 256, double-buffered stage
    else if (g.O <= 32 && !db_ok) CB_FUSED_CL(2, 2, 1, 1, 2, 0, 0, false);      // 32 x 32  |  32 x 64
    else if (g.O <= 32)           CB_FUSED_CL(2, 2, 1, 1, 2, 0, 0, true);       //   ... / 32 x 128, double-buffered stage
    else if (g.O <= 64 && !db_ok) CB_FUSED_CL(4, 1, 1, 1, 4, 0, 2, false);   // 64 x 16  |  64 x 64
    else if (g.O <= 64) {                                             // 64 x 16  |  64 x 64 / 64 x 128, double-buffered stage
        if (fused_db_lds(128) > lds) lds = fused_db_lds(128);
        CB_FUSED_CL(4, 1, 1, 1, 4, 0, 2, true);
    }
    else if (!db_ok) CB_FUSED_CL(4, 1, 2, 1, 4, 1, 2, false);         // 128 x 16 | 128 x 64
    else {                                                            // 128 x 16 | 128 x 128, double-buffered stage
        if (fused_db_lds(128) > lds) lds = fused_db_lds(128);         // (its tap masks hold 16 filter rows and columns)
        CB_FUSED_CL(4, 1, 2, 1, 4, 1, 2, true);
    }
#undef CB_FUSED_CL
    return hipGetLastError();
}

}  // namespace

hipError_t launch_fused_f32_cl(const Geom& g, const FusedPlan& plan, const float* shadow, const int32_t* idx,
                               const int* count, const void* KF, const float* bias, int relu, float* OUT, float* OUT2,
                               hipStream_t st, Tm tm)
{
    return launch_fused_cl<float>(g, plan, shadow, idx, count, KF, bias, relu, OUT, OUT2, st, tm);
}

hipError_t launch_fused_bf16_cl(const Geom& g, const FusedPlan& plan, const uint16_t* shadow, const int32_t* idx,
                                const int* count, const void* KF, const float* bias, int relu, uint16_t* OUT, uint16_t* OUT2,
                                hipStream_t st, Tm tm)
{
    return launch_fused_cl<uint16_t>(g, plan, shadow, idx, count, KF, bias, relu, OUT, OUT2, st, tm);
}

}  // namespace cb
