// Fused back end, float32: matrix generation, matrix multiplication and output
// update (Sec. III-A, last three processing steps) in one kernel.  The columns
// of X' for a tile of listed pixels are gathered from the input state straight
// into LDS, multiplied with the filter matrix on the MFMA units
// (v_mfma_f32_16x16x4_f32), and the result is written with bias + ReLU into the
// cached output at the listed pixels.  X' and Y' never exist in HBM.
//
// Work item = BN listed columns x BM output channels x all of K.  A workgroup is four wavefronts arranged
// WGM x WGN; a wavefront owns a (16*TM) x (16*TN) block of 16x16 MFMA tiles.
//   B operand (gathered receptive fields): LDS tile [k][n] holding a stage of up
//     to GU units of 64 rows, filled by all 256 threads (lane = column, so
//     consecutive lanes read consecutive pixels of the state).  A thread fetches
//     chunks -- runs of up to four horizontally adjacent filter taps of one
//     channel -- with one 16-byte load each; all loads of a stage are issued
//     together and stored behind one barrier pair.
//   A operand (filter matrix): pre-packed at layer creation in MFMA fragment
//     order, so a wavefront reads the fragments of 16 k-values of one 16-row tile
//     as one fully coalesced 16-byte-per-lane load straight into registers (it is
//     L2 resident); no LDS traffic for A.  Rolling prefetch, PF units deep.
// The grid is persistent; N is read from device memory.  Each XCD (workgroup id
// mod 8) takes a contiguous range of column tiles: the index list is sorted, so
// neighbouring tiles read neighbouring state rows, which then stay in that XCD's L2.
#include "cb_fused.h"

namespace cb {

namespace {

template <int CW> struct Chunk;
template <> struct Chunk<1> {
    float v;
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, unsigned off)
    { v = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 0)); }
    __device__ __forceinline__ unsigned get(int) const { return __float_as_uint(v); }
};
template <> struct Chunk<4> {
    uintx4 v;
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, unsigned off)
    { v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0); }
    __device__ __forceinline__ unsigned get(int e) const { return v[e]; }
};

template <int WGM, int WGN, int TM, int TN, int CW>
__device__ __forceinline__ void fused_f32_body(const Geom& g, const float* __restrict__ S,
                                               const int32_t* __restrict__ idx, const int N,
                                               const float4* __restrict__ KF, const int2* __restrict__ tabg,
                                               const int ntab, const float* __restrict__ bias, int relu,
                                               float* __restrict__ OUT, float* __restrict__ OUT2, const int GU)
{
    static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
    constexpr int BM = 16 * TM * WGM, BN = 16 * TN * WGN;
    constexpr int BNP = BN + (BN % 32 == 16 ? 0 : 16);   // row pitch: conflict-free fragment reads
    constexpr int RG = 256 / BN;                 // threads per column = chunks fetched side by side
    constexpr int CPS = fused_cps(false, CW);    // chunks per thread per stage at most
    constexpr int LV = KC / RG;                  // single elements: rows per thread per unit
    constexpr int GRP = CPS % 4 == 0 ? 4 : 3;    // runs: rounds tested together
    static_assert(CPS % GRP == 0 && (CW > 1 || CPS % LV == 0), "gather rounds come in whole groups");
    constexpr int UNIT = KC * BNP;               // floats of one unit in LDS
    constexpr bool TWO = TM * TN < 4;            // second accumulator chain where a wavefront has few tiles
    constexpr int PF = TM * TN >= 2 ? 2 : 4;     // units of filter fragments in flight (register budget)
    constexpr int KB = TN >= 4 ? 4 : 8;          // k-steps per group of B fragments read ahead of their MFMAs
    __shared__ int qs[BN];
    __shared__ float dump_slots[256];
    float* const dump = &dump_slots[threadIdx.x];
    extern __shared__ int2 dyn_lds[];            // chunk table, unit starts, then the B stage (GU units)

    const int nunits = (g.R + KC - 1) / KC;      // 64-row units of K
    int2* tab = dyn_lds;
    int* ustart = reinterpret_cast<int*>(dyn_lds + ntab + FUSED_TAB_PAD);
    float* Bs = reinterpret_cast<float*>(reinterpret_cast<char*>(dyn_lds) +
                                         ((((unsigned)ntab + (unsigned)FUSED_TAB_PAD) * 8u + ((unsigned)nunits + 1u) * 4u + 15u) & ~15u));
    // Raw buffer over the input state, 32-bit byte offsets, components beyond the end read
    // as 0.  A load whose FIRST byte lies before the buffer returns nothing at all, and the
    // chunk of the first channel's first image row starts up to `pad` elements early for
    // pixels at the left border: the buffer therefore begins FUSED_GUARD bytes ahead of the
    // state (inside the same allocation) and every offset is moved by as much.
    const __amdgpu_buffer_rsrc_t srsrc = __builtin_amdgcn_make_buffer_rsrc(
        reinterpret_cast<char*>(const_cast<float*>(S)) - FUSED_GUARD, 0,
        (int)((unsigned)g.C * (unsigned)g.P * 4u + (unsigned)FUSED_GUARD), 0x00020000);
    const int KG = nunits * 4;                   // 16-row groups of the packed filter matrix
    // The packed filter matrix is read through a buffer resource as well: the address of a
    // fragment is then a wave-uniform offset, computed on the scalar unit, plus constants.  (A
    // wavefront alone on its SIMD cannot overlap its own vector ALU instructions with its
    // MFMAs, so every address computed per lane costs MFMA time.)
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
    const int gn = tid % BN, gr = tid / BN;      // this thread's column and its place among the RG chunk fetchers

    // The listed pixel of this thread's column is requested one tile ahead -- for the first
    // tile ahead of the table copy -- so that its latency is not added to the chain
    // index list -> state -> LDS -> MFMA of every tile.
    auto fetch_q = [&](long tt) -> int {
        if (tt >= total) return 0;
        const int ntt = (int)(tt & 7) * per_xcd + (int)((tt >> 3) / MT);
        const int n = ntt * BN + gn;
        return (ntt < NT && n < N) ? idx[n] : 0;
    };
    int qnext = fetch_q(blockIdx.x);

    // the table is read once per chunk: keep it in LDS, so that no gather load depends on
    // an earlier global load
    // (eight loads in flight per thread: one load per trip would cost a memory latency per 256 entries)
    for (int r0 = threadIdx.x; r0 < ntab + FUSED_TAB_PAD; r0 += 8 * 256) {
        int2 e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
            e[j] = r0 + j * 256 < ntab + FUSED_TAB_PAD ? tabg[r0 + j * 256] : make_int2(0, 0);
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (r0 + j * 256 < ntab + FUSED_TAB_PAD) tab[r0 + j * 256] = e[j];
    }
    {
        const int* us = reinterpret_cast<const int*>(tabg + ntab + FUSED_TAB_PAD);
        for (int r = threadIdx.x; r < nunits + 1; r += 256) ustart[r] = us[r];
    }
    for (long t = blockIdx.x; t < total; t += gridDim.x) {
        const int xcd = (int)(t & 7);
        const long u = t >> 3;
        const int mt = (int)(u % MT);
        const int nt = xcd * per_xcd + (int)(u / MT);
        const int q = qnext;
        qnext = fetch_q(t + gridDim.x);
        if (nt >= NT) continue;
        const int n0 = nt * BN, m0 = mt * BM;
        const int ubeg = 0, uend = nunits;

        // filter fragments of unit c: 4 groups of 16 rows per 16-row output tile, one fully
        // coalesced 16-byte-per-lane load each; issued unconditionally (clamped unit index) so
        // that the rolling prefetch can be waited for with exact counts
        float4 areg[PF][TM][4];
        auto aload = [&](int c, float4 (&dst)[TM][4]) {
#pragma unroll
            for (int a = 0; a < TM; ++a) {
                // wave-uniform byte offset of the unit's four k-groups (scalar arithmetic); the lane's
                // 16 bytes and the k-group go into the instruction's own offset fields
                const unsigned soff = (unsigned)(((m0 >> 4) + wm_s * TM + a) * KG + c * 4) * 1024u;
#pragma unroll
                for (int kg = 0; kg < 4; ++kg)
                    dst[a][kg] = __builtin_bit_cast(float4, __builtin_amdgcn_raw_buffer_load_b128(krsrc, lane * 16 + kg * 1024, (int)soff, 0));
            }
        };

        // Cross-stage prefetch: when every full stage holds a multiple of PF units, the rolling
        // prefetch simply runs on into the next stage, and only the first fragments of a tile
        // are waited for -- they are requested here, ahead of the index list and the gather.
        const bool ring = GU % PF == 0;
#pragma unroll
        for (int p = 0; p < PF; ++p) aload(ubeg + p < uend - 1 ? ubeg + p : uend - 1, areg[p]);

        // this thread's column: top-left corner of the receptive field
        const bool colv = n0 + gn < N;
        const int yo = q / g.Wo, xo = q - yo * g.Wo;
        const int y0 = yo * g.s - g.p, x0 = xo * g.s - g.p;
        // Gather through a buffer resource over the state.  A chunk costs one LDS read of
        // its table entry, one add and one load; whatever a padding tap fetches (a
        // neighbouring row's pixel, or 0 beyond the buffer) is masked when the stage is
        // written to LDS, with one bit per tap of this pixel.
        const unsigned long long ok = taps_inside(g, colv, y0, x0);
        const unsigned base4 = (unsigned)(y0 * g.W + x0) * 4u + (unsigned)FUSED_GUARD;
        // (the barrier: the previous tile's epilogue has read qs; the table is filled)
        const bool interior = __syncthreads_and(!colv || ok == (1ull << (g.kh * g.kw)) - 1ull) != 0;
        if (tid < BN) qs[tid] = colv ? q : -1;    // threads 0..BN-1 own columns 0..BN-1

        // One stage = up to GU units of 64 rows: all its gather loads are issued together
        // (one memory latency per stage), parked in registers, and stored to LDS behind one
        // barrier pair; the MFMAs of the whole stage then run without further barriers.
        Chunk<CW> breg[CPS];
        // Single elements (CW == 1): chunk = row, a unit holds exactly 64 of them, so round v
        // of a stage is row gr + v*RG of the stage for every thread -- compile-time LDS
        // offsets, and a padding tap simply gets an out-of-range offset (reads as 0).
        // Runs (CW > 1): the chunks of a stage are dealt out RG at a time; the trip count is
        // uniform over the workgroup (a scalar test per round); threads beyond the stage's last
        // chunk fetch the table entry that follows and skip the store.
        const unsigned oklo = (unsigned)ok, okhi = (unsigned)(ok >> 32);
        auto gload_stage = [&](int u0) {
            const int ue = u0 + GU < uend ? u0 + GU : uend;
            if constexpr (CW == 1) {
                // one test per unit: the table reads and the loads of a unit stay in one basic
                // block, so their latencies overlap instead of adding up
                const int2* trow = tab + u0 * KC + gr;
#pragma unroll
                for (int uu = 0; uu < CPS / LV; ++uu) {
                    if (uu < ue - u0) {
#pragma unroll
                        for (int v = uu * LV; v < (uu + 1) * LV; ++v) {
                            const int2 ch = trow[v * RG];
                            const unsigned tap = (unsigned)ch.y >> 20;
                            breg[v].load(srsrc, (base4 + (unsigned)ch.x) | ~bit_ones((tap & 32u) ? okhi : oklo, tap & 31u));
                        }
                    }
                }
            } else {
                const int qb = __builtin_amdgcn_readfirstlane(ustart[u0]);
                const int nq = __builtin_amdgcn_readfirstlane(ustart[ue]) - qb;
                // rounds are tested GRP at a time (see above).  Fetchers beyond the stage's last
                // chunk load whatever entry follows (a chunk of the next stage, or one of the
                // entries that close the table: offset 0) and do not store it.
                const int2* tq = tab + qb + gr;
#pragma unroll
                for (int vb = 0; vb < CPS; vb += GRP) {
                    if (vb * RG < nq) {
#pragma unroll
                        for (int v = vb; v < vb + GRP; ++v) breg[v].load(srsrc, base4 + (unsigned)tq[v * RG].x);
                    }
                }
            }
        };
        auto lds_store_stage = [&](int u0) {
            const int ue = u0 + GU < uend ? u0 + GU : uend;
            if constexpr (CW == 1) {
                float* Bst = Bs + gr * BNP + gn;
#pragma unroll
                for (int uu = 0; uu < CPS / LV; ++uu) {
                    if (uu < ue - u0) {
#pragma unroll
                        for (int v = uu * LV; v < (uu + 1) * LV; ++v) Bst[v * RG * BNP] = __uint_as_float(breg[v].get(0));
                    }
                }
            } else {
                const int qb = __builtin_amdgcn_readfirstlane(ustart[u0]);
                const int nq = __builtin_amdgcn_readfirstlane(ustart[ue]) - qb;
                float* Bst = Bs + gn - u0 * UNIT;     // row r of X' lives at Bst[r * BNP]
                const int2* tq = tab + qb + gr;
                // Every vector ALU instruction here costs MFMA time (a wavefront cannot overlap
                // the two), so the common case -- no listed pixel of the tile touches the image
                // border -- stores the loaded elements as they are.
                if (interior) {
#pragma unroll
                    for (int vb = 0; vb < CPS; vb += GRP) {
                        if (vb * RG < nq) {
#pragma unroll
                            for (int v = vb; v < vb + GRP; ++v) {
                                const int y = tq[v * RG].y;   // first row | length << 16 | first tap << 20
                                const int len = gr + v * RG < nq ? (y >> 16) & 7 : 0;
                                float* dst = Bst + (y & 0xFFFF) * BNP;
                                // rows beyond the chunk's length go to a per-thread dump slot: no divergent branches
                                *(len > 0 ? dst : dump) = __uint_as_float(breg[v].get(0));
                                *(len > 1 ? dst + BNP : dump) = __uint_as_float(breg[v].get(1));
                                *(len > 2 ? dst + 2 * BNP : dump) = __uint_as_float(breg[v].get(2));
                                *(len > 3 ? dst + 3 * BNP : dump) = __uint_as_float(breg[v].get(3));
                            }
                        }
                    }
                } else {
#pragma unroll
                    for (int vb = 0; vb < CPS; vb += GRP) {
                        if (vb * RG < nq) {
#pragma unroll
                            for (int v = vb; v < vb + GRP; ++v) {
                                const int y = tq[v * RG].y;
                                const unsigned m = (unsigned)(ok >> ((unsigned)y >> 20));
                                const int len = gr + v * RG < nq ? (y >> 16) & 7 : 0;
                                float* dst = Bst + (y & 0xFFFF) * BNP;
                                // rows beyond the chunk's length go to a per-thread dump slot: no divergent branches
                                *(len > 0 ? dst : dump) = __uint_as_float(breg[v].get(0) & bit_ones(m, 0));
                                *(len > 1 ? dst + BNP : dump) = __uint_as_float(breg[v].get(1) & bit_ones(m, 1));
                                *(len > 2 ? dst + 2 * BNP : dump) = __uint_as_float(breg[v].get(2) & bit_ones(m, 2));
                                *(len > 3 ? dst + 3 * BNP : dump) = __uint_as_float(breg[v].get(3) & bit_ones(m, 3));
                            }
                        }
                    }
                }
                // rows R .. 64*nunits - 1 of the last unit have no chunks: they are zero
                if (ue == uend && g.R < uend * KC) {
                    const int rz = g.R - u0 * KC, nz = (uend - u0) * KC - rz;
                    for (int i = tid; i < nz * BN; i += 256) Bs[(rz + i / BN) * BNP + i % BN] = 0.f;
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

        // One unit = 16 k-steps in groups of KB.  The B fragments of the NEXT group are
        // requested from LDS before the MFMAs of the current one are issued (two register
        // sets); the scheduling barriers keep the compiler from sinking the reads down to
        // their first use, which would expose one LDS latency per k-step (wide tiles only:
        // with one or two tiles per wavefront the compiler's own order measured faster).
        // The first group of a unit's B fragments is requested during the last group of the
        // unit before it (same stage: the data is already in LDS), so that only the first unit
        // of a stage waits for an LDS read with nothing to issue meanwhile.
        constexpr int NG = 16 / KB;
        float bcarry[KB][TN];
        auto compute = [&](int uu, const float4 (&af)[TM][4], bool first, bool more) {
            const float* Bu = Bs + uu * UNIT + lq * BNP + wn * TN * 16 + l16;
            float bfr[2][KB][TN];
            auto bload = [&](const float* base, int grp, float (&dst)[KB][TN]) {
#pragma unroll
                for (int ks2 = 0; ks2 < KB; ++ks2)
#pragma unroll
                    for (int b = 0; b < TN; ++b)
                        dst[ks2][b] = base[(grp * KB + ks2) * 4 * BNP + b * 16];
            };
            if (first) bload(Bu, 0, bfr[0]);
            else {
#pragma unroll
                for (int ks2 = 0; ks2 < KB; ++ks2)
#pragma unroll
                    for (int b = 0; b < TN; ++b) bfr[0][ks2][b] = bcarry[ks2][b];
            }
#pragma unroll
            for (int grp = 0; grp < NG; ++grp) {
                if (grp + 1 < NG) bload(Bu, grp + 1, bfr[(grp + 1) & 1]);
                else if (more) bload(Bu + UNIT, 0, bcarry);
                if (TN >= 4) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int ks2 = 0; ks2 < KB; ++ks2) {
                    const int kg = (grp * KB + ks2) >> 2, kk = (grp * KB + ks2) & 3;
#pragma unroll
                    for (int a = 0; a < TM; ++a) {
                        const float av = kk == 0 ? af[a][kg].x : kk == 1 ? af[a][kg].y
                                       : kk == 2 ? af[a][kg].z : af[a][kg].w;
#pragma unroll
                        for (int b = 0; b < TN; ++b) {
                            if (TWO && (kk & 1))
                                acc1[TWO ? a : 0][TWO ? b : 0] = __builtin_amdgcn_mfma_f32_16x16x4f32(
                                    av, bfr[grp & 1][ks2][b], acc1[TWO ? a : 0][TWO ? b : 0], 0, 0, 0);
                            else
                                acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bfr[grp & 1][ks2][b], acc[a][b], 0, 0, 0);
                        }
                    }
                }
                if (TN >= 4) __builtin_amdgcn_sched_barrier(0);
            }
        };
        gload_stage(ubeg);
        for (int u0 = ubeg; u0 < uend; u0 += GU) {
            const int ucount = uend - u0 < GU ? uend - u0 : GU;
            const int ulast = u0 + ucount - 1;
            __syncthreads();                      // the previous stage's fragments have been read
            lds_store_stage(u0);
            __syncthreads();
            if (!ring && u0 != ubeg) {
#pragma unroll
                for (int p = 0; p < PF; ++p) aload(u0 + p < ulast ? u0 + p : ulast, areg[p]);
            }
            if (u0 + GU < uend) gload_stage(u0 + GU);   // in flight during this stage's MFMAs
            const int alast = ring ? uend - 1 : ulast;  // how far the rolling prefetch may run
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
                        OUT[(size_t)m * g.Po + qn] = v;
                        v4[r] = v;
                    }
                }
                // (a layer that keeps the pixel-major copy has a multiple of 16 output channels)
                if (OUT2 && mb < g.O) st_out4(OUT2 + (size_t)qn * g.O + mb, v4);
            }
        }
    }
}

// Columns per workgroup tile are chosen on the device from N: with few listed pixels small
// tiles (16*TNS columns per wavefront column) give every compute unit work and short
// per-tile latency; from FUSED_LARGE_N columns on, wide tiles (16*TNL) re-read the filter
// matrix less often.
template <int WGM, int WGN, int TM, int TNS, int TNL, int CW, int TMH, int TNM>
__global__ __launch_bounds__(256, 2) void fused_f32_kernel(Geom g, const float* __restrict__ S,
                                                        const int32_t* __restrict__ idx,
                                                        const int* __restrict__ count,
                                                        const float4* __restrict__ KF,
                                                        const int2* __restrict__ tab, int ntab,
                                                        const float* __restrict__ bias, int relu,
                                                        float* __restrict__ OUT, float* __restrict__ OUT2, int gu_small, int gu_large, int gu_mid)
{
    const int N = *count;
    if (N <= 0) return;
    if (TNM > 0 && gu_mid > 0 && N < FUSED_LARGE_N &&
        (long)((N + 16 * TNS * WGN - 1) / (16 * TNS * WGN)) * ((g.O + 16 * TM * WGM - 1) / (16 * TM * WGM)) > FUSED_MID_TILES) {
        fused_f32_body<WGM, WGN, TM, (TNM > 0 ? TNM : TNS), CW>(g, S, idx, N, KF, tab, ntab, bias, relu, OUT, OUT2, gu_mid);
    } else if (N < FUSED_LARGE_N) {
        // Few listed pixels mean few tiles, and the kernel takes as long as the busiest
        // compute unit: rows per tile are halved (TMH) where that shortens the longest queue.
        if (TMH > 0 && fused_half_rows(N, g.O, 16 * TNS * WGN, 16 * TM * WGM))
            fused_f32_body<WGM, WGN, (TMH > 0 ? TMH : TM), TNS, CW>(g, S, idx, N, KF, tab, ntab, bias, relu, OUT, OUT2, gu_small);
        else
            fused_f32_body<WGM, WGN, TM, TNS, CW>(g, S, idx, N, KF, tab, ntab, bias, relu, OUT, OUT2, gu_small);
    } else
        fused_f32_body<WGM, WGN, TM, TNL, CW>(g, S, idx, N, KF, tab, ntab, bias, relu, OUT, OUT2, gu_large);
}

}  // namespace

hipError_t launch_fused_f32(const Geom& g, const FusedPlan& plan, const float* src, const int32_t* idx,
                            const int* count, const void* KF, const int2* tab, const float* bias, int relu,
                            float* OUT, float* OUT2, hipStream_t st, Tm tm)
{
    const dim3 grid(1024), block(256);
    const float4* kf = (const float4*)KF;
#define CB_FUSED(wgm, wgn, tm_, tns, tnl, cw, tmh, tnm)                                                                   \
    hipExtLaunchKernelGGL((fused_f32_kernel<wgm, wgn, tm_, tns, tnl, cw, tmh, tnm>), grid, block, plan.lds_bytes, st, tm.start, \
                          tm.stop, 0, g, src, idx, count, kf, tab, plan.ntab, bias, relu, OUT, OUT2, plan.gu_small,      \
                          plan.gu_large, plan.gu_mid)
    // tile shapes (rows x columns): narrow | wide
    if (plan.cw == 1) {
        if (g.O <= 16)      CB_FUSED(1, 4, 1, 1, 2, 1, 0, 0);      // 16 x 64  |  16 x 128
        else if (g.O <= 32) CB_FUSED(2, 2, 1, 1, 2, 1, 0, 0);      // 32 x 32  |  32 x 64
        else if (g.O <= 64) CB_FUSED(4, 1, 1, 1, 4, 1, 0, 2);      // 64 x 16  |  64 x 64
        else                CB_FUSED(4, 1, 2, 1, 4, 1, 1, 2);      // 128 x 16 | 128 x 64
    } else {
        if (g.O <= 16)      CB_FUSED(1, 4, 1, 1, 2, 4, 0, 0);
        else if (g.O <= 32) CB_FUSED(2, 2, 1, 1, 2, 4, 0, 0);
        else if (g.O <= 64) CB_FUSED(4, 1, 1, 1, 4, 4, 0, 2);
        else                CB_FUSED(4, 1, 2, 1, 4, 4, 1, 2);
    }
#undef CB_FUSED
    return hipGetLastError();
}

}  // namespace cb
