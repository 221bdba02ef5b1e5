// Fused back end, bfloat16: same structure as the float32 kernel (matrix
// generation, matrix multiplication and output update of Sec. III-A in one
// kernel); differences:
//   * MFMA v_mfma_f32_16x16x32_bf16: a lane supplies 8 consecutive k of one row (A) /
//     one column (B), so the B stage in LDS is [n][k] with k contiguous (row pitch 72
//     elements = 144 bytes: eight lanes reading 16 bytes each then cover all 32 banks),
//     read with one 16-byte LDS load per fragment;
//   * a chunk is up to three horizontally adjacent taps, fetched as the two aligned
//     32-bit words that contain them and shifted into place when written to LDS;
//   * the filter matrix is packed as 16 bytes (8 k) per lane per 32-row group;
//   * accumulation stays float32; the cached output is rounded once to bfloat16.
//
#include "cb_fused.h"

namespace cb {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
constexpr int KPB = KC + 8;                      // k pitch of a column in LDS

template <int CW> struct Chunk;
template <> struct Chunk<1> {
    uint16_t v;
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, unsigned off)
    { v = __builtin_amdgcn_raw_buffer_load_b16(r, (int)off, 0, 0); }
};
template <> struct Chunk<3> {
    uintx2 v;                                    // the two aligned words that hold the three elements
    __device__ __forceinline__ void load(__amdgpu_buffer_rsrc_t r, unsigned off)
    { v = __builtin_amdgcn_raw_buffer_load_b64(r, (int)(off & ~3u), 0, 0); }
};

template <int WGM, int WGN, int TM, int TN, int CW>
__device__ __forceinline__ void fused_bf16_body(const Geom& g, const uint16_t* __restrict__ S,
                                               const int32_t* __restrict__ idx, const int N,
                                               const uint4* __restrict__ KF, const int2* __restrict__ tabg,
                                               const int ntab, const float* __restrict__ bias, int relu,
                                               uint16_t* __restrict__ OUT, uint16_t* __restrict__ OUT2, const int GU)
{
    static_assert(WGM * WGN == 4, "four wavefronts per workgroup");
    constexpr int BM = 16 * TM * WGM, BN = 16 * TN * WGN;
    constexpr int RG = 256 / BN;                 // threads per column = chunks fetched side by side
    constexpr int CPS = fused_cps(true, CW);    // chunks per thread per stage at most
    constexpr int LV = KC / RG;                  // single elements: rows per thread per unit
    constexpr int GRP = CPS % 4 == 0 ? 4 : 3;    // runs: rounds tested together
    static_assert(CPS % GRP == 0 && (CW > 1 || CPS % LV == 0), "gather rounds come in whole groups");
    constexpr int UNIT = BN * KPB;               // bf16 elements of one unit in LDS
    constexpr bool TWO = TM * TN < 4;            // second accumulator chain where a wavefront has few tiles
    constexpr int PF = TM * TN >= 2 ? 2 : 4;     // units of filter fragments in flight (register budget)
    __shared__ int qs[BN];
    __shared__ uint16_t dump_slots[256];
    uint16_t* const dump = &dump_slots[threadIdx.x];
    extern __shared__ int2 dyn_lds[];            // chunk table, unit starts, then the B stage (GU units)

    const int nunits = (g.R + KC - 1) / KC;      // 64-row units of K
    int2* tab = dyn_lds;
    int* ustart = reinterpret_cast<int*>(dyn_lds + ntab + FUSED_TAB_PAD);
    uint16_t* Bs = reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(dyn_lds) +
                                         ((((unsigned)ntab + (unsigned)FUSED_TAB_PAD) * 8u + ((unsigned)nunits + 1u) * 4u + 15u) & ~15u));
    // raw buffer over the input state: 32-bit byte offsets, out-of-range components read as 0
    // Raw buffer over the input state, 32-bit byte offsets, components beyond the end read
    // as 0.  A load whose FIRST byte lies before the buffer returns nothing at all, and the
    // chunk of the first channel's first image row starts up to `pad` elements early for
    // pixels at the left border: the buffer therefore begins FUSED_GUARD bytes ahead of the
    // state (inside the same allocation) and every offset is moved by as much.
    const __amdgpu_buffer_rsrc_t srsrc = __builtin_amdgcn_make_buffer_rsrc(
        reinterpret_cast<char*>(const_cast<uint16_t*>(S)) - FUSED_GUARD, 0,
        (int)((((unsigned)g.C * (unsigned)g.P * 2u + 3u) & ~3u) + (unsigned)FUSED_GUARD), 0x00020000);
    // (whole 32-bit words are fetched: an odd element count is rounded up, the state's
    // allocation is padded to 256 bytes)
    const int KG = nunits * 2;                   // 32-row groups of the packed filter matrix
    // The packed filter matrix is read through a buffer resource as well: the address of a
    // fragment is then a wave-uniform offset, computed on the scalar unit, plus constants (a
    // wavefront cannot overlap its own vector ALU instructions with its MFMAs).
    const __amdgpu_buffer_rsrc_t krsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint4*>(KF), 0, (int)((unsigned)((g.O + 127) / 128 * 8) * (unsigned)KG * 1024u), 0x00020000);
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

        // filter fragments of unit c: 2 groups of 32 rows per 16-row output tile, one fully
        // coalesced 16-byte-per-lane load each; issued unconditionally (clamped unit index) so
        // that the rolling prefetch can be waited for with exact counts
        uint4 areg[PF][TM][2];
        auto aload = [&](int c, uint4 (&dst)[TM][2]) {
#pragma unroll
            for (int a = 0; a < TM; ++a) {
                // wave-uniform byte offset of the unit's two k-groups (scalar arithmetic); the lane's
                // 16 bytes and the k-group go into the instruction's own offset fields
                const unsigned soff = (unsigned)(((m0 >> 4) + wm_s * TM + a) * KG + c * 2) * 1024u;
#pragma unroll
                for (int kg = 0; kg < 2; ++kg)
                    dst[a][kg] = __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(krsrc, lane * 16 + kg * 1024, (int)soff, 0));
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
        const unsigned base2 = (unsigned)(y0 * g.W + x0) * 2u + (unsigned)FUSED_GUARD;
        // (the barrier: the previous tile's epilogue has read qs; the table is filled.)  A tile none of
        // whose listed pixels touches the image border needs no masks for padding taps.
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
                            breg[v].load(srsrc, (base2 + (unsigned)ch.x) | ~bit_ones((tap & 32u) ? okhi : oklo, tap & 31u));
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
                        for (int v = vb; v < vb + GRP; ++v) breg[v].load(srsrc, base2 + (unsigned)tq[v * RG].x);
                    }
                }
            }
        };
        auto lds_store_stage = [&](int u0) {
            const int ue = u0 + GU < uend ? u0 + GU : uend;
            uint16_t* Bst = Bs + gn * KPB;
            if constexpr (CW == 1) {
#pragma unroll
                for (int uu = 0; uu < CPS / LV; ++uu) {
                    if (uu < ue - u0) {
#pragma unroll
                        for (int v = uu * LV; v < (uu + 1) * LV; ++v)
                            Bst[((v * RG) >> 6) * UNIT + ((v * RG) & 63) + gr] = breg[v].v;
                    }
                }
            } else {
                const int qb = __builtin_amdgcn_readfirstlane(ustart[u0]);
                const int nq = __builtin_amdgcn_readfirstlane(ustart[ue]) - qb;
                const int2* tq = tab + qb + gr;
#pragma unroll
                for (int vb = 0; vb < CPS; vb += GRP) {
                    if (vb * RG < nq) {
#pragma unroll
                      for (int v = vb; v < vb + GRP; ++v) {
                        const int2 ch = tq[v * RG];  // .y = first row | length << 16 | first tap << 20
                        const int rel = (ch.y & 0xFFFF) - u0 * KC;
                        uint16_t* dst = Bst + (rel >> 6) * UNIT + (rel & 63);
                        const unsigned sh = ((base2 + (unsigned)ch.x) & 2u) << 3;   // odd element: data starts 16 bits in
                        const unsigned lo = __builtin_amdgcn_alignbit(breg[v].v[1], breg[v].v[0], sh);
                        const unsigned hi = breg[v].v[1] >> sh;
                        const int len = gr + v * RG < nq ? (ch.y >> 16) & 7 : 0;
                        // elements beyond the chunk's length go to a per-thread dump slot: no divergent branches
                        if (interior && ((unsigned)ch.y >> 20) != (unsigned)FUSED_ZERO_TAP) {
                            *(len > 0 ? dst : dump) = (uint16_t)lo;
                            *(len > 1 ? dst + 1 : dump) = (uint16_t)(lo >> 16);
                            *(len > 2 ? dst + 2 : dump) = (uint16_t)hi;
                        } else {
                            const unsigned m = (unsigned)(ok >> ((unsigned)ch.y >> 20));
                            *(len > 0 ? dst : dump) = (uint16_t)(lo & bit_ones(m, 0));
                            *(len > 1 ? dst + 1 : dump) = (uint16_t)((lo >> 16) & bit_ones(m, 1));
                            *(len > 2 ? dst + 2 : dump) = (uint16_t)(hi & bit_ones(m, 2));
                        }
                      }
                    }
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

        // one unit = two k-steps of 32; its B fragments are read from LDS ahead of the MFMAs
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
                    if (TWO)
                        acc1[TWO ? a : 0][TWO ? b : 0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8, af[a][1]), __builtin_bit_cast(bf16x8, bfr[1][b]),
                            acc1[TWO ? a : 0][TWO ? b : 0], 0, 0, 0);
                    else
                        acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, af[a][1]),
                                                                            __builtin_bit_cast(bf16x8, bfr[1][b]), acc[a][b], 0, 0, 0);
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
                    compute(uu, areg[p]);
                    aload(u0 + uu + PF < alast ? u0 + uu + PF : alast, areg[p]);
                }
            }
#pragma unroll
            for (int p = 0; p < PF - 1; ++p)
                if (nfull * PF + p < ucount) compute(nfull * PF + p, areg[p]);
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

// Columns per workgroup tile are chosen on the device from N: with few listed pixels small
// tiles (16*TNS columns per wavefront column) give every compute unit work and short
// per-tile latency; from FUSED_LARGE_N columns on, wide tiles (16*TNL) re-read the filter
// matrix less often.
template <int WGM, int WGN, int TM, int TNS, int TNL, int CW, int TMH>
__global__ __launch_bounds__(256, 2) void fused_bf16_kernel(Geom g, const uint16_t* __restrict__ S,
                                                        const int32_t* __restrict__ idx,
                                                        const int* __restrict__ count,
                                                        const uint4* __restrict__ KF,
                                                        const int2* __restrict__ tab, int ntab,
                                                        const float* __restrict__ bias, int relu,
                                                        uint16_t* __restrict__ OUT, uint16_t* __restrict__ OUT2, int gu_small, int gu_large)
{
    const int N = *count;
    if (N <= 0) return;
    if (N < FUSED_LARGE_N) {
        // Few listed pixels mean few tiles, and the kernel takes as long as the busiest
        // compute unit: rows per tile are halved (TMH) where that shortens the longest queue.
        if (TMH > 0 && fused_half_rows(N, g.O, 16 * TNS * WGN, 16 * TM * WGM))
            fused_bf16_body<WGM, WGN, (TMH > 0 ? TMH : TM), TNS, CW>(g, S, idx, N, KF, tab, ntab, bias, relu, OUT, OUT2, gu_small);
        else
            fused_bf16_body<WGM, WGN, TM, TNS, CW>(g, S, idx, N, KF, tab, ntab, bias, relu, OUT, OUT2, gu_small);
    } else
        fused_bf16_body<WGM, WGN, TM, TNL, CW>(g, S, idx, N, KF, tab, ntab, bias, relu, OUT, OUT2, gu_large);
}

}  // namespace

hipError_t launch_fused_bf16(const Geom& g, const FusedPlan& plan, const uint16_t* src, const int32_t* idx,
                             const int* count, const void* KF, const int2* tab, const float* bias, int relu,
                             uint16_t* OUT, uint16_t* OUT2, hipStream_t st, Tm tm)
{
    const dim3 grid(1024), block(256);
    const uint4* kf = (const uint4*)KF;
#define CB_FUSED(wgm, wgn, tm_, tns, tnl, cw, tmh)                                                                     \
    hipExtLaunchKernelGGL((fused_bf16_kernel<wgm, wgn, tm_, tns, tnl, cw, tmh>), grid, block, plan.lds_bytes, st, tm.start, \
                          tm.stop, 0, g, src, idx, count, kf, tab, plan.ntab, bias, relu, OUT, OUT2, plan.gu_small,      \
                          plan.gu_large)
    // tile shapes (rows x columns): narrow | wide
    if (plan.cw == 1) {
        if (g.O <= 16)      CB_FUSED(1, 4, 1, 1, 2, 1, 0);      // 16 x 64  |  16 x 128
        else if (g.O <= 32) CB_FUSED(2, 2, 1, 1, 2, 1, 0);      // 32 x 32  |  32 x 64
        else if (g.O <= 64) CB_FUSED(4, 1, 1, 1, 4, 1, 0);      // 64 x 16  |  64 x 64
        else                CB_FUSED(4, 1, 2, 1, 4, 1, 1);      // 128 x 16 | 128 x 64
    } else {
        if (g.O <= 16)      CB_FUSED(1, 4, 1, 1, 2, 3, 0);
        else if (g.O <= 32) CB_FUSED(2, 2, 1, 1, 2, 3, 0);
        else if (g.O <= 64) CB_FUSED(4, 1, 1, 1, 4, 3, 0);
        else                CB_FUSED(4, 1, 2, 1, 4, 3, 1);
    }
#undef CB_FUSED
    return hipGetLastError();
}

}  // namespace cb
