// Fused back end, host side and the small kernels around the main one: filter
// matrix packing in MFMA fragment order, the chunk table that drives the gather
// (Sec. III-A, "Matrix Generation": which elements of the input state make up a
// column of X') and the plan of a launch (units per LDS stage).  The main kernels are in cb_fused_f32.hip and
// cb_fused_bf16.hip.
#include "cb_fused.h"

#include <vector>

namespace cb {

namespace {

// Filter matrix in MFMA fragment order for the float32 kernel:
//   KF[((mtile*KG + kgroup)*64 + lane)].{x,y,z,w}[kk] = K(m = mtile*16 + lane%16, k = kgroup*16 + kk*4 + lane/16)
// zero outside O x R.
__global__ __launch_bounds__(256) void pack_fused_f32_kernel(Geom g, int Mt16, int KG, const float* __restrict__ w,
                                                             float4* __restrict__ KF)
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
}

// Channel-last variant: K is walked tap-major, k' = (j*kw + i)*C + c, and a lane's four values of a
// k-group are four consecutive k':
//   KF[((mtile*KG + kgroup)*64 + lane)].{x,y,z,w}[kk] = K(m, c*kh*kw + tap) with k' = kgroup*16 + 4*(lane/16) + kk,
//   tap = k' / C, c = k' mod C; zero outside O x R.
__global__ __launch_bounds__(256) void pack_fused_f32_cl_kernel(Geom g, int Mt16, int KG, const float* __restrict__ w,
                                                                float4* __restrict__ KF)
{
    const long n = (long)Mt16 * KG * 64;
    const int taps = g.kh * g.kw;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long)gridDim.x * 256) {
        const int lane = (int)(e & 63);
        const long gk = e >> 6;
        const int kgroup = (int)(gk % KG), mtile = (int)(gk / KG);
        const int m = mtile * 16 + (lane & 15);
        float v[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int k = kgroup * 16 + 4 * (lane >> 4) + kk;
            const int tap = k / g.C, c = k - tap * g.C;
            v[kk] = (m < g.O && k < g.R) ? w[(size_t)m * g.R + (size_t)c * taps + tap] : 0.f;
        }
        KF[e] = make_float4(v[0], v[1], v[2], v[3]);
    }
}

// Filter matrix in fragment order for v_mfma_f32_16x16x32_bf16:
//   KF[(mtile*KG + kgroup)*64 + lane] = 8 bf16: K(m = mtile*16 + lane%16, k = kgroup*32 + 8*(lane/16) + 0..7)
__global__ __launch_bounds__(256) void pack_fused_bf16_kernel(Geom g, int Mt16, int KG, const uint16_t* __restrict__ w,
                                                              uint4* __restrict__ KF)
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
}

// Channel-last variant, bfloat16: 8 consecutive k' per lane, k' = (j*kw + i)*C + c.
__global__ __launch_bounds__(256) void pack_fused_bf16_cl_kernel(Geom g, int Mt16, int KG, const uint16_t* __restrict__ w,
                                                                 uint4* __restrict__ KF)
{
    const long n = (long)Mt16 * KG * 64;
    const int taps = g.kh * g.kw;
    for (long e = (long)blockIdx.x * 256 + threadIdx.x; e < n; e += (long)gridDim.x * 256) {
        const int lane = (int)(e & 63);
        const long gk = e >> 6;
        const int kgroup = (int)(gk % KG), mtile = (int)(gk / KG);
        const int m = mtile * 16 + (lane & 15);
        uint32_t v[4] = {0, 0, 0, 0};
#pragma unroll
        for (int qk = 0; qk < 8; ++qk) {
            const int k = kgroup * 32 + 8 * (lane >> 4) + qk;
            const int tap = k / g.C, c = k - tap * g.C;
            const uint32_t h = (m < g.O && k < g.R) ? w[(size_t)m * g.R + (size_t)c * taps + tap] : 0u;
            v[qk >> 1] |= h << ((qk & 1) * 16);
        }
        KF[e] = make_uint4(v[0], v[1], v[2], v[3]);
    }
}

// Elements per chunk: runs of up to four (float32) / three (bfloat16) horizontally adjacent
// taps per load wherever the filter is wider than one column.  The memory pipeline's cost is
// per load and cache line, not per byte; bfloat16 layers, whose MFMA rate leaves the gather
// as the bound, gain most (1.8x at many listed pixels), float32 layers mainly through the
// three to four times smaller table, which leaves LDS to the B stage when K is long.
int chunk_width(const Geom& g)
{
    if (g.kw == 1) return 1;
    return g.bf16 ? 3 : 4;
}

// The chunk table of a layer (see cb_fused.h), built on the host.
void build_chunks(const Geom& g, int cw, std::vector<int2>& tab, std::vector<int>& ustart)
{
    const int esz = g.bf16 ? 2 : 4;
    const int kk = g.kh * g.kw;
    const int nunits = (g.R + KC - 1) / KC, Rpad = nunits * KC;
    tab.clear();
    ustart.assign(nunits + 1, 0);
    const int rend = (!g.bf16 && cw > 1) ? g.R : Rpad;     // float32 runs: no zero chunks
    for (int r = 0; r < rend;) {
        if (r % KC == 0) ustart[r / KC] = (int)tab.size();
        int len = KC - r % KC;                       // never across a unit
        if (len > cw) len = cw;
        int2 e;
        if (r < g.R) {
            const int c = r / kk, ji = r - c * kk, j = ji / g.kw, i = ji - j * g.kw;
            if (len > g.kw - i) len = g.kw - i;      // never across a filter row
            e.x = (int)(((unsigned)c * (unsigned)g.P + (unsigned)(j * g.W + i)) * (unsigned)esz);
            e.y = r | (len << 16) | (ji << 20);
        } else {
            e.x = 0;
            e.y = r | (len << 16) | (FUSED_ZERO_TAP << 20);
        }
        tab.push_back(e);
        r += len;
    }
    ustart[nunits] = (int)tab.size();
    for (int i = 0; i < FUSED_TAB_PAD; ++i) tab.push_back(make_int2(0, 0));
}

unsigned table_lds_bytes(int ntab, int nunits)
{
    return (((unsigned)ntab + (unsigned)FUSED_TAB_PAD) * 8u + ((unsigned)nunits + 1u) * 4u + 15u) & ~15u;
}

// Largest number of units per stage for a tile of bn columns: the stage must fit the LDS
// window next to the table, and no thread may have to hold more than its register budget
// of chunks, whichever unit the stage starts at.
int stage_units(const Geom& g, int cw, int bn, unsigned tab_lds, const std::vector<int>& ustart)
{
    const int nunits = (int)ustart.size() - 1;
    int gu = (int)((FUSED_LDS_BYTES - tab_lds) / fused_unit_bytes(g.bf16, bn));
    if (gu > nunits) gu = nunits;
    const int room = fused_cps(g.bf16, cw) * (256 / bn);
    while (gu > 1) {
        int worst = 0;
        for (int u = 0; u < nunits; ++u) {
            const int ue = u + gu < nunits ? u + gu : nunits;
            if (ustart[ue] - ustart[u] > worst) worst = ustart[ue] - ustart[u];
        }
        if (worst <= room) break;
        --gu;
    }
    if (gu < 1) gu = 1;
    for (int u = 0; u < nunits; ++u)                 // a single unit must fit in any case
        if (ustart[u + 1] - ustart[u] > room) return 0;
    return gu;
}

}  // namespace

size_t fused_pack_bytes(const Geom& g)
{
    // (bfloat16: padded to 128 rows, the unit of the channel-last kernel)
    const size_t Rpad = g.bf16 ? (size_t)(g.R + 127) / 128 * 128 : (size_t)(g.R + KC - 1) / KC * KC;
    const size_t Mt16 = (size_t)(g.O + 127) / 128 * 8;     // 16-row tiles, padded to the largest row tile
    // 16 bytes per lane per k-group: 16 rows of float32, 32 rows of bfloat16
    return Mt16 * (Rpad / (g.bf16 ? 32 : 16)) * 64 * 16;
}

size_t fused_table_bytes(const Geom& g)
{
    // at most one chunk per row of the padded K, the closing entries, and the unit starts
    const size_t nunits = (size_t)(g.R + KC - 1) / KC;
    return (nunits * KC + FUSED_TAB_PAD) * 8 + (nunits + 1) * 4;
}

bool fused_supported(const Geom& g)
{
    // 32-bit byte offsets into the state (with room for a 16-byte load at the end); one bit
    // per filter tap in a 64-bit word whose top four bits stay clear; the chunk table must
    // fit its LDS window
    const int esz = g.bf16 ? 2 : 4;
    if ((unsigned long long)g.C * g.P * esz > 0xFFFFFF00ull) return false;
    if (g.kh * g.kw > FUSED_ZERO_TAP) return false;
    // chunks: one per run piece; bound without building the table
    const int cw = chunk_width(g);
    const size_t nunits = (size_t)(g.R + KC - 1) / KC;
    const size_t pieces = (size_t)g.C * g.kh * ((g.kw + cw - 1) / cw) + 2 * nunits + KC;
    return table_lds_bytes((int)pieces, (int)nunits) <= (unsigned)FUSED_TAB_LDS_MAX;
}

bool fused_channel_last(const Geom& g)
{
    // (bfloat16 from 32 channels on: change detection stages the shadow rows 16 bytes = 8 channels per lane)
    return g.C >= (g.bf16 ? 32 : 16) && (g.C & (g.C - 1)) == 0 && fused_supported(g);
}

hipError_t fused_prepare(const Geom& g, const void* w, void* KF, void* tab_dev, bool channel_last, hipStream_t st,
                         FusedPlan* plan)
{
    plan->cl = channel_last && fused_channel_last(g);
    // 16-row (float32) / 32-row (bfloat16) groups of K; the channel-last bfloat16 kernel walks K in units of 128 rows
    const int KG = (plan->cl && g.bf16) ? (g.R + 127) / 128 * 4 : (g.R + KC - 1) / KC * KC / (g.bf16 ? 32 : 16);
    const int Mt16 = (g.O + 127) / 128 * 8;
    long n = (long)Mt16 * KG * 64;
    unsigned grid = (unsigned)((n + 255) / 256);
    if (grid > 2048) grid = 2048;
    if (g.bf16 && plan->cl)
        hipLaunchKernelGGL(pack_fused_bf16_cl_kernel, dim3(grid), dim3(256), 0, st, g, Mt16, KG, (const uint16_t*)w,
                           (uint4*)KF);
    else if (g.bf16)
        hipLaunchKernelGGL(pack_fused_bf16_kernel, dim3(grid), dim3(256), 0, st, g, Mt16, KG, (const uint16_t*)w,
                           (uint4*)KF);
    else if (plan->cl)
        hipLaunchKernelGGL(pack_fused_f32_cl_kernel, dim3(grid), dim3(256), 0, st, g, Mt16, KG, (const float*)w,
                           (float4*)KF);
    else
        hipLaunchKernelGGL(pack_fused_f32_kernel, dim3(grid), dim3(256), 0, st, g, Mt16, KG, (const float*)w,
                           (float4*)KF);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (plan->cl) {
        // no table; units per stage from the LDS window and the gather's register budget
        plan->cw = 4;
        plan->ntab = 0;
        plan->nunits = g.bf16 ? (g.R + 127) / 128 : (g.R + KC - 1) / KC;   // 256-byte units of a column
        plan->tab_lds = 0;
        int bm, bns, bnl;
        fused_shape(g.O, bm, bns, bnl);
        auto units = [&](int cap, int pf) {
            int gu = cap < plan->nunits ? cap : plan->nunits;
            const int rounded = gu - gu % pf;    // a multiple of the prefetch depth, unless that costs a stage
            if (rounded >= pf && (plan->nunits + rounded - 1) / rounded == (plan->nunits + gu - 1) / gu) gu = rounded;
            return gu;
        };
        plan->gu_small = units(bns == 64 ? fused_cl_units(64) : bns == 32 ? fused_cl_units(32) : fused_cl_units(16),
                               g.O > 64 ? 2 : 4);
        plan->gu_large = units(bnl == 128 ? fused_cl_units(128) : fused_cl_units(64), 2);
        // (the 32-column tile at any length of K, both element types: a stage change is cheap in this kernel)
        plan->gu_mid = (g.O > 32) ? units(fused_cl_units(32), 2) : 0;
        plan->lds_bytes = FUSED_LDS_BYTES;
        return hipSuccess;                       // nothing built on the host: the packing kernel runs in stream order
    }

    std::vector<int2> tab;
    std::vector<int> ustart;
    plan->cw = chunk_width(g);
    build_chunks(g, plan->cw, tab, ustart);
    plan->ntab = (int)tab.size() - FUSED_TAB_PAD;
    plan->nunits = (int)ustart.size() - 1;
    plan->tab_lds = table_lds_bytes(plan->ntab, plan->nunits);
    if (plan->tab_lds > (unsigned)FUSED_TAB_LDS_MAX || tab.size() * 8 + ustart.size() * 4 > fused_table_bytes(g))
        return hipErrorInvalidValue;
    int bm, bns, bnl;
    fused_shape(g.O, bm, bns, bnl);
    plan->gu_small = stage_units(g, plan->cw, bns, plan->tab_lds, ustart);
    plan->gu_large = stage_units(g, plan->cw, bnl, plan->tab_lds, ustart);
    if (plan->gu_small < 1 || plan->gu_large < 1) return hipErrorInvalidValue;
    // a stage of a multiple of the filter-fragment prefetch depth lets the prefetch run across stages
    // (depth: 4 units where a wavefront owns a single 16x16 tile, else 2)
    const int pf_small = g.O > 64 ? 2 : 4, pf_large = 2;
    auto prefer_multiple = [&](int gu, int pf) {     // ... unless that costs a stage
        const int rounded = gu - gu % pf;
        if (rounded < pf) return gu;
        const int nu = plan->nunits;
        return (nu + rounded - 1) / rounded == (nu + gu - 1) / gu ? rounded : gu;
    };
    plan->gu_small = prefer_multiple(plan->gu_small, pf_small);
    plan->gu_large = prefer_multiple(plan->gu_large, pf_large);
    unsigned a = plan->gu_small * fused_unit_bytes(g.bf16, bns), b = plan->gu_large * fused_unit_bytes(g.bf16, bnl);
    // float32, more than 32 output channels, short K: a 32-column tile between the two.  It
    // halves what a tile's MFMAs read of the filter matrix; it holds a third of the narrow
    // tile's units per stage, which costs more than that gains once K is long (measured:
    // 9 - 14 % faster at K = 576 and 1152 with 12 000 listed pixels, even at K = 2304, 5 - 11 %
    // slower at K = 3136 and 4608).
    plan->gu_mid = 0;
    if (!g.bf16 && g.O > 32 && plan->nunits <= FUSED_MID_UNITS) {
        plan->gu_mid = stage_units(g, plan->cw, 32, plan->tab_lds, ustart);
        if (plan->gu_mid >= 1) {
            plan->gu_mid = prefer_multiple(plan->gu_mid, 2);
            const unsigned c = plan->gu_mid * fused_unit_bytes(false, 32);
            if (c > a) a = c;
        } else
            plan->gu_mid = 0;
    }
    plan->lds_bytes = plan->tab_lds + (a > b ? a : b);
    // table, then the unit starts (the copies are complete when the calls return: pageable source)
    e = hipMemcpyAsync(tab_dev, tab.data(), tab.size() * 8, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) return e;
    e = hipMemcpyAsync((char*)tab_dev + tab.size() * 8, ustart.data(), ustart.size() * 4, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) return e;
    return hipStreamSynchronize(st);
}

hipError_t launch_fused(const Geom& g, const FusedPlan& plan, const void* src, const void* shadow, const int32_t* idx,
                        const int* count, const void* KF, const void* tab, const float* bias, int relu, void* OUT,
                        void* OUT2, hipStream_t st, Tm tm)
{
    if (OUT2 && (g.O & 15) != 0) return hipErrorInvalidValue;
    if (plan.cl) {
        if (!shadow) return hipErrorInvalidValue;
        if (g.bf16)
            return launch_fused_bf16_cl(g, plan, (const uint16_t*)shadow, idx, count, KF, bias, relu, (uint16_t*)OUT,
                                        (uint16_t*)OUT2, st, tm);
        return launch_fused_f32_cl(g, plan, (const float*)shadow, idx, count, KF, bias, relu, (float*)OUT, (float*)OUT2, st, tm);
    }
    if (g.bf16)
        return launch_fused_bf16(g, plan, (const uint16_t*)src, idx, count, KF, (const int2*)tab, bias, relu,
                                 (uint16_t*)OUT, (uint16_t*)OUT2, st, tm);
    return launch_fused_f32(g, plan, (const float*)src, idx, count, KF, (const int2*)tab, bias, relu, (float*)OUT,
                            (float*)OUT2, st, tm);
}

}  // namespace cb
