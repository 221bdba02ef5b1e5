// Shared definitions of the fused back end (matrix generation, matrix
// multiplication and output update of Sec. III-A in one kernel): tile shapes,
// the chunk table that drives the gather, and the device
// helpers both element types use.
#pragma once
#include "cb_kernels.h"

namespace cb {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

constexpr int KC = 64;                  // rows of K per unit of the LDS stage
constexpr int FUSED_LARGE_N = 16384;    // from this many listed pixels on, the wide column tile is used
constexpr int FUSED_MID_TILES = 512;    // float32, short K: above this many narrow tiles (and below FUSED_LARGE_N pixels) a 32-column tile is used
constexpr int FUSED_MID_UNITS = 24;     // ... "short K": at most this many 64-row units
constexpr int FUSED_LDS_BYTES = 64 * 1024;   // dynamic LDS per workgroup: two workgroups per compute unit
constexpr int FUSED_TAB_LDS_MAX = 40 * 1024; // largest chunk table kept in LDS
constexpr int FUSED_GUARD = 128;        // bytes readable ahead of the gather source (pad <= 31 elements of 4 bytes)
constexpr int FUSED_ZERO_TAP = 60;      // tap index of the zero rows that pad K (never inside the image)
constexpr int FUSED_TAB_PAD = 64;       // entries of length 0 that close the chunk table: a group of gather rounds (up to 4 rounds of 16 fetchers) may read this far past the last chunk

// Channel-last variant (C a power of two: >= 16 float32, >= 32 bfloat16; layers that keep an input state): the
// gather reads a pixel-major shadow of the state, K is walked tap-major, no chunk table.
constexpr int FUSED_CL_LOADS = 12;      // 16-byte gather loads a thread holds per stage at most
// floats per column of its B stage ([n][k'] in LDS) for a tile of bn columns: the LDS window
// divided by the columns, less 28, which makes the pitch 4 mod 32 (conflict-free 16-byte reads)
__host__ __device__ constexpr int fused_cl_pitch(int bn) { return FUSED_LDS_BYTES / (bn * 4) - 28; }
__host__ __device__ constexpr int fused_cl_units(int bn)
{
    return fused_cl_pitch(bn) / KC < FUSED_CL_LOADS / (bn / 16) ? fused_cl_pitch(bn) / KC : FUSED_CL_LOADS / (bn / 16);
}

// Chunk table.  The rows of X' that belong to one input channel c and one filter row j,
// r = (c*kh + j)*kw + i for i = 0..kw-1 (construction of X below Eq. 2), are kw consecutive
// elements of the input state for every listed pixel.  A chunk is a piece of such a run --
// at most CW elements, never crossing a 64-row unit -- that a lane fetches with ONE load
// (up to 16 bytes) and then writes to 1..CW rows of the LDS tile.  The memory pipeline's
// cost is per load instruction and cache line touched, not per byte, so this is what
// bounds the gather.  Entry: .x = byte offset of the chunk's first element relative to
// the top-left element of the receptive field, .y = first row | length << 16 | first tap
// (j*kw + i) << 20.  Rows beyond R (K is padded to a multiple of 64) are zero chunks with
// tap FUSED_ZERO_TAP -- except in the float32 table of runs, which ends at row R: that
// kernel clears the padding rows of the last unit itself.  ustart[u] = index of the first
// chunk of unit u; FUSED_TAB_PAD entries of length 0 and offset 0 close the table.
struct FusedPlan {
    bool cl = false;            // channel-last variant: gathers from the pixel-major shadow of the state
    int cw = 1;                 // elements per chunk at most: 1, 4 (float32) or 3 (bfloat16)
    int ntab = 0;               // chunks, without the sentinel
    int nunits = 0;
    int gu_small = 1, gu_large = 1;   // units per LDS stage for the narrow and the wide column tile
    int gu_mid = 0;             // ... and for the 32-column tile of the float32 kernel (0: the layer does not use it)
    unsigned tab_lds = 0;       // bytes of table + ustart in LDS (16-byte multiple)
    unsigned lds_bytes = 0;     // dynamic LDS of the launch
};

// rows / narrow-tile columns / wide-tile columns of the workgroup tile used for O output channels
__host__ __device__ inline void fused_shape(int O, int& bm, int& bn_small, int& bn_large)
{
    if (O <= 16)      { bm = 16;  bn_small = 64; bn_large = 128; }
    else if (O <= 32) { bm = 32;  bn_small = 32; bn_large = 64; }
    else if (O <= 64) { bm = 64;  bn_small = 16; bn_large = 64; }
    else              { bm = 128; bn_small = 16; bn_large = 64; }
}
// Whether tiles of half the rows (bm / 2) finish a frame of N listed pixels sooner than tiles
// of bm rows: the kernel takes as long as the compute unit with the most tiles, a half tile
// costs a little over half (the gather is repeated per row tile).
__host__ __device__ inline bool fused_half_rows(int N, int O, int bn, int bm)
{
    const long nt = (N + bn - 1) / bn;
    const long full = nt * ((O + bm - 1) / bm), half = nt * ((O + bm / 2 - 1) / (bm / 2));
    const long cu = 256;
    return ((half + cu - 1) / cu) * 11 < ((full + cu - 1) / cu) * 20;
}
// chunks a thread can hold per stage (register budget of the gather)
__host__ __device__ constexpr int fused_cps(bool bf16, int cw) { return cw == 1 ? 64 : (bf16 ? 32 : 18); }
// bytes of one 64-row unit of the B stage in LDS for a tile of bn columns
__host__ __device__ constexpr unsigned fused_unit_bytes(bool bf16, int bn)
{
    return bf16 ? (unsigned)bn * (KC + 8) * 2u : (unsigned)KC * (unsigned)(bn + (bn % 32 == 16 ? 0 : 16)) * 4u;
}

#if defined(__HIPCC__)
// One bit per filter tap t = j*kw + i of a listed pixel: set when the tap lies inside the
// image.  Bits from kh*kw on are 0 (FUSED_ZERO_TAP among them); all 0 for a lane without pixel.
__device__ __forceinline__ unsigned long long taps_inside(const Geom& g, bool colv, int y0, int x0)
{
    unsigned long long ok = 0;
    if (colv) {
        unsigned colok = 0;
        for (int i = 0; i < g.kw; ++i) colok |= ((unsigned)(x0 + i) < (unsigned)g.W ? 1u : 0u) << i;
        for (int j = 0; j < g.kh; ++j)
            if ((unsigned)(y0 + j) < (unsigned)g.H) ok |= (unsigned long long)colok << (j * g.kw);
    }
    return ok;
}
// all ones when bit e of m is set
__device__ __forceinline__ unsigned bit_ones(unsigned m, unsigned e) { return (unsigned)__builtin_amdgcn_sbfe((int)m, e, 1u); }

// float32 -> bfloat16 bit pattern, round to nearest even (NaN stays NaN)
__device__ __forceinline__ uint16_t bf16_bits(float v)
{
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ void st_out(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_out(uint16_t* p, float v) { *p = bf16_bits(v); }
// Four consecutive output channels of one pixel into the pixel-major copy of the cached output
// (p is 16- / 8-byte aligned: the first channel is a multiple of four, and so is the channel count).
__device__ __forceinline__ void st_out4(float* p, const float (&v)[4])
{
    *reinterpret_cast<floatx4*>(p) = floatx4{v[0], v[1], v[2], v[3]};
}
__device__ __forceinline__ void st_out4(uint16_t* p, const float (&v)[4])
{
    *reinterpret_cast<uintx2*>(p) = uintx2{(unsigned)bf16_bits(v[0]) | ((unsigned)bf16_bits(v[1]) << 16),
                                           (unsigned)bf16_bits(v[2]) | ((unsigned)bf16_bits(v[3]) << 16)};
}
#endif

// Layer-creation side: availability, buffer sizes, packing of the filter matrix into MFMA
// fragment order, the chunk table and the launch plan (synchronises the stream once when it uploads a chunk
// table, i.e. for the channel-first kernels).
bool fused_supported(const Geom& g);
// whether a layer of this geometry that keeps an input state uses the channel-last variant
bool fused_channel_last(const Geom& g);
size_t fused_pack_bytes(const Geom& g);
size_t fused_table_bytes(const Geom& g);
hipError_t fused_prepare(const Geom& g, const void* w, void* KF, void* tab_dev, bool channel_last, hipStream_t st,
                         FusedPlan* plan);
// src: the channel-first source of the gather (input state, or a producer's output); shadow: the
// pixel-major copy of that source (used, and required, when plan.cl is set); OUT2: null, or the
// pixel-major copy of the cached output (Po x O; O a multiple of 16), which receives the same updates as OUT
hipError_t launch_fused(const Geom& g, const FusedPlan& plan, const void* src, const void* shadow, const int32_t* idx,
                        const int* count, const void* KF, const void* tab, const float* bias, int relu, void* OUT,
                        void* OUT2, hipStream_t st, Tm tm = Tm());

// launches of the two element types (cb_fused_f32.hip, cb_fused_bf16.hip, cb_fused_cl.hip)
hipError_t launch_fused_f32(const Geom& g, const FusedPlan& plan, const float* src, const int32_t* idx,
                            const int* count, const void* KF, const int2* tab, const float* bias, int relu,
                            float* OUT, float* OUT2, hipStream_t st, Tm tm);
hipError_t launch_fused_f32_cl(const Geom& g, const FusedPlan& plan, const float* shadow, const int32_t* idx,
                               const int* count, const void* KF, const float* bias, int relu, float* OUT, float* OUT2,
                               hipStream_t st, Tm tm);
hipError_t launch_fused_bf16_cl(const Geom& g, const FusedPlan& plan, const uint16_t* shadow, const int32_t* idx,
                                const int* count, const void* KF, const float* bias, int relu, uint16_t* OUT, uint16_t* OUT2,
                                hipStream_t st, Tm tm);
hipError_t launch_fused_bf16(const Geom& g, const FusedPlan& plan, const uint16_t* src, const int32_t* idx,
                             const int* count, const void* KF, const int2* tab, const float* bias, int relu,
                             uint16_t* OUT, uint16_t* OUT2, hipStream_t st, Tm tm);

}  // namespace cb
