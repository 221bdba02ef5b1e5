// Internal launcher interface between the C-ABI layer (cbconv.hip) and the
// gfx950 kernels.  Plain pointers and sizes only; every launcher enqueues on the
// given stream and returns the hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace cb {

// Optional pair of events that receive the begin and end time stamps of one
// kernel dispatch (per-step timing); null events make this a plain launch.
struct Tm {
    hipEvent_t start = nullptr, stop = nullptr;
};
#define CB_LAUNCH(kernel, grid, block, st, tm, ...) \
    hipExtLaunchKernelGGL(kernel, grid, block, 0, st, (tm).start, (tm).stop, 0, __VA_ARGS__)

// Geometry shared by all kernels of one layer (passed by value).
struct Geom {
    int C, O, kh, kw, s, p;
    int H, W, Ho, Wo;
    int P, Po;        // H*W, Ho*Wo
    int R;            // C*kh*kw
    int WWo;          // 64-bit words per output row of the bit-packed dilated map
    int Opad;         // O rounded up to 16: row pitch of the transposed filter matrix
    int bf16;         // element type: 0 float, 1 bfloat16 bit patterns
};

// Small device-resident control block of a layer (int32 slots).
enum Ctl {
    CTL_COUNT = 0,     // N of the current frame
    CTL_NIN_A = 1,     // changed-input counter, even frames
    CTL_NIN_B = 2,     // changed-input counter, odd frames
    CTL_LD = 3,        // leading dimension of X'/Y' of the last chunk
    CTL_NCOLS = 4,     // columns of the last chunk
    CTL_NSPLIT = 5,    // k-splits (partial products stacked in Y') of the last chunk
    CTL_DONE = 7,      // single-pass dilate + compact: workgroups that have finished
    CTL_EPOCH = 8,     //   epoch of the last completed launch
    CTL_FRAME = 10,    // frames processed by a layer that detects its own changes: its parity selects the input-map
                       //   buffer and the changed-pixel counter of the frame (advanced by the index extraction)
    CTL_RECOUNTS = 9,  //   predecessor counts a workgroup recomputed itself after its bounded wait ran out
    CTL_SLOTS = 64
};

// flags for detect
enum { DET_FORCE_ALL = 1,      // mark every pixel as changed (first frame)
       DET_COPY_ALL = 2,       // copy every pixel into the state (feed-forward)
       DET_STREAM_STATE = 4,   // the state is larger than the caches hold from one frame to the next: read it
                               // non-temporally too (1080p, 128 channels: 374 -> 318 us; a state that fits loses)
       DET_NO_UPDATE = 8 };    // compare and write the map only; launch_state_apply updates the state (and shadow)

// S2: null, or the channel-last shadow of the state (pixel-major, C values per pixel; C >= 16), which
// receives the same updates as S.
// mbits: the layer's two input maps, used by alternate frames and interleaved word by word (64-bit word w
// of the map of frame parity p at index 2*w + p: the index extraction, which does not know p when it
// starts, fetches both candidates with one 16-byte load); the frame count in ctl[CTL_FRAME] selects
// the map this frame fills and the changed-pixel counter it adds to.
hipError_t launch_detect(const Geom& g, const void* x, void* S, void* S2, uint64_t* mbits, int* ctl,
                         float tau, int flags, hipStream_t st, Tm tm = Tm());

// The state update of a frame whose detection ran with DET_NO_UPDATE (same stream, before the index
// extraction of that frame): copies the marked pixels of x into S and, if not null, the shadow S2.
hipError_t launch_state_apply(const Geom& g, const void* x, void* S, void* S2, const uint64_t* mbits, const int* ctl,
                              hipStream_t st, Tm tm = Tm());

// S2 = the channel-last copy of the whole state S (for a state that was written from outside).
hipError_t launch_shadow_rebuild(const Geom& g, const void* S, void* S2, hipStream_t st);

// Eq. 3 restricted to candidate pixels: the entries of a producer's index list (mapped through
// a w x w pooling stage when pool_w > 1: cand_W = the producer's output width); cand_cap = readable
// entries of the list (its count lives on the device).  Pixels that are not candidates keep their
// state and their (cleared) bit; the selected map must be all zero on entry.
hipError_t launch_detect_listed(const Geom& g, const void* x, void* S, void* S2, uint64_t* mbits, int* ctl,
                                float tau, int flags, const int32_t* cand, const int* cand_count, int cand_cap,
                                int pool_w, int cand_W, hipStream_t st, Tm tm = Tm());

// Dilation of a bit-packed map by the filter footprint + per-block popcounts.  own_map != 0: in_bits
// holds the layer's two interleaved input maps (see launch_detect); the frame count on the device
// selects the one to use, and housekeeping for the next frame rides along: the other map
// (clear_words words) and the other changed-pixel counter are zeroed, and the index extraction
// advances the frame count.  own_map == 0: in_bits is one plain map (a producer's).
// in_pitch_bits: bit distance between consecutive rows of the input map
// (W for the linear map written by detect, 64*words for a row-padded map).
hipError_t launch_dilate(const Geom& g, const uint64_t* in_bits, long in_pitch_bits, int full,
                         uint64_t* mt_bits, int* blk_cnt, int* ctl, int own_map, int clear_words, hipStream_t st,
                         Tm tm = Tm());
int dilate_num_blocks(const Geom& g);
// Maps small enough for the one-workgroup, one-launch dilate + compact kernel.
bool compact_single_launch(const Geom& g);
hipError_t launch_dilate_compact_small(const Geom& g, const uint64_t* in_bits, long in_pitch_bits,
                                       int full, uint64_t* mt_bits, int32_t* idx, int* ctl, int own_map,
                                       int clear_words, hipStream_t st, Tm tm = Tm());

// Maps of a size the single-pass kernel handles (dilation, scan, index list and N in one launch of
// many workgroups); `look` = compact_one_pass_bytes(g) bytes of the layer's own, zero-initialised
// state that no other layer touches (the kernel keeps epochs there between launches).  spin_limit: polls
// of a predecessor's count before a workgroup recomputes that count itself (the result is the same).
bool compact_one_pass(const Geom& g);
size_t compact_one_pass_bytes(const Geom& g);
hipError_t launch_dilate_compact(const Geom& g, const uint64_t* in_bits, long in_pitch_bits, int full,
                                 uint64_t* mt_bits, int32_t* idx, int* ctl, uint64_t* look, int own_map,
                                 int clear_words, int spin_limit, hipStream_t st, Tm tm = Tm());

// Ordered expansion of the dilated bit map into the index list; writes N.
hipError_t launch_compact(const Geom& g, const uint64_t* mt_bits, const int* blk_cnt,
                          int32_t* idx, int* ctl, int own_map, hipStream_t st, Tm tm = Tm());

// Matrix generation for columns [col0, col0+cap) of the index list.
hipError_t launch_gather(const Geom& g, const void* src, const int32_t* idx, const int* count,
                         int col0, int cap, void* X, int* ctl, hipStream_t st, Tm tm = Tm());

// Y' = K X' on the chunk; KT is the transposed filter matrix (R x Opad).
hipError_t launch_gemm(const Geom& g, const void* KT, const void* X, void* Y, const int* count,
                       int col0, int cap, int* ctl, hipStream_t st, Tm tm = Tm());

// Tile shape of the GEMM for a layer with O output channels, and the number of
// k-splits it uses for a chunk of ncols columns (the output update sums the
// partial products in a fixed order, so results do not depend on scheduling).
__host__ __device__ inline int gemm_bm(int O) { return O <= 16 ? 16 : (O <= 32 ? 32 : 64); }
__host__ __device__ inline int gemm_bn(int O) { return O <= 16 ? 256 : (O <= 32 ? 128 : 64); }
__host__ __device__ inline int gemm_nsplit(int ncols, int R, int O, int Opad, int cap)
{
    const int bm = gemm_bm(O), bn = gemm_bn(O);
    const int ld = (ncols + 255) & ~255;
    const int tiles = ((ncols + bn - 1) / bn) * (Opad / bm);
    int s = 512 / tiles;                 // aim at two workgroups per compute unit
    if (s > 8) s = 8;
    if (s > R / 128) s = R / 128;        // at least 128 rows of K per split
    if (s > cap / ld) s = cap / ld;      // partial products must fit the Y' buffer
    return s < 1 ? 1 : s;
}

// Output update with fused bias and ReLU for the chunk.
hipError_t launch_update(const Geom& g, const void* Y, const float* bias, const int32_t* idx,
                         const int* count, int col0, int cap, int relu, void* OUT, hipStream_t st, Tm tm = Tm());

// Change-based max-pool of window w (stride w, ceil mode): the pooled cells of the listed pixels; idx == null: all cells.
// POOL2: null, or a pixel-major copy of the pooled output that receives the same values.
hipError_t launch_pool(int O, int Ho, int Wo, int w, int bf16, const void* OUT, const int32_t* idx,
                       const int* count, void* POOL, void* POOL2, hipStream_t st);
// Pooled change map (row-padded bit words) from the producer's dilated map.
hipError_t launch_pool_mask(int Ho, int Wo, int WWo, int w, const uint64_t* mt_bits,
                            uint64_t* pm_bits, hipStream_t st);

// Bit map -> byte map (0/1).  pitch_bits as for launch_dilate.
hipError_t launch_expand_bits(const uint64_t* bits, long pitch_bits, int H, int W, uint8_t* bytes,
                              hipStream_t st);
// ... of the input map of the last frame of a layer that detects its own changes (two interleaved maps)
hipError_t launch_expand_own_map(const uint64_t* bits0, const int* ctl, long pitch_bits, int H, int W,
                                 uint8_t* bytes, hipStream_t st);
// Repack O x R filter matrix into R x Opad (zero padded), bias into float.
hipError_t launch_pack_weights(const Geom& g, const void* w, const void* bias, void* KT,
                               float* bias_f, hipStream_t st);
// acc[0] = (accumulate ? acc[0] : 0) + sum over i < n of (a[i] - b[i])^2 in float64, in a fixed order;
// partial: SSD_PARTIALS doubles.
constexpr int SSD_PARTIALS = 256;
hipError_t launch_ssd(const void* a, const void* b, size_t n, int bf16, double* partial, double* acc, int accumulate,
                      hipStream_t st);
// The current device's copy of the library's own, statically allocated metric scratch (partial sums and
// total), for the entry point that must not allocate.  Looked up once per device.
hipError_t ssd_static_scratch(double** partial, double** acc);
// Fill n 32-bit words with v (used instead of memset on paths that may be captured).
hipError_t launch_fill32(uint32_t* p, size_t n, uint32_t v, hipStream_t st);

}  // namespace cb
