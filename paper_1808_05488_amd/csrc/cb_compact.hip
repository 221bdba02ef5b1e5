// Change-map dilation by the filter footprint (Sec. III-A Eq. 4) and change-index
// extraction (Sec. III-A, "Change Indexes Extraction"), on bit-packed maps.
//
// The paper sets the k x k neighbourhood of every changed pixel (scatter form)
// and compacts with a library stream-compaction call.  Here the map is held as
// 64-pixel words: one thread produces one word of the dilated map from at most
// three input words per filter row (shifts and ORs), the words' popcounts are
// scanned (wavefront shuffles + LDS), and set bits are expanded into the ordered
// index list a word at a time by a whole wavefront (one-workgroup kernel: by its lane).  Two kernels, no atomics on
// the ordering path, so the list is strictly ascending by construction.
//
//   dilate_kernel : word (yo, wo) of the dilated map + per-block popcount
//   compact_kernel: block prefix over the popcounts, in-block scan, index write, N
//   dilate_compact_small_kernel: both in one workgroup, for maps of up to 1024 words
//                   (launch latency, not work, is what these steps cost there)
//   dilate_compact_kernel: both in one launch of many workgroups (single-pass scan), for
//                   maps of up to 262 144 words; the two-kernel form remains for larger ones
#include "cb_kernels.h"

namespace cb {

namespace {

struct U128 { uint64_t lo, hi; };

// 64-bit word wi of a bit map.  OWN: `w` holds the two input maps of a layer that detects its own
// changes, interleaved word by word (word wi of the map of frame parity p at index 2*wi + p).  One
// 16-byte load brings word wi of both; sel (the frame parity, which may still be on its way from
// memory when the load is issued) picks.  Otherwise `w` is one plain map.
template <bool OWN>
__device__ __forceinline__ uint64_t map_word(const uint64_t* __restrict__ w, long wi, int sel)
{
    if (OWN) {
        const ulonglong2 p = reinterpret_cast<const ulonglong2*>(w)[wi];
        return (sel & 1) ? p.y : p.x;
    }
    return w[wi];
}

// 128 bits starting at absolute bit position `bit` of a map that has at least two words of zero
// slack after its last used word.  Always three loads, no branch.
template <bool OWN>
__device__ __forceinline__ U128 read128(const uint64_t* __restrict__ w, long bit, int sel)
{
    const long wi = bit >> 6;
    const int sh = (int)(bit & 63);
    const uint64_t a = map_word<OWN>(w, wi, sel), b = map_word<OWN>(w, wi + 1, sel), c = map_word<OWN>(w, wi + 2, sel);
    const uint64_t bl = sh ? (b << (64 - sh)) : 0ull, cl = sh ? (c << (64 - sh)) : 0ull;
    return U128{(a >> sh) | bl, (b >> sh) | cl};
}

// Columns [x0, x0+128) of one row of a bit map as a 128-bit value (bit q =
// column x0+q); columns outside [0, W) read as zero, and so does everything when
// `valid` is false.  -63 <= x0.  Straight-line code: the loads of several rows can
// be in flight together.
template <bool OWN>
__device__ __forceinline__ U128 row_window(const uint64_t* __restrict__ bits, long rowstart, int W, int x0,
                                           bool valid, int sel)
{
    int a = x0 > 0 ? x0 : 0;
    const int pre = a - x0;
    int len = (x0 + 128 < W ? x0 + 128 : W) - a;
    if (a > W - 1) a = W - 1;                          // keep the address inside the row; len <= 0 masks it
    U128 v = read128<OWN>(bits, rowstart + a, sel);
    if (!valid) len = 0;
    const uint64_t mlo = len >= 64 ? ~0ull : (len > 0 ? (1ull << len) - 1ull : 0ull);
    const uint64_t mhi = len >= 128 ? ~0ull : (len > 64 ? (1ull << (len - 64)) - 1ull : 0ull);
    v.lo &= mlo;
    v.hi &= mhi;
    if (pre) { v.hi = (v.hi << pre) | (v.lo >> (64 - pre)); v.lo <<= pre; }
    return v;
}

template <bool OWN>
__device__ __forceinline__ bool test_bit(const uint64_t* __restrict__ bits, long bit, int sel)
{
    return (map_word<OWN>(bits, bit >> 6, sel) >> (bit & 63)) & 1ull;
}

// One word of the dilated map: output row yo, columns 64*wo .. 64*wo+63.
template <bool OWN>
__device__ __forceinline__ uint64_t dilated_word_t(const Geom& g, const uint64_t* __restrict__ in_bits, long pitch,
                                                   int yo, int wo, int sel)
{
    const int nvalid = g.Wo - 64 * wo < 64 ? g.Wo - 64 * wo : 64;
    const uint64_t vmask = nvalid == 64 ? ~0ull : ((1ull << nvalid) - 1ull);
    uint64_t word = 0;
    if (g.s == 1) {
        // filter rows in batches of four: their twelve loads are issued before the first use
        for (int j0 = 0; j0 < g.kh; j0 += 4) {
            U128 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int yi = yo - g.p + j0 + u;
                const bool valid = j0 + u < g.kh && yi >= 0 && yi < g.H;
                const int yc = yi < 0 ? 0 : (yi >= g.H ? g.H - 1 : yi);
                v[u] = row_window<OWN>(in_bits, (long)yc * pitch, g.W, 64 * wo - g.p, valid, sel);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                uint64_t h = v[u].lo;
                for (int i = 1; i < g.kw; ++i) h |= (v[u].lo >> i) | (v[u].hi << (64 - i));
                word |= h;
            }
        }
        return word & vmask;
    }
    for (int j = 0; j < g.kh; ++j) {
        const int yi = yo * g.s - g.p + j;
        if (yi < 0 || yi >= g.H) continue;
        const long rowstart = (long)yi * pitch;
        for (int b = 0; b < nvalid; ++b) {
            const int xb = (64 * wo + b) * g.s - g.p;
            bool any = false;
            for (int i = 0; i < g.kw; ++i) {
                const int xi = xb + i;
                if (xi >= 0 && xi < g.W && test_bit<OWN>(in_bits, rowstart + xi, sel)) any = true;
            }
            word |= (uint64_t)any << b;
        }
    }
    return word & vmask;
}

// own_map: in_bits holds the layer's two interleaved input maps and sel is the frame parity
__device__ __forceinline__ uint64_t dilated_word(const Geom& g, const uint64_t* __restrict__ in_bits, long pitch,
                                                 int yo, int wo, int own_map, int sel)
{
    return own_map ? dilated_word_t<true>(g, in_bits, pitch, yo, wo, sel)
                   : dilated_word_t<false>(g, in_bits, pitch, yo, wo, 0);
}


// Inclusive prefix sum over the 64 lanes of a wavefront with data-parallel-primitive moves: shifts by
// 1, 2, 4, 8 inside each row of 16 lanes, then lane 15 of a row broadcast into the next row and lane 31
// into the upper half (lanes without a source add 0).  Six register-to-register steps; the same scan
// through general shuffles costs six LDS round trips.
__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
    return v;
}
// ... and the sum over the wavefront, in every lane: the last lane of that scan
__device__ __forceinline__ int wave_sum(int v) { return __builtin_amdgcn_readlane(wave_inclusive_scan(v), 63); }

// Index-list entries of the 64 words held by a wavefront (word, its exclusive offset, the
// pixel index of its bit 0).  PER_LANE = false: the whole wavefront expands one non-empty word
// at a time (coalesced stores, a handful of cross-lane reads per word) -- the faster form
// when the words are spread over many compute units.  PER_LANE = true: every lane walks the
// bits of its own word, no cross-lane traffic -- the faster form in the one-workgroup kernel,
// where sixteen wavefronts share one compute unit's cross-lane hardware.
template <bool PER_LANE>
__device__ __forceinline__ void expand_words(uint64_t word, int off, int pixbase, int32_t* __restrict__ idx, int lane)
{
    if (PER_LANE) {
        while (word) {
            idx[off++] = pixbase + __builtin_ctzll(word);
            word &= word - 1;
        }
        return;
    }
    uint64_t nz = __ballot(word != 0);
    const uint64_t below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    while (nz) {
        // (nz comes from a ballot, so src is the same in every lane: plain lane reads into scalar registers,
        // not the cross-lane permutes of a general shuffle, which cost an LDS round trip each)
        const int src = __ffsll((long long)nz) - 1;
        nz &= nz - 1;
        const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)word, src);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(word >> 32), src);
        const uint64_t wsrc = ((uint64_t)hi << 32) | lo;
        const int o = __builtin_amdgcn_readlane(off, src);
        const int pb = __builtin_amdgcn_readlane(pixbase, src);
        if ((wsrc >> lane) & 1ull) idx[o + __popcll(wsrc & below)] = pb + lane;
    }
}

// A layer that detects its own changes keeps two input maps (interleaved word by word, see
// map_word) and two changed-pixel counters, used by alternate frames: change detection fills the
// pair that the frame count on the device (CTL_FRAME, advanced by the index extraction once per
// frame) selects, and the index extraction clears the other pair for the next frame.  Nothing about
// this lives on the host, so captured launches replay correctly whatever the number of frames in a
// capture.  A layer that takes its map from its producer (own_map == 0) has one plain map and
// nothing to clear.
__device__ __forceinline__ int frame_parity(const int* ctl, int own_map) { return own_map ? (ctl[CTL_FRAME] & 1) : 0; }
// the other map and the other counter start the next frame empty
__device__ __forceinline__ void clear_other_map(uint64_t* maps, int par, int clear_words, int first, int step)
{
    for (int i = first; i < clear_words; i += step) maps[2 * i + (par ^ 1)] = 0;
}

__global__ __launch_bounds__(256) void dilate_kernel(Geom g, const uint64_t* __restrict__ in_bits,
                                                     long pitch, int full, uint64_t* __restrict__ mt_bits,
                                                     int* __restrict__ blk_cnt, int* __restrict__ ctl, int own_map,
                                                     int clear_words)
{
    __shared__ int wsum[4];
    const int items = g.Ho * g.WWo;
    const int it = blockIdx.x * 256 + threadIdx.x;
    const int par = frame_parity(ctl, own_map);
    const int clear_slot = own_map ? CTL_NIN_A + (par ^ 1) : -1;
    uint64_t word = 0;
    if (it < items) {
        const int yo = it / g.WWo, wo = it - yo * g.WWo;
        if (full) {
            const int nvalid = g.Wo - 64 * wo < 64 ? g.Wo - 64 * wo : 64;
            word = nvalid == 64 ? ~0ull : ((1ull << nvalid) - 1ull);
        } else {
            word = dilated_word(g, in_bits, pitch, yo, wo, own_map, par);
        }
        mt_bits[it] = word;
    }
    if (own_map) clear_other_map(const_cast<uint64_t*>(in_bits), par, clear_words, it, (int)gridDim.x * 256);
    int s = wave_sum(__popcll(word));
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        blk_cnt[blockIdx.x] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
        if (blockIdx.x == 0 && clear_slot >= 0) ctl[clear_slot] = 0;
    }
}

__global__ __launch_bounds__(256) void compact_kernel(Geom g, const uint64_t* __restrict__ mt_bits,
                                                      const int* __restrict__ blk_cnt,
                                                      int32_t* __restrict__ idx, int* __restrict__ ctl, int own_map)
{
    __shared__ int red[4];
    __shared__ int wtot[4];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int items = g.Ho * g.WWo;

    // exclusive prefix of the counts of all earlier blocks
    int part = 0;
    for (int b = tid; b < (int)blockIdx.x; b += 256) part += blk_cnt[b];
    part = wave_sum(part);
    if (lane == 0) red[wv] = part;

    const int it = blockIdx.x * 256 + tid;
    uint64_t word = 0;
    int pixbase = 0;
    if (it < items) {
        word = mt_bits[it];
        const int yo = it / g.WWo, wo = it - yo * g.WWo;
        pixbase = yo * g.Wo + 64 * wo;
    }
    const int cnt = __popcll(word);
    const int inc = wave_inclusive_scan(cnt);                  // inclusive scan inside the wavefront
    if (lane == 63) wtot[wv] = inc;
    __syncthreads();
    int off = red[0] + red[1] + red[2] + red[3];
    for (int q = 0; q < wv; ++q) off += wtot[q];
    off += inc - cnt;                       // exclusive offset of this thread's word

    if (blockIdx.x == gridDim.x - 1 && tid == 255) {
        ctl[CTL_COUNT] = off + cnt;
        if (own_map) ctl[CTL_FRAME] = ctl[CTL_FRAME] + 1;     // (the dilation kernel, which read it, is complete)
    }

    expand_words<false>(word, off, pixbase, idx, lane);
}

// Dilation, scan and index write in ONE launch for maps of up to ONE_PASS_MAX_BLOCKS x 256 words.
// The scan over workgroups is a single-pass one: every workgroup publishes the popcount of its 256
// words and then adds up what its predecessors published, so nobody waits for a chain of prefixes.
// Progress: a workgroup publishes its own count before it waits for anybody, and it only waits for
// workgroups with lower numbers, which were dispatched no later than itself and publish before they
// wait in turn; on an idle GPU the whole grid (at most 1024 workgroups of 256 threads, a few dozen
// registers, 40 bytes of LDS) is resident at once anyway.  Correctness does not rest on either: the
// wait is bounded (spin_limit polls per predecessor), and a thread whose wait runs out -- other
// streams or processes may hold the compute units the predecessor is waiting for -- recomputes that
// predecessor's count itself from the input map (recount_block), which needs nobody else.  The list
// and N are therefore the same whatever the scheduling; CTL_RECOUNTS only counts how often that
// happened.  Published counts carry the launch's epoch in their upper half, so the slots never need
// clearing; the last workgroup to finish stores the epoch in device memory for the next launch
// (nothing launch-specific comes from the host, so a captured launch can be replayed).
constexpr int ONE_PASS_MAX_BLOCKS = 1024;

// Number of set bits in workgroup b's 256 words of the dilated map, from the input map alone.
// (inlined: a call would give the kernel a stack, and with it a slower launch, for a path that an idle GPU never takes)
__device__ __forceinline__ int recount_block(const Geom& g, const uint64_t* __restrict__ in_bits, long pitch, int full,
                                          int b, int own_map, int par)
{
    const int items = g.Ho * g.WWo;
    const int hi = b * 256 + 256 < items ? b * 256 + 256 : items;
    int total = 0;
    for (int it = b * 256; it < hi; ++it) {
        const int yo = it / g.WWo, wo = it - yo * g.WWo;
        if (full) total += g.Wo - 64 * wo < 64 ? g.Wo - 64 * wo : 64;
        else total += __popcll(dilated_word(g, in_bits, pitch, yo, wo, own_map, par));
    }
    return total;
}

__global__ __launch_bounds__(256) void dilate_compact_kernel(Geom g, const uint64_t* __restrict__ in_bits,
                                                             long pitch,
                                                             int full, uint64_t* __restrict__ mt_bits,
                                                             int32_t* __restrict__ idx, int* __restrict__ ctl,
                                                             unsigned long long* __restrict__ look, int own_map,
                                                             int clear_words, int spin_limit)
{
    // (needed only after the map words have been requested: both candidates come with one load)
    const int par = frame_parity(ctl, own_map);
    const int clear_slot = own_map ? CTL_NIN_A + (par ^ 1) : -1;
    __shared__ unsigned s_epoch;
    __shared__ int wtot[4];
    __shared__ int red[4];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int items = g.Ho * g.WWo;
    const int nblk = (int)gridDim.x;
    // written by the previous launch's last workgroup; the load is in flight during the dilation
    unsigned epoch_ld = tid == 0 ? (unsigned)ctl[CTL_EPOCH] : 0u;
    const int bid = (int)blockIdx.x;

    const int it = bid * 256 + tid;
    uint64_t word = 0;
    int pixbase = 0;
    if (it < items) {
        const int yo = it / g.WWo, wo = it - yo * g.WWo;
        if (full) {
            const int nvalid = g.Wo - 64 * wo < 64 ? g.Wo - 64 * wo : 64;
            word = nvalid == 64 ? ~0ull : ((1ull << nvalid) - 1ull);
        } else {
            word = dilated_word(g, in_bits, pitch, yo, wo, own_map, par);
        }
        mt_bits[it] = word;
        pixbase = yo * g.Wo + 64 * wo;
    }
    // housekeeping for the next frame: the other input map starts out empty
    if (own_map) clear_other_map(const_cast<uint64_t*>(in_bits), par, clear_words, bid * 256 + tid, nblk * 256);
    const int cnt = __popcll(word);
    const int inc = wave_inclusive_scan(cnt);                  // inclusive scan inside the wavefront
    if (lane == 63) wtot[wv] = inc;
    if (tid == 0) s_epoch = epoch_ld + 1u ? epoch_ld + 1u : 1u;   // 0 is what never-written slots hold
    __syncthreads();
    const unsigned epoch = s_epoch;
    if (tid == 0) {
        const unsigned total = (unsigned)(wtot[0] + wtot[1] + wtot[2] + wtot[3]);
        __hip_atomic_store(&look[bid], ((unsigned long long)epoch << 32) | total, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
    // counts of all earlier workgroups (count and epoch travel in one word: no ordering between words needed)
    int part = 0;
    for (int b = tid; b < bid; b += 256) {
        unsigned long long v = 0;
        int spins = 0;
        for (;;) {
            v = __hip_atomic_load(&look[b], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((unsigned)(v >> 32) == epoch) break;
            if (++spins > spin_limit) {
                v = (unsigned long long)(unsigned)recount_block(g, in_bits, pitch, full, b, own_map, par);
                atomicAdd(&ctl[CTL_RECOUNTS], 1);
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        part += (int)(unsigned)v;
    }
    part = wave_sum(part);
    if (lane == 0) red[wv] = part;
    __syncthreads();
    int off = red[0] + red[1] + red[2] + red[3];
    for (int q = 0; q < wv; ++q) off += wtot[q];
    off += inc - cnt;                                        // exclusive offset of this thread's word
    if (bid == nblk - 1 && tid == 255) ctl[CTL_COUNT] = off + cnt;

    expand_words<false>(word, off, pixbase, idx, lane);

    if (tid == 0) {
        if (bid == 0 && clear_slot >= 0) ctl[clear_slot] = 0;
        if (atomicAdd(&ctl[CTL_DONE], 1) == nblk - 1) {      // everybody has read the epoch and the frame count
            ctl[CTL_DONE] = 0;
            ctl[CTL_EPOCH] = (int)epoch;
            if (own_map) ctl[CTL_FRAME] = ctl[CTL_FRAME] + 1;
        }
    }
}

// Small maps: dilation, scan and index write in ONE workgroup of 1024 threads, so
// that the whole change-index extraction costs a single launch.  The workgroup walks
// the words in rounds of 1024, carrying the running count.
__global__ __launch_bounds__(1024) void dilate_compact_small_kernel(Geom g, const uint64_t* __restrict__ in_bits,
                                                                    long pitch, int full,
                                                                    uint64_t* __restrict__ mt_bits,
                                                                    int32_t* __restrict__ idx, int* __restrict__ ctl,
                                                                    int own_map, int clear_words)
{
    const int par = frame_parity(ctl, own_map);
    const int clear_slot = own_map ? CTL_NIN_A + (par ^ 1) : -1;
    __shared__ int wtot[16];
    __shared__ int carry;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int items = g.Ho * g.WWo;
    if (tid == 0) carry = 0;
    for (int r0 = 0; r0 < items; r0 += 1024) {
        const int it = r0 + tid;
        uint64_t word = 0;
        int pixbase = 0;
        if (it < items) {
            const int yo = it / g.WWo, wo = it - yo * g.WWo;
            if (full) {
                const int nvalid = g.Wo - 64 * wo < 64 ? g.Wo - 64 * wo : 64;
                word = nvalid == 64 ? ~0ull : ((1ull << nvalid) - 1ull);
            } else {
                word = dilated_word(g, in_bits, pitch, yo, wo, own_map, par);
            }
            mt_bits[it] = word;
            pixbase = yo * g.Wo + 64 * wo;
        }
        const int cnt = __popcll(word);
        const int inc = wave_inclusive_scan(cnt);                  // inclusive scan inside the wavefront
        __syncthreads();                 // previous round's wtot / carry have been consumed
        if (lane == 63) wtot[wv] = inc;
        __syncthreads();
        int off = carry;
        for (int q = 0; q < wv; ++q) off += wtot[q];
        off += inc - cnt;
        int round_total = 0;
        for (int q = 0; q < 16; ++q) round_total += wtot[q];
        expand_words<true>(word, off, pixbase, idx, lane);
        __syncthreads();                 // everyone has read carry
        if (tid == 0) carry += round_total;
    }
    if (own_map) clear_other_map(const_cast<uint64_t*>(in_bits), par, clear_words, tid, 1024);
    __syncthreads();
    if (tid == 0) {
        ctl[CTL_COUNT] = carry;
        if (clear_slot >= 0) ctl[clear_slot] = 0;
        if (own_map) ctl[CTL_FRAME] = ctl[CTL_FRAME] + 1;    // (one workgroup: everybody is past its reads)
    }
}

__global__ __launch_bounds__(256) void expand_bits_kernel(const uint64_t* __restrict__ bits, long pitch,
                                                          int H, int W, uint8_t* __restrict__ bytes)
{
    const long n = (long)H * W;
    for (long q = (long)blockIdx.x * 256 + threadIdx.x; q < n; q += (long)gridDim.x * 256) {
        const int y = (int)(q / W), x = (int)(q - (long)y * W);
        bytes[q] = test_bit<false>(bits, (long)y * pitch + x, 0) ? 1 : 0;
    }
}

// The input map of the last processed frame of a layer that detects its own changes: of its two
// interleaved maps the one that the frame count on the device selected for that frame.
__global__ __launch_bounds__(256) void expand_own_map_kernel(const uint64_t* __restrict__ bits,
                                                             const int* __restrict__ ctl, long pitch, int H, int W,
                                                             uint8_t* __restrict__ bytes)
{
    const int par = (ctl[CTL_FRAME] - 1) & 1;
    const long n = (long)H * W;
    for (long q = (long)blockIdx.x * 256 + threadIdx.x; q < n; q += (long)gridDim.x * 256) {
        const int y = (int)(q / W), x = (int)(q - (long)y * W);
        bytes[q] = test_bit<true>(bits, (long)y * pitch + x, par) ? 1 : 0;
    }
}

__global__ __launch_bounds__(256) void fill32_kernel(uint32_t* __restrict__ p, size_t n, uint32_t v)
{
    for (size_t q = (size_t)blockIdx.x * 256 + threadIdx.x; q < n; q += (size_t)gridDim.x * 256) p[q] = v;
}

// Pooled change map: bit (yp, xp) = OR over the w x w window of the producer's
// dilated map (row-padded words in, row-padded words out).
__global__ __launch_bounds__(256) void pool_mask_kernel(int Ho, int Wo, int WWo, int w, int Hp, int Wp, int WWp,
                                                        const uint64_t* __restrict__ mt_bits,
                                                        uint64_t* __restrict__ pm_bits)
{
    const int items = Hp * WWp;
    const int it = blockIdx.x * 256 + threadIdx.x;
    if (it >= items) return;
    const int yp = it / WWp, wp = it - yp * WWp;
    if (w == 2) {
        // word-parallel: OR the two producer rows, OR neighbouring bit pairs, squeeze the even bits
        // together (bits beyond Wo are 0 in the producer's words)
        uint64_t v[2] = {0, 0};
        for (int dy = 0; dy < 2; ++dy) {
            const int y = 2 * yp + dy;
            if (y >= Ho) break;
            for (int h = 0; h < 2; ++h)
                if (2 * wp + h < WWo) v[h] |= mt_bits[(long)y * WWo + 2 * wp + h];
        }
        uint64_t out = 0;
        for (int h = 0; h < 2; ++h) {
            uint64_t x = (v[h] | (v[h] >> 1)) & 0x5555555555555555ull;
            x = (x | (x >> 1)) & 0x3333333333333333ull;
            x = (x | (x >> 2)) & 0x0F0F0F0F0F0F0F0Full;
            x = (x | (x >> 4)) & 0x00FF00FF00FF00FFull;
            x = (x | (x >> 8)) & 0x0000FFFF0000FFFFull;
            x = (x | (x >> 16)) & 0x00000000FFFFFFFFull;
            out |= x << (32 * h);
        }
        pm_bits[it] = out;
        return;
    }
    uint64_t word = 0;
    for (int b = 0; b < 64; ++b) {
        const int xp = 64 * wp + b;
        if (xp >= Wp) break;
        bool any = false;
        for (int dy = 0; dy < w; ++dy)
            for (int dx = 0; dx < w; ++dx) {
                const int y = yp * w + dy, x = xp * w + dx;
                if (y < Ho && x < Wo && test_bit<false>(mt_bits, ((long)y * WWo << 6) + x, 0)) any = true;
            }
        word |= (uint64_t)any << b;
    }
    pm_bits[it] = word;
}

}  // namespace

int dilate_num_blocks(const Geom& g) { return (g.Ho * g.WWo + 255) / 256; }

// one round of the one-workgroup kernel; beyond that its serial rounds cost more than a second launch
bool compact_single_launch(const Geom& g) { return g.Ho * g.WWo <= 1024; }

hipError_t launch_dilate_compact_small(const Geom& g, const uint64_t* in_bits, long in_pitch_bits,
                                       int full, uint64_t* mt_bits, int32_t* idx, int* ctl, int own_map,
                                       int clear_words, hipStream_t st, Tm tm)
{
    CB_LAUNCH(dilate_compact_small_kernel, dim3(1), dim3(1024), st, tm, g, in_bits, in_pitch_bits, full,
              mt_bits, idx, ctl, own_map, clear_words);
    return hipGetLastError();
}

bool compact_one_pass(const Geom& g) { return dilate_num_blocks(g) <= ONE_PASS_MAX_BLOCKS; }
size_t compact_one_pass_bytes(const Geom& g) { return compact_one_pass(g) ? (size_t)dilate_num_blocks(g) * 8 : 0; }

hipError_t launch_dilate_compact(const Geom& g, const uint64_t* in_bits, long in_pitch_bits, int full,
                                 uint64_t* mt_bits, int32_t* idx, int* ctl, uint64_t* look, int own_map,
                                 int clear_words, int spin_limit, hipStream_t st, Tm tm)
{
    CB_LAUNCH(dilate_compact_kernel, dim3(dilate_num_blocks(g)), dim3(256), st, tm, g, in_bits,
              in_pitch_bits, full, mt_bits, idx, ctl, reinterpret_cast<unsigned long long*>(look), own_map, clear_words,
              spin_limit);
    return hipGetLastError();
}

hipError_t launch_dilate(const Geom& g, const uint64_t* in_bits, long in_pitch_bits, int full,
                         uint64_t* mt_bits, int* blk_cnt, int* ctl, int own_map, int clear_words, hipStream_t st, Tm tm)
{
    CB_LAUNCH(dilate_kernel, dim3(dilate_num_blocks(g)), dim3(256), st, tm, g, in_bits, in_pitch_bits,
              full, mt_bits, blk_cnt, ctl, own_map, clear_words);
    return hipGetLastError();
}

hipError_t launch_compact(const Geom& g, const uint64_t* mt_bits, const int* blk_cnt, int32_t* idx,
                          int* ctl, int own_map, hipStream_t st, Tm tm)
{
    CB_LAUNCH(compact_kernel, dim3(dilate_num_blocks(g)), dim3(256), st, tm, g, mt_bits, blk_cnt, idx, ctl, own_map);
    return hipGetLastError();
}

hipError_t launch_expand_own_map(const uint64_t* bits0, const int* ctl, long pitch_bits, int H, int W,
                                 uint8_t* bytes, hipStream_t st)
{
    long n = (long)H * W;
    unsigned grid = (unsigned)((n + 255) / 256);
    if (grid > 4096) grid = 4096;
    if (grid == 0) grid = 1;
    hipLaunchKernelGGL(expand_own_map_kernel, dim3(grid), dim3(256), 0, st, bits0, ctl, pitch_bits, H, W, bytes);
    return hipGetLastError();
}

hipError_t launch_expand_bits(const uint64_t* bits, long pitch_bits, int H, int W, uint8_t* bytes,
                              hipStream_t st)
{
    long n = (long)H * W;
    unsigned grid = (unsigned)((n + 255) / 256);
    if (grid > 4096) grid = 4096;
    if (grid == 0) grid = 1;
    hipLaunchKernelGGL(expand_bits_kernel, dim3(grid), dim3(256), 0, st, bits, pitch_bits, H, W, bytes);
    return hipGetLastError();
}

hipError_t launch_fill32(uint32_t* p, size_t n, uint32_t v, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    size_t grid = (n + 255) / 256;
    if (grid > 4096) grid = 4096;
    hipLaunchKernelGGL(fill32_kernel, dim3((unsigned)grid), dim3(256), 0, st, p, n, v);
    return hipGetLastError();
}

hipError_t launch_pool_mask(int Ho, int Wo, int WWo, int w, const uint64_t* mt_bits, uint64_t* pm_bits,
                            hipStream_t st)
{
    const int Hp = (Ho + w - 1) / w, Wp = (Wo + w - 1) / w, WWp = (Wp + 63) / 64;
    const int items = Hp * WWp;
    hipLaunchKernelGGL(pool_mask_kernel, dim3((items + 255) / 256), dim3(256), 0, st, Ho, Wo, WWo, w, Hp, Wp, WWp,
                       mt_bits, pm_bits);
    return hipGetLastError();
}

}  // namespace cb
