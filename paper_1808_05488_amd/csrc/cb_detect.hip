// Change detection with closed-loop state update (Sec. III-A Eq. 3, Sec. III-C).
//
// HBM-bound streaming kernel: reads the frame and the input state once over all
// channels (2*C*P elements), writes a bit-packed change map (P/8 bytes) and
// copies the channels of changed pixels into the state.
//
// Mapping: a block of 256 threads is CS channel groups x PL pixel lanes
// (PL = 256/CS, a multiple of the 64-wide wavefront).  A lane owns VEC
// consecutive pixels (one 16-byte load per channel for float, VEC = 4) and its
// group walks the channels g, g+CS, ...; the per-group flags are OR-ed through
// LDS.  Splitting channels over groups multiplies the number of wavefronts in
// flight for layers with many channels and few pixels.
#include "cb_kernels.h"
#include <algorithm>

namespace cb {

namespace {

__device__ __forceinline__ float widen(float v) { return v; }
__device__ __forceinline__ float widen(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

__device__ __forceinline__ float to_f(float v) { return v; }
__device__ __forceinline__ float to_f(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

template <typename T, int VEC> struct Pack;
template <> struct Pack<float, 4> { typedef float4 type; };
template <> struct Pack<float, 1> { typedef float type; };
template <> struct Pack<uint16_t, 4> { typedef uint2 type; };
template <> struct Pack<uint16_t, 1> { typedef uint16_t type; };

template <typename T, int VEC>
__device__ __forceinline__ void unpack(const typename Pack<T, VEC>::type& v, float (&f)[VEC]);
template <> __device__ __forceinline__ void unpack<float, 4>(const float4& v, float (&f)[4])
{ f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w; }
template <> __device__ __forceinline__ void unpack<float, 1>(const float& v, float (&f)[1]) { f[0] = v; }
template <> __device__ __forceinline__ void unpack<uint16_t, 4>(const uint2& v, float (&f)[4])
{
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
}
template <> __device__ __forceinline__ void unpack<uint16_t, 1>(const uint16_t& v, float (&f)[1])
{ f[0] = widen(v); }

// Load of a value that is used once (the new frame): marked non-temporal, so that it does not push
// the input state, which the next frame reads again, out of the caches.
template <typename V> __device__ __forceinline__ V ld_once(const V* p)
{
    typedef unsigned uvec __attribute__((ext_vector_type(sizeof(V) / 4 ? sizeof(V) / 4 : 1)));
    if constexpr (sizeof(V) >= 4) {
        const uvec u = __builtin_nontemporal_load(reinterpret_cast<const uvec*>(p));
        return __builtin_bit_cast(V, u);
    } else {
        return __builtin_nontemporal_load(p);
    }
}

// Workgroup barrier that orders LDS accesses only.  __syncthreads() also waits until every global
// store of the wavefront has been acknowledged, which here would put one store latency on
// each round of the shadow update.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// The value as the compiler cannot trace it back: what is computed from it stays where it is written.
__device__ __forceinline__ float opaque(float v) { asm volatile("" : "+v"(v)); return v; }
__device__ __forceinline__ uint16_t opaque(uint16_t v) { unsigned u = v; asm volatile("" : "+v"(u)); return (uint16_t)u; }

// bit i of a 16-bit value -> bit 4*i
__device__ __forceinline__ uint64_t spread4(uint64_t v)
{
    v = (v | (v << 24)) & 0x000000FF000000FFull;
    v = (v | (v << 12)) & 0x000F000F000F000Full;
    v = (v | (v << 6)) & 0x0303030303030303ull;
    v = (v | (v << 3)) & 0x1111111111111111ull;
    return v;
}

template <typename T, int VEC, int CS>
__global__ __launch_bounds__(256) void detect_kernel(const T* __restrict__ x, T* __restrict__ S, T* __restrict__ S2,
                                                     uint64_t* __restrict__ mbits0, int* __restrict__ ctl,
                                                     int C, int P, int nwords, float tau, int flags)
{
    typedef typename Pack<T, VEC>::type V;
    const int par = ctl[CTL_FRAME] & 1;          // which of the two map buffers and counters this frame fills
    uint64_t* __restrict__ mbits = mbits0 + par;  // the two maps are interleaved: word w of this frame's map at [2 * w]
    int* __restrict__ nin = ctl + CTL_NIN_A + par;
    constexpr int PL = 256 / CS;
    constexpr unsigned ALL = (1u << VEC) - 1u;
    const int tid = threadIdx.x;
    const int g = tid / PL;
    const int pl = tid - g * PL;
    const long p0 = ((long)blockIdx.x * PL + pl) * VEC;
    const bool valid = p0 < P;

    unsigned bits = 0;
    if (valid && !(flags & DET_FORCE_ALL)) {
#pragma unroll 4
        for (int c = g; c < C; c += CS) {
            const size_t off = (size_t)c * P + p0;
            V xv = ld_once(reinterpret_cast<const V*>(x + off));
            V sv = *reinterpret_cast<const V*>(S + off);
            float xf[VEC], sf[VEC];
            unpack<T, VEC>(xv, xf);
            unpack<T, VEC>(sv, sf);
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                float d = xf[v] - sf[v];          // one float32 subtract, then |.| > tau (strict)
                bits |= (fabsf(d) > tau ? 1u : 0u) << v;
            }
        }
    }
    if (CS > 1) {
        __shared__ unsigned sflag[256];
        sflag[tid] = bits;
        __syncthreads();
#pragma unroll
        for (int q = 0; q < CS; ++q) bits |= sflag[q * PL + pl];
    }
    if (flags & DET_FORCE_ALL) bits = valid ? ALL : 0u;

    // bit-packed change map, written by channel group 0
    if (g == 0) {
        const int lane = tid & 63;
        const long wave_p0 = ((long)blockIdx.x * PL + (pl & ~63)) * VEC;   // first pixel of this wavefront
        const long w0 = wave_p0 >> 6;
        if (VEC == 4) {
            uint64_t b0 = __ballot(bits & 1u), b1 = __ballot(bits & 2u);
            uint64_t b2 = __ballot(bits & 4u), b3 = __ballot(bits & 8u);
            if (lane < 4 && w0 + lane < nwords) {
                const int sh = 16 * lane;
                uint64_t w = spread4((b0 >> sh) & 0xFFFF) | (spread4((b1 >> sh) & 0xFFFF) << 1) |
                             (spread4((b2 >> sh) & 0xFFFF) << 2) | (spread4((b3 >> sh) & 0xFFFF) << 3);
                mbits[2 * (w0 + lane)] = w;
            }
            if (lane == 0) {
                int tot = __popcll(b0) + __popcll(b1) + __popcll(b2) + __popcll(b3);
                if (tot) atomicAdd(nin, tot);
            }
        } else {
            uint64_t b0 = __ballot(bits & 1u);
            if (lane == 0 && w0 < nwords) {
                mbits[2 * w0] = b0;
                int tot = __popcll(b0);
                if (tot) atomicAdd(nin, tot);
            }
        }
    }

    // state update: all channels of a changed pixel (closed loop), or every pixel
    unsigned upd = (flags & DET_NO_UPDATE) ? 0u : (flags & DET_COPY_ALL) ? (valid ? ALL : 0u) : bits;
    if (upd) {
        for (int c = g; c < C; c += CS) {
            const size_t off = (size_t)c * P + p0;
            if (upd == ALL) {
                *reinterpret_cast<V*>(S + off) = *reinterpret_cast<const V*>(x + off);
            } else {
#pragma unroll
                for (int v = 0; v < VEC; ++v)
                    if (upd & (1u << v)) S[off + v] = x[off + v];
            }
            if (S2) {
#pragma unroll
                for (int v = 0; v < VEC; ++v)
                    if (upd & (1u << v)) S2[(size_t)(p0 + v) * C + c] = x[off + v];
            }
        }
    }
}

// Register-resident variant: a lane keeps the CPT channel values it compared, so
// the state update is stores only (no second, latency-bound read of the frame).
// Workgroup = CS channel groups x PL pixel lanes.
// PLX = 16 (one pixel per lane only): 16 instead of 64 pixel lanes per workgroup, for maps with so
// few pixels that 64-pixel workgroups would leave most compute units idle; such a workgroup owns a
// quarter of a 64-pixel word of the bit map and stores it as a half word.
// SH: the layer keeps a channel-last shadow of its state (S2), C == CS*CPT, and channel q of group g is
// g*CPT + q instead of g + q*CS, so that a lane's channels are neighbours in the shadow.
template <typename T, int VEC, int CS, int CPT, int PLX = 0, bool SH = false>
__global__ __launch_bounds__((PLX ? PLX : (CS >= 4 ? 64 : 256 / CS)) * CS)
void detect_reg_kernel(const T* __restrict__ x, T* __restrict__ S, T* __restrict__ S2, uint64_t* __restrict__ mbits0,
                       int* __restrict__ ctl, int C, int P, int nwords, float tau, int flags)
{
    typedef typename Pack<T, VEC>::type V;
    // which of the two map buffers and counters this frame fills: the frame count lives on the device
    // (the index extraction advances it), so that a captured launch replays correctly whatever the
    // number of frames captured
    const int par = ctl[CTL_FRAME] & 1;
    uint64_t* __restrict__ mbits = mbits0 + par;  // the two maps are interleaved: word w of this frame's map at [2 * w]
    int* __restrict__ nin = ctl + CTL_NIN_A + par;
    constexpr int PL = PLX ? PLX : (CS >= 4 ? 64 : 256 / CS);
    static_assert(PLX == 0 || (PLX == 16 && VEC == 1 && CS > 1), "narrow workgroups: 16 lanes of one pixel each");
    constexpr int NT = PL * CS;
    constexpr unsigned ALL = (1u << VEC) - 1u;
    const int tid = threadIdx.x;
    const int g = tid / PL;
    const int pl = tid - g * PL;
    const long p0 = ((long)blockIdx.x * PL + pl) * VEC;
    const bool valid = p0 < P;

    V xv[CPT];
    unsigned bits = 0;
    if (valid) {
        if (flags & DET_FORCE_ALL) {
#pragma unroll
            for (int q = 0; q < CPT; ++q) {
                const int c = SH ? g * CPT + q : g + q * CS;
                if (c < C) xv[q] = *reinterpret_cast<const V*>(x + (size_t)c * P + p0);
            }
            // (first frame only.  Without this wait the compiler assumes these loads may still be in flight
            // in the other branch, and waits there between loads.)
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        } else {
            V sv[CPT];
#pragma unroll
            for (int q = 0; q < CPT; ++q) {
                const int c = SH ? g * CPT + q : g + q * CS;
                if (c < C) {
                    const size_t off = (size_t)c * P + p0;
                    xv[q] = ld_once(reinterpret_cast<const V*>(x + off));
                    sv[q] = (flags & DET_STREAM_STATE) ? ld_once(reinterpret_cast<const V*>(S + off))
                                                       : *reinterpret_cast<const V*>(S + off);
                }
            }
            // every load is issued before the first compare waits for one: the kernel lives on loads in flight
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < CPT; ++q) {
                const int c = SH ? g * CPT + q : g + q * CS;
                if (c < C) {
                    float xf[VEC], sf[VEC];
                    unpack<T, VEC>(xv[q], xf);
                    unpack<T, VEC>(sv[q], sf);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        float d = xf[v] - sf[v];      // one float32 subtract, then |.| > tau (strict)
                        bits |= (fabsf(d) > tau ? 1u : 0u) << v;
                    }
                }
            }
        }
    }
    if (CS > 1) {
        __shared__ unsigned sflag[NT];
        sflag[tid] = bits;
        __syncthreads();
#pragma unroll
        for (int q = 0; q < CS; ++q) bits |= sflag[q * PL + pl];
    }
    if (flags & DET_FORCE_ALL) bits = valid ? ALL : 0u;

    if (g == 0) {
        const int lane = tid & 63;
        const long wave_p0 = ((long)blockIdx.x * PL + (pl & ~63)) * VEC;
        const long w0 = wave_p0 >> 6;
        if (VEC == 4) {
            uint64_t b0 = __ballot(bits & 1u), b1 = __ballot(bits & 2u);
            uint64_t b2 = __ballot(bits & 4u), b3 = __ballot(bits & 8u);
            if (lane < 4 && w0 + lane < nwords) {
                const int sh = 16 * lane;
                uint64_t w = spread4((b0 >> sh) & 0xFFFF) | (spread4((b1 >> sh) & 0xFFFF) << 1) |
                             (spread4((b2 >> sh) & 0xFFFF) << 2) | (spread4((b3 >> sh) & 0xFFFF) << 3);
                mbits[2 * (w0 + lane)] = w;
            }
            if (lane == 0) {
                int tot = __popcll(b0) + __popcll(b1) + __popcll(b2) + __popcll(b3);
                if (tot) atomicAdd(nin, tot);
            }
        } else if (PLX == 16) {
            // the active lanes are lanes 0-15 of the first wavefront: 16 consecutive pixels
            const unsigned b0 = (unsigned)__ballot(bits & 1u) & 0xFFFFu;
            if (lane == 0) {
                reinterpret_cast<uint16_t*>(mbits + 2 * (blockIdx.x >> 2))[blockIdx.x & 3] = (uint16_t)b0;
                if (b0) atomicAdd(nin, __popc(b0));
            }
        } else {
            uint64_t b0 = __ballot(bits & 1u);
            if (lane == 0 && w0 < nwords) {
                mbits[2 * w0] = b0;
                int tot = __popcll(b0);
                if (tot) atomicAdd(nin, tot);
            }
        }
    }

    unsigned upd = (flags & DET_NO_UPDATE) ? 0u : (flags & DET_COPY_ALL) ? (valid ? ALL : 0u) : bits;
    if (upd) {
#pragma unroll
        for (int q = 0; q < CPT; ++q) {
            const int c = SH ? g * CPT + q : g + q * CS;
            if (c < C) {
                const size_t off = (size_t)c * P + p0;
                const T* xe = reinterpret_cast<const T*>(&xv[q]);
                if (upd == ALL) {
                    *reinterpret_cast<V*>(S + off) = xv[q];
                } else {
#pragma unroll
                    for (int v = 0; v < VEC; ++v)
                        if (upd & (1u << v)) S[off + v] = xe[v];
                }
            }
        }
    }

    // Channel-last shadow of the state (pixel-major: the C values of a pixel side by side), kept for
    // the gather of the fused back end.  The values of a changed pixel sit in CS different lanes of
    // CS different wavefronts.  The changed pixels of the workgroup are numbered (lane-major, from
    // ballots: upd is the same in every channel group, so every wavefront finds the same numbers),
    // their values are staged in LDS, KMAX pixels at a time in two alternating buffers (one
    // barrier per round; 16 bytes per store: a lane's channels are neighbours), and written out as
    // whole rows, 16 bytes per thread.  The phase is kept short in instructions: a workgroup that
    // lingers here has no loads in flight, and the kernel lives on loads in flight.
    if constexpr (SH) {
        static_assert(CS >= 4 && (CPT * sizeof(T)) % 16 == 0, "shadow rows are staged 16 bytes at a time");
        if (S2 != nullptr) {
            constexpr int EPV = 16 / (int)sizeof(T);  // elements per 16 bytes
            constexpr int CMAX = CS * CPT;
            constexpr int PITCH = CMAX + EPV;         // elements per staged pixel: 16-byte aligned rows, banks spread
            constexpr int KMAX = NT * 16 / (PITCH * (int)sizeof(T)) > 0 ? NT * 16 / (PITCH * (int)sizeof(T)) : 1;
            __shared__ int s_pix[PL * VEC];
            __shared__ __align__(16) T stage[2][KMAX * PITCH];
            // a channel group is a whole wavefront, or (16-lane groups) a quarter of one
            const int lane = tid & 63;
            const int seg_shift = PL >= 64 ? 0 : (lane & ~(PL - 1));
            const uint64_t seg_mask = PL >= 64 ? ~0ull : ((1ull << (PL & 63)) - 1ull);
            const uint64_t below = (1ull << (lane & (PL >= 64 ? 63 : PL - 1))) - 1ull;
            int before = 0, total = 0;
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const uint64_t bv = (__ballot((upd >> v) & 1u) >> seg_shift) & seg_mask;
                before += __popcll(bv & below);
                total += __popcll(bv);
            }
            if (g == 0) {
#pragma unroll
                for (int v = 0; v < VEC; ++v)
                    if (upd & (1u << v)) s_pix[before + __popc(upd & ((1u << v) - 1u))] = (int)(p0 + v);
            }
            const int lp = 31 - __builtin_clz((unsigned)(CMAX / EPV));     // 16-byte pieces per pixel = 1 << lp
            // The 16-byte LDS stores want the same pixel of EPV channels in neighbouring registers,
            // the loads delivered the VEC pixels of one channel there.  Made opaque here, the
            // values are rearranged here -- and not right behind each load, where the compiler
            // would otherwise put the moves, with a wait for every single load in front of them.
            T xs[CPT][VEC];
#pragma unroll
            for (int q = 0; q < CPT; ++q)
#pragma unroll
                for (int v = 0; v < VEC; ++v) xs[q][v] = opaque(reinterpret_cast<const T*>(&xv[q])[v]);
            int buf = 0;
            for (int k0 = 0; k0 < total; k0 += KMAX, buf ^= 1) {
#pragma unroll
                for (int v = 0; v < VEC; ++v)
                    if (upd & (1u << v)) {
                        const int k = before + __popc(upd & ((1u << v) - 1u)) - k0;
                        if ((unsigned)k < (unsigned)KMAX) {
#pragma unroll
                            for (int q0 = 0; q0 < CPT; q0 += EPV) {
                                __attribute__((aligned(16))) T e[EPV];
#pragma unroll
                                for (int j = 0; j < EPV; ++j) e[j] = xs[q0 + j][v];
                                *reinterpret_cast<uint4*>(&stage[buf][k * PITCH + g * CPT + q0]) = *reinterpret_cast<const uint4*>(e);
                            }
                        }
                    }
                lds_barrier();                    // (also: s_pix is written; the buffer's readers of two rounds ago are done)
                const int nrow = total - k0 < KMAX ? total - k0 : KMAX;
                for (int i = tid; i < (nrow << lp); i += NT) {
                    const int k = i >> lp, pc = i & ((1 << lp) - 1);
                    typedef unsigned uvec4 __attribute__((ext_vector_type(4)));
                    __builtin_nontemporal_store(*reinterpret_cast<const uvec4*>(&stage[buf][k * PITCH + pc * EPV]),
                                                reinterpret_cast<uvec4*>(S2 + (size_t)s_pix[k0 + k] * C + pc * EPV));
                }
            }
        }
    }
}

// State update as a kernel of its own, for frames whose change detection ran with DET_NO_UPDATE: all
// channels of every pixel that the change map marks are copied from the frame into the state (Sec. III-C)
// and, where the layer keeps one, into the channel-last shadow.  For states beyond the last-level
// cache, where the update inside the detection kernel costs far more than its bytes (a workgroup that
// stores anything leaves its compute unit without loads in flight): detection then is a pure
// stream, and this kernel touches the changed pixels only.
// A workgroup takes one 64-pixel word of the map at a time.  Phase 1, lane = pixel: the marked
// pixels' values of one channel go from the frame to the state (runs of pixels: part of a line)
// and into an LDS tile [changed pixel][channel]; phase 2, lane = channel: the tile's rows go to
// the shadow as contiguous pieces.  Channels in chunks of APPLY_CC.
constexpr int APPLY_CC = 128;
template <typename T>
__global__ __launch_bounds__(256) void state_apply_kernel(const T* __restrict__ x, T* __restrict__ S, T* __restrict__ S2,
                                                          const uint64_t* __restrict__ mbits0,
                                                          const int* __restrict__ ctl, int C, int P, int nwords)
{
    typedef typename Pack<T, 4>::type V4;                  // four consecutive pixels of one channel
    constexpr int E16 = 16 / (int)sizeof(T);               // elements per 16 bytes
    constexpr int PITCH = APPLY_CC + E16;                  // 16-byte aligned rows, banks spread
    __shared__ __align__(16) T stage[64 * PITCH];
    __shared__ int s_pix[64];
    const int tid = threadIdx.x;
    const int quad = tid & 15, cg = tid >> 4;              // 16 groups of four pixels x 16 channel groups
    const int par = ctl[CTL_FRAME] & 1;                    // (the index extraction, which advances it, runs later)
    // groups of four pixels are 16-byte (8-byte) aligned in the frame and in the state
    const bool vec_ok = (P & 3) == 0 && (((uintptr_t)x | (uintptr_t)S) & (4 * sizeof(T) - 1)) == 0;
    for (int w = blockIdx.x; w < nwords; w += gridDim.x) {
        const uint64_t word = mbits0[2 * (long)w + par];
        if (word == 0) continue;                           // (uniform over the workgroup)
        const unsigned nib = (unsigned)(word >> (4 * quad)) & 15u;          // this thread's four pixels
        const int k0 = __popcll(word & ((1ull << (4 * quad)) - 1ull));       // changed pixels before them
        const int nchg = __popcll(word);
        const long p0 = (long)w * 64 + 4 * quad;
        if (cg == 0 && nib) {
            int k = k0;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (nib & (1u << j)) s_pix[k++] = (int)(p0 + j);
        }
        for (int c0 = 0; c0 < C; c0 += APPLY_CC) {
            const int cn = C - c0 < APPLY_CC ? C - c0 : APPLY_CC;
            if (nib) {
                // eight channels at a time: eight loads in flight, then their stores
                for (int cb = cg; cb < cn; cb += 128) {
                    T v[8][4];
                    if (nib == 15u && vec_ok) {
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            if (cb + 16 * i < cn) {
                                const V4 t4 = ld_once(reinterpret_cast<const V4*>(x + (size_t)(c0 + cb + 16 * i) * P + p0));
                                const T* e = reinterpret_cast<const T*>(&t4);
#pragma unroll
                                for (int j = 0; j < 4; ++j) v[i][j] = e[j];
                            }
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            if (cb + 16 * i < cn) {
                                V4 t4;
                                T* e = reinterpret_cast<T*>(&t4);
#pragma unroll
                                for (int j = 0; j < 4; ++j) e[j] = v[i][j];
                                *reinterpret_cast<V4*>(S + (size_t)(c0 + cb + 16 * i) * P + p0) = t4;
                            }
                    } else {
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            if (cb + 16 * i < cn) {
#pragma unroll
                                for (int j = 0; j < 4; ++j)
                                    if (nib & (1u << j)) v[i][j] = x[(size_t)(c0 + cb + 16 * i) * P + p0 + j];
                            }
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            if (cb + 16 * i < cn) {
#pragma unroll
                                for (int j = 0; j < 4; ++j)
                                    if (nib & (1u << j)) S[(size_t)(c0 + cb + 16 * i) * P + p0 + j] = v[i][j];
                            }
                    }
                    if (S2) {
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            if (cb + 16 * i < cn) {
                                int k = k0;
#pragma unroll
                                for (int j = 0; j < 4; ++j)
                                    if (nib & (1u << j)) stage[(k++) * PITCH + cb + 16 * i] = v[i][j];
                            }
                    }
                }
            }
            if (S2) {
                __syncthreads();
                const int per = cn / E16;                  // 16-byte pieces per pixel (the shadow's C is a power of two >= 16 / 32)
                for (int i = tid; i < nchg * per; i += 256) {
                    const int kk = i / per, pc = i - kk * per;
                    typedef unsigned uvec4 __attribute__((ext_vector_type(4)));
                    const uvec4 v4 = *reinterpret_cast<const uvec4*>(&stage[kk * PITCH + pc * E16]);
                    __builtin_nontemporal_store(v4, reinterpret_cast<uvec4*>(S2 + (size_t)s_pix[kk] * C + c0 + pc * E16));
                }
                __syncthreads();                           // the tile and s_pix are rewritten by the next chunk / word
            }
        }
    }
}

// The whole shadow from the state: S (C x P) -> S2 (P x C), 64 x 64 tiles through LDS.  For a state that
// arrives from outside (an imported checkpoint); not on the per-frame path.
template <typename T>
__global__ __launch_bounds__(256) void shadow_rebuild_kernel(const T* __restrict__ S, T* __restrict__ S2, int C, int P)
{
    __shared__ T tile[64][65];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int ctiles = (C + 63) / 64;
    const long tiles = (((long)P + 63) / 64) * ctiles;
    for (long t = blockIdx.x; t < tiles; t += gridDim.x) {
        const long pt = t / ctiles;
        const int c0 = (int)(t - pt * ctiles) * 64;
        const long p0 = pt * 64;
        for (int r = ty; r < 64; r += 4)                   // row = channel, lane = pixel
            if (c0 + r < C && p0 + tx < P) tile[r][tx] = S[(size_t)(c0 + r) * P + p0 + tx];
        __syncthreads();
        for (int r = ty; r < 64; r += 4)                   // row = pixel, lane = channel
            if (c0 + tx < C && p0 + r < P) S2[(size_t)(p0 + r) * C + c0 + tx] = tile[tx][r];
        __syncthreads();
    }
}

template <typename T, int VEC, int CS, int CPT, int PLX = 0>
void launch_reg(const T* x, T* S, T* S2, uint64_t* mbits, int* ctl, int C, int P, float tau, int flags, hipStream_t st, Tm tm)
{
    constexpr int PL = PLX ? PLX : (CS >= 4 ? 64 : 256 / CS);
    const long px_per_block = (long)PL * VEC;
    const unsigned grid = (unsigned)((P + px_per_block - 1) / px_per_block);
    if constexpr (CS >= 4 && (CPT * sizeof(T)) % 16 == 0) {
        // (launch_t only passes a shadow on when the variant's registers hold exactly C channels)
        if (S2 != nullptr && C == CS * CPT) {
            CB_LAUNCH((detect_reg_kernel<T, VEC, CS, CPT, PLX, true>), dim3(grid), dim3(PL * CS), st, tm, x, S, S2, mbits,
                      ctl, C, P, (P + 63) / 64, tau, flags);
            return;
        }
    }
    CB_LAUNCH((detect_reg_kernel<T, VEC, CS, CPT, PLX>), dim3(grid), dim3(PL * CS), st, tm, x, S, (T*)nullptr, mbits,
              ctl, C, P, (P + 63) / 64, tau, flags);
}

template <typename T, int VEC>
void launch_v(const T* x, T* S, T* S2, uint64_t* mbits, int* ctl, int C, int P, float tau, int flags, hipStream_t st, Tm tm)
{
    // channel groups CS and channels per lane CPT with CS*CPT >= C
    if (C <= 4)        launch_reg<T, VEC, 1, 4>(x, S, S2, mbits, ctl, C, P, tau, flags, st, tm);
    else if (C <= 8)   launch_reg<T, VEC, 1, 8>(x, S, S2, mbits, ctl, C, P, tau, flags, st, tm);
    else if (C <= 16)  launch_reg<T, VEC, 4, 4>(x, S, S2, mbits, ctl, C, P, tau, flags, st, tm);
    else if (C <= 32)  launch_reg<T, VEC, 4, 8>(x, S, S2, mbits, ctl, C, P, tau, flags, st, tm);
    else if (C <= 64)  launch_reg<T, VEC, 8, 8>(x, S, S2, mbits, ctl, C, P, tau, flags, st, tm);
    // maps of fewer than 128 x 64 pixels with many channels: 16-pixel workgroups reach every compute unit
    else if (VEC == 1 && P < 8192 && C <= 128) launch_reg<T, 1, 16, 8, 16>(x, S, S2, mbits, ctl, C, P, tau, flags, st, tm);
    else if (VEC == 1 && P < 8192 && C <= 256) launch_reg<T, 1, 16, 16, 16>(x, S, S2, mbits, ctl, C, P, tau, flags, st, tm);
    else if (VEC == 1 && P < 8192 && C <= 512) launch_reg<T, 1, 16, 32, 16>(x, S, S2, mbits, ctl, C, P, tau, flags, st, tm);
    else if (C <= 128) launch_reg<T, VEC, 16, 8>(x, S, S2, mbits, ctl, C, P, tau, flags, st, tm);
    // one pixel per lane leaves registers for more channels per lane (deep layers: many channels, few pixels)
    else if (VEC == 1 && C <= 256) launch_reg<T, 1, 16, 16>(x, S, S2, mbits, ctl, C, P, tau, flags, st, tm);
    else if (VEC == 1 && C <= 512) launch_reg<T, 1, 16, 32>(x, S, S2, mbits, ctl, C, P, tau, flags, st, tm);
    else {
        // more channels than the register-resident variants hold: looped variant
        const long px_per_block = 64L * VEC;
        const unsigned grid = (unsigned)((P + px_per_block - 1) / px_per_block);
        CB_LAUNCH((detect_kernel<T, VEC, 4>), dim3(grid), dim3(256), st, tm, x, S, S2, mbits, ctl, C, P,
                  (P + 63) / 64, tau, flags);
    }
}

// Change detection restricted to candidate pixels (Eq. 3 where it can fire at all).  When a
// layer's input is the cached output of a change-based producer, only the producer's listed
// pixels were rewritten; every other input pixel holds the bits it held a frame ago, when it
// did not fire against the same state, so it cannot fire now.  Lane = candidate n, CS channel
// groups per workgroup; a first pass compares all channels of the candidate (flags OR-ed
// through LDS), a second pass copies the pixel into the state where it fired.  Bits are set
// with atomic ORs into the (pre-cleared) linear bit map, one per run of candidates that share
// a word; the changed-pixel count adds the bits that were newly set, so a pixel reached through
// several candidates (2x2 pooling maps up to four of them to one pixel) is counted once.  Duplicates race benignly: whoever copies the
// pixel first makes the others compare equal, and the bit is set either way.
// SH: the layer keeps a channel-last shadow S2 of its state (C a power of two).  The values of the candidates are
// staged in LDS ahead of the first barrier of a round and, once it is known which candidates fired, written to
// S2 with consecutive lanes on consecutive channels; two alternating buffers, so the barriers the round has anyway
// are enough.  (Written from the registers that hold them they are 4-byte stores to a different line per lane.)
template <typename T, int CS, int PLC, bool SH = false>
__global__ __launch_bounds__(CS * PLC) void detect_listed_kernel(const T* __restrict__ x, T* __restrict__ S,
                                                                 T* __restrict__ S2, uint64_t* __restrict__ mbits0,
                                                                 int* __restrict__ ctl,
                                                                 const int32_t* __restrict__ cand,
                                                                 const int* __restrict__ cand_count, int cand_cap,
                                                                 int C, int P, int W, float tau, int flags, int pool_w,
                                                                 int cand_W)
{
    constexpr int U = 8;                          // channels per lane held in registers (all of them when C <= 8*CS)
    const int par = ctl[CTL_FRAME] & 1;           // which of the two map buffers and counters this frame fills
    uint64_t* __restrict__ mbits = mbits0 + par;  // the two maps are interleaved: word w of this frame's map at [2 * w]
    int* __restrict__ nin = ctl + CTL_NIN_A + par;
    __shared__ unsigned sflag[CS * PLC];
    constexpr int PITCH = CS * U + 1;             // staged values per candidate: candidates a lane apart fall into different banks
    // (one buffer and a barrier at the end of the round where two would not fit)
    constexpr int NBUF = PLC * PITCH * (int)sizeof(T) * 2 <= 32768 ? 2 : 1;
    __shared__ T stage[SH ? NBUF : 1][SH ? PLC * PITCH : 1];
    __shared__ int s_q[SH ? NBUF : 1][SH ? PLC : 1];
    const int tid = threadIdx.x, g = tid / PLC, pl = tid - g * PLC;
    const int Cs = C < CS * U ? C : CS * U;       // channels held in registers (SH: a power of two)
    const int lcs = 31 - __builtin_clz((unsigned)Cs);
    int buf = 0;
    // the candidate of the first round is requested together with the count (the list has cand_cap
    // entries; those beyond the count are stale but readable), later ones a round ahead
    const int step = (int)gridDim.x * PLC;
    int nnext = (int)blockIdx.x * PLC + pl;
    int qnext = cand[nnext < cand_cap ? nnext : cand_cap - 1];
    const int nc = *cand_count;
    for (int t0 = blockIdx.x * PLC; t0 < nc; t0 += step) {
        const int n = t0 + pl;
        const bool valid = n < nc;
        int q = valid ? qnext : 0;
        nnext = n + step;
        qnext = cand[nnext < cand_cap ? nnext : cand_cap - 1];
        if (pool_w > 1) {
            const int yo = q / cand_W, xo = q - yo * cand_W;
            q = (yo / pool_w) * W + xo / pool_w;
        }
        unsigned fired = 0;
        T xr[U];
        if (valid) {
            T sr[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {         // surplus loads repeat channel 0 (a layer may have fewer
                const int c = g + u * CS;         // channels than the workgroup has channel groups)
                const size_t off = (size_t)(c < C ? c : 0) * P + q;
                xr[u] = x[off];
                sr[u] = S[off];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float d = to_f(xr[u]) - to_f(sr[u]);   // one float32 subtract, then |.| > tau (strict)
                fired |= (fabsf(d) > tau) ? 1u : 0u;
            }
            for (int c = g + U * CS; c < C; c += CS) {       // more channels than the registers hold
                const size_t off = (size_t)c * P + q;
                const float d = to_f(x[off]) - to_f(S[off]);
                fired |= (fabsf(d) > tau) ? 1u : 0u;
            }
        }
        if (SH && valid) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = g + u * CS;
                if (c < C) stage[SH ? buf : 0][SH ? pl * PITCH + c : 0] = xr[u];
            }
        }
        sflag[tid] = fired;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < CS; ++k) fired |= sflag[k * PLC + pl];
        if (SH && g == 0) s_q[SH ? buf : 0][SH ? pl : 0] = (valid && (fired || (flags & DET_COPY_ALL))) ? q : -1;
        __syncthreads();                          // sflag is rewritten in the next round
        // state update first: it does not depend on the bit map
        if (valid && (fired || (flags & DET_COPY_ALL))) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int c = g + u * CS;
                if (c < C) {
                    S[(size_t)c * P + q] = xr[u];
                    if (!SH && S2) S2[(size_t)q * C + c] = xr[u];
                }
            }
            for (int c = g + U * CS; c < C; c += CS) {
                const size_t off = (size_t)c * P + q;
                const T xc = x[off];
                S[off] = xc;
                if (S2) S2[(size_t)q * C + c] = xc;
            }
        }
        if (SH) {
            // rows of the candidates that fired (buffer `buf`: the next round fills the other one)
            for (int i = tid; i < (PLC << lcs); i += CS * PLC) {
                const int row = i >> lcs, c = i & (Cs - 1);
                const int qq = s_q[SH ? buf : 0][SH ? row : 0];
                if (qq >= 0) S2[(size_t)qq * C + c] = stage[SH ? buf : 0][SH ? row * PITCH + c : 0];
            }
            if (NBUF == 2) buf ^= 1;
            else lds_barrier();
        }
        if (g == 0) {
            // lanes 0..PLC-1 of the first wavefront.  Neighbouring candidates mostly fall into the same
            // 32-pixel word of the map: their bits are combined (segmented OR over runs of lanes with
            // equal word index) and the last lane of each run issues ONE atomic for the run -- a
            // few thousand atomics on a few hundred words otherwise queue up behind each other.
            const bool set = valid && fired;
            unsigned bits = set ? 1u << (q & 31) : 0u;
            const int word = set ? q >> 5 : -1 - pl;          // lanes without a bit never match a neighbour
#pragma unroll
            for (int o = 1; o < PLC; o <<= 1) {
                const unsigned b = __shfl_up(bits, o);
                const int w = __shfl_up(word, o);
                if (pl >= o && w == word) bits |= b;
            }
            const int wnext = __shfl_down(word, 1);
            int fresh = 0;
            if (set && (pl == PLC - 1 || wnext != word)) {
                const unsigned old = atomicOr(reinterpret_cast<uint32_t*>(mbits + 2 * (word >> 1)) + (word & 1), bits);
                fresh = __popc(bits & ~old);                  // a pixel reached through several candidates counts once
            }
#pragma unroll
            for (int o = 1; o < PLC; o <<= 1) fresh += __shfl_xor(fresh, o);
            if (pl == 0 && fresh) atomicAdd(nin, fresh);
        }
    }
}

template <typename T>
hipError_t launch_listed_t(const Geom& g, const T* x, T* S, T* S2, uint64_t* mbits, int* ctl, float tau, int flags,
                           const int32_t* cand, const int* cand_count, int cand_cap, int pool_w, int cand_W,
                           hipStream_t st, Tm tm)
{
    // channel groups so that a lane holds its (at most 8) channels in registers; few candidates per
    // workgroup, so that a few hundred candidates already spread over the chip
#define CB_LISTED(cs, plc)                                                                                          \
    do {                                                                                                            \
        {                                                                                                           \
            if (S2 != nullptr) {                                                                                    \
                CB_LAUNCH((detect_listed_kernel<T, cs, plc, true>), dim3(std::min(2048, (cand_cap + plc - 1) / plc)), \
                          dim3(cs * plc), st, tm, x, S, S2, mbits, ctl, cand, cand_count, cand_cap, g.C, g.P, g.W, tau, \
                          flags, pool_w, cand_W);                                                                   \
                break;                                                                                              \
            }                                                                                                       \
        }                                                                                                           \
        CB_LAUNCH((detect_listed_kernel<T, cs, plc>), dim3(std::min(2048, (cand_cap + plc - 1) / plc)), dim3(cs * plc), \
                  st, tm, x, S, S2, mbits, ctl, cand, cand_count, cand_cap, g.C, g.P, g.W, tau, flags, pool_w, cand_W); \
    } while (0)
    if (g.C <= 32)       CB_LISTED(4, 64);
    else if (g.C <= 64)  CB_LISTED(8, 32);
    else if (g.C <= 128) CB_LISTED(16, 16);
    else if (g.C <= 256) CB_LISTED(32, 16);
    else                 CB_LISTED(64, 16);
#undef CB_LISTED
    return hipGetLastError();
}

template <typename T>
hipError_t launch_t(const Geom& g, const T* x, T* S, T* S2, uint64_t* mbits, int* ctl, float tau, int flags,
                    hipStream_t st, Tm tm)
{
    const int P = g.P;
    const size_t valign = 4 * sizeof(T);
    // few pixels: one pixel per lane keeps more wavefronts busy than four
    // (with a shadow to update, more than 128 channels take the one-pixel-per-lane variants, which
    // stage the shadow rows through LDS; the looped variant writes them element by element)
    // 33 - 64 float32 channels: one pixel per lane on large maps too.  Workgroups of a quarter of the pixels
    // at 30 instead of 72 registers (four resident per compute unit instead of three) drain sooner at
    // the end of the launch, and the kernels behind it start sooner: 64 channels at 480x640, frame
    // 44.9 -> 42.4 - 42.7 us (two pixels per lane: 43.1 - 43.4 us); the kernel itself 26.9 -> 24.1 - 25.2 us.  No gain
    // for 128 channels (1080p) or for the first layers' 3 channels, so only here.
    const bool one_px = sizeof(T) == 4 && g.C > 32 && g.C <= 64;
    const bool vec4 = (P % 4 == 0) && ((uintptr_t)x % valign == 0) && ((uintptr_t)S % valign == 0) && P >= 65536 &&
                      !(S2 != nullptr && g.C > 128 && g.C <= 512) && !one_px;
    if (vec4) launch_v<T, 4>(x, S, S2, mbits, ctl, g.C, P, tau, flags, st, tm);
    else      launch_v<T, 1>(x, S, S2, mbits, ctl, g.C, P, tau, flags, st, tm);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_detect(const Geom& g, const void* x, void* S, void* S2, uint64_t* mbits, int* ctl,
                         float tau, int flags, hipStream_t st, Tm tm)
{
    // a shadow is kept for layers with a power-of-two channel count (see fused_channel_last)
    if (S2 && (g.C < (g.bf16 ? 32 : 16) || (g.C & (g.C - 1)) != 0)) return hipErrorInvalidValue;
    if (g.bf16)
        return launch_t<uint16_t>(g, (const uint16_t*)x, (uint16_t*)S, (uint16_t*)S2, mbits, ctl, tau, flags,
                                  st, tm);
    return launch_t<float>(g, (const float*)x, (float*)S, (float*)S2, mbits, ctl, tau, flags, st, tm);
}

hipError_t launch_state_apply(const Geom& g, const void* x, void* S, void* S2, const uint64_t* mbits, const int* ctl,
                              hipStream_t st, Tm tm)
{
    const int nwords = (g.P + 63) / 64;
    const unsigned grid = (unsigned)std::min(nwords, 8192);
    if (g.bf16)
        CB_LAUNCH(state_apply_kernel<uint16_t>, dim3(grid), dim3(256), st, tm, (const uint16_t*)x, (uint16_t*)S, (uint16_t*)S2,
                  mbits, ctl, g.C, g.P, nwords);
    else
        CB_LAUNCH(state_apply_kernel<float>, dim3(grid), dim3(256), st, tm, (const float*)x, (float*)S, (float*)S2, mbits, ctl,
                  g.C, g.P, nwords);
    return hipGetLastError();
}

hipError_t launch_shadow_rebuild(const Geom& g, const void* S, void* S2, hipStream_t st)
{
    const long tiles = (((long)g.P + 63) / 64) * ((g.C + 63) / 64);
    const unsigned grid = (unsigned)std::min(tiles, 8192L);
    if (g.bf16)
        hipLaunchKernelGGL(shadow_rebuild_kernel<uint16_t>, dim3(grid), dim3(256), 0, st, (const uint16_t*)S, (uint16_t*)S2,
                           g.C, g.P);
    else
        hipLaunchKernelGGL(shadow_rebuild_kernel<float>, dim3(grid), dim3(256), 0, st, (const float*)S, (float*)S2, g.C, g.P);
    return hipGetLastError();
}

hipError_t launch_detect_listed(const Geom& g, const void* x, void* S, void* S2, uint64_t* mbits, int* ctl,
                                float tau, int flags, const int32_t* cand, const int* cand_count, int cand_cap,
                                int pool_w, int cand_W, hipStream_t st, Tm tm)
{
    if (cand_cap < 1) return hipErrorInvalidValue;
    if (g.bf16)
        return launch_listed_t<uint16_t>(g, (const uint16_t*)x, (uint16_t*)S, (uint16_t*)S2, mbits, ctl, tau,
                                         flags, cand, cand_count, cand_cap, pool_w, cand_W, st, tm);
    return launch_listed_t<float>(g, (const float*)x, (float*)S, (float*)S2, mbits, ctl, tau, flags, cand,
                                  cand_count, cand_cap, pool_w, cand_W, st, tm);
}

}  // namespace cb
