// C-ABI layer of the change-based convolution library (see include/cbconv.h):
// descriptor validation, carve-up of the caller's state and scratch buffers, and
// the per-frame launch sequence of Sec. III-A with the closed-loop state of
// Sec. III-C.  No device allocation, no host<->device synchronisation and no
// memset on the per-frame path: the column count N stays in device memory and the
// matrix kernels are launched with persistent grids that read it there.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/cbconv.h"
#include "cb_kernels.h"
#include "cb_fused.h"

namespace {

thread_local int g_last_hip = 0;
// polls of a predecessor's count in the single-pass index extraction before the count is recomputed
std::atomic<int> g_scan_wait_limit{1 << 20};

inline int hip_fail(hipError_t e) { g_last_hip = (int)e; return CB_EHIP; }
#define CB_HIP(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return hip_fail(e_); } while (0)

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct StateLayout {
    size_t S, S2, OUT, OUT2, mbits, mtbits, idx, ctl, look, KT, bias, m_u8, mt_u8, KF, rowtab, total;
};

struct ScratchLayout {
    size_t blk, X, Y, total;
    int cap;       // columns per chunk, multiple of 256
};

constexpr size_t kXprimeBudget = (size_t)4 << 30;   // recommended upper size of one X' chunk
// A state of this size or more no longer stays in the 256 MB last-level cache from one frame to the next
constexpr size_t kStateBeyondCache = (size_t)128 << 20;

int validate(const cb_layer_desc* d, cb::Geom* g)
{
    if (!d) return CB_EINVAL;
    if (d->c_in < 1 || d->c_out < 1 || d->kh < 1 || d->kw < 1 || d->kh > 31 || d->kw > 31) return CB_EINVAL;
    if (d->stride < 1 || d->pad < 0 || d->pad > 31 || d->h_in < 1 || d->w_in < 1) return CB_EINVAL;
    if (d->dtype != CB_F32 && d->dtype != CB_BF16) return CB_EINVAL;
    if (d->relu != 0 && d->relu != 1) return CB_EINVAL;
    if (d->mode != CB_CLOSED_LOOP && d->mode != CB_FEED_FORWARD && d->mode != CB_PROPAGATE) return CB_EINVAL;
    if (d->backend != CB_BACKEND_AUTO && d->backend != CB_BACKEND_EXPLICIT && d->backend != CB_BACKEND_FUSED)
        return CB_EINVAL;
    for (int i = 0; i < 2; ++i) if (d->reserved[i] != 0) return CB_EINVAL;
    if ((d->keep_output_channel_last != 0 && d->keep_output_channel_last != 1) ||
        (d->gather_channel_last != 0 && d->gather_channel_last != 1)) return CB_EINVAL;
    if (d->h_in + 2 * d->pad < d->kh || d->w_in + 2 * d->pad < d->kw) return CB_EINVAL;
    const long P = (long)d->h_in * d->w_in;
    const long Ho = (d->h_in + 2 * d->pad - d->kh) / d->stride + 1;
    const long Wo = (d->w_in + 2 * d->pad - d->kw) / d->stride + 1;
    const long R = (long)d->c_in * d->kh * d->kw;
    if (P >= (1L << 30) || Ho * Wo >= (1L << 30) || R >= (1L << 24) || d->c_out >= (1 << 20)) return CB_EINVAL;
    // 32-bit byte offsets into the input state, with room for the guard ahead of it and a 16-byte load at its end
    if ((unsigned long long)d->c_in * P * (d->dtype == CB_BF16 ? 2 : 4) > 0xFFFFFF00ull) return CB_EINVAL;
    g->C = d->c_in; g->O = d->c_out; g->kh = d->kh; g->kw = d->kw; g->s = d->stride; g->p = d->pad;
    g->H = d->h_in; g->W = d->w_in; g->Ho = (int)Ho; g->Wo = (int)Wo;
    g->P = (int)P; g->Po = (int)(Ho * Wo); g->R = (int)R;
    g->WWo = (int)((Wo + 63) / 64);
    const int bm = cb::gemm_bm(d->c_out);
    g->Opad = (d->c_out + bm - 1) / bm * bm;
    g->bf16 = d->dtype == CB_BF16;
    if (d->backend == CB_BACKEND_FUSED && !cb::fused_supported(*g)) return CB_EINVAL;
    const bool fused = d->backend != CB_BACKEND_EXPLICIT && cb::fused_supported(*g);
    // the pixel-major copy of the cached output is written by the fused kernel's epilogue, four channels at a time
    if (d->keep_output_channel_last &&
        (!fused || d->c_out < (g->bf16 ? 32 : 16) || (d->c_out & (d->c_out - 1)) != 0)) return CB_EINVAL;
    // ... and read by the channel-last fused kernel of a consumer that keeps no state of its own
    if (d->gather_channel_last && (d->mode != CB_PROPAGATE || !fused || !cb::fused_channel_last(*g))) return CB_EINVAL;
    return CB_OK;
}

bool use_fused(const cb_layer_desc* d, const cb::Geom& g)
{
    return d->backend == CB_BACKEND_FUSED || (d->backend == CB_BACKEND_AUTO && cb::fused_supported(g));
}

// Closed-loop layers on the fused back end whose channel count allows it keep a second,
// pixel-major copy of the input state for the gather of the fused kernel.  Not feed-forward
// layers, which rewrite the whole state every frame.
bool use_shadow(const cb_layer_desc* d, const cb::Geom& g)
{
    return use_fused(d, g) && d->mode == CB_CLOSED_LOOP && cb::fused_channel_last(g);
}

StateLayout state_layout(const cb_layer_desc* d, const cb::Geom& g)
{
    const size_t b = g.bf16 ? 2 : 4;
    StateLayout L;
    // the fused kernel's gather may read up to cb::FUSED_GUARD bytes ahead of its source
    // (the input state, or the cached output when a CB_PROPAGATE consumer reads it)
    size_t o = 256;
    L.S = o;      o += d->mode == CB_PROPAGATE ? 0 : align256((size_t)g.C * g.P * b);
    L.S2 = o;     o += use_shadow(d, g) ? align256((size_t)g.C * g.P * b) : 0;
    L.OUT = o;    o += align256((size_t)g.O * g.Po * b);
    L.OUT2 = o;   o += d->keep_output_channel_last ? align256((size_t)g.O * g.Po * b) : 0;
    L.mbits = o;  o += align256(((size_t)(g.P + 63) / 64 + 4) * 16);  // two maps, word-interleaved: frames alternate between them
    L.mtbits = o; o += align256(((size_t)g.Ho * g.WWo + 4) * 8);
    L.idx = o;    o += align256((size_t)g.Po * 4);
    L.ctl = o;    o += align256(cb::CTL_SLOTS * 4);
    L.look = o;   o += align256(cb::compact_one_pass_bytes(g));
    L.KT = o;     o += align256((size_t)g.R * g.Opad * b);
    L.bias = o;   o += align256((size_t)g.Opad * 4);
    L.m_u8 = o;   o += align256((size_t)g.P);
    L.mt_u8 = o;  o += align256((size_t)g.Po);
    const bool fused = use_fused(d, g);
    L.KF = o;     o += fused ? align256(cb::fused_pack_bytes(g)) : 0;
    L.rowtab = o; o += fused ? align256(cb::fused_table_bytes(g)) : 0;
    L.total = o;
    return L;
}

size_t col_bytes(const cb::Geom& g) { return (size_t)g.R * (g.bf16 ? 2 : 4) + (size_t)g.O * 4; }
int po_pad(const cb::Geom& g) { return (g.Po + 255) & ~255; }

// fused layers need the block counters only
ScratchLayout scratch_layout(const cb::Geom& g, int cap, bool fused)
{
    ScratchLayout L;
    L.cap = cap;
    size_t o = 0;
    L.blk = o; o += align256((size_t)cb::dilate_num_blocks(g) * 4);
    L.X = o;   o += fused ? 0 : align256((size_t)g.R * cap * (g.bf16 ? 2 : 4));
    L.Y = o;   o += fused ? 0 : align256((size_t)g.O * cap * 4);
    L.total = o;
    return L;
}

int recommended_cap(const cb::Geom& g)
{
    size_t per_col = (size_t)g.R * (g.bf16 ? 2 : 4);
    size_t cols = kXprimeBudget / per_col;
    cols &= ~(size_t)255;
    if (cols < 256) cols = 256;
    if (cols > (size_t)po_pad(g)) cols = po_pad(g);
    return (int)cols;
}

}  // namespace

struct cb_layer {
    cb_layer_desc d;
    cb::Geom g;
    hipStream_t st;
    char* state;
    StateLayout sl;
    char* scratch;
    ScratchLayout sc;
    int nchunks;
    bool fused;            // back end: one fused kernel instead of gather / GEMM / update
    bool shadow;           // the layer keeps a pixel-major copy of its input state for the fused kernel
    const void* ext_cl;    // CB_PROPAGATE layer that gathers channel-last: the producer's pixel-major output (per call)
    cb::FusedPlan plan;
    bool primed;
    bool timing;
    std::vector<hipEvent_t> ev;      // begin/end event pairs, one pair per kernel dispatch
    std::vector<int> ev_step;        // step each pair belongs to
    int ev_used;
    // change set of the last frame (own buffers, or the producer's for a 1x1 CB_PROPAGATE layer).
    // cur_in_own: the input map is the layer's own, i.e. one of its two alternating buffers -- which
    // one, the frame count in the control block on the device tells (cb_kernels.h, CTL_FRAME)
    const uint64_t* cur_in_bits;  long cur_in_pitch;  bool cur_in_own;
    const uint64_t* cur_mtbits;
    const int32_t* cur_idx;
    const int* cur_count;
    long frames;
    // lockstep with a producer, for cb_process_frame_chained: which producer fed the last frame and
    // how many frames it had processed then
    const void* chain_src;
    long chain_frames;
    float chain_tau;       // threshold of this layer's last frame

    void* S() const { return state + sl.S; }
    void* S2() const { return shadow ? state + sl.S2 : nullptr; }
    void* OUT() const { return state + sl.OUT; }
    // pixel-major copy of the cached output (for consumers that gather channel-last), or null
    void* OUT2() const { return d.keep_output_channel_last ? state + sl.OUT2 : nullptr; }
    // the two input change maps, filled by alternate frames and interleaved word by word (the other
    // one is cleared for the next frame)
    uint64_t* mbits() const { return (uint64_t*)(state + sl.mbits); }
    int mbits_words() const { return (g.P + 63) / 64; }
    uint64_t* mtbits() const { return (uint64_t*)(state + sl.mtbits); }
    int32_t* idx() const { return (int32_t*)(state + sl.idx); }
    int* ctl() const { return (int*)(state + sl.ctl); }
    uint64_t* look() const { return (uint64_t*)(state + sl.look); }
    void* KT() const { return state + sl.KT; }
    float* bias() const { return (float*)(state + sl.bias); }
    uint8_t* m_u8() const { return (uint8_t*)(state + sl.m_u8); }
    uint8_t* mt_u8() const { return (uint8_t*)(state + sl.mt_u8); }
    void* KF() const { return state + sl.KF; }
    void* rowtab() const { return state + sl.rowtab; }
    int* blk() const { return (int*)(scratch + sc.blk); }
    void* X() const { return scratch + sc.X; }
    void* Y() const { return scratch + sc.Y; }
};

struct cb_pool {
    const cb_layer* prod;
    int w, O, Ho, Wo, WWo, Hp, Wp, WWp, bf16;
    hipStream_t st;
    char* state;
    size_t off_pool, off_pool2, off_bits, off_u8, total;
    bool cl;               // keeps a pixel-major copy of the pooled output (the producer keeps one of its output)
    long done_frames;      // producer frame count at the last cb_pool_process
    bool primed;

    void* POOL() const { return state + off_pool; }
    void* POOL2() const { return cl ? state + off_pool2 : nullptr; }
    uint64_t* pmbits() const { return (uint64_t*)(state + off_bits); }
    uint8_t* pm_u8() const { return (uint8_t*)(state + off_u8); }
};

namespace {

void pool_layout(cb_pool* p)
{
    const size_t b = p->bf16 ? 2 : 4;
    size_t o = 256;      // readable bytes ahead of the pooled output (gather of a fused CB_PROPAGATE consumer)
    p->off_pool = o; o += align256((size_t)p->O * p->Hp * p->Wp * b);
    p->off_pool2 = o; o += p->cl ? align256((size_t)p->O * p->Hp * p->Wp * b) : 0;
    p->off_bits = o; o += align256(((size_t)p->Hp * p->WWp + 4) * 8);
    p->off_u8 = o;   o += align256((size_t)p->Hp * p->Wp);
    p->total = o;
}

// Next pair of begin/end events for one kernel dispatch (null events when timing is off).
cb::Tm next_tm(cb_layer* L, int step)
{
    cb::Tm tm;
    if (!L->timing || L->ev_used + 2 > (int)L->ev.size()) return tm;
    tm.start = L->ev[L->ev_used];
    tm.stop = L->ev[L->ev_used + 1];
    L->ev_step[L->ev_used / 2] = step;
    L->ev_used += 2;
    return tm;
}

// dilate + compact into the layer's own buffers, then the chunked
// gather / GEMM / update sequence from `src`.
int run_back_end(cb_layer* L, const void* src, bool have_list)
{
    const cb::Geom& g = L->g;
    if (!have_list) {
        const int own_map = L->cur_in_own ? 1 : 0;
        const int clear_words = own_map ? L->mbits_words() : 0;
        if (cb::compact_single_launch(g)) {
            CB_HIP(cb::launch_dilate_compact_small(g, L->cur_in_bits, L->cur_in_pitch, L->primed ? 0 : 1,
                                                   L->mtbits(), L->idx(), L->ctl(), own_map, clear_words, L->st,
                                                   next_tm(L, CB_STEP_DILATE)));
        } else if (cb::compact_one_pass(g)) {
            CB_HIP(cb::launch_dilate_compact(g, L->cur_in_bits, L->cur_in_pitch, L->primed ? 0 : 1,
                                             L->mtbits(), L->idx(), L->ctl(), L->look(), own_map, clear_words,
                                             g_scan_wait_limit.load(std::memory_order_relaxed), L->st,
                                             next_tm(L, CB_STEP_DILATE)));
        } else {
            CB_HIP(cb::launch_dilate(g, L->cur_in_bits, L->cur_in_pitch, L->primed ? 0 : 1, L->mtbits(),
                                     L->blk(), L->ctl(), own_map, clear_words, L->st, next_tm(L, CB_STEP_DILATE)));
            CB_HIP(cb::launch_compact(g, L->mtbits(), L->blk(), L->idx(), L->ctl(), own_map, L->st,
                                      next_tm(L, CB_STEP_COMPACT)));
        }
        L->cur_mtbits = L->mtbits();
        L->cur_idx = L->idx();
        L->cur_count = L->ctl() + cb::CTL_COUNT;
    }
    if (L->fused) {
        CB_HIP(cb::launch_fused(g, L->plan, src, L->d.gather_channel_last ? L->ext_cl : L->S2(), L->cur_idx, L->cur_count,
                                L->KF(), L->rowtab(), L->bias(), L->d.relu, L->OUT(), L->OUT2(), L->st,
                                next_tm(L, CB_STEP_FUSED)));
        L->primed = true;
        L->frames++;
        return CB_OK;
    }
    for (int q = 0; q < L->nchunks; ++q) {
        const int col0 = q * L->sc.cap;
        CB_HIP(cb::launch_gather(g, src, L->cur_idx, L->cur_count, col0, L->sc.cap, L->X(), L->ctl(), L->st,
                                 next_tm(L, CB_STEP_GATHER)));
        CB_HIP(cb::launch_gemm(g, L->KT(), L->X(), L->Y(), L->cur_count, col0, L->sc.cap, L->ctl(), L->st,
                               next_tm(L, CB_STEP_GEMM)));
        CB_HIP(cb::launch_update(g, L->Y(), L->bias(), L->cur_idx, L->cur_count, col0, L->sc.cap, L->d.relu,
                                 L->OUT(), L->st, next_tm(L, CB_STEP_UPDATE)));
    }
    L->primed = true;
    L->frames++;
    return CB_OK;
}

// Change detection (whole input, or candidates only) + state update, then the back end.
int detect_and_update(cb_layer* L, const void* input_dev, float tau, const int32_t* cand, const int* cand_count,
                      int cand_cap, int pool_w, int cand_W, const void** output_dev)
{
    L->ev_used = 0;
    int flags = 0;
    if (!L->primed) flags = cb::DET_FORCE_ALL | cb::DET_COPY_ALL;
    else if (L->d.mode == CB_FEED_FORWARD) flags = cb::DET_COPY_ALL;
    if ((size_t)L->g.C * L->g.P * (L->g.bf16 ? 2 : 4) >= kStateBeyondCache) flags |= cb::DET_STREAM_STATE;
    if (cand)
        CB_HIP(cb::launch_detect_listed(L->g, input_dev, L->S(), L->S2(), L->mbits(), L->ctl(), tau,
                                        flags, cand, cand_count, cand_cap, pool_w, cand_W, L->st,
                                        next_tm(L, CB_STEP_DETECT)));
    else if (L->shadow && L->primed && !L->g.bf16 && (flags & cb::DET_STREAM_STATE)) {
        // a float32 state beyond the caches, with a shadow: detection as a pure stream, the update of the changed
        // pixels (state and shadow) in a kernel of its own (1080p x 128 channels: the detection variant that
        // updates the shadow itself costs 17 us more even when nothing changes, this one 0 - 10 us up to 1 % changed;
        // bfloat16, whose variant is the cheaper one at every density, keeps the update inside)
        CB_HIP(cb::launch_detect(L->g, input_dev, L->S(), nullptr, L->mbits(), L->ctl(), tau, flags | cb::DET_NO_UPDATE,
                                 L->st, next_tm(L, CB_STEP_DETECT)));
        CB_HIP(cb::launch_state_apply(L->g, input_dev, L->S(), L->S2(), L->mbits(), L->ctl(), L->st,
                                      next_tm(L, CB_STEP_STATE)));
    } else
        CB_HIP(cb::launch_detect(L->g, input_dev, L->S(), L->S2(), L->mbits(), L->ctl(), tau, flags,
                                 L->st, next_tm(L, CB_STEP_DETECT)));
    L->cur_in_bits = L->mbits();
    L->cur_in_pitch = L->g.W;
    L->cur_in_own = true;
    const int rc = run_back_end(L, L->S(), false);
    if (rc) return rc;
    if (output_dev) *output_dev = L->OUT();
    return CB_OK;
}

// Pooled change map of the producer's last frame.  Computed on every request: a count of frames kept
// on the host would not see the frames of a replayed HIP graph.
int pool_mask(const cb_pool* p)
{
    CB_HIP(cb::launch_pool_mask(p->Ho, p->Wo, p->WWo, p->w, p->prod->cur_mtbits, p->pmbits(), p->st));
    return CB_OK;
}

}  // namespace

extern "C" {

int cb_version(void) { return 100; }

int cb_last_hip_error(void) { return g_last_hip; }

const char* cb_strerror(int status)
{
    switch (status) {
        case CB_OK: return "success";
        case CB_EINVAL: return "invalid argument";
        case CB_ENOMEM: return "state or scratch buffer too small";
        case CB_EHIP: return "HIP runtime error";
        case CB_ESTATE: return "call out of order";
        default: return "unknown status";
    }
}

int cb_layer_workspace_bytes(const cb_layer_desc* desc, size_t* state_bytes, size_t* scratch_bytes)
{
    cb::Geom g;
    int rc = validate(desc, &g);
    if (rc) return rc;
    if (state_bytes) *state_bytes = state_layout(desc, g).total;
    if (scratch_bytes) *scratch_bytes = scratch_layout(g, recommended_cap(g), use_fused(desc, g)).total;
    return CB_OK;
}

int cb_layer_min_scratch_bytes(const cb_layer_desc* desc, size_t* scratch_bytes)
{
    cb::Geom g;
    int rc = validate(desc, &g);
    if (rc) return rc;
    if (scratch_bytes) *scratch_bytes = scratch_layout(g, 256, use_fused(desc, g)).total;
    return CB_OK;
}

int cb_layer_create(const cb_layer_desc* desc, const void* w_oihw_dev, const void* bias_dev,
                    void* state_dev, size_t state_bytes, void* scratch_dev, size_t scratch_bytes,
                    void* hip_stream, cb_layer_t** out)
{
    if (!out) return CB_EINVAL;
    *out = nullptr;
    cb::Geom g;
    int rc = validate(desc, &g);
    if (rc) return rc;
    if (!w_oihw_dev || !state_dev || !scratch_dev) return CB_EINVAL;
    if (((uintptr_t)state_dev & 255) || ((uintptr_t)scratch_dev & 255)) return CB_EINVAL;
    const size_t esz = g.bf16 ? 2 : 4;
    if (((uintptr_t)w_oihw_dev % esz) || (bias_dev && ((uintptr_t)bias_dev % esz))) return CB_EINVAL;
    StateLayout sl = state_layout(desc, g);
    if (state_bytes < sl.total) return CB_ENOMEM;
    const bool fused = use_fused(desc, g);
    if (scratch_bytes < scratch_layout(g, 256, fused).total) return CB_ENOMEM;
    // largest chunk capacity (multiple of 256 columns) that fits the given scratch
    size_t cols = (scratch_bytes / col_bytes(g) + 255) & ~(size_t)255;
    if (cols > (size_t)po_pad(g)) cols = po_pad(g);
    if (cols < 256) cols = 256;
    while (cols > 256 && scratch_layout(g, (int)cols, fused).total > scratch_bytes) cols -= 256;

    cb_layer* L = new (std::nothrow) cb_layer();
    if (!L) return CB_ENOMEM;
    L->d = *desc;
    L->g = g;
    L->st = (hipStream_t)hip_stream;
    L->state = (char*)state_dev;
    L->sl = sl;
    L->scratch = (char*)scratch_dev;
    L->sc = scratch_layout(g, (int)cols, fused);
    L->fused = fused;
    L->shadow = use_shadow(desc, g);
    L->ext_cl = nullptr;
    L->nchunks = (po_pad(g) + L->sc.cap - 1) / L->sc.cap;
    L->primed = false;
    L->timing = false;
    L->ev_used = 0;
    L->cur_in_bits = L->mbits();
    L->cur_in_pitch = g.W;
    L->cur_in_own = desc->mode != CB_PROPAGATE;
    L->cur_mtbits = L->mtbits();
    L->cur_idx = L->idx();
    L->cur_count = L->ctl() + cb::CTL_COUNT;
    L->frames = 0;
    L->chain_src = nullptr;
    L->chain_frames = 0;
    L->chain_tau = 0.0f;

    hipError_t e = hipMemsetAsync(state_dev, 0, sl.total, L->st);
    if (e == hipSuccess) e = cb::launch_pack_weights(g, w_oihw_dev, bias_dev, L->KT(), L->bias(), L->st);
    if (e == hipSuccess && fused) e = cb::fused_prepare(g, w_oihw_dev, L->KF(), L->rowtab(), L->shadow || desc->gather_channel_last, L->st, &L->plan);
    if (e != hipSuccess) { delete L; return hip_fail(e); }
    *out = L;
    return CB_OK;
}

int cb_process_frame(cb_layer_t* L, const void* input_dev, float tau, const void** output_dev)
{
    if (!L || !input_dev) return CB_EINVAL;
    if (L->d.mode == CB_PROPAGATE) return CB_EINVAL;
    if (!(tau >= 0.0f) || std::isinf(tau)) return CB_EINVAL;
    if ((uintptr_t)input_dev % (L->g.bf16 ? 2 : 4)) return CB_EINVAL;
    {   // the input must not alias the layer's own state
        const char* a = (const char*)input_dev;
        const size_t n = (size_t)L->g.C * L->g.P * (L->g.bf16 ? 2 : 4);
        if (a < L->state + L->sl.total && a + n > L->state) return CB_EINVAL;
    }
    L->chain_src = nullptr;               // a frame from an arbitrary source ends any lockstep with a producer
    L->chain_tau = tau;
    return detect_and_update(L, input_dev, tau, nullptr, nullptr, 0, 0, 0, output_dev);
}

int cb_process_frame_chained(cb_layer_t* L, const void* input_dev, const cb_layer_t* pl, const cb_pool_t* pp,
                             float tau, const void** output_dev)
{
    if (!L || !input_dev) return CB_EINVAL;
    if (L->d.mode == CB_PROPAGATE) return CB_EINVAL;
    if ((pl == nullptr) == (pp == nullptr)) return CB_EINVAL;
    if (!(tau >= 0.0f) || std::isinf(tau)) return CB_EINVAL;
    const cb::Geom& g = L->g;
    const cb_layer* conv = pl ? pl : pp->prod;       // whose index list names the rewritten pixels
    const void* src = pl ? (const void*)pl : (const void*)pp;
    long src_frames;
    if (pl) {
        if (pl->g.O != g.C || pl->g.Ho != g.H || pl->g.Wo != g.W || pl->g.bf16 != g.bf16) return CB_EINVAL;
        if (pl->st != L->st) return CB_EINVAL;
        if (!pl->primed) return CB_ESTATE;
        if (input_dev != pl->OUT()) return CB_EINVAL;
        src_frames = pl->frames;
    } else {
        if (pp->O != g.C || pp->Hp != g.H || pp->Wp != g.W || pp->bf16 != g.bf16) return CB_EINVAL;
        if (pp->st != L->st) return CB_EINVAL;
        if (!pp->primed) return CB_ESTATE;
        if (input_dev != pp->POOL()) return CB_EINVAL;
        if (pp->done_frames != pp->prod->frames) return CB_ESTATE;   // the pooling stage has not seen the producer's last frame
        src_frames = pp->done_frames;
    }
    // Restricted detection is exact only if this layer has seen every frame of the producer since
    // its own last frame; otherwise (first frame, a skipped frame, another source in between) the
    // whole input is compared, and the lockstep starts again.
    // A closed-loop layer also needs a threshold that has not dropped: an untouched pixel is only known
    // to be within the LAST frame's tau of the state (a feed-forward layer's state equals its last input,
    // so there an untouched pixel has difference zero).
    const bool lockstep = L->primed && L->chain_src == src && src_frames == L->chain_frames + 1 &&
                          (L->d.mode == CB_FEED_FORWARD || tau >= L->chain_tau);
    L->chain_src = src;
    L->chain_frames = src_frames;
    L->chain_tau = tau;
    if (!lockstep) return detect_and_update(L, input_dev, tau, nullptr, nullptr, 0, 0, 0, output_dev);
    return detect_and_update(L, input_dev, tau, conv->cur_idx, conv->cur_count, conv->g.Po, pp ? pp->w : 1,
                             conv->g.Wo, output_dev);
}

int cb_process_frame_propagated(cb_layer_t* L, const void* input_dev, const cb_layer_t* pl,
                                const cb_pool_t* pp, const void** output_dev)
{
    if (!L || !input_dev) return CB_EINVAL;
    if (L->d.mode != CB_PROPAGATE) return CB_EINVAL;
    if ((pl == nullptr) == (pp == nullptr)) return CB_EINVAL;
    const cb::Geom& g = L->g;
    const void* src = pl ? (const void*)pl : (const void*)pp;
    long src_frames;
    int rc;
    if (pl) {
        if (pl->g.O != g.C || pl->g.Ho != g.H || pl->g.Wo != g.W || pl->g.bf16 != g.bf16) return CB_EINVAL;
        if (pl->st != L->st) return CB_EINVAL;
        if (!pl->primed) return CB_ESTATE;
        if (input_dev != pl->OUT()) return CB_EINVAL;     // the input is the producer's cached output
        if (L->d.gather_channel_last && !pl->OUT2()) return CB_EINVAL;   // ... of which the producer must keep the pixel-major copy
        L->ext_cl = pl->OUT2();
        L->cur_in_bits = pl->cur_mtbits;
        L->cur_in_pitch = 64L * pl->g.WWo;
        L->cur_in_own = false;
        src_frames = pl->frames;
    } else {
        if (pp->O != g.C || pp->Hp != g.H || pp->Wp != g.W || pp->bf16 != g.bf16) return CB_EINVAL;
        if (pp->st != L->st) return CB_EINVAL;
        if (!pp->primed) return CB_ESTATE;
        if (input_dev != pp->POOL()) return CB_EINVAL;    // the input is the producer's pooled output
        if (L->d.gather_channel_last && !pp->POOL2()) return CB_EINVAL;
        L->ext_cl = pp->POOL2();
        if (pp->done_frames != pp->prod->frames) return CB_ESTATE;   // the pooling stage has not seen the producer's last frame
        if ((rc = pool_mask(pp))) return rc;
        L->cur_in_bits = pp->pmbits();
        L->cur_in_pitch = 64L * pp->WWp;
        L->cur_in_own = false;
        src_frames = pp->done_frames;
    }
    // The producer's change set of ITS last frame stands for everything that changed in the input since
    // this layer's last frame only if this layer has seen every frame of that producer; after a skipped
    // frame (or another producer) every output is recomputed once, as on the first frame.
    if (L->chain_src != src || src_frames != L->chain_frames + 1) L->primed = false;
    L->chain_src = src;
    L->chain_frames = src_frames;
    L->ev_used = 0;
    const bool pointwise = g.kh == 1 && g.kw == 1 && g.s == 1 && g.p == 0;
    bool have_list = false;
    if (pl && pointwise && L->primed) {
        // Sec. III-E case 2: the change map and the index list are the producer's
        L->cur_mtbits = pl->cur_mtbits;
        L->cur_idx = pl->cur_idx;
        L->cur_count = pl->cur_count;
        have_list = true;
    }
    rc = run_back_end(L, input_dev, have_list);
    if (rc) return rc;
    if (output_dev) *output_dev = L->OUT();
    return CB_OK;
}

int cb_layer_changes(cb_layer_t* L, const uint8_t** m_in_dev, const uint8_t** m_out_dev,
                     const int32_t** idx_dev, const int32_t** count_dev)
{
    if (!L) return CB_EINVAL;
    if (!L->primed) return CB_ESTATE;
    if (m_in_dev) {
        if (L->cur_in_own)
            CB_HIP(cb::launch_expand_own_map(L->cur_in_bits, L->ctl(), L->cur_in_pitch, L->g.H, L->g.W,
                                             L->m_u8(), L->st));
        else
            CB_HIP(cb::launch_expand_bits(L->cur_in_bits, L->cur_in_pitch, L->g.H, L->g.W, L->m_u8(), L->st));
        *m_in_dev = L->m_u8();
    }
    if (m_out_dev) {
        CB_HIP(cb::launch_expand_bits(L->cur_mtbits, 64L * L->g.WWo, L->g.Ho, L->g.Wo, L->mt_u8(), L->st));
        *m_out_dev = L->mt_u8();
    }
    if (idx_dev) *idx_dev = L->cur_idx;
    if (count_dev) *count_dev = L->cur_count;
    return CB_OK;
}

int cb_layer_state(const cb_layer_t* L, const void** state_dev)
{
    if (!L || !state_dev) return CB_EINVAL;
    if (L->d.mode == CB_PROPAGATE) return CB_EINVAL;     // such a layer keeps no input state
    *state_dev = L->S();
    return CB_OK;
}

int cb_layer_export_state(cb_layer_t* L, void* state_out_dev, void* output_out_dev)
{
    if (!L || !output_out_dev) return CB_EINVAL;
    const bool has_state = L->d.mode != CB_PROPAGATE;
    if (has_state != (state_out_dev != nullptr)) return CB_EINVAL;
    if (!L->primed) return CB_ESTATE;
    const size_t b = L->g.bf16 ? 2 : 4;
    if (has_state)
        CB_HIP(hipMemcpyAsync(state_out_dev, L->S(), (size_t)L->g.C * L->g.P * b, hipMemcpyDeviceToDevice, L->st));
    CB_HIP(hipMemcpyAsync(output_out_dev, L->OUT(), (size_t)L->g.O * L->g.Po * b, hipMemcpyDeviceToDevice, L->st));
    return CB_OK;
}

int cb_layer_import_state(cb_layer_t* L, const void* state_in_dev, const void* output_in_dev)
{
    if (!L || !output_in_dev) return CB_EINVAL;
    const bool has_state = L->d.mode != CB_PROPAGATE;
    if (has_state != (state_in_dev != nullptr)) return CB_EINVAL;
    const cb::Geom& g = L->g;
    const size_t b = g.bf16 ? 2 : 4;
    const size_t nS = (size_t)g.C * g.P * b, nO = (size_t)g.O * g.Po * b;
    {   // the sources must not lie inside the layer's own buffer
        const char *a = (const char*)state_in_dev, *o = (const char*)output_in_dev;
        if (a && a < L->state + L->sl.total && a + nS > L->state) return CB_EINVAL;
        if (o < L->state + L->sl.total && o + nO > L->state) return CB_EINVAL;
    }
    if (has_state) {
        CB_HIP(hipMemcpyAsync(L->S(), state_in_dev, nS, hipMemcpyDeviceToDevice, L->st));
        if (L->shadow) CB_HIP(cb::launch_shadow_rebuild(g, L->S(), L->S2(), L->st));
    }
    CB_HIP(hipMemcpyAsync(L->OUT(), output_in_dev, nO, hipMemcpyDeviceToDevice, L->st));
    if (L->OUT2()) {
        cb::Geom go = g;                      // the same transposition, on the output's shape
        go.C = g.O; go.P = g.Po;
        CB_HIP(cb::launch_shadow_rebuild(go, L->OUT(), L->OUT2(), L->st));
    }
    // the change set of "the last frame" is empty: both input maps, the dilated map, N and the two counters of M
    CB_HIP(cb::launch_fill32((uint32_t*)L->mbits(), ((size_t)(g.P + 63) / 64) * 4, 0u, L->st));
    CB_HIP(cb::launch_fill32((uint32_t*)L->mtbits(), (size_t)g.Ho * g.WWo * 2, 0u, L->st));
    CB_HIP(cb::launch_fill32((uint32_t*)L->ctl(), 3, 0u, L->st));       // CTL_COUNT, CTL_NIN_A, CTL_NIN_B
    L->cur_in_bits = L->mbits();
    L->cur_in_pitch = g.W;
    L->cur_in_own = has_state;
    L->cur_mtbits = L->mtbits();
    L->cur_idx = L->idx();
    L->cur_count = L->ctl() + cb::CTL_COUNT;
    L->primed = true;
    // For the layers and pooling stages that consume this one, the import is a frame they cannot follow
    // through its change set: a count that skips one makes them compare (or recompute, or pool) everything once.
    L->frames += 2;
    L->chain_src = nullptr;
    L->chain_frames = 0;
    L->ev_used = 0;
    return CB_OK;
}

int cb_layer_matrices(const cb_layer_t* L, const void** xprime_dev, const void** yprime_dev,
                      const int32_t** ld_ncols_dev)
{
    if (!L) return CB_EINVAL;
    if (L->fused) return CB_ESTATE;
    if (xprime_dev) *xprime_dev = L->X();
    if (yprime_dev) *yprime_dev = L->Y();
    if (ld_ncols_dev) *ld_ncols_dev = L->ctl() + cb::CTL_LD;
    return CB_OK;
}

int cb_layer_out_shape(const cb_layer_t* L, int32_t* c_out, int32_t* h_out, int32_t* w_out)
{
    if (!L) return CB_EINVAL;
    if (c_out) *c_out = L->g.O;
    if (h_out) *h_out = L->g.Ho;
    if (w_out) *w_out = L->g.Wo;
    return CB_OK;
}

int cb_layer_set_timing(cb_layer_t* L, int32_t on)
{
    if (!L) return CB_EINVAL;
    if (on && L->ev.empty()) {
        const int n = 2 * (4 + 3 * L->nchunks);
        L->ev.resize(n);
        L->ev_step.assign(n / 2, 0);
        for (int i = 0; i < n; ++i) {
            hipError_t e = hipEventCreate(&L->ev[i]);
            if (e != hipSuccess) {
                for (int j = 0; j < i; ++j) (void)hipEventDestroy(L->ev[j]);
                L->ev.clear();
                return hip_fail(e);
            }
        }
    }
    L->timing = on != 0;
    L->ev_used = 0;
    return CB_OK;
}

int cb_layer_stats(cb_layer_t* L, cb_stats* stats)
{
    if (!L || !stats) return CB_EINVAL;
    std::memset(stats, 0, sizeof(*stats));
    CB_HIP(hipStreamSynchronize(L->st));
    if (!L->primed) return CB_OK;
    int ctl[cb::CTL_SLOTS];
    CB_HIP(hipMemcpy(ctl, L->ctl(), sizeof(ctl), hipMemcpyDeviceToHost));
    stats->scan_recounts = ctl[cb::CTL_RECOUNTS];
    int n = 0;
    CB_HIP(hipMemcpy(&n, L->cur_count, sizeof(int), hipMemcpyDeviceToHost));
    stats->n_changed_out = n;
    // (the counter of the last frame: the one that the frame count, already advanced, selected for it)
    stats->n_changed_in = L->d.mode == CB_PROPAGATE ? -1 : ctl[cb::CTL_NIN_A + ((ctl[cb::CTL_FRAME] - 1) & 1)];
    stats->ops = 2LL * L->g.O * L->g.R * (long long)n;
    if (L->timing && L->ev_used >= 2) {
        // each pair holds the begin and end time stamps of one kernel dispatch
        for (int i = 0; i + 1 < L->ev_used; i += 2) {
            float ms = 0.f;
            CB_HIP(hipEventElapsedTime(&ms, L->ev[i], L->ev[i + 1]));
            stats->us_step[L->ev_step[i / 2]] += ms * 1000.f;
        }
        float ms = 0.f;
        CB_HIP(hipEventElapsedTime(&ms, L->ev[0], L->ev[L->ev_used - 1]));
        stats->us_step[CB_STEP_TOTAL] = ms * 1000.f;
    }
    return CB_OK;
}

int cb_set_scan_wait_limit(int32_t polls)
{
    if (polls < 0) return CB_EINVAL;
    g_scan_wait_limit.store(polls, std::memory_order_relaxed);
    return CB_OK;
}

int cb_layer_reset(cb_layer_t* L)
{
    if (!L) return CB_EINVAL;
    L->primed = false;
    return CB_OK;
}

int cb_layer_destroy(cb_layer_t* L)
{
    if (!L) return CB_EINVAL;
    for (hipEvent_t e : L->ev) (void)hipEventDestroy(e);
    delete L;
    return CB_OK;
}

int cb_pool_workspace_bytes(const cb_layer_t* prod, int32_t window, size_t* state_bytes)
{
    if (!prod || window < 1 || window > 8) return CB_EINVAL;
    cb_pool p;
    p.O = prod->g.O; p.Ho = prod->g.Ho; p.Wo = prod->g.Wo; p.bf16 = prod->g.bf16;
    p.cl = prod->d.keep_output_channel_last != 0;
    p.Hp = (p.Ho + window - 1) / window; p.Wp = (p.Wo + window - 1) / window; p.WWp = (p.Wp + 63) / 64;
    pool_layout(&p);
    if (state_bytes) *state_bytes = p.total;
    return CB_OK;
}

int cb_pool_create(const cb_layer_t* prod, int32_t window, void* state_dev, size_t state_bytes,
                   void* hip_stream, cb_pool_t** out)
{
    if (!out) return CB_EINVAL;
    *out = nullptr;
    if (!prod || window < 1 || window > 8 || !state_dev) return CB_EINVAL;
    if ((uintptr_t)state_dev & 255) return CB_EINVAL;
    if ((hipStream_t)hip_stream != prod->st) return CB_EINVAL;   // consumes the producer's list in stream order
    cb_pool* p = new (std::nothrow) cb_pool();
    if (!p) return CB_ENOMEM;
    p->prod = prod; p->w = window;
    p->O = prod->g.O; p->Ho = prod->g.Ho; p->Wo = prod->g.Wo; p->WWo = prod->g.WWo; p->bf16 = prod->g.bf16;
    p->cl = prod->d.keep_output_channel_last != 0;
    p->Hp = (p->Ho + window - 1) / window; p->Wp = (p->Wo + window - 1) / window; p->WWp = (p->Wp + 63) / 64;
    p->st = (hipStream_t)hip_stream;
    p->state = (char*)state_dev;
    p->done_frames = -1;
    p->primed = false;
    pool_layout(p);
    if (state_bytes < p->total) { delete p; return CB_ENOMEM; }
    hipError_t e = hipMemsetAsync(state_dev, 0, p->total, p->st);
    if (e != hipSuccess) { delete p; return hip_fail(e); }
    *out = p;
    return CB_OK;
}

int cb_pool_process(cb_pool_t* p, const void** output_dev)
{
    if (!p) return CB_EINVAL;
    if (!p->prod->primed) return CB_ESTATE;
    // The producer's index list names what its LAST frame rewrote: before the first call and after a missed
    // producer frame (or an imported producer state) every pooled cell is recomputed.
    const bool all = !p->primed || p->done_frames + 1 != p->prod->frames;
    CB_HIP(cb::launch_pool(p->O, p->Ho, p->Wo, p->w, p->bf16, p->prod->OUT(), all ? nullptr : p->prod->cur_idx,
                           p->prod->cur_count, p->POOL(), p->POOL2(), p->st));
    p->primed = true;
    p->done_frames = p->prod->frames;
    if (output_dev) *output_dev = p->POOL();
    return CB_OK;
}

int cb_pool_changes(cb_pool_t* p, const uint8_t** pm_dev)
{
    if (!p || !pm_dev) return CB_EINVAL;
    if (!p->primed) return CB_ESTATE;
    int rc = pool_mask(p);
    if (rc) return rc;
    CB_HIP(cb::launch_expand_bits(p->pmbits(), 64L * p->WWp, p->Hp, p->Wp, p->pm_u8(), p->st));
    *pm_dev = p->pm_u8();
    return CB_OK;
}

int cb_pool_out_shape(const cb_pool_t* p, int32_t* c, int32_t* h_out, int32_t* w_out)
{
    if (!p) return CB_EINVAL;
    if (c) *c = p->O;
    if (h_out) *h_out = p->Hp;
    if (w_out) *w_out = p->Wp;
    return CB_OK;
}

int cb_pool_destroy(cb_pool_t* p)
{
    if (!p) return CB_EINVAL;
    delete p;
    return CB_OK;
}

}  // extern "C"

// ------------------------------------------------------------------ chains of layers and threshold selection
namespace {

struct ChainOut {
    const void* ptr;
    size_t elems;
    int bf16;
};

int check_chain(const cb_stage* st, int n)
{
    if (!st || n < 1) return CB_EINVAL;
    for (int s = 0; s < n; ++s) {
        if (!st[s].layer) return CB_EINVAL;
        if (st[s].layer->st != st[0].layer->st) return CB_EINVAL;
        if (st[s].pool && (st[s].pool->prod != st[s].layer || st[s].pool->st != st[0].layer->st)) return CB_EINVAL;
        if (s == 0 && st[s].layer->d.mode == CB_PROPAGATE) return CB_EINVAL;
    }
    return CB_OK;
}

ChainOut chain_output(const cb_stage* st, int n)
{
    const cb_stage& e = st[n - 1];
    ChainOut o;
    o.bf16 = e.layer->g.bf16;
    if (e.pool) { o.ptr = e.pool->POOL(); o.elems = (size_t)e.pool->O * e.pool->Hp * e.pool->Wp; }
    else { o.ptr = e.layer->OUT(); o.elems = (size_t)e.layer->g.O * e.layer->g.Po; }
    return o;
}

struct SelectLayout {
    size_t refs, ref_pitch, partial, acc, total;
};

SelectLayout select_layout(const cb_stage* st, int n, int n_sequences)
{
    const ChainOut o = chain_output(st, n);
    SelectLayout L;
    L.ref_pitch = align256(o.elems * (o.bf16 ? 2 : 4));
    size_t off = 0;
    L.refs = off;    off += L.ref_pitch * (size_t)n_sequences;
    L.partial = off; off += align256(cb::SSD_PARTIALS * sizeof(double));
    L.acc = off;     off += 256;
    L.total = off;
    return L;
}

// all frames of one sequence from a reset chain; the output of the last frame stays in the last stage
int run_sequence(const cb_stage* st, int n, const void* const* frames, int n_frames, const float* taus)
{
    for (int s = 0; s < n; ++s) st[s].layer->primed = false;
    for (int t = 0; t < n_frames; ++t) {
        const int rc = cb_network_forward(st, n, frames[t], taus, nullptr);
        if (rc) return rc;
    }
    return CB_OK;
}

// mean squared difference between the chain's last-frame outputs and the stored references
int chain_quality(const cb_stage* st, int n, const void* const* frames, int n_sequences, int n_frames,
                  const float* taus, char* ws, const SelectLayout& L, double* q)
{
    hipStream_t stream = st[0].layer->st;
    const ChainOut o = chain_output(st, n);
    double* acc = reinterpret_cast<double*>(ws + L.acc);
    CB_HIP(hipMemsetAsync(acc, 0, sizeof(double), stream));
    for (int i = 0; i < n_sequences; ++i) {
        const int rc = run_sequence(st, n, frames + (size_t)i * n_frames, n_frames, taus);
        if (rc) return rc;
        CB_HIP(cb::launch_ssd(o.ptr, ws + L.refs + L.ref_pitch * i, o.elems, o.bf16,
                              reinterpret_cast<double*>(ws + L.partial), acc, 1, stream));
    }
    double sum = 0.0;
    CB_HIP(hipMemcpyAsync(&sum, acc, sizeof(double), hipMemcpyDeviceToHost, stream));
    CB_HIP(hipStreamSynchronize(stream));
    *q = sum / ((double)n_sequences * (double)o.elems);
    return CB_OK;
}

}  // namespace

extern "C" {

int cb_network_forward(const cb_stage* stages, int32_t n_stages, const void* input_dev, const float* taus,
                       const void** output_dev)
{
    int rc = check_chain(stages, n_stages);
    if (rc) return rc;
    if (!input_dev || !taus) return CB_EINVAL;
    const void* x = input_dev;
    for (int s = 0; s < n_stages; ++s) {
        cb_layer* L = stages[s].layer;
        const cb_layer* pl = (s > 0 && !stages[s - 1].pool) ? stages[s - 1].layer : nullptr;
        const cb_pool* pp = s > 0 ? stages[s - 1].pool : nullptr;
        const void* out = nullptr;
        if (s == 0) rc = cb_process_frame(L, x, taus[0], &out);
        else if (L->d.mode == CB_PROPAGATE) rc = cb_process_frame_propagated(L, x, pl, pp, &out);
        else rc = cb_process_frame_chained(L, x, pl, pp, taus[s], &out);
        if (rc) return rc;
        x = out;
        if (stages[s].pool) {
            rc = cb_pool_process(stages[s].pool, &out);
            if (rc) return rc;
            x = out;
        }
    }
    if (output_dev) *output_dev = x;
    return CB_OK;
}

int cb_sum_squared_diff(const void* a_dev, const void* b_dev, size_t n, int32_t dtype, void* workspace_dev,
                        double* sum_host, void* hip_stream)
{
    if (!a_dev || !b_dev || !workspace_dev || !sum_host) return CB_EINVAL;
    if (dtype != CB_F32 && dtype != CB_BF16) return CB_EINVAL;
    if ((uintptr_t)workspace_dev & 255) return CB_EINVAL;
    hipStream_t stream = (hipStream_t)hip_stream;
    double* partial = reinterpret_cast<double*>(workspace_dev);
    double* acc = partial + cb::SSD_PARTIALS;
    CB_HIP(cb::launch_ssd(a_dev, b_dev, n, dtype == CB_BF16, partial, acc, 0, stream));
    CB_HIP(hipMemcpyAsync(sum_host, acc, sizeof(double), hipMemcpyDeviceToHost, stream));
    CB_HIP(hipStreamSynchronize(stream));
    return CB_OK;
}

int cb_sum_squared_diff_noalloc(const void* a_dev, const void* b_dev, size_t n, int32_t dtype, double* sum_host,
                                void* hip_stream)
{
    if (!a_dev || !b_dev || !sum_host) return CB_EINVAL;
    if (dtype != CB_F32 && dtype != CB_BF16) return CB_EINVAL;
    if (n > CB_METRIC_NOALLOC_MAX_ELEMS) return CB_ENOMEM;
    hipStream_t stream = (hipStream_t)hip_stream;
    double *partial = nullptr, *acc = nullptr;
    CB_HIP(cb::ssd_static_scratch(&partial, &acc));
    // the partial sums and the total are overwritten, never accumulated: nothing to clear from the last call
    CB_HIP(cb::launch_ssd(a_dev, b_dev, n, dtype == CB_BF16, partial, acc, 0, stream));
    CB_HIP(hipMemcpyAsync(sum_host, acc, sizeof(double), hipMemcpyDeviceToHost, stream));
    CB_HIP(hipStreamSynchronize(stream));
    return CB_OK;
}

int cb_select_workspace_bytes(const cb_stage* stages, int32_t n_stages, int32_t n_sequences, size_t* bytes)
{
    const int rc = check_chain(stages, n_stages);
    if (rc) return rc;
    if (n_sequences < 1 || !bytes) return CB_EINVAL;
    *bytes = select_layout(stages, n_stages, n_sequences).total;
    return CB_OK;
}

int cb_select_thresholds(const cb_stage* stages, int32_t n_stages, const void* const* frames_dev,
                         int32_t n_sequences, int32_t n_frames, const cb_select_params* params,
                         const double* max_loss, void* workspace_dev, size_t workspace_bytes, float* taus_out,
                         double* loss_out, int32_t* steps_out)
{
    int rc = check_chain(stages, n_stages);
    if (rc) return rc;
    if (!frames_dev || n_sequences < 1 || n_frames < 1 || !params || !max_loss || !workspace_dev || !taus_out)
        return CB_EINVAL;
    if (!(params->tau0 > 0.0f) || !(params->factor > 1.0f) || std::isinf(params->tau0) || std::isinf(params->factor) ||
        params->max_steps < 1 || params->reserved != 0)
        return CB_EINVAL;
    for (long i = 0; i < (long)n_sequences * n_frames; ++i) if (!frames_dev[i]) return CB_EINVAL;
    if ((uintptr_t)workspace_dev & 255) return CB_EINVAL;
    const SelectLayout L = select_layout(stages, n_stages, n_sequences);
    if (workspace_bytes < L.total) return CB_ENOMEM;
    char* ws = static_cast<char*>(workspace_dev);
    hipStream_t stream = stages[0].layer->st;
    const ChainOut o = chain_output(stages, n_stages);

    std::vector<float> taus((size_t)n_stages, 0.0f);
    // the original model's outputs: every threshold zero (Sec. III-F, first paragraph)
    for (int i = 0; i < n_sequences; ++i) {
        rc = run_sequence(stages, n_stages, frames_dev + (size_t)i * n_frames, n_frames, taus.data());
        if (rc) return rc;
        CB_HIP(hipMemcpyAsync(ws + L.refs + L.ref_pitch * i, o.ptr, o.elems * (o.bf16 ? 2 : 4),
                              hipMemcpyDeviceToDevice, stream));
    }
    // first to last layer: raise this layer's threshold by the factor until the loss it adds, relative
    // to the same chain with this layer at zero, exceeds its limit; keep the value before that
    for (int s = 0; s < n_stages; ++s) {
        if (loss_out) loss_out[s] = 0.0;
        if (steps_out) steps_out[s] = 0;
        if (stages[s].layer->d.mode == CB_PROPAGATE) continue;      // no threshold of its own
        double base = 0.0;
        rc = chain_quality(stages, n_stages, frames_dev, n_sequences, n_frames, taus.data(), ws, L, &base);
        if (rc) return rc;
        float tau = params->tau0, kept = 0.0f;
        for (int step = 0; step < params->max_steps; ++step) {
            taus[s] = tau;
            double q = 0.0;
            rc = chain_quality(stages, n_stages, frames_dev, n_sequences, n_frames, taus.data(), ws, L, &q);
            if (rc) return rc;
            if (steps_out) steps_out[s] = step + 1;
            if (q - base > max_loss[s]) break;
            kept = tau;
            if (loss_out) loss_out[s] = q - base;
            tau = tau * params->factor;                             // float32, as the layers take it
            if (std::isinf(tau)) break;
        }
        taus[s] = kept;
    }
    for (int s = 0; s < n_stages; ++s) taus_out[s] = taus[s];
    return CB_OK;
}

}  // extern "C"
