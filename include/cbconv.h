/*
 * cbconv.h -- C ABI of the change-based convolution (CBconv) library for
 * AMD Instinct MI355X (gfx950).
 *
 * One cb_layer is the stateful replacement of a convolution layer that the
 * paper describes in Sec. III-A ("Processing Steps") with the closed-loop input
 * state of Sec. III-C: per frame it runs change detection (Eq. 3), change-map
 * dilation by the filter footprint (Eq. 4), change-index extraction, matrix
 * generation for the listed output pixels only, the matrix multiplication of
 * Eq. 2 on that reduced matrix, and the output update with fused bias + ReLU.
 * One cb_pool is the change-based 2x2 max-pooling of Sec. III-E that re-uses
 * its producer's change indexes.
 *
 * General rules
 *  - Every pointer named *_dev is DEVICE memory on the GPU that was current
 *    when the layer was created; everything else is host memory.
 *  - Tensors are dense, batch 1, channel-major: C x H x W, row-major
 *    ("NCHW"; the paper processes single frames, Sec. III-B item 1).
 *    Element type is the layer's dtype (float32, or bfloat16 bit patterns).
 *  - All work is enqueued on the HIP stream given at create time and is
 *    asynchronous; only the calls that hand a number to the host wait for the
 *    stream (cb_layer_stats, cb_sum_squared_diff*, cb_select_thresholds)
 *    (and cb_layer_create, once, when the layer uses the fused back end's
 *    channel-first kernel: it uploads a small table built on the host).
 *    No entry point allocates or frees device memory: the caller provides the
 *    state and scratch buffers (cb_layer_workspace_bytes says how large).
 *    Nothing on the per-frame path uses hipMemsetAsync, and nothing that varies
 *    from frame to frame is decided on the host (the number of listed pixels and
 *    the alternation of a layer's two map buffers live in device memory), so the
 *    per-frame calls may be captured into a HIP graph, any number of frames per
 *    capture, and replays may be mixed with eager calls on the same layer.  What
 *    a capture does freeze is what the host decides per call from the calls it
 *    has seen: whether a frame is a full update (the first one after create or
 *    reset -- capture later frames), and, for cb_process_frame_chained and
 *    cb_process_frame_propagated, whether the consumer is in lockstep with its
 *    producer, and for cb_pool_process whether the stage has seen every frame of
 *    its producer -- capture producer, pooling stage and consumer together,
 *    after a first eager frame of all of them, and replay them together.  (The
 *    other way round nothing breaks, it is only slower: a stage called eagerly
 *    on a producer whose frames come from a replayed graph cannot see those
 *    frames on the host and compares, recomputes or pools everything.)
 *  - Every function returns CB_OK (0) or a negative cb_status; nothing throws
 *    or aborts.  After CB_EHIP, cb_last_hip_error() gives the HIP error code.
 *  - Calls on one layer are not thread-safe; different layers on different
 *    streams are independent, provided they do not share a scratch buffer.
 */
#ifndef CBCONV_H
#define CBCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cb_layer cb_layer_t;
typedef struct cb_pool cb_pool_t;

typedef enum {
    CB_OK = 0,
    CB_EINVAL = -1,   /* bad descriptor, NULL pointer, misaligned buffer, tau < 0 or NaN */
    CB_ENOMEM = -2,   /* state or scratch buffer smaller than required */
    CB_EHIP = -3,     /* a HIP runtime call failed; see cb_last_hip_error() */
    CB_ESTATE = -4    /* call out of order (e.g. pooling before the producer's first frame) */
} cb_status;

typedef enum { CB_F32 = 0, CB_BF16 = 1 } cb_dtype;

/* Where the layer's change map comes from. */
typedef enum {
    CB_CLOSED_LOOP = 0,   /* Sec. III-C: compare against the input state, which is
                             updated only at pixels that triggered (default) */
    CB_FEED_FORWARD = 1,  /* Sec. III-A / Fig. 2a: compare against the previous
                             input, keep the whole current input */
    CB_PROPAGATE = 2      /* Sec. III-E: no detection; the producer's dilated map is
                             taken as this layer's change map (for a 1x1 filter the
                             producer's index list is re-used as is) */
} cb_mode;

/* How the last three processing steps are executed. */
typedef enum {
    CB_BACKEND_AUTO = 0,      /* fused where available, else explicit */
    CB_BACKEND_EXPLICIT = 1,  /* three kernels; X' and Y' are materialised in the scratch buffer */
    CB_BACKEND_FUSED = 2      /* one kernel: receptive fields gathered into LDS, MFMA, bias/ReLU, scatter;
                                 X' and Y' never exist in memory (CB_EINVAL where it is not available:
                                 kh*kw above 60, or a gather table beyond 40 KB of
                                 LDS: c_in above about 4800 for 1x1 filters, c_in*kh*kw above about
                                 13 000 for 3x3 and wider ones) */
} cb_backend;

/* Geometry of one layer.  Output size: Ho = (h_in + 2*pad - kh)/stride + 1, same
 * for Wo.  Limits: 1 <= kh,kw <= 31, 0 <= pad <= 31, stride >= 1, the padded input
 * not smaller than the filter, h_in*w_in and Ho*Wo below 2^30, the input tensor
 * c_in*h_in*w_in not above 2^32 - 256 bytes (the kernels address the input state
 * with 32-bit byte offsets), c_in*kh*kw below 2^24. */
typedef struct {
    int32_t c_in, c_out, kh, kw, stride, pad, h_in, w_in;
    int32_t dtype;   /* cb_dtype */
    int32_t relu;    /* 1: ReLU fused into the output update (Sec. III-A, Output Updating) */
    int32_t mode;    /* cb_mode */
    int32_t backend; /* cb_backend */
    int32_t keep_output_channel_last;  /* 1: the layer also keeps its cached output pixel-major (Ho*Wo x c_out), updated
                                          at the same pixels, for CB_PROPAGATE consumers that gather from it; a
                                          pooling stage on such a layer keeps its output both ways too.  Fused back
                                          end only; c_out a power of two, at least 16 (float32) / 32 (bfloat16) */
    int32_t gather_channel_last;       /* 1 (CB_PROPAGATE layers only): gather from the producer's pixel-major output,
                                          which the producer must keep (CB_EINVAL from cb_process_frame_propagated
                                          otherwise).  Fused back end only; c_in a power of two, at least 16 / 32 */
    int32_t reserved[2];   /* must be zero */
} cb_layer_desc;

/* Per-frame statistics of the last processed frame. */
enum { CB_STEP_DETECT = 0, CB_STEP_DILATE, CB_STEP_COMPACT, CB_STEP_GATHER, CB_STEP_GEMM,
       CB_STEP_UPDATE, CB_STEP_FUSED /* gather+GEMM+update of the fused back end */,
       CB_STEP_STATE /* state (and shadow) update of the changed pixels where it is a kernel of its own: float32
                        layers with a shadow whose state is beyond the last-level cache; elsewhere part of DETECT */,
       CB_STEP_TOTAL, CB_NUM_STEPS };
typedef struct {
    int32_t n_changed_in;    /* M: input pixels with m = 1 (Eq. 3) */
    int32_t n_changed_out;   /* N: listed output pixels (Eq. 4) */
    int64_t ops;             /* 2 * c_out * (c_in*kh*kw) * N multiply-adds counted as 2 */
    float us_step[CB_NUM_STEPS];   /* GPU time of each step's kernel dispatches in microseconds
                                      (begin/end time stamps of the dispatches; TOTAL = first begin
                                      to last end); zeros unless cb_layer_set_timing switched it on */
    int32_t scan_recounts;   /* since create: how often a workgroup of the index extraction recomputed a
                                predecessor's count itself because its bounded wait for it ran out (see
                                cb_set_scan_wait_limit); 0 on an idle GPU; the results are the same */
    int32_t reserved;
} cb_stats;

/* Sizes of the two caller-provided device buffers for a layer.
 *  state_bytes   : per-layer, lives as long as the layer (input state, cached
 *                  output, bit-packed change maps, index list, repacked filter
 *                  matrix -- the "variables to be stored per-layer" of Fig. 2;
 *                  closed-loop layers on the fused back end with a power-of-two
 *                  number of input channels -- float32 from 16 on, bfloat16
 *                  from 32 on -- keep a second, pixel-major copy of the input
 *                  state for the gather).
 *  scratch_bytes : X' and Y' matrices and block counters; may be shared by
 *                  layers that run on the same stream (Sec. III-B).  This is the
 *                  recommended size; cb_layer_create accepts any size not below
 *                  cb_layer_min_scratch_bytes and processes the listed pixels in
 *                  column chunks that fit.
 * Both buffers must be 256-byte aligned. */
int cb_layer_workspace_bytes(const cb_layer_desc *desc, size_t *state_bytes, size_t *scratch_bytes);
int cb_layer_min_scratch_bytes(const cb_layer_desc *desc, size_t *scratch_bytes);

/* Create a layer.  w_oihw_dev: c_out x c_in x kh x kw filter tensor == the filter
 * matrix K of Eq. 2; bias_dev: c_out values or NULL (zero bias); both in the
 * layer's dtype, both copied (repacked) during the call's stream work -- they may
 * be freed once the stream has passed this point.  The state buffer is cleared.
 * hip_stream is a hipStream_t (NULL = default stream).  On success *out receives
 * the layer, to be released with cb_layer_destroy (which frees host memory only). */
int cb_layer_create(const cb_layer_desc *desc, const void *w_oihw_dev, const void *bias_dev,
                    void *state_dev, size_t state_bytes, void *scratch_dev, size_t scratch_bytes,
                    void *hip_stream, cb_layer_t **out);

/* Process one frame (Sec. III-A steps 1-5 with the state update of Sec. III-C).
 * input_dev: c_in x h_in x w_in, borrowed until the enqueued work has run; it must
 * not alias this layer's own state.  tau >= 0 is the change threshold of Eq. 3
 * (strict '>' on |difference| in float32; tau = 0 reproduces the dense layer,
 * Sec. III-F).  The first frame after create / reset is a full update.
 * *output_dev receives the cached output c_out x Ho x Wo (post bias, post ReLU),
 * owned by the layer, valid until the next call on this layer; it is what the next
 * layer takes as its input.
 * For a CB_PROPAGATE layer use cb_process_frame_propagated instead. */
int cb_process_frame(cb_layer_t *layer, const void *input_dev, float tau, const void **output_dev);

/* Sec. III-E: process a frame whose change set is taken from `producer` (the
 * layer, or the pooling stage, that wrote input_dev) instead of being detected.
 * input_dev must be that producer's output pointer (CB_EINVAL otherwise).
 * Exactly one of producer_layer / producer_pool is non-NULL; its output geometry
 * must equal this layer's input geometry, and it must have processed its frame
 * on the same stream.  The layer must have been created with CB_PROPAGATE.
 * Lockstep: the producer's change set describes its LAST frame only, so the layer
 * has to be called once per producer frame.  If the producer has processed any
 * other number of frames since this layer's last call (or the producer is another
 * one), every output of this layer is recomputed once, as on its first frame.
 * CB_ESTATE if a producing pooling stage has not processed its producer's last
 * frame.  (Frames are counted on the host: frames of a replayed HIP graph do not
 * count, so eager and replayed calls of one chain must not be mixed without a
 * cb_layer_reset of the consumers in between.) */
int cb_process_frame_propagated(cb_layer_t *layer, const void *input_dev,
                                const cb_layer_t *producer_layer, const cb_pool_t *producer_pool,
                                const void **output_dev);

/* Same result as cb_process_frame for a layer whose input is the cached output of
 * `producer` (a change-based layer, or the pooling stage after one), at a fraction
 * of the cost: Eq. 3 is evaluated at the producer's listed pixels only.  Every
 * other input pixel was left untouched by the producer, so it holds the bits it
 * held a frame ago, when it did not exceed tau against the same input state, and
 * cannot exceed it now (the observation behind Sec. III-E, used here without
 * giving up the threshold).  input_dev must be the producer's output pointer, the
 * layer a CB_CLOSED_LOOP or CB_FEED_FORWARD one, same stream.  The restriction is
 * applied only while this layer has seen every frame of the producer since its
 * own last frame and (closed loop) tau is not below that frame's; after create /
 * reset, a skipped producer frame, a call of cb_process_frame in between or a
 * lowered tau, the whole input is compared once and the lockstep starts again.  CB_ESTATE if a producing pooling stage has not processed its
 * producer's last frame. */
int cb_process_frame_chained(cb_layer_t *layer, const void *input_dev,
                             const cb_layer_t *producer_layer, const cb_pool_t *producer_pool,
                             float tau, const void **output_dev);

/* Change set of the last frame, for parity checks and chaining.  m_in_dev: h_in x
 * w_in bytes (0/1), Eq. 3; m_out_dev: Ho x Wo bytes (0/1), Eq. 4; idx_dev: int32
 * linear output indices yo*Wo+xo in ascending order; count_dev: one int32, N.
 * The byte maps are expanded from the internal bit-packed maps by work enqueued in
 * this call.  Any of the four out-pointers may be NULL. */
int cb_layer_changes(cb_layer_t *layer, const uint8_t **m_in_dev, const uint8_t **m_out_dev,
                     const int32_t **idx_dev, const int32_t **count_dev);

/* The layer's input state (c_in x h_in x w_in) and, for inspection in tests, the
 * X' (R x ld) and Y' (c_out x ld) matrices of the last processed column chunk with
 * their leading dimension, column count and number of k-splits (device int32[3]: {ld, ncols,
 * nsplit}; Y' holds nsplit partial products of O x ld each, which the output update adds).
 * Only layers with the explicit back end have these matrices (CB_ESTATE otherwise). */
int cb_layer_state(const cb_layer_t *layer, const void **state_dev);
int cb_layer_matrices(const cb_layer_t *layer, const void **xprime_dev, const void **yprime_dev,
                      const int32_t **ld_ncols_dev);

/* Checkpoint and resume.  What a layer carries from one frame to the next is its input state (Sec. III-C: the
 * values its last detected changes were measured against) and its cached output (Sec. III-A, Output
 * Updating); a change-based network does not accumulate error in anything else (Sec. III-C, III-F).
 * cb_layer_export_state copies both into caller buffers (device memory, the layer's element type:
 * c_in x h_in x w_in and c_out x Ho x Wo, dense); cb_layer_import_state copies them back in -- into the
 * same layer later, or into a layer of the same description in another process -- brings the layer's other
 * copies of the state up to date, and leaves the layer as if it had just processed a frame in which nothing
 * changed (empty change maps, N = M = 0): the next frame is an ordinary change-based frame, no full update.
 * CB_PROPAGATE layers keep no input state: pass NULL for it (CB_EINVAL otherwise, and for a missing state on
 * the other modes).  Both calls are stream-ordered (device-to-device copies and small kernels, no
 * synchronisation, no allocation); the buffers are the caller's and must not overlap the layer's own.
 * Export needs a layer that has processed a frame (CB_ESTATE otherwise).  Consumers of an imported layer
 * (cb_process_frame_chained / _propagated, pooling stages) treat the import like a frame of the producer they
 * missed: their next call compares, recomputes or pools everything once. */
int cb_layer_export_state(cb_layer_t *layer, void *state_out_dev, void *output_out_dev);
int cb_layer_import_state(cb_layer_t *layer, const void *state_in_dev, const void *output_in_dev);

/* Output geometry. */
int cb_layer_out_shape(const cb_layer_t *layer, int32_t *c_out, int32_t *h_out, int32_t *w_out);

/* Switch per-step timing (a begin/end event pair per kernel dispatch) on or off. */
int cb_layer_set_timing(cb_layer_t *layer, int32_t on);
/* Waits for the layer's stream, then fills *stats for the last frame. */
int cb_layer_stats(cb_layer_t *layer, cb_stats *stats);
/* The one-launch index extraction (Sec. III-A, "Change Indexes Extraction") scans the per-workgroup
 * counts in a single pass: a workgroup polls for the counts of the workgroups before it.  After
 * `polls` unsuccessful polls of one count it recomputes that count from the change map instead, so
 * the index list and N never depend on how the GPU schedules workgroups (other streams or processes
 * may hold compute units).  Process-wide; default 2^20 (tens of milliseconds); 0 = never wait.  Meant
 * for tests of that path; cb_stats.scan_recounts tells how often it was taken. */
int cb_set_scan_wait_limit(int32_t polls);
/* The next frame will be a full update (as after create). */
int cb_layer_reset(cb_layer_t *layer);
int cb_layer_destroy(cb_layer_t *layer);

/* Change-based max-pooling (Sec. III-E, last paragraph; Table I geometry):
 * window x window, stride = window, ceil mode with clipped border windows, on the
 * cached output of `producer`.  state buffer: pooled output c x Hp x Wp plus the
 * pooled change map; size from cb_pool_workspace_bytes; 256-byte aligned. */
int cb_pool_workspace_bytes(const cb_layer_t *producer, int32_t window, size_t *state_bytes);
int cb_pool_create(const cb_layer_t *producer, int32_t window, void *state_dev, size_t state_bytes,
                   void *hip_stream, cb_pool_t **out);
/* Recompute the pooled cells that hold a listed producer pixel of the producer's
 * last frame -- every cell on the first call and whenever the stage has not been called
 * for each frame of the producer (the list describes the last frame only).
 * *output_dev: c x Hp x Wp, owned by the pooling stage. */
int cb_pool_process(cb_pool_t *pool, const void **output_dev);
/* Pooled change map of the last frame: Hp x Wp bytes (0/1), the OR of the
 * producer's dilated map over each window. */
int cb_pool_changes(cb_pool_t *pool, const uint8_t **pm_dev);
int cb_pool_out_shape(const cb_pool_t *pool, int32_t *c, int32_t *h_out, int32_t *w_out);
int cb_pool_destroy(cb_pool_t *pool);

/* ---- chains of layers, and the threshold selection of Sec. III-F -------------- */

/* One stage of a chain: a change-based convolution and, optionally, the change-based
 * pooling stage fed by it (NULL = none).  All stages of a chain share one stream;
 * stage s+1 takes the output of stage s as its input. */
typedef struct {
    cb_layer_t *layer;
    cb_pool_t *pool;
} cb_stage;

/* One frame through a chain of n_stages stages (Sec. III-E, Fig. 3: the layers of a
 * network run one after the other, each on the cached output of the one before).
 * taus[s] is the threshold of stage s (ignored by CB_PROPAGATE layers, which take
 * their change set from the stage before; stage 0 must not be one).  Stages after
 * the first evaluate Eq. 3 at the pixels their producer rewrote
 * (cb_process_frame_chained: same result as comparing the whole input).
 * *output_dev (may be NULL) receives the last stage's output.  Asynchronous. */
int cb_network_forward(const cb_stage *stages, int32_t n_stages, const void *input_dev, const float *taus,
                       const void **output_dev);

/* The quality metric Sec. III-F offers for sequences without annotated frames: the
 * change-based model's output is measured against the output of the unmodified
 * model.  Here as a sum of squared differences of two device tensors of n
 * elements of `dtype`, accumulated in float64 in a fixed order (the result does not
 * depend on scheduling).  workspace_dev: CB_METRIC_WORKSPACE_BYTES bytes, 256-byte
 * aligned.  Waits for the stream; *sum_host is host memory. */
#define CB_METRIC_WORKSPACE_BYTES 4096
int cb_sum_squared_diff(const void *a_dev, const void *b_dev, size_t n, int32_t dtype, void *workspace_dev,
                        double *sum_host, void *hip_stream);

/* cb_sum_squared_diff for callers that cannot provide or allocate a workspace
 * (tight serving loops, harnesses that forbid hipMalloc): same kernels, same
 * result bit for bit, but the partial sums live in a statically allocated device
 * array of the library (2304 bytes on every GPU the library is used on, held until
 * the process ends; its address is looked up on the first call on each device).
 * Allocates and frees nothing.  n above CB_METRIC_NOALLOC_MAX_ELEMS is refused
 * with CB_ENOMEM.  All calls on one GPU share that array: calls that overlap in
 * time on one GPU (different streams or host threads) race and must be serialised
 * by the caller.  Waits for the stream; *sum_host is host memory. */
#define CB_METRIC_NOALLOC_MAX_ELEMS ((size_t)1 << 32)
int cb_sum_squared_diff_noalloc(const void *a_dev, const void *b_dev, size_t n, int32_t dtype, double *sum_host,
                                void *hip_stream);

/* Threshold selection, Sec. III-F ("Threshold Selection"): all thresholds start at
 * zero; the stages are visited from first to last; the threshold of the stage being
 * visited starts at tau0 and is multiplied by `factor` (float32 arithmetic) until
 * the quality loss the stage introduces -- the metric with this threshold minus the
 * metric with this stage's threshold at zero, earlier stages at their selected
 * values, later ones at zero -- exceeds max_loss[stage]; the value before that is
 * kept (zero if already tau0 exceeds the limit).  At most max_steps values are tried
 * per stage.  The metric is the mean squared difference between the chain's output
 * for the LAST frame of every sequence and the original model's output for the same
 * frame, which is the chain run with all thresholds zero (Sec. III-F: a threshold of
 * zero yields results identical to the non-change-based layer).  Every sequence is
 * played from a reset chain.
 *  frames_dev   : n_sequences * n_frames device pointers, sequence after sequence,
 *                 each a stage-0 input tensor
 *  max_loss     : n_stages acceptable loss increments (the paper allows them to
 *                 differ per layer)
 *  workspace_dev: cb_select_workspace_bytes bytes, 256-byte aligned
 *  taus_out     : n_stages selected thresholds (0 for CB_PROPAGATE stages)
 *  loss_out     : (may be NULL) loss at the selected threshold of each stage
 *  steps_out    : (may be NULL) thresholds tried per stage
 * Synchronises the stream after every evaluation of the metric; leaves the layers
 * in the state of the last evaluation (reset them before further use). */
typedef struct {
    float tau0;
    float factor;        /* > 1 (the paper's example: 1.1) */
    int32_t max_steps;
    int32_t reserved;    /* must be zero */
} cb_select_params;
int cb_select_workspace_bytes(const cb_stage *stages, int32_t n_stages, int32_t n_sequences, size_t *bytes);
int cb_select_thresholds(const cb_stage *stages, int32_t n_stages, const void *const *frames_dev,
                         int32_t n_sequences, int32_t n_frames, const cb_select_params *params,
                         const double *max_loss, void *workspace_dev, size_t workspace_bytes, float *taus_out,
                         double *loss_out, int32_t *steps_out);

const char *cb_strerror(int status);
int cb_last_hip_error(void);
/* Library version: major*10000 + minor*100 + patch. */
int cb_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CBCONV_H */
