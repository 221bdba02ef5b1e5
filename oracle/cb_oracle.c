/*
 * CPU oracle for change-based convolution (CBconv).  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, step-by-step implementation of what one CBconv layer computes
 * per frame, written from the paper (Sec. III-A "Processing Steps", Sec. III-C
 * "Closed-Loop Formulation", Sec. III-E "Propagating Changes & Pooling").  It
 * shares no code with the HIP library, never builds the X matrix, and
 * accumulates every output in double precision, rounding once.  Only tests,
 * the smoke check and the benchmark's cpu_baseline leg may use it; the product
 * path never calls into this file.
 *
 * Conventions (0-based indices everywhere):
 *   x, S   : C x H x W, row-major (NCHW with batch 1, Sec. III-B item 1)
 *   OUT    : O x Ho x Wo
 *   K      : O x C x kh x kw  == the filter matrix K(o,(c*kh+j)*kw+i) of Eq. 2
 *   output pixel (yo,xo) reads inputs (yo*s-p+j, xo*s-p+i), zero outside
 *   (cross-correlation, the matrix form below Eq. 2)
 *
 * Pins (tests/test_oracle_pins.py): threshold zero reproduces a dense
 * convolution (Sec. III-F); cached output == convolution of the input state
 * (Sec. III-C); the printed footprint counts 9 / 49 / 169 (Sec. III);
 * 1x1 filters leave the change map unchanged (Sec. III-E); scatter-form
 * brute force of Eq. 4; Table I's pooled resolutions; library conv/pool
 * routines as the textbook special cases.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct cbo_layer {
    int C, O, kh, kw, s, p, H, W, Ho, Wo;
    int relu;       /* fused ReLU in the output update (Sec. III-A, Output Updating) */
    int bf16;       /* 1: outputs are rounded to bfloat16 instead of float32 */
    int mode;       /* 0 closed loop (Sec. III-C), 1 feed-forward (Sec. III-A) */
    int primed;     /* 0 until the first frame has been processed */
    float *S;       /* input state (closed loop) / previous input (feed-forward) */
    float *OUT;     /* cached output, post bias, post ReLU */
    float *Kw;      /* O x R filter matrix */
    float *b;       /* O */
    uint8_t *m;     /* H x W   change map, Eq. 3 */
    uint8_t *mt;    /* Ho x Wo dilated change map, Eq. 4 */
    int32_t *idx;   /* ascending linear output indices with mt == 1 */
    int32_t N;      /* number of listed output pixels */
    int32_t M;      /* number of changed input pixels */
} cbo_layer;

/* ---------------------------------------------------------------- helpers */
int cbo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void cbo_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* nearest bfloat16 (8 significant bits, float32 exponent range), ties to even,
 * straight from the double so that there is a single rounding. */
static float round_bf16(double v)
{
    if (v == 0.0 || isnan(v) || isinf(v)) return (float)v;
    int e;
    double f = frexp(v, &e);            /* v = f * 2^e, 0.5 <= |f| < 1 */
    int qexp = e - 8;                   /* quantum 2^(e-8) for 8 significant bits */
    if (qexp < -133) qexp = -133;       /* bf16 subnormal quantum */
    (void)f;
    double q = ldexp(1.0, qexp);
    double r = nearbyint(v / q) * q;    /* default rounding mode: ties to even */
    return (float)r;                    /* exact: r has <= 8 significant bits */
}

static inline float finish(double acc, int relu, int bf16)
{
    if (relu && acc < 0.0) acc = 0.0;
    return bf16 ? round_bf16(acc) : (float)acc;
}

/* ---------------------------------------------------------------- steps */

/* Eq. 3 with the closed-loop state update of Sec. III-C: a pixel is changed if
 * any channel differs from the state by more than tau (strict), in float32;
 * all channels of a changed pixel are then copied into the state.
 * Returns the number of changed pixels. */
int32_t cbo_detect(int C, int P, const float *x, float *S, float tau, uint8_t *m)
{
    int32_t M = 0;
    for (int p = 0; p < P; ++p) {
        int ch = 0;
        for (int c = 0; c < C; ++c) {
            float d = x[(size_t)c * P + p] - S[(size_t)c * P + p];
            if (fabsf(d) > tau) ch = 1;
        }
        m[p] = (uint8_t)ch;
        M += ch;
    }
    for (int p = 0; p < P; ++p)
        if (m[p])
            for (int c = 0; c < C; ++c) S[(size_t)c * P + p] = x[(size_t)c * P + p];
    return M;
}

/* Feed-forward variant (Sec. III-A, Fig. 2a): compare against the previous
 * input, then keep the whole current input. */
int32_t cbo_detect_ff(int C, int P, const float *x, float *S, float tau, uint8_t *m)
{
    int32_t M = 0;
    for (int p = 0; p < P; ++p) {
        int ch = 0;
        for (int c = 0; c < C; ++c) {
            float d = x[(size_t)c * P + p] - S[(size_t)c * P + p];
            if (fabsf(d) > tau) ch = 1;
        }
        m[p] = (uint8_t)ch;
        M += ch;
    }
    memcpy(S, x, (size_t)C * P * sizeof(float));
    return M;
}

/* Eq. 4: an output pixel is marked iff its receptive field holds a changed
 * input pixel; positions in the zero padding never count as changed. */
void cbo_dilate(int H, int W, int Ho, int Wo, int kh, int kw, int s, int p,
                const uint8_t *m, uint8_t *mt)
{
    for (int yo = 0; yo < Ho; ++yo)
        for (int xo = 0; xo < Wo; ++xo) {
            int any = 0;
            for (int j = 0; j < kh; ++j)
                for (int i = 0; i < kw; ++i) {
                    int yi = yo * s - p + j, xi = xo * s - p + i;
                    if (yi >= 0 && yi < H && xi >= 0 && xi < W && m[yi * W + xi]) any = 1;
                }
            mt[yo * Wo + xo] = (uint8_t)any;
        }
}

/* Change-index extraction (Sec. III-A): order-preserving selection of the
 * linear indices yo*Wo+xo with mt == 1, and their count. */
int32_t cbo_extract(int Po, const uint8_t *mt, int32_t *idx)
{
    int32_t n = 0;
    for (int q = 0; q < Po; ++q)
        if (mt[q]) idx[n++] = q;
    return n;
}

/* Eq. 1 in the matrix form of Eq. 2, evaluated directly at one output pixel:
 * acc = b[o] + sum_{c,j,i} K(o,(c*kh+j)*kw+i) * S(c, yo*s-p+j, xo*s-p+i). */
static double conv_point(int C, int H, int W, int kh, int kw, int s, int p,
                         const float *S, const float *Ko, double b, int yo, int xo)
{
    double acc = b;
    for (int c = 0; c < C; ++c)
        for (int j = 0; j < kh; ++j) {
            int yi = yo * s - p + j;
            if (yi < 0 || yi >= H) continue;
            for (int i = 0; i < kw; ++i) {
                int xi = xo * s - p + i;
                if (xi < 0 || xi >= W) continue;
                acc += (double)Ko[(c * kh + j) * kw + i] * (double)S[((size_t)c * H + yi) * W + xi];
            }
        }
    return acc;
}

/* Values of the listed output pixels: vals[o*n + q] for pixel idx[q]. */
void cbo_conv_at(int C, int O, int H, int W, int kh, int kw, int s, int p, int relu, int bf16,
                 const float *S, const float *Kw, const float *b,
                 const int32_t *idx, int32_t n, float *vals)
{
    int Wo = (W + 2 * p - kw) / s + 1;
    int R = C * kh * kw;
#pragma omp parallel for schedule(static)
    for (int q = 0; q < n; ++q) {
        int yo = idx[q] / Wo, xo = idx[q] % Wo;
        for (int o = 0; o < O; ++o) {
            double acc = conv_point(C, H, W, kh, kw, s, p, S, Kw + (size_t)o * R,
                                    b ? (double)b[o] : 0.0, yo, xo);
            vals[(size_t)o * n + q] = finish(acc, relu, bf16);
        }
    }
}

/* Dense direct convolution of a whole frame (the non-change-based layer). */
void cbo_dense_conv(int C, int O, int H, int W, int kh, int kw, int s, int p, int relu, int bf16,
                    const float *x, const float *Kw, const float *b, float *out)
{
    int Ho = (H + 2 * p - kh) / s + 1, Wo = (W + 2 * p - kw) / s + 1;
    int R = C * kh * kw;
#pragma omp parallel for schedule(static)
    for (int q = 0; q < Ho * Wo; ++q) {
        int yo = q / Wo, xo = q % Wo;
        for (int o = 0; o < O; ++o) {
            double acc = conv_point(C, H, W, kh, kw, s, p, x, Kw + (size_t)o * R,
                                    b ? (double)b[o] : 0.0, yo, xo);
            out[(size_t)o * Ho * Wo + q] = finish(acc, relu, bf16);
        }
    }
}

/* ---------------------------------------------------------------- layer */
cbo_layer *cbo_create(int C, int O, int kh, int kw, int s, int p, int H, int W,
                      int relu, int bf16, int mode, const float *Kw, const float *b)
{
    if (C < 1 || O < 1 || kh < 1 || kw < 1 || s < 1 || p < 0 || H < 1 || W < 1) return NULL;
    if (H + 2 * p < kh || W + 2 * p < kw) return NULL;
    cbo_layer *L = (cbo_layer *)calloc(1, sizeof(*L));
    if (!L) return NULL;
    L->C = C; L->O = O; L->kh = kh; L->kw = kw; L->s = s; L->p = p; L->H = H; L->W = W;
    L->Ho = (H + 2 * p - kh) / s + 1;
    L->Wo = (W + 2 * p - kw) / s + 1;
    L->relu = relu; L->bf16 = bf16; L->mode = mode;
    size_t P = (size_t)H * W, Po = (size_t)L->Ho * L->Wo, R = (size_t)C * kh * kw;
    L->S = (float *)calloc(C * P, sizeof(float));
    L->OUT = (float *)calloc(O * Po, sizeof(float));
    L->Kw = (float *)malloc(O * R * sizeof(float));
    L->b = (float *)calloc(O, sizeof(float));
    L->m = (uint8_t *)calloc(P, 1);
    L->mt = (uint8_t *)calloc(Po, 1);
    L->idx = (int32_t *)calloc(Po, sizeof(int32_t));
    memcpy(L->Kw, Kw, O * R * sizeof(float));
    if (b) memcpy(L->b, b, O * sizeof(float));
    return L;
}

void cbo_destroy(cbo_layer *L)
{
    if (!L) return;
    free(L->S); free(L->OUT); free(L->Kw); free(L->b); free(L->m); free(L->mt); free(L->idx);
    free(L);
}

void cbo_reset(cbo_layer *L) { L->primed = 0; }

/* Steps shared by both entry points after the change map m is known: Eq. 4,
 * index extraction, recomputation of the listed outputs from the input state,
 * output update.  On a full update every output pixel is listed, also those
 * whose receptive field lies entirely in the zero padding (they equal the
 * bias and can never be reached through Eq. 4). */
static int32_t finish_frame(cbo_layer *L, int full)
{
    int Po = L->Ho * L->Wo;
    if (full)
        memset(L->mt, 1, (size_t)Po);
    else
        cbo_dilate(L->H, L->W, L->Ho, L->Wo, L->kh, L->kw, L->s, L->p, L->m, L->mt);
    L->N = cbo_extract(Po, L->mt, L->idx);
    if (L->N > 0) {
        float *vals = (float *)malloc((size_t)L->O * L->N * sizeof(float));
        cbo_conv_at(L->C, L->O, L->H, L->W, L->kh, L->kw, L->s, L->p, L->relu, L->bf16,
                    L->S, L->Kw, L->b, L->idx, L->N, vals);
        for (int o = 0; o < L->O; ++o)
            for (int q = 0; q < L->N; ++q)
                L->OUT[(size_t)o * Po + L->idx[q]] = vals[(size_t)o * L->N + q];
        free(vals);
    }
    return L->N;
}

/* One frame through the layer: detect (+ state update), dilate, extract,
 * recompute the listed outputs from the input state, update the cached output
 * with fused bias and ReLU.  The first frame after create/reset is a full
 * update (every input pixel changed, every output pixel listed).  Returns N. */
int32_t cbo_process(cbo_layer *L, const float *x, float tau)
{
    int P = L->H * L->W;
    int full = !L->primed;
    if (full) {
        memset(L->m, 1, (size_t)P);
        memcpy(L->S, x, (size_t)L->C * P * sizeof(float));
        L->M = P;
        L->primed = 1;
    } else if (L->mode == 0) {
        L->M = cbo_detect(L->C, P, x, L->S, tau, L->m);
    } else {
        L->M = cbo_detect_ff(L->C, P, x, L->S, tau, L->m);
    }
    return finish_frame(L, full);
}

/* Layer whose change set comes from its producer instead of its own detection
 * (Sec. III-E): case 1 -- `m` is the producer's dilated map and is propagated
 * through Eq. 4; the oracle's copy of the input takes the pixels the map marks
 * (the producer rewrote no others, so it equals the whole input).  For a 1x1 filter
 * this is case 2 (the map and therefore the index list are the producer's). */
int32_t cbo_process_propagated(cbo_layer *L, const float *x, const uint8_t *m_producer)
{
    int P = L->H * L->W;
    int full = !L->primed;
    if (full) {
        memset(L->m, 1, (size_t)P);
        L->primed = 1;
    } else {
        memcpy(L->m, m_producer, (size_t)P);
    }
    L->M = 0;
    for (int q = 0; q < P; ++q) L->M += L->m[q];
    for (int q = 0; q < P; ++q)
        if (L->m[q])
            for (int c = 0; c < L->C; ++c) L->S[(size_t)c * P + q] = x[(size_t)c * P + q];
    return finish_frame(L, full);
}

/* accessors */
const float *cbo_state(const cbo_layer *L) { return L->S; }
const float *cbo_out(const cbo_layer *L) { return L->OUT; }
const uint8_t *cbo_m(const cbo_layer *L) { return L->m; }
const uint8_t *cbo_mt(const cbo_layer *L) { return L->mt; }
const int32_t *cbo_idx(const cbo_layer *L) { return L->idx; }
int32_t cbo_count(const cbo_layer *L) { return L->N; }
int32_t cbo_n_in(const cbo_layer *L) { return L->M; }
int cbo_ho(const cbo_layer *L) { return L->Ho; }
int cbo_wo(const cbo_layer *L) { return L->Wo; }

/* ---------------------------------------------------------------- pooling */

/* Change-based max-pool (Sec. III-E, last paragraph): w x w window, stride w,
 * ceil mode with windows clipped at the border (Table I: 541x871 -> 271x436 ->
 * 136x218).  For every listed producer pixel the pooled cell holding it is
 * recomputed from the producer's cached output; `pm` receives the pooled change
 * map (OR over each window of the producer's dilated map). */
void cbo_pool_update(int O, int Ho, int Wo, int w, const float *OUT,
                     const int32_t *idx, int32_t n, const uint8_t *mt,
                     float *POOL, uint8_t *pm)
{
    int Hp = (Ho + w - 1) / w, Wp = (Wo + w - 1) / w;
    for (int q = 0; q < n; ++q) {
        int yp = (idx[q] / Wo) / w, xp = (idx[q] % Wo) / w;
        for (int o = 0; o < O; ++o) {
            float best = -INFINITY;
            for (int dy = 0; dy < w; ++dy)
                for (int dx = 0; dx < w; ++dx) {
                    int y = yp * w + dy, x = xp * w + dx;
                    if (y < Ho && x < Wo) {
                        float v = OUT[((size_t)o * Ho + y) * Wo + x];
                        if (v > best) best = v;
                    }
                }
            POOL[((size_t)o * Hp + yp) * Wp + xp] = best;
        }
    }
    if (pm) {
        for (int yp = 0; yp < Hp; ++yp)
            for (int xp = 0; xp < Wp; ++xp) {
                int any = 0;
                for (int dy = 0; dy < w; ++dy)
                    for (int dx = 0; dx < w; ++dx) {
                        int y = yp * w + dy, x = xp * w + dx;
                        if (y < Ho && x < Wo && mt[y * Wo + x]) any = 1;
                    }
                pm[yp * Wp + xp] = (uint8_t)any;
            }
    }
}

/* Dense max-pool of a whole tensor, same geometry. */
void cbo_pool_dense(int O, int Ho, int Wo, int w, const float *OUT, float *POOL)
{
    int Hp = (Ho + w - 1) / w, Wp = (Wo + w - 1) / w;
    for (int o = 0; o < O; ++o)
        for (int yp = 0; yp < Hp; ++yp)
            for (int xp = 0; xp < Wp; ++xp) {
                float best = -INFINITY;
                for (int dy = 0; dy < w; ++dy)
                    for (int dx = 0; dx < w; ++dx) {
                        int y = yp * w + dy, x = xp * w + dx;
                        if (y < Ho && x < Wo) {
                            float v = OUT[((size_t)o * Ho + y) * Wo + x];
                            if (v > best) best = v;
                        }
                    }
                POOL[((size_t)o * Hp + yp) * Wp + xp] = best;
            }
}
