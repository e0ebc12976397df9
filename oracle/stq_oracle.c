/*
 * stq_oracle.c -- plain CPU oracle of the quantized Adam step of STQuant.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, obviously-correct reference
 * that the GPU library is compared against.  It shares no code, header, table
 * generator or helper with the HIP path, and nothing in the product may call it.
 *
 * What it follows (paper: "STQuant: Spatio-Temporal Adaptive Framework for
 * Optimizer Quantization ..."):
 *   - Algorithm 1, the per-layer loop body: moment update, Quantize(m,'linear'),
 *     Quantize(v,'log'), bias correction of the QUANTIZED moments, decoupled
 *     weight-decay parameter update.
 *   - Section 3.5 (Quantization Engine): block-wise quantization over contiguous
 *     sub-blocks with one scaling factor per block; linear symmetric for the first
 *     moment, logarithmic for the second moment.
 *   - Section 3.3 Eq. 2, 3, 8 and Section 3.4 (score, Map) and Algorithm 1 for the
 *     bit-width decision.
 *
 * The paper gives no formula for the two quantizers, no storage layout and no
 * conversion rule for a bit-width change.  The readings taken here:
 *   linear : scale s = max|x| over the block; qmax = 2^(b-1)-1; integer grid
 *            {-qmax..qmax}; stored code u = q + qmax; value = s * R_b[u] with
 *            R_b[u] = fl32((u-qmax)/qmax); rounding half-to-even.
 *   log    : scale s = max x over the block (x >= 0); 2^b levels s*2^(-k*D_b),
 *            k = 0..2^b-1, D_b = 2^(4-b) octaves; stored code c = 2^b-1-k; nearest
 *            level in the log domain, i.e. thresholds at geometric midpoints; a
 *            value exactly on a threshold takes the larger level; values below
 *            the bottom level clamp to it; there is no zero code.
 *            All levels and thresholds are entries of ONE table
 *            G[j] = fl32(2^(-j/32)): level k of width b is G[k << (9-b)], threshold
 *            k is G[(2k+1) << (8-b)].  Decisions are exact fp32 compares.
 *   widths 16, 32: the two wide members of the paper's width set B = {4, 8, 16, 32} are not
 *            quantized block-wise: at 32 bits a state is kept as the fp32 value itself, at 16
 *            bits as its bfloat16 rounding (round to nearest even; bfloat16 rather than
 *            half precision because second moments reach 1e-13 and below).  No scales.
 *   tiny blocks: a block whose max is below the smallest normal fp32 (2^-126) is
 *            stored as an all-zero block (scale 0), so 1/s never overflows.
 *   arithmetic: IEEE binary32, round to nearest even, every operation rounded on
 *            its own (no fused multiply-add), denormals kept.  Build with
 *            -ffp-contract=off and without -ffast-math.
 *
 * All functions work on UNPACKED codes (one uint8 per element); the storage
 * layout is implemented separately by stq_oracle_pack/unpack below.
 */
#include <math.h>
#include <float.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ tables */

#define STQ_G_LEN 511 /* j = 0 .. 510: the largest index used is 255<<1 (level, b=8) */

static float G_tab[STQ_G_LEN];
static int G_ready = 0;

static void ensure_G(void) {
  if (G_ready) return;
  for (int j = 0; j < STQ_G_LEN; ++j) G_tab[j] = (float)exp2(-(double)j / 32.0);
  G_ready = 1;
}

/* G[j] = fl32(2^(-j/32)) */
float stq_oracle_G(int j) { ensure_G(); return G_tab[j]; }

static int qmax_of(int b) { return (1 << (b - 1)) - 1; }

/* value of linear code u at width b, for scale 1 */
float stq_oracle_R(int b, int u) {
  int qmax = qmax_of(b);
  return (float)(u - qmax) / (float)qmax; /* one correctly rounded fp32 division */
}

/* value of log code c at width b, for scale 1 */
float stq_oracle_L(int b, int c) {
  ensure_G();
  int k = ((1 << b) - 1) - c;
  return G_tab[k << (9 - b)];
}

/* threshold between log levels k and k+1 at width b, for scale 1 */
float stq_oracle_T(int b, int k) {
  ensure_G();
  return G_tab[(2 * k + 1) << (8 - b)];
}

/* ------------------------------------------------- block quantizers (Sec. 3.5) */

/* scale of a block after the tiny-block rule */
static float block_scale(float s) { return (s < FLT_MIN) ? 0.0f : s; }

/* Quantize(x, b, 'linear') on ONE block of n values.  Returns the scale. */
float stq_oracle_quant_linear_block(const float* x, int n, int b, uint8_t* u) {
  int qmax = qmax_of(b);
  float s = 0.0f;
  for (int i = 0; i < n; ++i) { float a = fabsf(x[i]); if (a > s) s = a; }
  s = block_scale(s);
  float inv = (s > 0.0f) ? 1.0f / s : 0.0f;
  for (int i = 0; i < n; ++i) {
    float t = (x[i] * inv) * (float)qmax;
    float r = rintf(t); /* half to even */
    if (r > (float)qmax) r = (float)qmax;
    if (r < -(float)qmax) r = -(float)qmax;
    u[i] = (uint8_t)((int)r + qmax);
  }
  return s;
}

/* Quantize(x, b, 'log') on ONE block of n non-negative values.  Returns the scale. */
float stq_oracle_quant_log_block(const float* x, int n, int b, uint8_t* c) {
  int kmax = (1 << b) - 1;
  float s = 0.0f;
  for (int i = 0; i < n; ++i) if (x[i] > s) s = x[i];
  s = block_scale(s);
  float inv = (s > 0.0f) ? 1.0f / s : 0.0f;
  for (int i = 0; i < n; ++i) {
    float rho = x[i] * inv;
    int k = 0;
    while (k < kmax && rho < stq_oracle_T(b, k)) ++k;
    c[i] = (uint8_t)(kmax - k);
  }
  return s;
}

void stq_oracle_dequant_linear_block(const uint8_t* u, int n, int b, float s, float* x) {
  for (int i = 0; i < n; ++i) x[i] = s * stq_oracle_R(b, u[i]);
}

void stq_oracle_dequant_log_block(const uint8_t* c, int n, int b, float s, float* x) {
  for (int i = 0; i < n; ++i) x[i] = s * stq_oracle_L(b, c[i]);
}

/* --------------------------------------------------------- statistics record */

typedef struct {
  uint64_t count;
  double g_sum, g_abs_sum, g_sq_sum; float g_absmax;  /* gradient: Eq. 2, 3, 8 inputs */
  double m_sum, m_sq_sum, m_err_sq;  float m_absmax;  /* first moment before quantization, and its quantization error */
  double v_sum, v_sq_sum, v_err_sq;  float v_absmax;  /* second moment, same */
} stq_oracle_stats;

/* ------------------------------------------------ the step (Alg. 1 inner loop) */

typedef struct {
  float lr, beta1, beta2, eps, weight_decay;
  uint32_t step;  /* t >= 1 */
} stq_oracle_hparams;

static float bf16_to_f32(uint16_t h) {
  uint32_t w = (uint32_t)h << 16; float f; memcpy(&f, &w, 4); return f;
}

/* The statistics of one layer's gradient alone (the inputs of Eq. 2, 3 and 8), for the order in which
 * Algorithm 1 is written: statistics and Map first, then the layer loop of the same step.  The other
 * fields of *st are left as they are. */
void stq_oracle_grad_stats(const void* grad, int grad_is_bf16, uint64_t n, stq_oracle_stats* st) {
  for (uint64_t i = 0; i < n; ++i) {
    float gf = grad_is_bf16 ? bf16_to_f32(((const uint16_t*)grad)[i]) : ((const float*)grad)[i];
    double gd = (double)gf;
    st->g_sum += gd; st->g_abs_sum += fabs(gd); st->g_sq_sum += gd * gd;
    if (fabsf(gf) > st->g_absmax) st->g_absmax = fabsf(gf);
  }
  st->count += n;
}

/*
 * One Adam step on one tensor ("layer") of `numel` elements with blocks of K
 * consecutive elements (the last block may be shorter).
 *   param : fp32, updated in place
 *   grad  : fp32 (grad_bf16 = 0) or bf16 bit patterns (grad_bf16 = 1)
 *   um,sm : first-moment codes (one byte per element) and per-block scales, in/out
 *   cv,sv : second-moment codes and scales, in/out
 *   bm_old,bv_old : widths of the stored codes m_{t-1}, v_{t-1} (2..8)
 *   bm,bv : widths b_{l,t} that Quantize uses in this step (2..8).  Algorithm 1 maps the
 *           layer's new width before its layer loop, so in a step where the width changes
 *           the stored moments are read at the old width and written at the new one; the
 *           codes arrays hold one byte per element, so they are reused in place
 *   st    : if non-NULL, receives the statistics of this tensor for this step
 */
/* value kept for a state of width 16 or 32 */
float stq_oracle_wide_value(float x, int b) {
  if (b == 32) return x;
  uint32_t u; memcpy(&u, &x, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);   /* bfloat16: round to nearest, ties to even */
  u &= 0xFFFF0000u;
  float y; memcpy(&y, &u, 4);
  return y;
}

/* As stq_oracle_step_widths; states of width 16 or 32 live in mwide / vwide (one float per
 * element: the stored value itself), their codes and scales are neither read nor written. */
void stq_oracle_step_wide(float* param, const void* grad, int grad_bf16, uint64_t numel,
                          uint8_t* um, float* sm, uint8_t* cv, float* sv, float* mwide, float* vwide,
                          int bm_old, int bv_old, int bm, int bv, int K,
                          const stq_oracle_hparams* hp, stq_oracle_stats* st) {
  const float beta1 = hp->beta1, beta2 = hp->beta2;
  const float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
  const float decay = 1.0f - hp->lr * hp->weight_decay;
  /* reciprocal bias corrections: computed in double, rounded once to fp32 */
  const float ibc1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)hp->step)));
  const float ibc2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)hp->step)));
  const float lr = hp->lr, eps = hp->eps;

  float* m = (float*)malloc(sizeof(float) * (size_t)K);
  float* v = (float*)malloc(sizeof(float) * (size_t)K);
  float* g = (float*)malloc(sizeof(float) * (size_t)K);

  if (st) { memset(st, 0, sizeof(*st)); st->count = numel; }

  uint64_t nblocks = (numel + (uint64_t)K - 1) / (uint64_t)K;
  for (uint64_t j = 0; j < nblocks; ++j) {
    uint64_t lo = j * (uint64_t)K;
    int n = (int)((numel - lo < (uint64_t)K) ? (numel - lo) : (uint64_t)K);

    /* m_t = beta1 m_{t-1} + (1-beta1) g ;  v_t = beta2 v_{t-1} + (1-beta2) g^2,
       where m_{t-1}, v_{t-1} are the stored (quantized) states */
    for (int i = 0; i < n; ++i) {
      g[i] = grad_bf16 ? bf16_to_f32(((const uint16_t*)grad)[lo + i]) : ((const float*)grad)[lo + i];
      float mh = (bm_old >= 16) ? mwide[lo + i] : sm[j] * stq_oracle_R(bm_old, um[lo + i]);
      float vh = (bv_old >= 16) ? vwide[lo + i] : sv[j] * stq_oracle_L(bv_old, cv[lo + i]);
      float a = beta1 * mh, c = omb1 * g[i];
      m[i] = a + c;
      float gg = g[i] * g[i];
      float d = beta2 * vh, e = omb2 * gg;
      v[i] = d + e;
    }

    /* \hat m_t = Quantize(m_t, 'linear'), \hat v_t = Quantize(v_t, 'log') */
    float s_m = 0.0f, s_v = 0.0f;
    if (bm < 16) { s_m = stq_oracle_quant_linear_block(m, n, bm, um + lo); sm[j] = s_m; }
    else for (int i = 0; i < n; ++i) mwide[lo + i] = stq_oracle_wide_value(m[i], bm);
    if (bv < 16) { s_v = stq_oracle_quant_log_block(v, n, bv, cv + lo); sv[j] = s_v; }
    else for (int i = 0; i < n; ++i) vwide[lo + i] = stq_oracle_wide_value(v[i], bv);

    /* bias correction of the quantized moments and the parameter update */
    for (int i = 0; i < n; ++i) {
      float mq = (bm >= 16) ? mwide[lo + i] : s_m * stq_oracle_R(bm, um[lo + i]);
      float vq = (bv >= 16) ? vwide[lo + i] : s_v * stq_oracle_L(bv, cv[lo + i]);
      float mt = mq * ibc1;
      float vt = vq * ibc2;
      float den = sqrtf(vt) + eps;
      float ratio = mt / den;
      float upd = lr * ratio;
      float dec = param[lo + i] * decay;
      param[lo + i] = dec - upd;

      if (st) {
        double gd = (double)g[i], md = (double)m[i], vd = (double)v[i];
        st->g_sum += gd; st->g_abs_sum += fabs(gd); st->g_sq_sum += gd * gd;
        if (fabsf(g[i]) > st->g_absmax) st->g_absmax = fabsf(g[i]);
        st->m_sum += md; st->m_sq_sum += md * md;
        st->m_err_sq += (md - (double)mq) * (md - (double)mq);
        if (fabsf(m[i]) > st->m_absmax) st->m_absmax = fabsf(m[i]);
        st->v_sum += vd; st->v_sq_sum += vd * vd;
        st->v_err_sq += (vd - (double)vq) * (vd - (double)vq);
        if (v[i] > st->v_absmax) st->v_absmax = v[i];
      }
    }
  }
  free(m); free(v); free(g);
}

/* The step between quantized widths (2..8). */
void stq_oracle_step_widths(float* param, const void* grad, int grad_bf16, uint64_t numel,
                            uint8_t* um, float* sm, uint8_t* cv, float* sv,
                            int bm_old, int bv_old, int bm, int bv, int K,
                            const stq_oracle_hparams* hp, stq_oracle_stats* st) {
  stq_oracle_step_wide(param, grad, grad_bf16, numel, um, sm, cv, sv, NULL, NULL, bm_old, bv_old, bm, bv, K, hp, st);
}

/* The step with unchanged widths. */
void stq_oracle_step(float* param, const void* grad, int grad_bf16, uint64_t numel,
                     uint8_t* um, float* sm, uint8_t* cv, float* sv,
                     int bm, int bv, int K, const stq_oracle_hparams* hp,
                     stq_oracle_stats* st) {
  stq_oracle_step_widths(param, grad, grad_bf16, numel, um, sm, cv, sv, bm, bv, bm, bv, K, hp, st);
}

/* ---------------------------------------------------------- storage layout
 *
 * A state of `numel` codes of width b is stored in tiles of 2048 elements.  A
 * tile is 64 "lanes" x 32 codes: lane j owns the elements
 *     tile*2048 + 256*i + 4*j + e,   i = 0..7, e = 0..3,
 * and writes its codes, in the order n = 4*i + e, LSB first into a stream of
 * 32*b bits = b 32-bit words.  Word p of lane j sits at word index
 *     tile*64*b + p*64 + j
 * of the code buffer.  Elements at or beyond numel (the pad of the last tile)
 * have code bits 0.  Scales are a separate fp32 array, one per block of K
 * consecutive elements, padded with zeros to 2048/K entries per tile.
 */
#define TILE 2048

uint64_t stq_oracle_code_words(uint64_t numel, int b) {
  uint64_t tiles = (numel + TILE - 1) / TILE;
  return tiles * 64u * (uint64_t)b;
}

void stq_oracle_pack(const uint8_t* codes, uint64_t numel, int b, uint32_t* words) {
  uint64_t nw = stq_oracle_code_words(numel, b);
  memset(words, 0, nw * 4);
  for (uint64_t idx = 0; idx < numel; ++idx) {
    uint64_t tile = idx / TILE;
    uint32_t r = (uint32_t)(idx % TILE);
    uint32_t i = r / 256, j = (r % 256) / 4, e = r % 4;
    uint32_t n = 4 * i + e;
    uint32_t bit = n * (uint32_t)b;
    for (int k = 0; k < b; ++k, ++bit) {            /* one bit at a time */
      if ((codes[idx] >> k) & 1u) {
        uint64_t w = tile * 64u * (uint64_t)b + (uint64_t)(bit / 32) * 64u + j;
        words[w] |= 1u << (bit % 32);
      }
    }
  }
}

void stq_oracle_unpack(const uint32_t* words, uint64_t numel, int b, uint8_t* codes) {
  for (uint64_t idx = 0; idx < numel; ++idx) {
    uint64_t tile = idx / TILE;
    uint32_t r = (uint32_t)(idx % TILE);
    uint32_t i = r / 256, j = (r % 256) / 4, e = r % 4;
    uint32_t n = 4 * i + e;
    uint32_t bit = n * (uint32_t)b;
    unsigned c = 0;
    for (int k = 0; k < b; ++k, ++bit) {
      uint64_t w = tile * 64u * (uint64_t)b + (uint64_t)(bit / 32) * 64u + j;
      c |= ((words[w] >> (bit % 32)) & 1u) << k;
    }
    codes[idx] = (uint8_t)c;
  }
}

/* States of width 16 or 32 use the same tile format with 16- or 32-bit "codes": the fp32 bit
 * pattern, or its upper half for bfloat16. */
void stq_oracle_pack_wide(const float* vals, uint64_t numel, int b, uint32_t* words) {
  uint64_t nw = stq_oracle_code_words(numel, b);
  memset(words, 0, nw * 4);
  for (uint64_t idx = 0; idx < numel; ++idx) {
    uint64_t tile = idx / TILE;
    uint32_t r = (uint32_t)(idx % TILE);
    uint32_t i = r / 256, j = (r % 256) / 4, e = r % 4;
    uint32_t n = 4 * i + e;
    uint32_t u; memcpy(&u, &vals[idx], 4);
    uint32_t code = (b == 32) ? u : (u >> 16);
    uint32_t bit = n * (uint32_t)b;
    uint64_t w = tile * 64u * (uint64_t)b + (uint64_t)(bit / 32) * 64u + j;
    words[w] |= code << (bit % 32);   /* 16 | 32: a code never straddles a word */
  }
}

void stq_oracle_unpack_wide(const uint32_t* words, uint64_t numel, int b, float* vals) {
  for (uint64_t idx = 0; idx < numel; ++idx) {
    uint64_t tile = idx / TILE;
    uint32_t r = (uint32_t)(idx % TILE);
    uint32_t i = r / 256, j = (r % 256) / 4, e = r % 4;
    uint32_t n = 4 * i + e;
    uint32_t bit = n * (uint32_t)b;
    uint64_t w = tile * 64u * (uint64_t)b + (uint64_t)(bit / 32) * 64u + j;
    uint32_t u = (b == 32) ? words[w] : ((words[w] >> (bit % 32)) & 0xFFFFu) << 16;
    memcpy(&vals[idx], &u, 4);
  }
}

/* ------------------------------------------- bit-width transition (re-pack)
 *
 * When a layer's width changes from b_old to b_new the stored codes are
 * converted in the code domain and the block scales stay as they are: the new
 * code is the one the quantizer of width b_new assigns to the old code's value
 * in a block of scale 1.  (The largest value of a block decodes to exactly the
 * scale in both modes, so the scale remains the block maximum.)
 */
void stq_oracle_repack(const uint8_t* in, uint64_t numel, int state /*0 = m linear, 1 = v log*/,
                       int b_old, int b_new, uint8_t* out) {
  for (uint64_t i = 0; i < numel; ++i) {
    if (state == 0) {
      int qn = qmax_of(b_new);
      float x = stq_oracle_R(b_old, in[i]);          /* value at scale 1 */
      float r = rintf((x * 1.0f) * (float)qn);
      if (r > (float)qn) r = (float)qn;
      if (r < -(float)qn) r = -(float)qn;
      out[i] = (uint8_t)((int)r + qn);
    } else {
      int kmax = (1 << b_new) - 1;
      float rho = stq_oracle_L(b_old, in[i]);
      int k = 0;
      while (k < kmax && rho < stq_oracle_T(b_new, k)) ++k;
      out[i] = (uint8_t)(kmax - k);
    }
  }
}

/* ------------------------------------------------ bit-width decision (Alg. 1)
 *
 * Score Engine + Map.  For every layer l, from the gradient sums of the step:
 *   n_l = sqrt(mean g^2)                      (Eq. 2)
 *   r_l = sigma(|g|) / (mu(|g|) + eps)        (Eq. 3; r_mode 1 uses Alg. 1's
 *                                              sigma(g) / (E|g| + eps) instead)
 *   v_l = mean g^2                            (Eq. 8)
 * then the three global EMAs (Eq. 4 and the one for V), S_t = 1 + sech(t/tau)
 * (Eq. 7), the score of Sec. 3.4 with Alg. 1's eps in the denominators, and the
 * step function Map: width = bits[ number of thresholds <= score ].
 * The second-moment width uses score + v_offset.
 * The update cadence of Alg. 1 (decide when t mod U = 0 or t < 5) is stq_oracle_decide_due.
 */
typedef struct { double n_ema, r_ema, v_ema; } stq_oracle_ema;

typedef struct {
  double alpha, tau, phi, eps, v_offset;
  int r_mode;       /* 0: Eq. 3, 1: Alg. 1 line for r_l */
  int n_thr;        /* number of thresholds; bits has n_thr+1 entries */
  int drop;         /* ablations of Sec. 4 (Table "w/o ..."): bit 0 drops the dual factor (the
                       intensity and variation terms), bit 1 the temporal term log2 S_t, bit 2 the
                       spatial term log2(v_l / v_global) */
  int pad_;
  const double* thr;
  const uint8_t* bits;
} stq_oracle_decide_cfg;

int stq_oracle_decide_due(uint32_t step, uint32_t U) { return (U != 0 && step % U == 0) || step < 5; }

static uint8_t map_score(double score, const stq_oracle_decide_cfg* c) {
  int k = 0;
  for (int i = 0; i < c->n_thr; ++i) if (c->thr[i] <= score) ++k;
  return c->bits[k];
}

void stq_oracle_decide(stq_oracle_ema* ema, const stq_oracle_stats* st, int L,
                       const stq_oracle_decide_cfg* c, uint32_t step,
                       uint8_t* bits_m, uint8_t* bits_v, double* score_out /*nullable, L*/) {
  double* n = (double*)malloc(sizeof(double) * (size_t)L);
  double* r = (double*)malloc(sizeof(double) * (size_t)L);
  double* v = (double*)malloc(sizeof(double) * (size_t)L);
  double an = 0, ar = 0, av = 0;
  for (int l = 0; l < L; ++l) {
    double N = (double)st[l].count;
    double msq = st[l].g_sq_sum / N;
    double mabs = st[l].g_abs_sum / N;
    double mean = st[l].g_sum / N;
    n[l] = sqrt(msq);
    v[l] = msq;
    double var = (c->r_mode == 0) ? (msq - mabs * mabs) : (msq - mean * mean);
    if (var < 0) var = 0;
    r[l] = sqrt(var) / (mabs + c->eps);
    an += n[l]; ar += r[l]; av += v[l];
  }
  an /= L; ar /= L; av /= L;
  ema->n_ema = c->alpha * an + (1.0 - c->alpha) * ema->n_ema;
  ema->r_ema = c->alpha * ar + (1.0 - c->alpha) * ema->r_ema;
  ema->v_ema = c->alpha * av + (1.0 - c->alpha) * ema->v_ema;
  double S = 1.0 + 1.0 / cosh((double)step / c->tau);
  for (int l = 0; l < L; ++l) {
    double score = c->phi;
    if (!(c->drop & 1)) score += log2(r[l] / (ema->r_ema + c->eps)) + log2(n[l] / (ema->n_ema + c->eps));
    if (!(c->drop & 2)) score += log2(S);
    if (!(c->drop & 4)) score += log2(v[l] / (ema->v_ema + c->eps));
    if (score_out) score_out[l] = score;
    bits_m[l] = map_score(score, c);
    bits_v[l] = map_score(score + c->v_offset, c);
  }
  free(n); free(r); free(v);
}
