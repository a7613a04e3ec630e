/*
 * OScaR CPU oracle -- TEST INFRASTRUCTURE, NOT A PRODUCT PATH.
 *
 * A plain, slow, single-purpose C implementation of what the OScaR KV-cache
 * hot path computes, written from the paper and sharing no code with the HIP
 * library.  Only the test-suite, the smoke check and the benchmark's
 * cpu_baseline leg may load it.
 *
 * Two halves with different precision regimes:
 *   - the ENCODER (Canalized Rotation, Omni-Token Scaling, per-channel key
 *     quantization, per-token value quantization, residual bookkeeping) is an
 *     encoding, so it is written step by step in one fixed fp32 operation
 *     order (compile with -ffp-contract=off, no -ffast-math);
 *   - the DECODE is the plain definition softmax(scale * Q_h K^T) V on the
 *     dequantized cache, accumulated in double.
 *
 * Paper passages followed (section / equation / algorithm names):
 *   [Eq.3-4]   block-wise per-channel quantization, Sec. "Block-Wise
 *              Per-Channel Quantization" (Delta, integer zero-point z, clamp,
 *              reconstruction), restated in App. "Preliminaries on Low-Bit
 *              Quantization".
 *   [Key-xf]   App. "Implementation Details of OScaR's CUDA Kernels",
 *              "Overall Design": K_h = H(K)/sqrt(D), n_k = ||K_h||_2,
 *              K_u = K_h / n_k ; Q_h = H(Q)/sqrt(D) ;
 *              logits = (Q_h . dequant(K_u)) * n_k.
 *   [Fmt]      same appendix, "Quantization Format and Cache Organization":
 *              keys per-channel over groups of G tokens, values per-token over
 *              groups of G channels, packed cache + FP16 residual cache.
 *   [Alg.1]    Algorithm "The OScaR algorithm": OScaR-Inference, BufferQuantK,
 *              BufferQuantV (prefill split at len % R, decode append + flush
 *              when the residual reaches R).
 *   [Flow]     same appendix, "Prefill and Decode Workflows" / "Residual
 *              Flush": residual keys are already normalized, flush only
 *              quantizes.
 *   [Abl]      App. "Ablation Study": rotation and scaling switched off one at a
 *              time; alternative scaling coefficients (maximum absolute value /
 *              mean absolute value across the channels of a token).
 *   [Fused-HN] same appendix, "Fused Hadamard-Norm Kernel": all kv heads of a
 *              token are transformed, their squared sums accumulated across
 *              heads, one token-wise norm normalizes every head (the
 *              OREF_NORM_ALL_KV_HEADS variant; [Key-xf]'s per-vector norm is
 *              the default).
 *
 * Readings taken where the paper is silent (each is listed in the design
 * notes of the repository):
 *   - Hadamard matrix = Sylvester natural order, normalized by 1/sqrt(d).
 *   - floor-ceil brackets = round half to even.
 *   - x/Delta is evaluated as x * (1/Delta) with one IEEE reciprocal per group.
 *   - Delta, z and n are rounded to their storage type BEFORE they are used.
 *   - K_u is rounded to fp16 before quantization (it always passes through the
 *     FP16 residual format), so bulk and token-by-token ingestion agree.
 *   - max == min: Delta := |min| (1 if that is 0), so a constant group
 *     round-trips exactly.
 *   - zero-norm token: K_u = 0.
 *   - a parameter (Delta, z, n) beyond the largest finite value of its storage type is
 *     stored as that value (saturation); K_u is then K_h over the saturated norm, so
 *     n * K_u still restores K_h.
 *   - mean absolute value: |x_j| summed in the same balanced tree as the squared
 *     sum, times 1/d.
 *   - norm over all kv heads: the per-head squared sums (each in its tree
 *     order) are added in head order, then one sqrt; the same stored norm is
 *     kept with every head of the token.
 *
 * Parity status: every function below is pinned by tests under tests/ against
 * closed forms, invariants, the worked example of App. "Detailed Analysis of
 * Scaling-Induced Outlier Artifact" and brute force.  Agreement with the
 * authors' own (unpublished here) kernels is "parity unpinned": the paper
 * prints no codes, scales or attention outputs.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { OREF_F32 = 0, OREF_BF16 = 1, OREF_F16 = 2 };
enum { OREF_ZP_INT = 0, OREF_ZP_MIN = 1 };
enum { OREF_SCALE_NONE = 0, OREF_SCALE_L2 = 1, OREF_SCALE_MAX = 2, OREF_SCALE_MEAN_ABS = 3 };
enum { OREF_NORM_PER_HEAD = 0, OREF_NORM_ALL_KV_HEADS = 1 };

typedef struct {
  /* parameters of Alg.1 (G, R, d_h) and of Eq.3-4 (b) */
  int32_t d;          /* head dimension, power of two */
  int32_t bits;       /* b: 2, 4 or 8 */
  int32_t k_group;    /* G for keys: tokens per per-channel group, divides R */
  int32_t v_group;    /* G for values: channels per per-token group, divides d */
  int32_t R;          /* residual length = flush block */
  int32_t meta_dtype; /* storage type of Delta, z, n: OREF_F32 or OREF_F16 */
  int32_t zp_mode;    /* OREF_ZP_INT = Eq.3-4 ; OREF_ZP_MIN = float zero-point (cost section of App. complexity) */
  int32_t rotate;     /* 1 = Canalized Rotation on (ablation switch) */
  int32_t scale_mode; /* OREF_SCALE_L2 = Omni-Token Scaling as in the method; NONE = off;
                         MAX / MEAN_ABS = the alternative coefficients of [Abl] */
  int32_t norm_scope; /* OREF_NORM_PER_HEAD: n = ||K_h|| of one head's vector [Key-xf];
                         OREF_NORM_ALL_KV_HEADS: one n per token from the squared sums of all
                         kv heads (the fused preprocessing kernel's description, [Fused-HN]) */
  /* shape */
  int32_t batch, n_kv_heads, cap_tokens; /* cap_tokens multiple of R */
  /* state, per sequence */
  int32_t *n_packed;  /* [batch] tokens in the packed cache (multiple of R) */
  int32_t *n_res;     /* [batch] tokens in the residual cache, 0..R */
  /* canonical UNPACKED cache, one code per byte */
  uint8_t *k_codes;   /* [batch][n_kv][cap][d] */
  float *k_delta;     /* [batch][n_kv][cap/k_group][d] */
  float *k_zero;      /* same shape */
  float *k_norm;      /* [batch][n_kv][cap] */
  uint8_t *v_codes;   /* [batch][n_kv][cap][d] */
  float *v_delta;     /* [batch][n_kv][cap][d/v_group] */
  float *v_zero;      /* same shape */
  /* residual cache (values exactly representable in their storage type) */
  float *res_k;       /* [batch][n_kv][R][d]  K_u, fp16 values */
  float *res_v;       /* [batch][n_kv][R][d]  V, input precision */
  float *res_norm;    /* [batch][n_kv][R] */
} oref_cache;

/* ------------------------------------------------------------------------ */
/* Storage rounding (IEEE round-to-nearest-even), written from the formats'  */
/* definitions: binary16 has 11 significand bits and e_min = -14, bfloat16   */
/* has 8 significand bits and e_min = -126.                                  */
/* ------------------------------------------------------------------------ */

static float round_to_format(float f, int sig_bits, int e_min, double max_finite) {
  if (f == 0.0f || isnan(f) || isinf(f)) return f;
  int e2;
  (void)frexp((double)f, &e2);       /* |f| = m * 2^e2, m in [0.5,1) */
  int e = e2 - 1;                    /* |f| in [2^e, 2^(e+1)) */
  if (e < e_min) e = e_min;          /* subnormal range: fixed spacing */
  double ulp = ldexp(1.0, e - (sig_bits - 1));
  double q = nearbyint((double)f / ulp); /* ties to even (default rounding mode) */
  double r = q * ulp;
  if (fabs(r) > max_finite) r = (f > 0) ? INFINITY : -INFINITY;
  return (float)r;
}

float oref_round_f16(float f) { return round_to_format(f, 11, -14, 65504.0); }
float oref_round_bf16(float f) { return round_to_format(f, 8, -126, 3.3895313892515355e38); }

float oref_round_dtype(float f, int dtype) {
  if (dtype == OREF_F16) return oref_round_f16(f);
  if (dtype == OREF_BF16) return oref_round_bf16(f);
  return f;
}

/* Metadata (Delta, zero-point, token norm) is stored in `dtype` [Fmt]; a value beyond the
 * largest finite number of that type is stored as that number (saturation), so that no
 * stored parameter is ever infinite and the decode stays finite.  The paper is silent on
 * metadata overflow; an fp32 store is unchanged. */
float oref_round_meta(float f, int dtype) {
  float r = oref_round_dtype(f, dtype);
  if (isinf(r) && !isinf(f)) {
    float big = (dtype == OREF_F16) ? 65504.0f : 3.3895313892515355e38f;
    r = (f > 0) ? big : -big;
  }
  return r;
}

/* ------------------------------------------------------------------------ */
/* Canalized Rotation [Key-xf]: x <- H_d x / sqrt(d), Sylvester Hadamard.    */
/* Butterfly stages h = 1,2,4,...,d/2; pair (i, i|h): (a,b) -> (a+b, a-b).   */
/* ------------------------------------------------------------------------ */
void oref_fwht(float *x, int d) {
  for (int h = 1; h < d; h <<= 1)
    for (int i = 0; i < d; ++i)
      if ((i & h) == 0) {
        float a = x[i], b = x[i | h];
        x[i] = a + b;
        x[i | h] = a - b;
      }
  float c = (float)(1.0 / sqrt((double)d)); /* fp32(1/sqrt(d)) */
  for (int i = 0; i < d; ++i) x[i] = x[i] * c;
}

/* Sum of squares in a fixed balanced tree, adjacent pairs first:
 * t[i] <- t[i] + t[i^h] for h = 1,2,...,d/2 (every slot ends with the total). */
float oref_sumsq_tree(const float *x, int d) {
  float t[1024], s[1024];
  for (int i = 0; i < d; ++i) t[i] = x[i] * x[i];
  for (int h = 1; h < d; h <<= 1) {
    for (int i = 0; i < d; ++i) s[i] = t[i] + t[i ^ h];
    memcpy(t, s, sizeof(float) * (size_t)d);
  }
  return t[0];
}

/* Sum of |x_j| in the same balanced tree. */
float oref_sumabs_tree(const float *x, int d) {
  float t[1024], s[1024];
  for (int i = 0; i < d; ++i) t[i] = fabsf(x[i]);
  for (int h = 1; h < d; h <<= 1) {
    for (int i = 0; i < d; ++i) s[i] = t[i] + t[i ^ h];
    memcpy(t, s, sizeof(float) * (size_t)d);
  }
  return t[0];
}

/* Key transform of one token of one head [Key-xf], [Alg.1: X_K <- FHT(X_K);
 * s_K <- ||X_K||_2; X_K <- X_K / s_K].
 * in : k[d]  (already exactly representable in the input dtype)
 * out: u[d]  = fp16(K_h / n_st),  *n_st = norm rounded to the metadata type.
 * Ablation switches [Abl]: rotate=0 skips the Hadamard, scale_mode=NONE keeps n=1,
 * MAX / MEAN_ABS replace the L2 norm by another per-token coefficient. */
void oref_key_transform(const float *k, int d, int rotate, int scale_mode,
                        int meta_dtype, float *u, float *n_st) {
  float x[1024];
  for (int j = 0; j < d; ++j) x[j] = k[j];
  if (rotate) oref_fwht(x, d);
  float nf = 1.0f;
  if (scale_mode != OREF_SCALE_NONE) {
    float n;
    if (scale_mode == OREF_SCALE_L2) {
      n = sqrtf(oref_sumsq_tree(x, d));
    } else if (scale_mode == OREF_SCALE_MAX) {          /* [Abl] max_j |x_j| */
      n = 0.0f;
      for (int j = 0; j < d; ++j)
        if (fabsf(x[j]) > n) n = fabsf(x[j]);
    } else {                                            /* [Abl] mean_j |x_j| */
      n = oref_sumabs_tree(x, d) * (1.0f / (float)d);
    }
    nf = oref_round_meta(n, meta_dtype);
    float inv = (nf > 0.0f && !isinf(nf)) ? 1.0f / nf : 0.0f;
    for (int j = 0; j < d; ++j) x[j] = x[j] * inv;
  }
  for (int j = 0; j < d; ++j) u[j] = oref_round_f16(x[j]); /* FP16 residual format [Fmt] */
  *n_st = nf;
}

/* The token-wise norm of [Fused-HN]: k_heads = the n_heads head vectors of one token
 * (head h at k_heads + h*head_stride); each head is transformed, its squared sum taken in
 * the tree order, the sums added in head order; returns the norm rounded to the metadata type. */
float oref_token_norm_all_heads(const float *k_heads, int n_heads, size_t head_stride, int d,
                                int rotate, int meta_dtype) {
  float x[1024];
  float s = 0.0f;
  for (int h = 0; h < n_heads; ++h) {
    for (int j = 0; j < d; ++j) x[j] = k_heads[(size_t)h * head_stride + j];
    if (rotate) oref_fwht(x, d);
    float sh = oref_sumsq_tree(x, d);
    s = (h == 0) ? sh : s + sh;
  }
  return oref_round_meta(sqrtf(s), meta_dtype);
}

/* Key transform of one head vector with a norm that was computed elsewhere (nf, already
 * rounded to the metadata type): u = fp16(K_h / nf). */
void oref_key_transform_given_norm(const float *k, int d, int rotate, float nf, float *u) {
  float x[1024];
  for (int j = 0; j < d; ++j) x[j] = k[j];
  if (rotate) oref_fwht(x, d);
  float inv = (nf > 0.0f && !isinf(nf)) ? 1.0f / nf : 0.0f;
  for (int j = 0; j < d; ++j) u[j] = oref_round_f16(x[j] * inv);
}

/* Query transform [Key-xf]: Q_h = H(Q)/sqrt(D), no normalization. */
void oref_query_transform(const float *q, int d, int rotate, float *qh) {
  for (int j = 0; j < d; ++j) qh[j] = q[j];
  if (rotate) oref_fwht(qh, d);
}

/* ------------------------------------------------------------------------ */
/* Asymmetric uniform quantizer of one group [Eq.3-4].                        */
/* ------------------------------------------------------------------------ */

/* Parameters from the group's range; both are rounded to the metadata type
 * before use.  ZP_INT: zero = round(-min/Delta) (an integer).  ZP_MIN: zero = min. */
void oref_quant_params(float mn, float mx, int bits, int meta_dtype, int zp_mode,
                       float *delta, float *zero) {
  float qmax = (float)((1 << bits) - 1);
  float dl = (mx - mn) / qmax;
  float df = oref_round_meta(dl, meta_dtype);
  if (df == 0.0f) {                       /* constant (or underflowing) group */
    df = oref_round_meta(fabsf(mn), meta_dtype);
    if (df == 0.0f || isinf(df)) df = 1.0f;
  }
  float rd = 1.0f / df;
  float z;
  if (zp_mode == OREF_ZP_INT) z = oref_round_meta(rintf(-mn * rd), meta_dtype);
  else z = oref_round_meta(mn, meta_dtype);
  *delta = df;
  *zero = z;
}

uint8_t oref_quant_code(float x, float delta, float zero, int bits, int zp_mode) {
  float qmax = (float)((1 << bits) - 1);
  float rd = 1.0f / delta;
  float c;
  if (zp_mode == OREF_ZP_INT) c = rintf(x * rd) + zero;
  else c = rintf((x - zero) * rd);
  if (c < 0.0f) c = 0.0f;
  if (c > qmax) c = qmax;
  return (uint8_t)c;
}

double oref_dequant(uint8_t c, float delta, float zero, int zp_mode) {
  if (zp_mode == OREF_ZP_INT) return (double)delta * ((double)c - (double)zero);
  return (double)delta * (double)c + (double)zero;
}

/* Quantize `count` values x[i*stride] as one group. */
void oref_quant_group(const float *x, int count, int stride, int bits, int meta_dtype,
                      int zp_mode, float *delta, float *zero, uint8_t *codes,
                      int code_stride) {
  float mn = x[0], mx = x[0];
  for (int i = 1; i < count; ++i) {
    float v = x[(size_t)i * stride];
    if (v < mn) mn = v;
    if (v > mx) mx = v;
  }
  oref_quant_params(mn, mx, bits, meta_dtype, zp_mode, delta, zero);
  for (int i = 0; i < count; ++i)
    codes[(size_t)i * code_stride] =
        oref_quant_code(x[(size_t)i * stride], *delta, *zero, bits, zp_mode);
}

/* ------------------------------------------------------------------------ */
/* Cache bookkeeping [Alg.1: BufferQuantK / BufferQuantV], one (seq, head).  */
/* ------------------------------------------------------------------------ */

typedef struct {
  const oref_cache *c;
  uint8_t *k_codes; float *k_delta, *k_zero, *k_norm;
  uint8_t *v_codes; float *v_delta, *v_zero;
  float *res_k, *res_v, *res_norm;
} stream_view;

static stream_view view_of(const oref_cache *c, int b, int h) {
  stream_view s;
  size_t sh = (size_t)b * c->n_kv_heads + h;
  size_t cap = (size_t)c->cap_tokens, d = (size_t)c->d;
  s.c = c;
  s.k_codes = c->k_codes + sh * cap * d;
  s.k_delta = c->k_delta + sh * (cap / c->k_group) * d;
  s.k_zero = c->k_zero + sh * (cap / c->k_group) * d;
  s.k_norm = c->k_norm + sh * cap;
  s.v_codes = c->v_codes + sh * cap * d;
  s.v_delta = c->v_delta + sh * cap * (d / c->v_group);
  s.v_zero = c->v_zero + sh * cap * (d / c->v_group);
  s.res_k = c->res_k + sh * (size_t)c->R * d;
  s.res_v = c->res_v + sh * (size_t)c->R * d;
  s.res_norm = c->res_norm + sh * (size_t)c->R;
  return s;
}

/* GroupQuant of a full block of R tokens held in the residual arrays
 * (already rotated/normalized keys, raw values) into packed position `pos`. */
static void quantize_block(const stream_view *s, int pos) {
  const oref_cache *c = s->c;
  int d = c->d, R = c->R;
  /* keys: dim=channel, numGroup = R / G */
  for (int g = 0; g < R / c->k_group; ++g)
    for (int j = 0; j < d; ++j) {
      size_t grp = (size_t)(pos / c->k_group + g);
      oref_quant_group(s->res_k + (size_t)g * c->k_group * d + j, c->k_group, d, c->bits,
                       c->meta_dtype, c->zp_mode, &s->k_delta[grp * d + j],
                       &s->k_zero[grp * d + j],
                       s->k_codes + ((size_t)pos + (size_t)g * c->k_group) * d + j, d);
    }
  /* values: dim=token, numGroup = d / G */
  int ngv = d / c->v_group;
  for (int t = 0; t < R; ++t)
    for (int g = 0; g < ngv; ++g)
      oref_quant_group(s->res_v + (size_t)t * d + (size_t)g * c->v_group, c->v_group, 1,
                       c->bits, c->meta_dtype, c->zp_mode,
                       &s->v_delta[((size_t)pos + t) * ngv + g],
                       &s->v_zero[((size_t)pos + t) * ngv + g],
                       s->v_codes + ((size_t)pos + t) * d + (size_t)g * c->v_group, 1);
  for (int t = 0; t < R; ++t) s->k_norm[pos + t] = s->res_norm[t];
}

/* Append `n` tokens (k, v: [n][d] with row stride `row_stride` floats) to one
 * (sequence, head).  `np`/`nr` are that sequence's packed / residual counts on
 * entry; the new counts are returned through them.
 *   eager = 1 : prefill rule, every completed block of R tokens is quantized,
 *               the tail (< R) stays in the residual.  The algorithm acts on arriving
 *               tokens: with n = 0 nothing happens under either rule.
 *   eager = 0 : decode rule, a block completed by this call stays in the
 *               residual (so the attention that follows still sees it in FP16,
 *               as in OScaR-Inference where attention precedes BufferQuant)
 *               and is flushed at the start of the next append. */
static void stream_append(const stream_view *s, const float *k, const float *v, int n,
                          size_t row_stride, const float *tok_norm, int eager, int *np,
                          int *nr) {
  const oref_cache *c = s->c;
  int d = c->d, R = c->R;
  for (int t = 0; t < n; ++t) {
    if (*nr == R) {              /* deferred flush of a full residual */
      quantize_block(s, *np);
      *np += R;
      *nr = 0;
    }
    if (tok_norm) {              /* one norm per token over all kv heads [Fused-HN] */
      oref_key_transform_given_norm(k + (size_t)t * row_stride, d, c->rotate, tok_norm[t],
                                    s->res_k + (size_t)(*nr) * d);
      s->res_norm[*nr] = tok_norm[t];
    } else {
      oref_key_transform(k + (size_t)t * row_stride, d, c->rotate, c->scale_mode,
                         c->meta_dtype, s->res_k + (size_t)(*nr) * d, &s->res_norm[*nr]);
    }
    for (int j = 0; j < d; ++j) s->res_v[(size_t)(*nr) * d + j] = v[(size_t)t * row_stride + j];
    *nr += 1;
  }
  if (eager && n > 0 && *nr == R) {   /* (a call that brings no token changes nothing) */
    quantize_block(s, *np);
    *np += R;
    *nr = 0;
  }
}

/* k, v: [batch][T][n_kv][d]; new_lens[batch] (NULL = T for every sequence).
 * Returns 0, or -1 if a sequence would exceed cap_tokens. */
int oref_append(oref_cache *c, const float *k, const float *v, int T,
                const int32_t *new_lens, int eager, int nthreads) {
  for (int b = 0; b < c->batch; ++b) {
    int n = new_lens ? new_lens[b] : T;
    if (n < 0 || n > T) return -1;
    if (c->n_packed[b] + c->n_res[b] + n > c->cap_tokens) return -1;
  }
  int units = c->batch * c->n_kv_heads;
  float *tok_norm = NULL;       /* [batch][T], only for the all-heads norm */
  if (c->norm_scope == OREF_NORM_ALL_KV_HEADS && c->scale_mode == OREF_SCALE_L2) {
    tok_norm = (float *)malloc(sizeof(float) * (size_t)c->batch * (size_t)(T > 0 ? T : 1));
    for (int b = 0; b < c->batch; ++b)
      for (int t = 0; t < (new_lens ? new_lens[b] : T); ++t)
        tok_norm[(size_t)b * T + t] = oref_token_norm_all_heads(
            k + ((size_t)b * T + t) * c->n_kv_heads * c->d, c->n_kv_heads, (size_t)c->d, c->d,
            c->rotate, c->meta_dtype);
  }
  int32_t *np_out = (int32_t *)malloc(sizeof(int32_t) * (size_t)units);
  int32_t *nr_out = (int32_t *)malloc(sizeof(int32_t) * (size_t)units);
#ifdef _OPENMP
#pragma omp parallel for num_threads(nthreads > 0 ? nthreads : 1) schedule(dynamic, 1)
#endif
  for (int u = 0; u < units; ++u) {
    int b = u / c->n_kv_heads, h = u % c->n_kv_heads;
    int n = new_lens ? new_lens[b] : T;
    stream_view s = view_of(c, b, h);
    size_t row = (size_t)c->n_kv_heads * c->d;
    const float *kb = k + ((size_t)b * T * c->n_kv_heads + h) * c->d;
    const float *vb = v + ((size_t)b * T * c->n_kv_heads + h) * c->d;
    int np = c->n_packed[b], nr = c->n_res[b];
    stream_append(&s, kb, vb, n, row, tok_norm ? tok_norm + (size_t)b * T : NULL, eager, &np, &nr);
    np_out[u] = np;
    nr_out[u] = nr;
  }
  for (int b = 0; b < c->batch; ++b) {
    c->n_packed[b] = np_out[b * c->n_kv_heads];
    c->n_res[b] = nr_out[b * c->n_kv_heads];
  }
  free(np_out);
  free(nr_out);
  free(tok_norm);
  return 0;
}

/* ------------------------------------------------------------------------ */
/* Decode attention [Alg.1: K_all, V_all, Attention], [Key-xf: logits].      */
/* out = softmax(scale * Q_h K_hat^T) V_hat over packed + residual tokens,   */
/* K_hat_i = n_i * dequant(codes_i) or n_i * K_u residual, double precision. */
/* q: [batch][n_q][d] ; out: [batch][n_q][d] (fp32). q head h uses kv h/g.   */
/* ------------------------------------------------------------------------ */
static void attend_one(const stream_view *s, int np, int nr, const float *q, double scale,
                       float *out) {
  const oref_cache *c = s->c;
  int d = c->d, ngv = d / c->v_group;
  int total = np + nr;
  float qh[1024];
  oref_query_transform(q, d, c->rotate, qh);
  double *logit = (double *)malloc(sizeof(double) * (size_t)(total > 0 ? total : 1));
  double mx = -INFINITY;
  for (int i = 0; i < total; ++i) {
    double acc = 0.0;
    if (i < np) {
      size_t grp = (size_t)(i / c->k_group);
      for (int j = 0; j < d; ++j) {
        double kh = (double)s->k_norm[i] *
                    oref_dequant(s->k_codes[(size_t)i * d + j], s->k_delta[grp * d + j],
                                 s->k_zero[grp * d + j], c->zp_mode);
        acc += (double)qh[j] * kh;
      }
    } else {
      int r = i - np;
      for (int j = 0; j < d; ++j)
        acc += (double)qh[j] * ((double)s->res_norm[r] * (double)s->res_k[(size_t)r * d + j]);
    }
    logit[i] = scale * acc;
    if (logit[i] > mx) mx = logit[i];
  }
  double den = 0.0;
  double o[1024];
  for (int j = 0; j < d; ++j) o[j] = 0.0;
  for (int i = 0; i < total; ++i) {
    double p = exp(logit[i] - mx);
    den += p;
    if (i < np) {
      for (int j = 0; j < d; ++j) {
        int g = j / c->v_group;
        o[j] += p * oref_dequant(s->v_codes[(size_t)i * d + j], s->v_delta[(size_t)i * ngv + g],
                                 s->v_zero[(size_t)i * ngv + g], c->zp_mode);
      }
    } else {
      int r = i - np;
      for (int j = 0; j < d; ++j) o[j] += p * (double)s->res_v[(size_t)r * d + j];
    }
  }
  for (int j = 0; j < d; ++j) out[j] = (total > 0) ? (float)(o[j] / den) : 0.0f;
  free(logit);
}

void oref_decode_attn(const oref_cache *c, const float *q, int n_q_heads, float scale,
                      float *out, int nthreads) {
  int g = n_q_heads / c->n_kv_heads;
  int units = c->batch * n_q_heads;
  double sc = (scale > 0.0f) ? (double)scale : 1.0 / sqrt((double)c->d);
#ifdef _OPENMP
#pragma omp parallel for num_threads(nthreads > 0 ? nthreads : 1) schedule(dynamic, 1)
#endif
  for (int u = 0; u < units; ++u) {
    int b = u / n_q_heads, h = u % n_q_heads;
    stream_view s = view_of(c, b, h / g);
    attend_one(&s, c->n_packed[b], c->n_res[b], q + (size_t)u * c->d, sc,
               out + (size_t)u * c->d);
  }
}

/* Dequantized view of one (sequence, head): k_hat[total][d] (= n * K_u_hat, in
 * the ROTATED basis), v_hat[total][d]; for tests that need the decoded cache. */
void oref_dequantize_stream(const oref_cache *c, int b, int h, double *k_hat, double *v_hat) {
  stream_view s = view_of(c, b, h);
  int d = c->d, ngv = d / c->v_group, np = c->n_packed[b], nr = c->n_res[b];
  for (int i = 0; i < np + nr; ++i)
    for (int j = 0; j < d; ++j) {
      if (i < np) {
        size_t grp = (size_t)(i / c->k_group);
        k_hat[(size_t)i * d + j] =
            (double)s.k_norm[i] * oref_dequant(s.k_codes[(size_t)i * d + j],
                                               s.k_delta[grp * d + j], s.k_zero[grp * d + j],
                                               c->zp_mode);
        v_hat[(size_t)i * d + j] =
            oref_dequant(s.v_codes[(size_t)i * d + j], s.v_delta[(size_t)i * ngv + j / c->v_group],
                         s.v_zero[(size_t)i * ngv + j / c->v_group], c->zp_mode);
      } else {
        int r = i - np;
        k_hat[(size_t)i * d + j] = (double)s.res_norm[r] * (double)s.res_k[(size_t)r * d + j];
        v_hat[(size_t)i * d + j] = (double)s.res_v[(size_t)r * d + j];
      }
    }
}

/* ------------------------------------------------------------------------ */
/* BF16 comparator oracle: plain attention on un-rotated K, V (the baseline  */
/* of the paper's efficiency section), double accumulation.                  */
/* k, v: [batch][S][n_kv][d] ; q, out: [batch][n_q][d].                       */
/* ------------------------------------------------------------------------ */
void oref_plain_attn(const float *q, const float *k, const float *v, int batch, int S,
                     int n_q_heads, int n_kv_heads, int d, const int32_t *seq_lens,
                     float scale, float *out, int nthreads) {
  int g = n_q_heads / n_kv_heads;
  double sc = (scale > 0.0f) ? (double)scale : 1.0 / sqrt((double)d);
  int units = batch * n_q_heads;
#ifdef _OPENMP
#pragma omp parallel for num_threads(nthreads > 0 ? nthreads : 1) schedule(dynamic, 1)
#endif
  for (int u = 0; u < units; ++u) {
    int b = u / n_q_heads, h = u % n_q_heads, kvh = h / g;
    int len = seq_lens ? seq_lens[b] : S;
    const float *qv = q + (size_t)u * d;
    double *logit = (double *)malloc(sizeof(double) * (size_t)(len > 0 ? len : 1));
    double mx = -INFINITY;
    for (int i = 0; i < len; ++i) {
      const float *kr = k + (((size_t)b * S + i) * n_kv_heads + kvh) * d;
      double acc = 0.0;
      for (int j = 0; j < d; ++j) acc += (double)qv[j] * (double)kr[j];
      logit[i] = sc * acc;
      if (logit[i] > mx) mx = logit[i];
    }
    double den = 0.0, o[1024];
    for (int j = 0; j < d; ++j) o[j] = 0.0;
    for (int i = 0; i < len; ++i) {
      const float *vr = v + (((size_t)b * S + i) * n_kv_heads + kvh) * d;
      double p = exp(logit[i] - mx);
      den += p;
      for (int j = 0; j < d; ++j) o[j] += p * (double)vr[j];
    }
    for (int j = 0; j < d; ++j) out[(size_t)u * d + j] = len > 0 ? (float)(o[j] / den) : 0.0f;
    free(logit);
  }
}

int oref_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
