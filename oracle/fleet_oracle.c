/*
 * CPU oracle for the Fleet decode step.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the plain definition of what one decode step of a Qwen3-style
 * decoder stack computes (paper section 2.2, the per-layer operator list:
 * RMSNorm, QKV projection, attention over the KV cache, output projection,
 * RMSNorm + gate/up projection, SiLU x multiply, down projection + residual;
 * model shape from section 5.2).  The paper's scheduling, tiling, fusion and
 * cache policy only change where and when bytes move (section 3.1: a
 * device-task assembles its output in place without reduction; section 3.2:
 * each chiplet computes its columns with the full K reduction), so the
 * reference result is the plain definition written out with no blocking,
 * fusion or reordering.
 *
 * Arithmetic: bf16-rounded inputs, fp32 accumulation in index order, tensors
 * that cross an operator boundary rounded to bf16 (round-to-nearest-even):
 * norm outputs, q/k/v, attention output, the SwiGLU product.  The residual
 * stream and the logits stay fp32.  Flag ORACLE_HI switches every
 * accumulation to double and drops all intermediate rounding (used to bound
 * the effect of the rounding points); flag ORACLE_REVERSE_K sums GEMM
 * reductions from the last index down (used to estimate how far a different
 * but equally valid fp32 summation order moves the result).
 *
 * Nothing here is shared with the GPU path: own bf16 helpers, own RoPE
 * angles, own loops.  Only tests, the smoke check and the benchmark's CPU
 * baseline leg may call this library.
 *
 * Every function below is pinned by tests/test_oracle_pins.py against closed
 * forms, invariants, fp64 brute force and library routines.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_HI 1
#define ORACLE_REVERSE_K 2

typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
  int32_t max_batch, max_seq;
  float rms_eps, rope_theta;
} oracle_shape_t;

/* Host pointers to bf16 (uint16_t bit patterns). Per-layer arrays hold
 * n_layers pointers.  Matrices are [out_features, in_features], in_features
 * contiguous (section 4.3: chiplet k's partition starts at
 * base + k*(N/8)*K elements, i.e. rows of length K). */
typedef struct {
  const uint16_t *embed;           /* [vocab, hidden] or NULL */
  const uint16_t *const *ln1;      /* [hidden] */
  const uint16_t *const *wqkv;     /* [(nq+2nkv)*hd, hidden], rows Q|K|V */
  const uint16_t *const *q_norm;   /* [hd] */
  const uint16_t *const *k_norm;   /* [hd] */
  const uint16_t *const *wo;       /* [hidden, nq*hd] */
  const uint16_t *const *ln2;      /* [hidden] */
  const uint16_t *const *wgu;      /* [2*ffn, hidden], rows gate|up */
  const uint16_t *const *wdown;    /* [hidden, ffn] */
  const uint16_t *final_norm;      /* [hidden] or NULL when vocab == 0 */
  const uint16_t *lm_head;         /* [vocab, hidden] or NULL */
} oracle_weights_t;

/* ---- bf16 <-> fp32 ------------------------------------------------------ */

static inline float bf2f(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* round-to-nearest-even on the upper 16 bits; NaN kept quiet */
static inline uint16_t f2bf(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  return (uint16_t)(u >> 16);
}

static inline float round_bf(float f) { return bf2f(f2bf(f)); }

uint16_t oracle_f2bf(float f) { return f2bf(f); }
float oracle_bf2f(uint16_t h) { return bf2f(h); }
int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---- RMSNorm (section 2.2 step 1; eps inside the root, gain last) ------- */
/* x fp32 [n], gain bf16 [n] -> out fp32 [n] (NOT yet rounded). */
static void rmsnorm_f32(const float *x, const uint16_t *g, int n, float eps,
                        int hi, float *out) {
  if (hi) {
    double ss = 0.0;
    for (int i = 0; i < n; ++i) ss += (double)x[i] * (double)x[i];
    double r = 1.0 / sqrt(ss / n + (double)eps);
    for (int i = 0; i < n; ++i) out[i] = (float)((double)x[i] * r * (double)bf2f(g[i]));
  } else {
    float ss = 0.f;
    for (int i = 0; i < n; ++i) ss += x[i] * x[i];
    float r = 1.0f / sqrtf(ss / (float)n + eps);
    for (int i = 0; i < n; ++i) out[i] = x[i] * r * bf2f(g[i]);
  }
}

/* public: x fp32 [rows, n] -> out fp32 [rows, n], rounded to bf16 values
 * unless hi. */
void oracle_rmsnorm(const float *x, const uint16_t *gain, int rows, int n,
                    float eps, int flags, float *out) {
  int hi = flags & ORACLE_HI;
  for (int r = 0; r < rows; ++r) {
    rmsnorm_f32(x + (size_t)r * n, gain, n, eps, hi, out + (size_t)r * n);
    if (!hi)
      for (int i = 0; i < n; ++i) out[(size_t)r * n + i] = round_bf(out[(size_t)r * n + i]);
  }
}

/* ---- Linear: y[b,n] = sum_k x[b,k] * W[n,k]  (section 2.2 steps 2,4,5,7) - */
/* x fp32 values (already bf16-representable unless hi), W bf16 [N,K]. */
void oracle_linear(const float *x, const uint16_t *w, int B, int K, int N,
                   int flags, float *y) {
  const int hi = flags & ORACLE_HI;
  const int rev = flags & ORACLE_REVERSE_K;
#pragma omp parallel for schedule(static)
  for (int n = 0; n < N; ++n) {
    const uint16_t *wr = w + (size_t)n * K;
    for (int b = 0; b < B; ++b) {
      const float *xr = x + (size_t)b * K;
      if (hi) {
        double acc = 0.0;
        for (int k = 0; k < K; ++k) acc += (double)xr[k] * (double)bf2f(wr[k]);
        y[(size_t)b * N + n] = (float)acc;
      } else if (rev) {
        float acc = 0.f;
        for (int k = K - 1; k >= 0; --k) acc += xr[k] * bf2f(wr[k]);
        y[(size_t)b * N + n] = acc;
      } else {
        float acc = 0.f;
        for (int k = 0; k < K; ++k) acc += xr[k] * bf2f(wr[k]);
        y[(size_t)b * N + n] = acc;
      }
    }
  }
}

/* ---- per-head RMSNorm then rotary embedding ------------------------------ */
/* t fp32 [hd] in place.  Norm over the head's hd values with gain [hd];
 * rotation pairs (i, i+hd/2), angle = pos * theta^(-2i/hd), computed in
 * double and applied in fp32 (double when hi). */
void oracle_head_norm_rope(float *t, const uint16_t *gain, int hd, float eps,
                           float theta, int pos, int flags) {
  const int hi = flags & ORACLE_HI;
  float tmp[1024];
  rmsnorm_f32(t, gain, hd, eps, hi, tmp);
  const int half = hd / 2;
  for (int i = 0; i < half; ++i) {
    double inv = pow((double)theta, -2.0 * (double)i / (double)hd);
    double ang = (double)pos * inv;
    double c = cos(ang), s = sin(ang);
    if (hi) {
      double a = tmp[i], b = tmp[i + half];
      t[i] = (float)(a * c - b * s);
      t[i + half] = (float)(b * c + a * s);
    } else {
      float cf = (float)c, sf = (float)s;
      float a = tmp[i], b = tmp[i + half];
      t[i] = a * cf - b * sf;
      t[i + half] = b * cf + a * sf;
    }
  }
}

/* ---- decode attention for one query head (section 2.2 step 3) ------------ */
/* q fp32 [hd]; kc, vc bf16 [n_keys, hd] (slots 0..n_keys-1 of one KV head);
 * out fp32 [hd] = softmax(q.K^T / sqrt(hd)) . V, max-subtracted softmax. */
void oracle_attend_head(const float *q, const uint16_t *kc, const uint16_t *vc,
                        int n_keys, int hd, int flags, float *out) {
  const int hi = flags & ORACLE_HI;
  if (hi) {
    double *s = (double *)malloc(sizeof(double) * (size_t)n_keys);
    double scale = 1.0 / sqrt((double)hd), m = -INFINITY;
    for (int j = 0; j < n_keys; ++j) {
      double a = 0.0;
      for (int d = 0; d < hd; ++d) a += (double)q[d] * (double)bf2f(kc[(size_t)j * hd + d]);
      s[j] = a * scale;
      if (s[j] > m) m = s[j];
    }
    double l = 0.0;
    for (int j = 0; j < n_keys; ++j) { s[j] = exp(s[j] - m); l += s[j]; }
    for (int d = 0; d < hd; ++d) {
      double a = 0.0;
      for (int j = 0; j < n_keys; ++j) a += s[j] * (double)bf2f(vc[(size_t)j * hd + d]);
      out[d] = (float)(a / l);
    }
    free(s);
  } else {
    float *s = (float *)malloc(sizeof(float) * (size_t)n_keys);
    float scale = 1.0f / sqrtf((float)hd), m = -INFINITY;
    for (int j = 0; j < n_keys; ++j) {
      float a = 0.f;
      for (int d = 0; d < hd; ++d) a += q[d] * bf2f(kc[(size_t)j * hd + d]);
      s[j] = a * scale;
      if (s[j] > m) m = s[j];
    }
    float l = 0.f;
    for (int j = 0; j < n_keys; ++j) { s[j] = expf(s[j] - m); l += s[j]; }
    for (int d = 0; d < hd; ++d) {
      float a = 0.f;
      for (int j = 0; j < n_keys; ++j) a += s[j] * bf2f(vc[(size_t)j * hd + d]);
      out[d] = a / l;
    }
    free(s);
  }
}

/* softmax probabilities only (for the row-sum pin): s fp32 [n] in place */
void oracle_softmax(float *s, int n) {
  float m = -INFINITY, l = 0.f;
  for (int j = 0; j < n; ++j) if (s[j] > m) m = s[j];
  for (int j = 0; j < n; ++j) { s[j] = expf(s[j] - m); l += s[j]; }
  for (int j = 0; j < n; ++j) s[j] /= l;
}

/* ---- SwiGLU (section 2.2 step 6, fused: section 3.2 "Operator fusion") --- */
/* gu fp32 [B, 2*ffn] (gate | up) -> h fp32 [B, ffn]; silu(z) = z/(1+e^-z) on
 * the unrounded accumulators, product rounded to bf16 unless hi. */
void oracle_swiglu(const float *gu, int B, int ffn, int flags, float *h) {
  const int hi = flags & ORACLE_HI;
  for (int b = 0; b < B; ++b)
    for (int i = 0; i < ffn; ++i) {
      float g = gu[(size_t)b * 2 * ffn + i], u = gu[(size_t)b * 2 * ffn + ffn + i];
      if (hi) {
        double v = ((double)g / (1.0 + exp(-(double)g))) * (double)u;
        h[(size_t)b * ffn + i] = (float)v;
      } else {
        float v = (g / (1.0f + expf(-g))) * u;
        h[(size_t)b * ffn + i] = round_bf(v);
      }
    }
}

/* ---- the decode step ---------------------------------------------------------- */
/*
 * Layers [layer_begin, layer_end) applied to the fp32 residual stream.
 *
 * x_in   fp32 [B, hidden]: residual stream entering layer_begin
 * k_cache/v_cache bf16 [n_layers][max_batch][n_kv][max_seq][hd], updated at
 *   slot positions[b] for every layer run
 * positions int32 [B]: index of the new token = number of valid cache slots
 *   before the step; the new token attends to slots 0..positions[b] inclusive
 * x_out  fp32 [B, hidden]: residual stream after layer_end-1
 * x_trace fp32 [layer_end-layer_begin+1][B, hidden] or NULL: the residual
 *   stream at every layer boundary (entry 0 = x_in)
 * logits fp32 [B, vocab] or NULL; computed only when layer_end == n_layers
 * Rows are independent; every row is computed on its own.
 * Returns 0, or -1 on a bad argument.
 */
int oracle_decode_layers(const oracle_shape_t *sh, const oracle_weights_t *w,
                         int B, int layer_begin, int layer_end, const float *x_in,
                         uint16_t *k_cache, uint16_t *v_cache,
                         const int32_t *positions, float *x_out, float *x_trace,
                         float *logits, int flags) {
  if (!sh || !w || !x_in || !x_out || B < 1 || B > sh->max_batch) return -1;
  if (layer_begin < 0 || layer_end > sh->n_layers || layer_begin > layer_end) return -1;
  const int hi = flags & ORACLE_HI;
  const int H = sh->hidden, hd = sh->head_dim, nq = sh->n_q_heads,
            nkv = sh->n_kv_heads, F = sh->ffn;
  if (hd > 1024 || (hd & 1) || nq % nkv) return -1;
  const int NQKV = (nq + 2 * nkv) * hd, QD = nq * hd, grp = nq / nkv;
  for (int b = 0; b < B; ++b)
    if (positions[b] < 0 || positions[b] >= sh->max_seq) return -1;

  float *x = (float *)malloc(sizeof(float) * (size_t)B * H);
  float *n = (float *)malloc(sizeof(float) * (size_t)B * H);
  float *qkv = (float *)malloc(sizeof(float) * (size_t)B * NQKV);
  float *att = (float *)malloc(sizeof(float) * (size_t)B * QD);
  float *proj = (float *)malloc(sizeof(float) * (size_t)B * H);
  float *gu = (float *)malloc(sizeof(float) * (size_t)B * 2 * F);
  float *h = (float *)malloc(sizeof(float) * (size_t)B * F);
  memcpy(x, x_in, sizeof(float) * (size_t)B * H);
  if (x_trace) memcpy(x_trace, x, sizeof(float) * (size_t)B * H);

  for (int l = layer_begin; l < layer_end; ++l) {
    oracle_rmsnorm(x, w->ln1[l], B, H, sh->rms_eps, flags, n);
    oracle_linear(n, w->wqkv[l], B, H, NQKV, flags, qkv);
    for (int b = 0; b < B; ++b) {
      const int p = positions[b];
      float *row = qkv + (size_t)b * NQKV;
      for (int hh = 0; hh < nq + nkv; ++hh) {
        float *t = row + (size_t)hh * hd;
        oracle_head_norm_rope(t, hh < nq ? w->q_norm[l] : w->k_norm[l], hd,
                              sh->rms_eps, sh->rope_theta, p, flags);
      }
      if (!hi)
        for (int i = 0; i < NQKV; ++i) row[i] = round_bf(row[i]);
      /* append k, v of the new token at slot p (the cache stores bf16) */
      for (int g = 0; g < nkv; ++g) {
        size_t slot = ((((size_t)l * sh->max_batch + b) * nkv + g) * sh->max_seq + p) * hd;
        for (int d = 0; d < hd; ++d) {
          k_cache[slot + d] = f2bf(row[(size_t)(nq + g) * hd + d]);
          v_cache[slot + d] = f2bf(row[(size_t)(nq + nkv + g) * hd + d]);
        }
      }
    }
#pragma omp parallel for schedule(static) collapse(2)
    for (int b = 0; b < B; ++b)
      for (int hh = 0; hh < nq; ++hh) {
        const int g = hh / grp, p = positions[b];
        size_t base = (((size_t)l * sh->max_batch + b) * nkv + g) * sh->max_seq * hd;
        float *o = att + (size_t)b * QD + (size_t)hh * hd;
        oracle_attend_head(qkv + (size_t)b * NQKV + (size_t)hh * hd, k_cache + base,
                           v_cache + base, p + 1, hd, flags, o);
        if (!hi)
          for (int d = 0; d < hd; ++d) o[d] = round_bf(o[d]);
      }
    oracle_linear(att, w->wo[l], B, QD, H, flags, proj);
    for (size_t i = 0; i < (size_t)B * H; ++i) x[i] = x[i] + proj[i];
    oracle_rmsnorm(x, w->ln2[l], B, H, sh->rms_eps, flags, n);
    oracle_linear(n, w->wgu[l], B, H, 2 * F, flags, gu);
    oracle_swiglu(gu, B, F, flags, h);
    oracle_linear(h, w->wdown[l], B, F, H, flags, proj);
    for (size_t i = 0; i < (size_t)B * H; ++i) x[i] = x[i] + proj[i];
    if (x_trace)
      memcpy(x_trace + (size_t)(l - layer_begin + 1) * B * H, x, sizeof(float) * (size_t)B * H);
  }
  memcpy(x_out, x, sizeof(float) * (size_t)B * H);
  if (logits && layer_end == sh->n_layers && sh->vocab > 0 && w->lm_head && w->final_norm) {
    oracle_rmsnorm(x, w->final_norm, B, H, sh->rms_eps, flags, n);
    oracle_linear(n, w->lm_head, B, H, sh->vocab, flags, logits);
  }
  free(x); free(n); free(qkv); free(att); free(proj); free(gu); free(h);
  return 0;
}

/*
 * The whole step: the residual stream starts as float(hidden_in[b]) (bf16
 * [B, hidden]) or, when tokens != NULL, as float(embed[tokens[b]]); then all
 * layers, then final norm + LM head.  hidden_out is the fp32 residual stream
 * after the last layer.
 */
int oracle_decode_step(const oracle_shape_t *sh, const oracle_weights_t *w,
                       int B, const uint16_t *hidden_in, const int32_t *tokens,
                       uint16_t *k_cache, uint16_t *v_cache,
                       const int32_t *positions, float *hidden_out,
                       float *x_trace, float *logits, int flags) {
  if (!sh || !w || B < 1 || B > sh->max_batch) return -1;
  if (!hidden_in && !(tokens && w->embed)) return -1;
  const int H = sh->hidden;
  if (tokens)
    for (int b = 0; b < B; ++b)
      if (tokens[b] < 0 || tokens[b] >= sh->vocab) return -1;
  float *x = (float *)malloc(sizeof(float) * (size_t)B * H);
  for (int b = 0; b < B; ++b)
    for (int i = 0; i < H; ++i)
      x[(size_t)b * H + i] = tokens ? bf2f(w->embed[(size_t)tokens[b] * H + i])
                                    : bf2f(hidden_in[(size_t)b * H + i]);
  int rc = oracle_decode_layers(sh, w, B, 0, sh->n_layers, x, k_cache, v_cache,
                                positions, hidden_out, x_trace, logits, flags);
  free(x);
  return rc;
}
