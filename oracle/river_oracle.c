/*
 * CPU oracle for early-exit decode with a KV-Shared Exit River.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the decode path must
 * compute; it is slow and plain on purpose.  It shares no code with the HIP
 * library and must never be called from the product path.
 *
 * What it follows (River-LLM paper):
 *   - "KV-Shared Exit Layer" subsection of the method section: every backbone
 *     block l has a twin with the same architecture whose seven projection
 *     matrices are 4-bit weight-only quantised copies; the twin reads and
 *     writes the SAME KV-cache slot (layer l, position p) as the backbone.
 *   - "Inference with Seamless Exit" subsection and Eq. 1: after backbone
 *     block l the cosine similarity s between the block's input and output
 *     hidden states is compared with tau; on exit the remaining blocks run as
 *     river twins, chained serially, and the ORIGINAL final norm + LM head
 *     produce the logits.  Generation phase = token-level exit; the prompt is
 *     processed at one unified depth given by the caller (default: the full depth L).
 *   - Table "Evaluation results ... Exit Position" caption: the exit position
 *     is the number of executed backbone layers.
 *
 * Readings where the paper is silent (listed in the design notes too):
 *   blocks 1..L, h(0) = embedding; test only for L_s <= l < L, first hit wins,
 *   strict '>'; s = 0 if a norm is 0, clamped to [-1,1]; pre-norm Llama block
 *   (RMSNorm, rotate-half RoPE, GQA, SwiGLU, no biases); K/V are rounded to the
 *   cache dtype (round-to-nearest-even) when stored and attention reads the
 *   stored value also for the current position; argmax ties -> lowest index;
 *   river quantiser = asymmetric round-to-nearest over groups of consecutive
 *   input elements of one output row.
 *
 * Arithmetic: fp64 everywhere except the declared rounding points (weights
 * and cache entries are values of the storage dtype; dequantisation of a river
 * weight is (q - zero) * scale evaluated in fp32 as the format defines it).
 *
 * parity unpinned: the QUALITY of the river approximation on trained weights
 * (K/V cosine >= 0.97, 98 % next-token match) cannot be pinned here: it needs
 * the pretrained models.  Everything the algorithm computes is pinned by the
 * tests under tests/ that are not marked gpu.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ENOSPC (-2)

typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rope_base, rms_eps;
  int32_t dtype; /* 0 fp32, 1 bf16 */
  int32_t max_seq;
  int32_t min_exit_layer; /* L_s */
  float tau;
  int32_t river_group;
  int32_t kv_dtype; /* KV-cache storage: 0 = the weight dtype, 1 = IEEE half (fp16), the type the
                       paper keeps its cache in ("KV-Shared Exit Layer": W4A16, KV cache in FP16) */
} orc_config;

/* per-layer pointer table, host memory, element type = cfg.dtype */
typedef struct {
  const void *attn_norm, *wq, *wk, *wv, *wo, *ffn_norm, *w_gate, *w_up, *w_down;
} orc_layer;

/* river twin of one matrix: packed codes (two per byte, even index in the low
 * nibble), scale and zero per (row, group) in cfg.dtype */
typedef struct {
  const uint8_t *codes;
  const void *scale, *zero;
} orc_qmat;

typedef struct {
  orc_qmat m[7]; /* wq wk wv wo w_gate w_up w_down */
} orc_qlayer;

typedef struct {
  orc_config c;
  const void *tok_emb, *final_norm, *lm_head;
  orc_layer *layers;
  orc_qlayer *river; /* NULL entries (codes==NULL) for layers without twin */
  float *kcache, *vcache; /* [L][max_seq][n_kv*hd], values already rounded */
  uint8_t *written;       /* [L][max_seq] write counters (KV integrity check) */
  int32_t pos;            /* next position to be written */
  double *hid;            /* [L+1][d] hidden states of the last step */
  double *logits;         /* [vocab] of the last step */
  double *sims;           /* [L] similarity per executed backbone block, NaN else */
} orc_ctx;

/* ---------------------------------------------------------------- storage */

static inline float bf16_to_f32(uint16_t w) {
  uint32_t u = (uint32_t)w << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* round-to-nearest-even float -> bf16 word */
uint16_t orc_f32_to_bf16(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40); /* NaN */
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  return (uint16_t)(u >> 16);
}

static inline double ld(const void *p, int64_t i, int dtype) {
  return dtype ? (double)bf16_to_f32(((const uint16_t *)p)[i]) : (double)((const float *)p)[i];
}

/* round-to-nearest-even float -> IEEE binary16 word (1 sign, 5 exponent, 10 mantissa bits;
 * subnormals kept, overflow to infinity) */
uint16_t orc_f32_to_f16(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
  uint32_t a = u & 0x7fffffffu;
  if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);          /* NaN */
  if (a >= 0x477ff000u) return (uint16_t)(sign | 0x7c00u);         /* >= 65520 rounds to infinity */
  if (a < 0x33000001u) return sign;                                /* <= 2^-25 rounds to zero */
  int e = (int)(a >> 23) - 127;                                    /* unbiased exponent */
  uint32_t m = (a & 0x7fffffu) | 0x800000u;                        /* 24-bit significand */
  int shift = e >= -14 ? 13 : 13 + (-14 - e);                      /* bits dropped (subnormal: more) */
  uint32_t keep = m >> shift, rem = m & ((1u << shift) - 1u), half = 1u << (shift - 1);
  if (rem > half || (rem == half && (keep & 1u))) keep += 1;
  /* normal: keep holds 1.mmmmmmmmmm (11 bits), exponent field e + 15; a carry out of the
   * significand moves into the exponent by plain addition, subnormals likewise */
  uint32_t h = e >= -14 ? ((uint32_t)(e + 15) << 10) + (keep - 0x400u) : keep;
  return (uint16_t)(sign | h);
}

float orc_f16_to_f32(uint16_t h) {
  int sign = (h >> 15) & 1, e = (h >> 10) & 31, m = h & 1023;
  double v;
  if (e == 0) v = ldexp((double)m, -24);
  else if (e == 31) v = m ? NAN : INFINITY;
  else v = ldexp((double)(m | 1024), e - 25);
  return (float)(sign ? -v : v);
}

/* value -> value representable in the cache's storage type */
static inline float round_cache(double v, int dtype, int kv_dtype) {
  float f = (float)v;
  if (kv_dtype == 1) return orc_f16_to_f32(orc_f32_to_f16(f));
  return dtype ? bf16_to_f32(orc_f32_to_bf16(f)) : f;
}

/* ------------------------------------------------------------ quantiser */

/*
 * 4-bit asymmetric round-to-nearest quantiser of one [rows, cols] matrix
 * ("KV-Shared Exit Layer": W4A16 weight-only PTQ of a copied block).
 * Group = `group` consecutive input elements of one row (the last group of a
 * row is shorter when group does not divide cols).  Per group, in fp32:
 *   scale = (max - min) / 15   (1 if max == min), stored in the weight dtype
 *   zero  = -min / scale       (with the STORED scale), stored in the weight dtype
 *   code  = clamp(rint(w / scale + zero), 0, 15)   with the stored scale, zero
 */
int orc_quantize_w4(const void *w, int64_t rows, int64_t cols, int group, int dtype,
                    uint8_t *codes, void *scale, void *zero) {
  if (!w || !codes || !scale || !zero || group <= 0 || cols % 2 || group % 2) return ORC_EINVAL;
  int64_t gpr = (cols + group - 1) / group; /* the last group of a row may be shorter */
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r) {
    for (int64_t g = 0; g < gpr; ++g) {
      int64_t base = r * cols + g * group;
      int glen = (int)((g + 1) * group <= cols ? group : cols - g * group);
      float mn = (float)ld(w, base, dtype), mx = mn;
      for (int i = 1; i < glen; ++i) {
        float v = (float)ld(w, base + i, dtype);
        if (v < mn) mn = v;
        if (v > mx) mx = v;
      }
      float s = (mx > mn) ? (mx - mn) / 15.0f : 1.0f;
      if (dtype) s = bf16_to_f32(orc_f32_to_bf16(s));
      float z = -mn / s;
      if (dtype) z = bf16_to_f32(orc_f32_to_bf16(z));
      if (dtype) {
        ((uint16_t *)scale)[r * gpr + g] = orc_f32_to_bf16(s);
        ((uint16_t *)zero)[r * gpr + g] = orc_f32_to_bf16(z);
      } else {
        ((float *)scale)[r * gpr + g] = s;
        ((float *)zero)[r * gpr + g] = z;
      }
      for (int i = 0; i < glen; i += 2) {
        int q[2];
        for (int k = 0; k < 2; ++k) {
          float v = (float)ld(w, base + i + k, dtype);
          float t = rintf(v / s + z);
          q[k] = t < 0.0f ? 0 : (t > 15.0f ? 15 : (int)t);
        }
        codes[(base + i) / 2] = (uint8_t)(q[0] | (q[1] << 4));
      }
    }
  }
  return ORC_OK;
}

/* river weight (row r, column c) as the format defines it: (q - zero) * scale in fp32 */
static inline double dq(const orc_qmat *m, int64_t r, int64_t c, int64_t cols, int group, int dtype) {
  int64_t idx = r * cols + c;
  uint8_t b = m->codes[idx >> 1];
  int q = (idx & 1) ? (b >> 4) : (b & 15);
  int64_t g = r * ((cols + group - 1) / group) + c / group;
  float s = (float)ld(m->scale, g, dtype), z = (float)ld(m->zero, g, dtype);
  float wv = ((float)q - z) * s;
  return (double)wv;
}

int orc_dequantize_w4(const uint8_t *codes, const void *scale, const void *zero, int64_t rows,
                      int64_t cols, int group, int dtype, double *out) {
  orc_qmat m = {codes, scale, zero};
  for (int64_t r = 0; r < rows; ++r)
    for (int64_t c = 0; c < cols; ++c) out[r * cols + c] = dq(&m, r, c, cols, group, dtype);
  return ORC_OK;
}

/* --------------------------------------------------------- block pieces */

/* y = W x, W [rows, cols] dense in dtype */
static void matvec(const void *w, int dtype, int64_t rows, int64_t cols, const double *x, double *y) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r) {
    double acc = 0.0;
    for (int64_t c = 0; c < cols; ++c) acc += ld(w, r * cols + c, dtype) * x[c];
    y[r] = acc;
  }
}

/* y = W^ x, W^ the dequantised river matrix */
static void matvec_q(const orc_qmat *m, int dtype, int group, int64_t rows, int64_t cols,
                     const double *x, double *y) {
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < rows; ++r) {
    double acc = 0.0;
    for (int64_t c = 0; c < cols; ++c) acc += dq(m, r, c, cols, group, dtype) * x[c];
    y[r] = acc;
  }
}

/* out = x * rsqrt(mean(x^2) + eps) * g */
void orc_rmsnorm(const double *x, const void *g, int dtype, int n, double eps, double *out) {
  double ss = 0.0;
  for (int i = 0; i < n; ++i) ss += x[i] * x[i];
  double r = 1.0 / sqrt(ss / n + eps);
  for (int i = 0; i < n; ++i) out[i] = x[i] * r * ld(g, i, dtype);
}

/* rotate-half RoPE on n_heads vectors of length hd at position pos:
 * pair (i, i + hd/2) is rotated by the angle pos * base^(-2i/hd) */
void orc_rope(double *v, int n_heads, int hd, int pos, double base) {
  int half = hd / 2;
  for (int h = 0; h < n_heads; ++h) {
    double *p = v + (int64_t)h * hd;
    for (int i = 0; i < half; ++i) {
      double ang = (double)pos * pow(base, -2.0 * i / hd);
      double c = cos(ang), s = sin(ang);
      double a = p[i], b = p[i + half];
      p[i] = a * c - b * s;
      p[i + half] = a * s + b * c;
    }
  }
}

/* causal single-query GQA attention over cache rows 0..T-1 (row stride n_kv*hd):
 * o_i = sum_j softmax_j(q_i . K_j / sqrt(hd)) V_j, q head i uses kv head i / (nq/nkv) */
void orc_attention(const double *q, const float *K, const float *V, int T, int nq, int nkv, int hd,
                   double *o) {
  int rep = nq / nkv, stride = nkv * hd;
  double inv = 1.0 / sqrt((double)hd);
#pragma omp parallel for schedule(static)
  for (int i = 0; i < nq; ++i) {
    int kvh = i / rep;
    double *sc = (double *)malloc(sizeof(double) * (size_t)T);
    double mx = -INFINITY;
    for (int j = 0; j < T; ++j) {
      const float *kr = K + (int64_t)j * stride + kvh * hd;
      double d = 0.0;
      for (int e = 0; e < hd; ++e) d += q[i * hd + e] * (double)kr[e];
      sc[j] = d * inv;
      if (sc[j] > mx) mx = sc[j];
    }
    double den = 0.0;
    for (int j = 0; j < T; ++j) {
      sc[j] = exp(sc[j] - mx);
      den += sc[j];
    }
    for (int e = 0; e < hd; ++e) {
      double acc = 0.0;
      for (int j = 0; j < T; ++j) acc += sc[j] * (double)V[(int64_t)j * stride + kvh * hd + e];
      o[i * hd + e] = acc / den;
    }
    free(sc);
  }
}

/* silu(g) * u */
void orc_swiglu(const double *g, const double *u, int n, double *out) {
  for (int i = 0; i < n; ++i) out[i] = g[i] / (1.0 + exp(-g[i])) * u[i];
}

/* Eq. 1 similarity: <a,b> / (|a| |b|), 0 if a norm vanishes, clamped to [-1,1] */
double orc_cosine(const double *a, const double *b, int n) {
  double ab = 0, aa = 0, bb = 0;
  for (int i = 0; i < n; ++i) {
    ab += a[i] * b[i];
    aa += a[i] * a[i];
    bb += b[i] * b[i];
  }
  if (aa == 0.0 || bb == 0.0) return 0.0;
  double s = ab / (sqrt(aa) * sqrt(bb));
  return s > 1.0 ? 1.0 : (s < -1.0 ? -1.0 : s);
}

/*
 * One decoder block at position p; `river` selects the twin's matrices.
 * Writes slot (l, p) of the shared cache whichever path runs.
 */
static void block(orc_ctx *x, int l, int p, int river, const double *h, double *hout) {
  const orc_config *c = &x->c;
  int d = c->d_model, nq = c->n_q_heads, nkv = c->n_kv_heads, hd = c->head_dim, f = c->d_ffn;
  int dt = c->dtype, G = c->river_group;
  const orc_layer *W = &x->layers[l];
  const orc_qlayer *Q = river ? &x->river[l] : NULL;
  int qd = nq * hd, kvd = nkv * hd;
  double *xn = malloc(sizeof(double) * d), *q = malloc(sizeof(double) * qd);
  double *k = malloc(sizeof(double) * kvd), *v = malloc(sizeof(double) * kvd);
  double *o = malloc(sizeof(double) * qd), *t = malloc(sizeof(double) * d);
  double *h1 = malloc(sizeof(double) * d), *g = malloc(sizeof(double) * f);
  double *u = malloc(sizeof(double) * f), *a = malloc(sizeof(double) * f);

  orc_rmsnorm(h, W->attn_norm, dt, d, c->rms_eps, xn); /* norm gains: always the backbone's */
  if (river) {
    matvec_q(&Q->m[0], dt, G, qd, d, xn, q);
    matvec_q(&Q->m[1], dt, G, kvd, d, xn, k);
    matvec_q(&Q->m[2], dt, G, kvd, d, xn, v);
  } else {
    matvec(W->wq, dt, qd, d, xn, q);
    matvec(W->wk, dt, kvd, d, xn, k);
    matvec(W->wv, dt, kvd, d, xn, v);
  }
  orc_rope(q, nq, hd, p, c->rope_base);
  orc_rope(k, nkv, hd, p, c->rope_base);
  float *Kl = x->kcache + (int64_t)l * c->max_seq * kvd, *Vl = x->vcache + (int64_t)l * c->max_seq * kvd;
  for (int i = 0; i < kvd; ++i) {
    Kl[(int64_t)p * kvd + i] = round_cache(k[i], dt, c->kv_dtype);
    Vl[(int64_t)p * kvd + i] = round_cache(v[i], dt, c->kv_dtype);
  }
  if (x->written[(int64_t)l * c->max_seq + p] < 255) x->written[(int64_t)l * c->max_seq + p]++;
  orc_attention(q, Kl, Vl, p + 1, nq, nkv, hd, o);
  if (river) matvec_q(&Q->m[3], dt, G, d, qd, o, t);
  else matvec(W->wo, dt, d, qd, o, t);
  for (int i = 0; i < d; ++i) h1[i] = h[i] + t[i];
  orc_rmsnorm(h1, W->ffn_norm, dt, d, c->rms_eps, xn);
  if (river) {
    matvec_q(&Q->m[4], dt, G, f, d, xn, g);
    matvec_q(&Q->m[5], dt, G, f, d, xn, u);
  } else {
    matvec(W->w_gate, dt, f, d, xn, g);
    matvec(W->w_up, dt, f, d, xn, u);
  }
  orc_swiglu(g, u, f, a);
  if (river) matvec_q(&Q->m[6], dt, G, d, f, a, t);
  else matvec(W->w_down, dt, d, f, a, t);
  for (int i = 0; i < d; ++i) hout[i] = h1[i] + t[i];
  free(xn); free(q); free(k); free(v); free(o); free(t); free(h1); free(g); free(u); free(a);
}

/* test hook: one block on a caller-supplied hidden state (uses and writes the cache) */
int orc_block(orc_ctx *x, int layer1, int pos, int river, const double *h, double *hout) {
  if (!x || layer1 < 1 || layer1 > x->c.n_layers || pos < 0 || pos >= x->c.max_seq) return ORC_EINVAL;
  if (river && !x->river[layer1 - 1].m[0].codes) return ORC_EINVAL;
  block(x, layer1 - 1, pos, river, h, hout);
  return ORC_OK;
}

/* ------------------------------------------------------------ lifecycle */

int orc_create(const orc_config *cfg, const void *tok_emb, const void *final_norm,
               const void *lm_head, const orc_layer *layers, const orc_qlayer *river,
               orc_ctx **out) {
  if (!cfg || !tok_emb || !final_norm || !lm_head || !layers || !out) return ORC_EINVAL;
  if (cfg->n_layers < 1 || cfg->n_q_heads % cfg->n_kv_heads || cfg->head_dim % 2 ||
      cfg->min_exit_layer < 0 || cfg->min_exit_layer > cfg->n_layers || cfg->max_seq < 1 ||
      (cfg->kv_dtype != 0 && cfg->kv_dtype != 1))
    return ORC_EINVAL;
  orc_ctx *x = calloc(1, sizeof(*x));
  x->c = *cfg;
  x->tok_emb = tok_emb; x->final_norm = final_norm; x->lm_head = lm_head;
  int L = cfg->n_layers;
  x->layers = malloc(sizeof(orc_layer) * L);
  memcpy(x->layers, layers, sizeof(orc_layer) * L);
  x->river = calloc(L, sizeof(orc_qlayer));
  if (river) memcpy(x->river, river, sizeof(orc_qlayer) * L);
  int64_t kvd = (int64_t)cfg->n_kv_heads * cfg->head_dim;
  x->kcache = calloc((size_t)L * cfg->max_seq * kvd, sizeof(float));
  x->vcache = calloc((size_t)L * cfg->max_seq * kvd, sizeof(float));
  x->written = calloc((size_t)L * cfg->max_seq, 1);
  x->hid = calloc((size_t)(L + 1) * cfg->d_model, sizeof(double));
  x->logits = calloc(cfg->vocab, sizeof(double));
  x->sims = calloc(L, sizeof(double));
  if (!x->kcache || !x->vcache || !x->written || !x->hid || !x->logits || !x->sims) return ORC_ENOSPC;
  *out = x;
  return ORC_OK;
}

void orc_destroy(orc_ctx *x) {
  if (!x) return;
  free(x->layers); free(x->river); free(x->kcache); free(x->vcache); free(x->written);
  free(x->hid); free(x->logits); free(x->sims); free(x);
}

/*
 * One token through the model at position x->pos.
 * forced_e < 0: Eq. 1 decides; otherwise the token leaves the backbone after
 * exactly forced_e blocks (forced_e == L: never; 0 only if L_s == 0).
 * want_logits == 0 skips the head (prompt positions other than the last).
 */
static int step(orc_ctx *x, int token, int forced_e, int want_logits, int *out_token, int *out_e) {
  const orc_config *c = &x->c;
  int L = c->n_layers, d = c->d_model, dt = c->dtype;
  if (token < 0 || token >= c->vocab) return ORC_EINVAL;
  if (x->pos >= c->max_seq) return ORC_ENOSPC;
  if (forced_e >= 0 && forced_e != L && (forced_e < c->min_exit_layer || forced_e > L)) return ORC_EINVAL;
  int p = x->pos;
  double *h = x->hid;
  for (int i = 0; i < d; ++i) h[i] = ld(x->tok_emb, (int64_t)token * d + i, dt);
  int exited = (forced_e == 0), e = exited ? 0 : L;
  for (int l = 1; l <= L; ++l) {
    double *hin = x->hid + (int64_t)(l - 1) * d, *hout = x->hid + (int64_t)l * d;
    x->sims[l - 1] = NAN;
    if (!exited) {
      block(x, l - 1, p, 0, hin, hout);
      double s = orc_cosine(hin, hout, d);
      x->sims[l - 1] = s;
      if (l >= c->min_exit_layer && l < L &&
          ((forced_e < 0 && s > (double)c->tau) || forced_e == l)) {
        exited = 1;
        e = l;
      }
    } else {
      if (!x->river[l - 1].m[0].codes) return ORC_EINVAL;
      block(x, l - 1, p, 1, hin, hout);
    }
  }
  x->pos = p + 1;
  if (out_e) *out_e = e;
  if (want_logits) {
    double *xn = malloc(sizeof(double) * d);
    orc_rmsnorm(x->hid + (int64_t)L * d, x->final_norm, dt, d, c->rms_eps, xn);
    matvec(x->lm_head, dt, c->vocab, d, xn, x->logits);
    free(xn);
    int best = 0;
    for (int i = 1; i < c->vocab; ++i)
      if (x->logits[i] > x->logits[best]) best = i; /* strict: lowest index wins ties */
    if (out_token) *out_token = best;
  }
  return ORC_OK;
}

/*
 * Prefill phase ("Inference with Seamless Exit", the list of phases: the prompt is
 * processed by sequence-level exit, every prompt token leaving the backbone at one
 * unified depth).  exit_layer is that depth e_p: every prompt position runs backbone
 * blocks 1..e_p and river twins e_p+1..L, each writing its K/V to the shared slot.
 * e_p = L (or negative) is the full depth.  How e_p is chosen the paper does not say:
 * it is the caller's.  Returns the greedy token after the last prompt position.
 */
int orc_prefill(orc_ctx *x, const int32_t *tokens, int n, int exit_layer, int32_t *out_token) {
  if (!x || !tokens || n < 1) return ORC_EINVAL;
  int ep = exit_layer < 0 ? x->c.n_layers : exit_layer;
  x->pos = 0;
  memset(x->written, 0, (size_t)x->c.n_layers * x->c.max_seq);
  for (int i = 0; i < n; ++i) {
    int tok = 0, e = 0;
    int rc = step(x, tokens[i], ep, i == n - 1, &tok, &e);
    if (rc) return rc;
    if (i == n - 1 && out_token) *out_token = tok;
  }
  return ORC_OK;
}

int orc_decode_step(orc_ctx *x, int32_t token, int32_t forced_e, int32_t *out_token,
                    int32_t *out_e, double *out_sims) {
  if (!x) return ORC_EINVAL;
  int tok = 0, e = 0;
  int rc = step(x, token, forced_e, 1, &tok, &e);
  if (rc) return rc;
  if (out_token) *out_token = tok;
  if (out_e) *out_e = e;
  if (out_sims) memcpy(out_sims, x->sims, sizeof(double) * x->c.n_layers);
  return ORC_OK;
}

/*
 * The pieces of step() on their own, for the batched form of Eq. 1: there the exit decision
 * after block l looks at every sequence of the batch (the minimum of their similarities),
 * so a batch is stepped block by block over one context per sequence (oracle/batch_oracle.py):
 * orc_embed, orc_block for l = 1..L at position orc_pos, orc_head, orc_advance.
 */
int orc_embed(const orc_ctx *x, int token, double *h) {
  if (!x || !h || token < 0 || token >= x->c.vocab) return ORC_EINVAL;
  for (int i = 0; i < x->c.d_model; ++i) h[i] = ld(x->tok_emb, (int64_t)token * x->c.d_model + i, x->c.dtype);
  return ORC_OK;
}

/* logits = W_head RMSNorm(h) g_final (kept in the context), greedy token, lowest index on ties */
int orc_head(orc_ctx *x, const double *h, int32_t *out_token) {
  if (!x || !h) return ORC_EINVAL;
  const orc_config *c = &x->c;
  double *xn = malloc(sizeof(double) * c->d_model);
  orc_rmsnorm(h, x->final_norm, c->dtype, c->d_model, c->rms_eps, xn);
  matvec(x->lm_head, c->dtype, c->vocab, c->d_model, xn, x->logits);
  free(xn);
  int best = 0;
  for (int i = 1; i < c->vocab; ++i)
    if (x->logits[i] > x->logits[best]) best = i;
  if (out_token) *out_token = best;
  return ORC_OK;
}

int orc_advance(orc_ctx *x) {
  if (!x || x->pos >= x->c.max_seq) return ORC_ENOSPC;
  x->pos += 1;
  return ORC_OK;
}

int orc_rewind(orc_ctx *x, int new_len) {
  if (!x || new_len < 0 || new_len > x->pos) return ORC_EINVAL;
  for (int l = 0; l < x->c.n_layers; ++l)
    for (int p = new_len; p < x->pos; ++p) x->written[(int64_t)l * x->c.max_seq + p] = 0;
  x->pos = new_len;
  return ORC_OK;
}

int orc_pos(const orc_ctx *x) { return x ? x->pos : ORC_EINVAL; }
const double *orc_hidden(const orc_ctx *x) { return x->hid; }   /* [L+1][d] */
const double *orc_logits(const orc_ctx *x) { return x->logits; } /* [vocab]  */
const float *orc_kcache(const orc_ctx *x) { return x->kcache; } /* [L][max_seq][kvd] */
const float *orc_vcache(const orc_ctx *x) { return x->vcache; }
const uint8_t *orc_written(const orc_ctx *x) { return x->written; } /* [L][max_seq] */
