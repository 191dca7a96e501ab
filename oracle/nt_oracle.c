/*
 * CPU oracle for the student-Transformer translation path.  TEST INFRASTRUCTURE ONLY:
 * it defines what the GPU library must compute and is used by the tests, the smoke
 * check and the CPU-baseline leg of the benchmark.  It shares no code with the HIP
 * library and is never called by the product path.
 *
 * Plain C, one sentence at a time, no blocking, no fusion, no BLAS.  Weights are the
 * fp16 values of the blob widened exactly to fp32; every activation and every
 * reduction is fp64.
 *
 * What is computed (citations are to the paper, arXiv 2109.08003):
 *   - architecture: deep encoder / one-layer decoder student, single head, FFN removed
 *     (Sec. 1; Sec. 2.2 "Fast Student Models"; Table 2), with the vanilla-Transformer
 *     defaults the paper refers to (Sec. 2.1, Table 1 caption): sinusoidal positions,
 *     sqrt(d) embedding scale, pre-LayerNorm residual blocks with a final LayerNorm
 *     per stack (reading fixed by the benchmark configuration);
 *   - 1/sqrt(d_k) applied to the query, softmax in full precision (Sec. 3.1 "FP16 Inference");
 *   - greedy search with no log-softmax on the output layer (Sec. 3.3 "Graph Optimization",
 *     "Greedy Search"); ties go to the lowest id;
 *   - relative position keys with clipping distance 8 for the teacher shape (Sec. 2.1);
 *   - multi-head attention and ReLU FFN for the ablation / teacher shapes (Table 1, Table 2).
 *
 * Parity pins live in tests/test_oracle_*.py.  Parity unpinned: translation quality
 * (BLEU) - it needs trained weights and test sets that are not available.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t n_enc, n_dec, d_model, n_heads, d_ffn, vocab, max_len, rpr_clip, tie_output, bos_id;
  /* decoder shape where it differs from the encoder's (Table 2, Sec. 5: the submitted students put a base
     encoder in front of a one-head decoder whose FFN is 512 wide or absent):
     dec_n_heads 0 = n_heads;  dec_d_ffn 0 = d_ffn, -1 = no decoder FFN, else the width */
  int32_t dec_n_heads, dec_d_ffn;
  /* 1: every layer normalisation divides by the scaled mean absolute deviation instead of the standard
     deviation (Sec. 3.1 "FP16 Inference": the L1-norm replacement; see ora_layer_norm_l1) */
  int32_t ln_l1;
  /* 1: the output layer is an 8-bit matrix multiplication (Sec. 3.2 "8-bit Matrix Multiplication with Packing",
     Eq. 3-6; see the q8 functions below) */
  int32_t q8_output;
  double ln_eps;
} ora_config;

static int dec_heads(const ora_config *c) { return c->dec_n_heads > 0 ? c->dec_n_heads : c->n_heads; }
static int dec_ffn(const ora_config *c) { return c->dec_d_ffn == 0 ? c->d_ffn : (c->dec_d_ffn < 0 ? 0 : c->dec_d_ffn); }

typedef struct { const float *g, *b; } ln_t;
typedef struct { const float *Wq, *bq, *Wk, *bk, *Wv, *bv, *Wo, *bo, *rk; } attn_t;
typedef struct { const float *W1, *b1, *W2, *b2; } ffn_t;
typedef struct { ln_t ln1; attn_t self; ln_t ln2; ffn_t ffn; } enc_layer;
typedef struct { ln_t ln1; attn_t self; ln_t ln2; attn_t cross; ln_t ln3; ffn_t ffn; } dec_layer;

typedef struct ora_model {
  ora_config c;
  float *w;               /* whole blob widened to fp32 */
  const float *E, *Wout;  /* [V][d] each; Wout == E when tied */
  /* 8-bit output layer: codes [V][d], scale and zero point per vocabulary entry */
  int8_t *q8_w;
  float *q8_scale;
  int32_t *q8_zero;
  enc_layer *enc;
  ln_t enc_final;
  dec_layer *dec;
  ln_t dec_final;
} ora_model;

/* ---- fp16 -> fp32, exact ---- */
float ora_half_to_float(uint16_t h) {
  uint32_t sign = (uint32_t)(h >> 15) << 31, e = (h >> 10) & 31u, m = h & 1023u, bits;
  if (e == 0) {
    if (m == 0) bits = sign;
    else { /* subnormal: value = m * 2^-24 */
      float f = (float)m * 5.9604644775390625e-8f;
      memcpy(&bits, &f, 4); bits |= sign;
    }
  } else if (e == 31) bits = sign | 0x7f800000u | (m << 13);
  else bits = sign | ((e + 112u) << 23) | (m << 13);
  float out; memcpy(&out, &bits, 4); return out;
}

/* ---- closed-form parameter count of the blob (matrices, biases, LayerNorms) ---- */
int64_t ora_param_count(const ora_config *c) {
  int64_t d = c->d_model, V = c->vocab, F = c->d_ffn, dh = d / c->n_heads;
  int64_t Fd = dec_ffn(c), dhd = d / dec_heads(c);
  int64_t attn = 4 * (d * d + d), ln = 2 * d, ffn = F > 0 ? (2 * d * F + F + d + ln) : 0;
  int64_t ffnd = Fd > 0 ? (2 * d * Fd + Fd + d + ln) : 0;
  int64_t rk = c->rpr_clip > 0 ? (2 * c->rpr_clip + 1) * dh : 0;
  int64_t rkd = c->rpr_clip > 0 ? (2 * c->rpr_clip + 1) * dhd : 0;
  int64_t n = V * d * (c->tie_output ? 1 : 2);
  n += c->n_enc * (ln + attn + rk + ffn) + ln;
  n += c->n_dec * (ln + attn + rkd + ln + attn + ffnd) + ln;
  return n;
}

/* number of greedy steps for a source of `len` tokens: ceil(1.2*len)+2 in integers */
int32_t ora_n_steps(int32_t len) { return (6 * len + 4) / 5 + 2; }

/* ---- blob parsing ---- */
static const float *take(const float **p, int64_t n) { const float *r = *p; *p += n; return r; }
static void take_ln(const float **p, int64_t d, ln_t *l) { l->g = take(p, d); l->b = take(p, d); }
static void take_attn(const float **p, int64_t d, int64_t rk, attn_t *a) {
  a->Wq = take(p, d * d); a->bq = take(p, d);
  a->Wk = take(p, d * d); a->bk = take(p, d);
  a->Wv = take(p, d * d); a->bv = take(p, d);
  a->Wo = take(p, d * d); a->bo = take(p, d);
  a->rk = rk ? take(p, rk) : NULL;
}
static void take_ffn(const float **p, int64_t d, int64_t F, ffn_t *f) {
  f->W1 = take(p, d * F); f->b1 = take(p, F); f->W2 = take(p, F * d); f->b2 = take(p, d);
}

void ora_q8_weight_row(const float *w, int32_t d, int8_t *q, float *scale_out, int32_t *zero_out);
static void q8_logits(const ora_model *m, const double *h, double *logits);

ora_model *ora_load(const ora_config *c, const uint16_t *blob, int64_t n_halfs) {
  if (!c || !blob) return NULL;
  if (c->d_model <= 0 || c->n_heads <= 0 || c->d_model % c->n_heads || c->vocab <= 0 ||
      c->n_enc < 0 || c->n_dec < 1 || c->d_ffn < 0 || c->rpr_clip < 0) return NULL;
  if (c->dec_n_heads < 0 || c->d_model % dec_heads(c) || c->dec_d_ffn < -1 || c->ln_l1 < 0 || c->ln_l1 > 1 ||
      c->q8_output < 0 || c->q8_output > 1) return NULL;
  if (n_halfs != ora_param_count(c)) return NULL;
  ora_model *m = (ora_model *)calloc(1, sizeof *m);
  m->c = *c;
  m->w = (float *)malloc(sizeof(float) * (size_t)n_halfs);
  for (int64_t i = 0; i < n_halfs; i++) m->w[i] = ora_half_to_float(blob[i]);
  int64_t d = c->d_model, V = c->vocab, F = c->d_ffn, Fd = dec_ffn(c);
  int64_t rk = c->rpr_clip > 0 ? (2 * c->rpr_clip + 1) * (d / c->n_heads) : 0;
  int64_t rkd = c->rpr_clip > 0 ? (2 * c->rpr_clip + 1) * (d / dec_heads(c)) : 0;
  const float *p = m->w;
  m->E = take(&p, V * d);
  m->Wout = c->tie_output ? m->E : take(&p, V * d);
  m->enc = (enc_layer *)calloc((size_t)(c->n_enc > 0 ? c->n_enc : 1), sizeof(enc_layer));
  m->dec = (dec_layer *)calloc((size_t)c->n_dec, sizeof(dec_layer));
  for (int l = 0; l < c->n_enc; l++) {
    take_ln(&p, d, &m->enc[l].ln1);
    take_attn(&p, d, rk, &m->enc[l].self);
    if (F > 0) { take_ln(&p, d, &m->enc[l].ln2); take_ffn(&p, d, F, &m->enc[l].ffn); }
  }
  take_ln(&p, d, &m->enc_final);
  for (int l = 0; l < c->n_dec; l++) {
    take_ln(&p, d, &m->dec[l].ln1);
    take_attn(&p, d, rkd, &m->dec[l].self);
    take_ln(&p, d, &m->dec[l].ln2);
    take_attn(&p, d, 0, &m->dec[l].cross);
    if (Fd > 0) { take_ln(&p, d, &m->dec[l].ln3); take_ffn(&p, d, Fd, &m->dec[l].ffn); }
  }
  take_ln(&p, d, &m->dec_final);
  if (p - m->w != n_halfs) { free(m->enc); free(m->dec); free(m->w); free(m); return NULL; }
  if (c->q8_output) {
    m->q8_w = (int8_t *)malloc((size_t)(V * d));
    m->q8_scale = (float *)malloc(sizeof(float) * (size_t)V);
    m->q8_zero = (int32_t *)malloc(sizeof(int32_t) * (size_t)V);
    for (int64_t v = 0; v < V; v++)
      ora_q8_weight_row(m->Wout + v * d, (int32_t)d, m->q8_w + v * d, &m->q8_scale[v], &m->q8_zero[v]);
  }
  return m;
}

void ora_free(ora_model *m) {
  if (!m) return;
  free(m->q8_w); free(m->q8_scale); free(m->q8_zero);
  free(m->enc); free(m->dec); free(m->w); free(m);
}

/* ---- primitives (exported so that tests can pin each against a library routine) ---- */

/* sinusoidal position row: out[2k] = sin(pos / 10000^(2k/d)), out[2k+1] = cos(same) */
void ora_pe(int32_t pos, int32_t d, double *out) {
  for (int k = 0; 2 * k < d; k++) {
    double ang = (double)pos / pow(10000.0, (2.0 * k) / (double)d);
    out[2 * k] = sin(ang);
    if (2 * k + 1 < d) out[2 * k + 1] = cos(ang);
  }
}

/* y = g * (x - mean) / sqrt(biased_var + eps) + b */
void ora_layer_norm(const double *x, const float *g, const float *b, int32_t d, double eps, double *y) {
  double mean = 0.0, var = 0.0;
  for (int i = 0; i < d; i++) mean += x[i];
  mean /= d;
  for (int i = 0; i < d; i++) var += (x[i] - mean) * (x[i] - mean);
  var /= d;
  double r = 1.0 / sqrt(var + eps);
  for (int i = 0; i < d; i++) y[i] = (double)g[i] * ((x[i] - mean) * r) + (double)b[i];
}

/* L1-norm layer normalisation (Sec. 3.1 "FP16 Inference" names the replacement and cites Lin et al., IJCAI 2020,
   without printing a formula; this is the reading taken here): the standard deviation is replaced by the mean
   absolute deviation scaled by sqrt(pi/2), the factor that makes the two agree for normally distributed
   activations:   y = g * (x - mean) / (sqrt(pi/2) * mean|x - mean| + eps) + b */
void ora_layer_norm_l1(const double *x, const float *g, const float *b, int32_t d, double eps, double *y) {
  double mean = 0.0, mad = 0.0;
  for (int i = 0; i < d; i++) mean += x[i];
  mean /= d;
  for (int i = 0; i < d; i++) mad += fabs(x[i] - mean);
  mad /= d;
  double r = 1.0 / (sqrt(acos(-1.0) / 2.0) * mad + eps);
  for (int i = 0; i < d; i++) y[i] = (double)g[i] * ((x[i] - mean) * r) + (double)b[i];
}

/* the model's layer normalisation: vanilla or L1-norm, as configured */
static void norm(const ora_config *c, const double *x, const float *g, const float *b, double *y) {
  if (c->ln_l1) ora_layer_norm_l1(x, g, b, c->d_model, c->ln_eps, y);
  else ora_layer_norm(x, g, b, c->d_model, c->ln_eps, y);
}

/* y[n] = b[n] + sum_k x[k] W[k][n],  W stored [n_in][n_out] */
void ora_linear(const double *x, const float *W, const float *b, int32_t n_in, int32_t n_out, double *y) {
  for (int n = 0; n < n_out; n++) y[n] = b ? (double)b[n] : 0.0;
  for (int k = 0; k < n_in; k++) {
    const float *row = W + (int64_t)k * n_out;
    double xk = x[k];
    for (int n = 0; n < n_out; n++) y[n] += xk * (double)row[n];
  }
}

/* in-place softmax over s[0..n); entries equal to -INFINITY get probability exactly 0 */
void ora_softmax(double *s, int32_t n) {
  double mx = -INFINITY, sum = 0.0;
  for (int j = 0; j < n; j++) if (s[j] > mx) mx = s[j];
  for (int j = 0; j < n; j++) { s[j] = (s[j] == -INFINITY) ? 0.0 : exp(s[j] - mx); sum += s[j]; }
  for (int j = 0; j < n; j++) s[j] /= sum;
}

/*
 * One query against n_keys keys, all heads.  q is already scaled by 1/sqrt(d_h).
 * Key j sits at position j; the query sits at position qpos.  With relative position
 * keys (rk != NULL, clip c): score_j += q_h . rk[clamp(j - qpos, -c, c) + c].
 * K, V: [n_keys][d]; out c: [d] (heads concatenated).  probs (optional): [heads][n_keys].
 */
void ora_attend(const double *q, const double *K, const double *V, int32_t n_keys, int32_t d,
                int32_t heads, const float *rk, int32_t clip, int32_t qpos, double *c, double *probs) {
  int dh = d / heads;
  double *s = (double *)malloc(sizeof(double) * (size_t)n_keys);
  for (int h = 0; h < heads; h++) {
    const double *qh = q + h * dh;
    for (int j = 0; j < n_keys; j++) {
      const double *kj = K + (int64_t)j * d + h * dh;
      double acc = 0.0;
      for (int e = 0; e < dh; e++) acc += qh[e] * kj[e];
      if (rk) {
        int off = j - qpos;
        if (off < -clip) off = -clip;
        if (off > clip) off = clip;
        const float *r = rk + (int64_t)(off + clip) * dh;
        for (int e = 0; e < dh; e++) acc += qh[e] * (double)r[e];
      }
      s[j] = acc;
    }
    ora_softmax(s, n_keys);
    if (probs) memcpy(probs + (int64_t)h * n_keys, s, sizeof(double) * (size_t)n_keys);
    for (int e = 0; e < dh; e++) c[h * dh + e] = 0.0;
    for (int j = 0; j < n_keys; j++) {
      const double *vj = V + (int64_t)j * d + h * dh;
      for (int e = 0; e < dh; e++) c[h * dh + e] += s[j] * vj[e];
    }
  }
  free(s);
}

/* ---- model pieces ---- */

static void embed(const ora_model *m, int32_t id, int32_t pos, double *x) {
  int d = m->c.d_model;
  double sc = sqrt((double)d);
  ora_pe(pos, d, x);
  for (int i = 0; i < d; i++) x[i] += sc * (double)m->E[(int64_t)id * d + i];
}

/* x += relu(LN(x) W1 + b1) W2 + b2 */
static void ffn_block(const ora_model *m, const ln_t *ln, const ffn_t *f, int F, double *x) {
  int d = m->c.d_model;
  double *a = (double *)malloc(sizeof(double) * (size_t)(2 * d + F)), *u = a + d, *o = u + F;
  norm(&m->c, x, ln->g, ln->b, a);
  ora_linear(a, f->W1, f->b1, d, F, u);
  for (int i = 0; i < F; i++) if (u[i] < 0.0) u[i] = 0.0;
  ora_linear(u, f->W2, f->b2, F, d, o);
  for (int i = 0; i < d; i++) x[i] += o[i];
  free(a);
}

/* encoder over one sentence; x: [len][d] in/out scratch, enc: [len][d] result */
static int encode(const ora_model *m, const int32_t *src, int32_t len, double *enc) {
  const ora_config *c = &m->c;
  int d = c->d_model, H = c->n_heads;
  double qs = 1.0 / sqrt((double)(d / H));
  for (int i = 0; i < len; i++) if (src[i] < 0 || src[i] >= c->vocab) return -1;
  size_t n = (size_t)len * d;
  double *x = (double *)malloc(sizeof(double) * n * 5);
  double *q = x + n, *k = q + n, *v = k + n, *a = v + n;
  double *ctx = (double *)malloc(sizeof(double) * 2 * (size_t)d), *o = ctx + d;
  for (int i = 0; i < len; i++) embed(m, src[i], i, x + (size_t)i * d);
  for (int l = 0; l < c->n_enc; l++) {
    const enc_layer *L = &m->enc[l];
    for (int i = 0; i < len; i++) {
      double *ai = a + (size_t)i * d;
      norm(c, x + (size_t)i * d, L->ln1.g, L->ln1.b, ai);
      ora_linear(ai, L->self.Wq, L->self.bq, d, d, q + (size_t)i * d);
      ora_linear(ai, L->self.Wk, L->self.bk, d, d, k + (size_t)i * d);
      ora_linear(ai, L->self.Wv, L->self.bv, d, d, v + (size_t)i * d);
      for (int e = 0; e < d; e++) q[(size_t)i * d + e] *= qs;
    }
    for (int i = 0; i < len; i++) {
      ora_attend(q + (size_t)i * d, k, v, len, d, H, L->self.rk, c->rpr_clip, i, ctx, NULL);
      ora_linear(ctx, L->self.Wo, L->self.bo, d, d, o);
      for (int e = 0; e < d; e++) x[(size_t)i * d + e] += o[e];
    }
    if (c->d_ffn > 0)
      for (int i = 0; i < len; i++) ffn_block(m, &L->ln2, &L->ffn, c->d_ffn, x + (size_t)i * d);
  }
  for (int i = 0; i < len; i++)
    norm(c, x + (size_t)i * d, m->enc_final.g, m->enc_final.b, enc + (size_t)i * d);
  free(ctx); free(x);
  return 0;
}

/* decoder state for one sentence: cross keys/values per layer, growing self caches */
typedef struct {
  int32_t len, cap;
  double *ck, *cv;  /* [n_dec][len][d] */
  double *sk, *sv;  /* [n_dec][cap][d] */
} dec_state;

static dec_state *dec_begin(const ora_model *m, const double *enc, int32_t len, int32_t cap) {
  int d = m->c.d_model, Ld = m->c.n_dec;
  dec_state *s = (dec_state *)calloc(1, sizeof *s);
  s->len = len; s->cap = cap;
  s->ck = (double *)malloc(sizeof(double) * 2 * (size_t)Ld * len * d);
  s->cv = s->ck + (size_t)Ld * len * d;
  s->sk = (double *)malloc(sizeof(double) * 2 * (size_t)Ld * cap * d);
  s->sv = s->sk + (size_t)Ld * cap * d;
  for (int l = 0; l < Ld; l++)
    for (int j = 0; j < len; j++) {
      const attn_t *A = &m->dec[l].cross;
      ora_linear(enc + (size_t)j * d, A->Wk, A->bk, d, d, s->ck + ((size_t)l * len + j) * d);
      ora_linear(enc + (size_t)j * d, A->Wv, A->bv, d, d, s->cv + ((size_t)l * len + j) * d);
    }
  return s;
}
static void dec_end(dec_state *s) { free(s->ck); free(s->sk); free(s); }

/* one incremental decoder step at position t with previous token y_prev -> logits[V] */
static void dec_step(const ora_model *m, dec_state *s, int32_t y_prev, int32_t t, double *logits) {
  const ora_config *c = &m->c;
  int d = c->d_model, H = dec_heads(c), V = c->vocab;
  double qs = 1.0 / sqrt((double)(d / H));
  double *z = (double *)malloc(sizeof(double) * 5 * (size_t)d);
  double *a = z + d, *q = a + d, *ctx = q + d, *o = ctx + d;
  embed(m, y_prev, t, z);
  for (int l = 0; l < c->n_dec; l++) {
    const dec_layer *L = &m->dec[l];
    double *sk = s->sk + (size_t)l * s->cap * d, *sv = s->sv + (size_t)l * s->cap * d;
    /* causal self-attention over positions 0..t; earlier keys/values are the cached ones */
    norm(c, z, L->ln1.g, L->ln1.b, a);
    ora_linear(a, L->self.Wq, L->self.bq, d, d, q);
    ora_linear(a, L->self.Wk, L->self.bk, d, d, sk + (size_t)t * d);
    ora_linear(a, L->self.Wv, L->self.bv, d, d, sv + (size_t)t * d);
    for (int e = 0; e < d; e++) q[e] *= qs;
    ora_attend(q, sk, sv, t + 1, d, H, L->self.rk, c->rpr_clip, t, ctx, NULL);
    ora_linear(ctx, L->self.Wo, L->self.bo, d, d, o);
    for (int e = 0; e < d; e++) z[e] += o[e];
    /* cross-attention over the encoder output (no relative positions) */
    norm(c, z, L->ln2.g, L->ln2.b, a);
    ora_linear(a, L->cross.Wq, L->cross.bq, d, d, q);
    for (int e = 0; e < d; e++) q[e] *= qs;
    ora_attend(q, s->ck + (size_t)l * s->len * d, s->cv + (size_t)l * s->len * d, s->len, d, H,
               NULL, 0, 0, ctx, NULL);
    ora_linear(ctx, L->cross.Wo, L->cross.bo, d, d, o);
    for (int e = 0; e < d; e++) z[e] += o[e];
    if (dec_ffn(c) > 0) ffn_block(m, &L->ln3, &L->ffn, dec_ffn(c), z);
  }
  norm(c, z, m->dec_final.g, m->dec_final.b, a);
  /* output layer: plain logits, no bias, no log-softmax */
  if (m->q8_w) q8_logits(m, a, logits);
  else for (int v = 0; v < V; v++) {
    const float *w = m->Wout + (int64_t)v * d;
    double acc = 0.0;
    for (int e = 0; e < d; e++) acc += a[e] * (double)w[e];
    logits[v] = acc;
  }
  free(z);
}

/* ---- 8-bit output layer (Sec. 3.2 "8-bit Matrix Multiplication with Packing") ----------------------------
 * The paper quantises every column of a weight matrix on its own (Eq. 3, 4) and the input matrix with one scale
 * and zero point (Eq. 5, 6).  Readings taken here:
 *  - a column of the output layer's matrix is one vocabulary entry v (the d weights that produce its logit);
 *  - Eq. 4 and Eq. 6 as printed divide the whole bracket by the scale, which maps neither end of the range onto
 *    an end of the 8-bit range; they are read as  zero = 127 - (mean + 7 sd) / scale  and
 *    zero = 255 - x_max / scale, which send mean + 7 sd to 127 and x_max to 255 (and so mean - 7 sd to -128
 *    and x_min to 0); zero points are rounded to integers and, like the codes, kept inside the 8-bit range
 *    (the convention of the FBGEMM library the paper uses: a zero point is itself a code; this only matters
 *    for a column or row whose values all lie far to one side of zero); codes are round-to-nearest-even, clamped;
 *  - the input is quantised per row (one decoder state) instead of per matrix, so that a sentence's result does
 *    not depend on its batch mates; weights are signed 8-bit codes, activations unsigned 8-bit codes;
 *  - weight statistics and codes are computed in double, in index order; Eq. 5, 6 state no precision, and a code
 *    is an integer decided by floating-point arithmetic, so this leg is specified to fp32, one rounding per
 *    operation in the order written here, which lets any implementation be compared with it bit for bit:
 *        a_scale = (max - min) / 255      a_zero = rint(255 - max / a_scale)      u_k = rint(h_k / a_scale + a_zero)
 *    (pinned against the same equations evaluated in double: codes and zero point within one step, and on every
 *    row that straddles zero the zero point needs no clamping);
 *  - logit[v] = a_scale * (b_scale[v] * float(I_v)),  I_v = sum_k (u_k - a_zero) (q_vk - zero_v)  exactly in
 *    integers; the arg-max is taken on t_v = b_scale[v] * float(I_v) in fp32 (a_scale > 0 is common to the row).
 */
/* (built with -std=c11: gcc then contracts no multiply-add, so every operation below rounds once) */

/* Eq. 3, 4 for one vocabulary entry: w[d] -> codes q[d], scale, zero point */
void ora_q8_weight_row(const float *w, int32_t d, int8_t *q, float *scale_out, int32_t *zero_out) {
  double mean = 0.0, var = 0.0;
  for (int k = 0; k < d; k++) mean += (double)w[k];
  mean /= (double)d;
  for (int k = 0; k < d; k++) {
    double c = (double)w[k] - mean;
    var += c * c;
  }
  var /= (double)d;
  double sd = sqrt(var);
  double scale = sd > 0.0 ? 14.0 * sd / 255.0 : 1.0;
  double zero = rint(127.0 - (mean + 7.0 * sd) / scale);
  zero = zero < -128.0 ? -128.0 : (zero > 127.0 ? 127.0 : zero); /* a zero point is a code of the same 8 bits */
  for (int k = 0; k < d; k++) {
    double c = rint((double)w[k] / scale + zero);
    q[k] = (int8_t)(c < -128.0 ? -128.0 : (c > 127.0 ? 127.0 : c));
  }
  *scale_out = (float)scale;
  *zero_out = (int32_t)zero;
}

/* Eq. 5, 6 for one row of activations, in fp32: h[d] -> codes u[d] in [0, 255], scale, zero point */
void ora_q8_activation_row(const float *h, int32_t d, uint8_t *u, float *scale_out, int32_t *zero_out) {
  float mn = h[0], mx = h[0];
  for (int k = 1; k < d; k++) {
    mn = h[k] < mn ? h[k] : mn;
    mx = h[k] > mx ? h[k] : mx;
  }
  float range = mx - mn;
  float scale = range > 0.0f ? range / 255.0f : 1.0f;
  float ratio = mx / scale;
  float zero = rintf(255.0f - ratio);
  zero = zero < 0.0f ? 0.0f : (zero > 255.0f ? 255.0f : zero);
  for (int k = 0; k < d; k++) {
    float c = h[k] / scale;
    c = rintf(c + zero);
    u[k] = (uint8_t)(c < 0.0f ? 0.0f : (c > 255.0f ? 255.0f : c));
  }
  *scale_out = scale;
  *zero_out = (int32_t)zero;
}

/* logits[V] of the 8-bit output layer for one decoder state h[d] (given in double, rounded to fp32 first) */
static void q8_logits(const ora_model *m, const double *h, double *logits) {
  int d = m->c.d_model, V = m->c.vocab;
  float *hf = (float *)malloc(sizeof(float) * (size_t)d);
  uint8_t *u = (uint8_t *)malloc((size_t)d);
  for (int k = 0; k < d; k++) hf[k] = (float)h[k];
  float a_scale;
  int32_t a_zero;
  ora_q8_activation_row(hf, d, u, &a_scale, &a_zero);
  for (int v = 0; v < V; v++) {
    const int8_t *q = m->q8_w + (int64_t)v * d;
    int64_t I = 0;
    for (int k = 0; k < d; k++) I += (int64_t)((int32_t)u[k] - a_zero) * (int64_t)((int32_t)q[k] - m->q8_zero[v]);
    float t = m->q8_scale[v] * (float)I;
    logits[v] = (double)a_scale * (double)t; /* exact in double: the order of the t_v is kept */
  }
  free(u); free(hf);
}

/* the same for a caller's fp32 rows (tests): h [R][d] -> logits [R][V] as fp32 = a_scale * t_v rounded once */
int ora_q8_output_layer(const ora_model *m, const float *h, int32_t R, float *logits, int32_t *argmax) {
  if (!m || !m->q8_w) return -1;
  int d = m->c.d_model, V = m->c.vocab;
  double *hd = (double *)malloc(sizeof(double) * (size_t)d), *lg = (double *)malloc(sizeof(double) * (size_t)V);
  for (int r = 0; r < R; r++) {
    for (int k = 0; k < d; k++) hd[k] = (double)h[(int64_t)r * d + k];
    q8_logits(m, hd, lg);
    int best = 0;
    for (int v = 1; v < V; v++) if (lg[v] > lg[best]) best = v;
    if (argmax) argmax[r] = best;
    if (logits) for (int v = 0; v < V; v++) logits[(int64_t)r * V + v] = (float)lg[v];
  }
  free(lg); free(hd);
  return 0;
}

/* the stored codes of one vocabulary entry (tests) */
int ora_q8_weights(const ora_model *m, int32_t v, int8_t *q, float *scale, int32_t *zero) {
  if (!m || !m->q8_w || v < 0 || v >= m->c.vocab) return -1;
  memcpy(q, m->q8_w + (int64_t)v * m->c.d_model, (size_t)m->c.d_model);
  *scale = m->q8_scale[v];
  *zero = m->q8_zero[v];
  return 0;
}

/* ---- public calls ---- */

/* enc_out: [len][d] fp64.  Returns 0, or -1 for an id outside [0,V) / bad length. */
int ora_encode(const ora_model *m, const int32_t *src, int32_t len, double *enc_out) {
  if (!m || len < 1 || len > m->c.max_len) return -1;
  return encode(m, src, len, enc_out);
}

/*
 * Greedy search from BOS (Sec. 3.3 "Greedy Search"): at every step the token with the largest logit, lowest id on
 * ties.  eos_id < 0: exactly n_steps steps, EOS an ordinary token (the benchmark's fixed-length rule).
 * eos_id >= 0: the sentence ends with the first EOS, which is stored, or after n_steps tokens, whichever comes
 * first.  out: [n_steps]; margin (optional): [n_steps] top-1 minus top-2 logit at each step taken.
 * Returns the number of tokens stored, or a negative error.
 */
static int greedy_search(const ora_model *m, const int32_t *src, int32_t len, int32_t n_steps, int32_t eos_id,
                         int32_t *out, double *margin) {
  if (!m || len < 1 || len > m->c.max_len || n_steps < 0 || n_steps > m->c.max_len) return -1;
  int d = m->c.d_model, V = m->c.vocab;
  double *enc = (double *)malloc(sizeof(double) * (size_t)len * d);
  if (encode(m, src, len, enc)) { free(enc); return -1; }
  dec_state *s = dec_begin(m, enc, len, n_steps > 0 ? n_steps : 1);
  double *logits = (double *)malloc(sizeof(double) * (size_t)V);
  int32_t y = m->c.bos_id;
  int rc = 0, t = 0;
  while (t < n_steps) {
    dec_step(m, s, y, t, logits);
    int best = 0;
    double second = -INFINITY;
    if (logits[0] != logits[0]) rc = -2; /* NaN must never appear on valid input */
    for (int v = 1; v < V; v++) {
      if (logits[v] != logits[v]) rc = -2;
      if (logits[v] > logits[best]) { second = logits[best]; best = v; }
      else if (logits[v] > second) second = logits[v];
    }
    out[t] = y = best;
    if (margin) margin[t] = logits[best] - second;
    t++;
    if (eos_id >= 0 && y == eos_id) break;
  }
  free(logits); dec_end(s); free(enc);
  return rc ? rc : t;
}

int ora_greedy(const ora_model *m, const int32_t *src, int32_t len, int32_t n_steps, int32_t *out,
               double *margin) {
  int n = greedy_search(m, src, len, n_steps, -1, out, margin);
  return n < 0 ? n : 0;
}

/* EOS-terminated greedy search; returns the number of tokens stored (the last one is EOS unless the cap cut it) */
int ora_greedy_eos(const ora_model *m, const int32_t *src, int32_t len, int32_t max_steps, int32_t eos_id,
                   int32_t *out, double *margin) {
  if (!m || eos_id < 0 || eos_id >= m->c.vocab) return -1;
  return greedy_search(m, src, len, max_steps, eos_id, out, margin);
}

/* logits[t] for t < T when the decoder is fed tgt_in[0..T) (tgt_in[0] is normally BOS) */
int ora_teacher_forced(const ora_model *m, const int32_t *src, int32_t len, const int32_t *tgt_in,
                       int32_t T, double *logits) {
  if (!m || len < 1 || len > m->c.max_len || T < 1 || T > m->c.max_len) return -1;
  for (int t = 0; t < T; t++) if (tgt_in[t] < 0 || tgt_in[t] >= m->c.vocab) return -1;
  int d = m->c.d_model, V = m->c.vocab;
  double *enc = (double *)malloc(sizeof(double) * (size_t)len * d);
  if (encode(m, src, len, enc)) { free(enc); return -1; }
  dec_state *s = dec_begin(m, enc, len, T);
  for (int t = 0; t < T; t++) dec_step(m, s, tgt_in[t], t, logits + (size_t)t * V);
  dec_end(s); free(enc);
  return 0;
}

/*
 * Translate N sentences (tokens concatenated, offsets[N+1]); sentence i gets
 * ora_n_steps(len_i) output tokens at out[out_offsets[i]..out_offsets[i+1]).
 * out_offsets is written here.  Sentences of length 0 produce nothing.  Parallel over
 * sentences only.  Returns the number of threads used, or a negative error.
 */
static int translate(const ora_model *m, const int32_t *tokens, const int64_t *offsets, int64_t N, int32_t eos_id,
                     int32_t pad_id, int32_t *out, int64_t *out_offsets, int32_t *out_len, int32_t n_threads) {
  if (!m) return -1;
  out_offsets[0] = 0;
  for (int64_t i = 0; i < N; i++) {
    int64_t len = offsets[i + 1] - offsets[i];
    if (len < 0 || len > m->c.max_len) return -1;
    out_offsets[i + 1] = out_offsets[i] + (len > 0 ? ora_n_steps((int32_t)len) : 0);
  }
  int used = 1, err = 0;
#ifdef _OPENMP
  if (n_threads > 0) omp_set_num_threads(n_threads);
  used = omp_get_max_threads();
#endif
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t i = 0; i < N; i++) {
    int32_t len = (int32_t)(offsets[i + 1] - offsets[i]);
    if (len == 0) continue;
    int n = greedy_search(m, tokens + offsets[i], len, ora_n_steps(len), eos_id, out + out_offsets[i], NULL);
    if (n < 0) {
#pragma omp atomic write
      err = 1;
    } else if (out_len) {
      out_len[i] = n;
      for (int64_t k = out_offsets[i] + n; k < out_offsets[i + 1]; k++) out[k] = pad_id;
    }
  }
  return err ? -2 : used;
}

int ora_translate(const ora_model *m, const int32_t *tokens, const int64_t *offsets, int64_t N,
                  int32_t *out, int64_t *out_offsets, int32_t n_threads) {
  return translate(m, tokens, offsets, N, -1, 0, out, out_offsets, NULL, n_threads);
}

/*
 * The same with EOS-terminated greedy search: sentence i keeps its ora_n_steps(len_i) output slots, out_len[i]
 * of them hold its tokens (ending with EOS unless the cap cut it) and the rest hold pad_id.  A sentence of
 * length 0 gets out_len 0.
 */
int ora_translate_eos(const ora_model *m, const int32_t *tokens, const int64_t *offsets, int64_t N, int32_t eos_id,
                      int32_t pad_id, int32_t *out, int64_t *out_offsets, int32_t *out_len, int32_t n_threads) {
  if (!m || !out_len || eos_id < 0 || eos_id >= m->c.vocab || pad_id < 0 || pad_id >= m->c.vocab) return -1;
  for (int64_t i = 0; i < N; i++) out_len[i] = 0;
  return translate(m, tokens, offsets, N, eos_id, pad_id, out, out_offsets, out_len, n_threads);
}
