/*
 * TEST INFRASTRUCTURE -- CPU oracle for one LLM decode step.
 *
 * Plain, slow, loop-per-definition implementation of the decoder operators that the task-graph
 * mega-kernel executes (the paper names these operators -- Section 4 Fig. 4 caption, Section 6.5
 * "operator decomposition" -- but defines none of them numerically; each function below is the
 * standard textbook definition, and every such reading is listed in the design notes).
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this file.  It shares
 * no code with the GPU library.
 *
 * `real` is float by default (the precision the target states for the oracle) and double when
 * built with -DORC_F64 (used to bound the fp32 oracle's own rounding error).
 *
 * Conventions: weights are bf16 bit patterns (uint16_t), row-major [out][in]; activations are
 * `real`; the KV cache is bf16 [n_kv][max_seq][d] per sequence; no blocking, no reordering:
 * every sum runs in increasing index order.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>

#ifdef ORC_F64
typedef double real;
#define R_EXP exp
#define R_SQRT sqrt
#else
typedef float real;
#define R_EXP expf
#define R_SQRT sqrtf
#endif

int orc_real_bytes(void) { return (int)sizeof(real); }

#ifdef _OPENMP
#include <omp.h>
int orc_threads(void) { return omp_get_max_threads(); }
#else
int orc_threads(void) { return 1; }
#endif

/* bf16 -> fp32 is exact: the 16 bits become the high half of the fp32 pattern. */
static inline float bf16_to_f32(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

/* fp32 -> bf16, round to nearest, ties to even; NaN stays NaN (quiet), inf stays inf. */
static inline uint16_t f32_to_bf16_rne(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) return (uint16_t)((u >> 16) | 0x0040u);
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7FFFu + lsb;
  return (uint16_t)(u >> 16);
}

float orc_bf16_to_f32(uint16_t b) { return bf16_to_f32(b); }
uint16_t orc_f32_to_bf16(float f) { return f32_to_bf16_rne(f); }

/* x = E[token]  (embedding lookup, widened exactly). */
void orc_embed(const uint16_t *E, int hidden, int token, real *x) {
  for (int i = 0; i < hidden; ++i) x[i] = (real)bf16_to_f32(E[(size_t)token * hidden + i]);
}

/* RMSNorm: y_i = x_i * (1 / sqrt(mean_j x_j^2 + eps)) * g_i. */
void orc_rmsnorm(const real *x, const uint16_t *g, int n, float eps, real *y) {
  real ss = 0;
  for (int j = 0; j < n; ++j) ss += x[j] * x[j];
  real inv = (real)1 / R_SQRT(ss / (real)n + (real)eps);
  for (int i = 0; i < n; ++i) y[i] = x[i] * inv * (real)bf16_to_f32(g[i]);
}

/* Linear: y_r = sum_j W[r][j] * x_j, j increasing, no bias.  Rows are independent, so the
 * OpenMP split over rows does not change any row's summation order. */
void orc_linear(const uint16_t *W, int out, int in, const real *x, real *y) {
#pragma omp parallel for schedule(static)
  for (int r = 0; r < out; ++r) {
    const uint16_t *w = W + (size_t)r * in;
    real acc = 0;
    for (int j = 0; j < in; ++j) acc += (real)bf16_to_f32(w[j]) * x[j];
    y[r] = acc;
  }
}

/* Rotary embedding, half-split pairing (i, i + d/2), on one head vector in place.
 * f_i = theta^(-2i/d); angle = pos * f_i evaluated in double, then cos/sin rounded to `real`. */
void orc_rope(real *u, int d, int pos, double theta) {
  int h = d / 2;
  for (int i = 0; i < h; ++i) {
    double f = pow(theta, -2.0 * (double)i / (double)d);
    double a = (double)pos * f;
    real c = (real)cos(a), s = (real)sin(a);
    real u0 = u[i], u1 = u[i + h];
    u[i] = u0 * c - u1 * s;
    u[i + h] = u1 * c + u0 * s;
  }
}

/* Store one head vector into a cache row as bf16 (round to nearest even). */
void orc_kv_store(uint16_t *row, const real *u, int d) {
  for (int i = 0; i < d; ++i) row[i] = f32_to_bf16_rne((float)u[i]);
}

/* Decode attention for one query head over cache rows 0..n_pos-1 of its KV head:
 *   s_t = (q . K_t) / sqrt(d);  P = softmax(s) with max subtraction;  o = sum_t P_t V_t.
 * K, V point at row 0 of that KV head ([max_seq][d], contiguous rows). */
void orc_attention_head(const real *q, const uint16_t *K, const uint16_t *V, int n_pos, int d,
                        real *scratch /* n_pos */, real *o) {
  real inv_sqrt_d = (real)1 / R_SQRT((real)d);
  real m = -INFINITY;
  for (int t = 0; t < n_pos; ++t) {
    real acc = 0;
    for (int i = 0; i < d; ++i) acc += q[i] * (real)bf16_to_f32(K[(size_t)t * d + i]);
    scratch[t] = acc * inv_sqrt_d;
    if (scratch[t] > m) m = scratch[t];
  }
  real l = 0;
  for (int t = 0; t < n_pos; ++t) {
    scratch[t] = R_EXP(scratch[t] - m);
    l += scratch[t];
  }
  for (int i = 0; i < d; ++i) {
    real acc = 0;
    for (int t = 0; t < n_pos; ++t) acc += scratch[t] * (real)bf16_to_f32(V[(size_t)t * d + i]);
    o[i] = acc / l;
  }
}

/* SwiGLU activation: gu = [gate(0..F) | up(F..2F)];  h_i = gate_i / (1 + exp(-gate_i)) * up_i. */
void orc_swiglu(const real *gu, int F, real *h) {
  for (int i = 0; i < F; ++i) {
    real g = gu[i];
    h[i] = g / ((real)1 + R_EXP(-g)) * gu[F + i];
  }
}

void orc_add(const real *a, const real *b, int n, real *y) {
  for (int i = 0; i < n; ++i) y[i] = a[i] + b[i];
}

/* Greedy token: arg max, lowest index on ties. */
int orc_argmax(const real *x, int n) {
  int best = 0;
  for (int i = 1; i < n; ++i)
    if (x[i] > x[best]) best = i;
  return best;
}

/* MoE router: p = softmax(logits) over all E experts; pick the k largest (ties -> lower index);
 * renormalise the k weights to sum to one.  sel[] comes back in ascending expert index. */
void orc_router_topk(const real *logits, int E, int k, int *sel, real *w) {
  real m = -INFINITY;
  for (int e = 0; e < E; ++e)
    if (logits[e] > m) m = logits[e];
  real p[4096];
  real l = 0;
  for (int e = 0; e < E; ++e) {
    p[e] = R_EXP(logits[e] - m);
    l += p[e];
  }
  for (int e = 0; e < E; ++e) p[e] /= l;
  char taken[4096];
  for (int e = 0; e < E; ++e) taken[e] = 0;
  for (int j = 0; j < k; ++j) {
    int best = -1;
    for (int e = 0; e < E; ++e)
      if (!taken[e] && (best < 0 || p[e] > p[best])) best = e;
    taken[best] = 1;
  }
  real s = 0;
  int n = 0;
  for (int e = 0; e < E; ++e)
    if (taken[e]) {
      sel[n] = e;
      w[n] = p[e];
      s += p[e];
      ++n;
    }
  for (int j = 0; j < k; ++j) w[j] /= s;
}

/* ------------------------------------------------------------------------------------------
 * One decoder layer for one sequence, composed only of the functions above, in the operator
 * order  attn_norm, qkv_proj, (per-head q/k RMSNorm,) rope + kv append, attention, o_proj, residual, mlp_norm,
 * gate_up_proj, swiglu, down_proj, residual  (or the MoE block in place of the dense MLP).
 * pos = number of rows already cached; the new K/V row is written at `pos` and attention reads
 * rows 0..pos of the ROUNDED cache.  kc/vc: this sequence's cache [n_kv][max_seq][d].
 * work: caller scratch of at least  4*hidden + 2*qkv_rows + 3*ffn_like + max_seq  reals.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int hidden, n_q, n_kv, d, ffn, max_seq;
  float eps;
  double theta;
  int n_experts, top_k, expert_ffn;
  int qk_norm; /* 1: RMSNorm over head_dim of every q and k head (gains q_norm / k_norm) before RoPE */
} orc_layer_cfg;

typedef struct {
  const uint16_t *attn_norm, *wqkv, *wo, *mlp_norm, *wgu, *wd;
  const uint16_t *router, *exp_wgu, *exp_wd;
  const uint16_t *q_norm, *k_norm;
} orc_layer_w;

/* The two places of a layer where floating point decides something discrete -- the bf16 rounding
 * of the appended K/V row and the top-k expert set -- can be held fixed by the caller (`held`):
 * two correct implementations that sum in different orders may round a value that sits on a bf16
 * rounding boundary either way, or order two near-equal router outputs either way, and everything
 * downstream of such a decision then legitimately differs.  A comparison hands the decisions of
 * the implementation under test to the oracle, checks that each is a valid one against what the
 * oracle reports here (the unrounded rows; the router outputs), and compares the rest tightly.
 * All members may be NULL; with held == NULL the oracle decides everything itself. */
typedef struct {
  const uint16_t *k_rows, *v_rows; /* in: [n_kv][d] bf16 rows to append instead of the oracle's own */
  const int *experts;              /* in: top_k experts (ascending) to use instead of the oracle's own */
  real *k_exact, *v_exact;         /* out: [n_kv][d] the oracle's rows before rounding */
} orc_held;

void orc_layer(const orc_layer_cfg *c, const orc_layer_w *w, uint16_t *kc, uint16_t *vc, int pos,
               real *x /* in: layer input, out: layer output */, real *work,
               int *moe_sel /* top_k, may be NULL */,
               real *moe_logits /* n_experts router outputs, may be NULL */,
               const orc_held *held /* may be NULL */) {
  int H = c->hidden, d = c->d, nq = c->n_q, nkv = c->n_kv;
  int qkv_rows = (nq + 2 * nkv) * d;
  real *xn = work;
  real *qkv = xn + H;
  real *o = qkv + qkv_rows;
  real *a = o + nq * d;
  real *x1 = a + H;
  real *scr = x1 + H;
  real *rest = scr + c->max_seq;

  orc_rmsnorm(x, w->attn_norm, H, c->eps, xn);
  orc_linear(w->wqkv, qkv_rows, H, xn, qkv);
  real *q = qkv, *k = qkv + nq * d, *v = k + nkv * d;
  if (c->qk_norm) { /* element-wise, so in place is fine */
    for (int h = 0; h < nq; ++h) orc_rmsnorm(q + h * d, w->q_norm, d, c->eps, q + h * d);
    for (int g = 0; g < nkv; ++g) orc_rmsnorm(k + g * d, w->k_norm, d, c->eps, k + g * d);
  }
  for (int h = 0; h < nq; ++h) orc_rope(q + h * d, d, pos, c->theta);
  for (int g = 0; g < nkv; ++g) {
    orc_rope(k + g * d, d, pos, c->theta);
    uint16_t *krow = kc + ((size_t)g * c->max_seq + pos) * d, *vrow = vc + ((size_t)g * c->max_seq + pos) * d;
    orc_kv_store(krow, k + g * d, d);
    orc_kv_store(vrow, v + g * d, d);
    if (held && held->k_exact) memcpy(held->k_exact + (size_t)g * d, k + g * d, sizeof(real) * d);
    if (held && held->v_exact) memcpy(held->v_exact + (size_t)g * d, v + g * d, sizeof(real) * d);
    if (held && held->k_rows) memcpy(krow, held->k_rows + (size_t)g * d, sizeof(uint16_t) * d);
    if (held && held->v_rows) memcpy(vrow, held->v_rows + (size_t)g * d, sizeof(uint16_t) * d);
  }
  int group = nq / nkv;
  for (int h = 0; h < nq; ++h) {
    int g = h / group;
    orc_attention_head(q + h * d, kc + (size_t)g * c->max_seq * d, vc + (size_t)g * c->max_seq * d,
                       pos + 1, d, scr, o + h * d);
  }
  orc_linear(w->wo, H, nq * d, o, a);
  orc_add(x, a, H, x1);
  orc_rmsnorm(x1, w->mlp_norm, H, c->eps, xn);
  if (c->n_experts == 0) {
    int F = c->ffn;
    real *gu = rest, *hh = gu + 2 * F, *m = hh + F;
    orc_linear(w->wgu, 2 * F, H, xn, gu);
    orc_swiglu(gu, F, hh);
    orc_linear(w->wd, H, F, hh, m);
    orc_add(x1, m, H, x);
  } else {
    int E = c->n_experts, K = c->top_k, F = c->expert_ffn;
    real *rl = rest, *gu = rl + E, *hh = gu + 2 * F, *m = hh + F, *y = m + H;
    int sel_local[64];
    real wts[64];
    int *sel = moe_sel ? moe_sel : sel_local;
    orc_linear(w->router, E, H, xn, rl);
    if (moe_logits)
      for (int e = 0; e < E; ++e) moe_logits[e] = rl[e];
    orc_router_topk(rl, E, K, sel, wts);
    if (held && held->experts) { /* the held set, weighted as the router weights it: softmax, renormalised */
      real mx = -INFINITY, l = 0, ssum = 0;
      for (int e = 0; e < E; ++e)
        if (rl[e] > mx) mx = rl[e];
      for (int e = 0; e < E; ++e) l += R_EXP(rl[e] - mx);
      for (int j = 0; j < K; ++j) {
        sel[j] = held->experts[j];
        wts[j] = R_EXP(rl[sel[j]] - mx) / l;
        ssum += wts[j];
      }
      for (int j = 0; j < K; ++j) wts[j] /= ssum;
    }
    for (int i = 0; i < H; ++i) y[i] = 0;
    for (int j = 0; j < K; ++j) { /* ascending expert index */
      int e = sel[j];
      orc_linear(w->exp_wgu + (size_t)e * 2 * F * H, 2 * F, H, xn, gu);
      orc_swiglu(gu, F, hh);
      orc_linear(w->exp_wd + (size_t)e * H * F, H, F, hh, m);
      for (int i = 0; i < H; ++i) y[i] += wts[j] * m[i];
    }
    orc_add(x1, y, H, x);
  }
}
