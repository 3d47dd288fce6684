/*
 * CPU oracle for one pipeline stage of decoder blocks.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP library is checked against.  It shares no code, header, table or helper
 * with the GPU path, and nothing in the product may call it.
 *
 * What it computes follows the paper's description of a decoder block
 * (Sec. III-A and the Fig. 2 caption): RMS Norm before the attention and before
 * the feed-forward sub-layer, grouped-query attention that incorporates rotary
 * position encoding, a SwiGLU feed-forward network, blocks stacked strictly in
 * sequence (Eq. 1), and a stage being the contiguous block range of Eq. 6 run on
 * an activation tensor batch x sequence x hidden (Sec. IV-A).  The paper prints
 * no formula for the inside of a block; the conventions of the model family it
 * names (Llama 3 / Phi-3) are used: pre-norm residuals, eps inside the square
 * root, no biases, rotate-half RoPE pairing (i, i + d/2) with plain base,
 * contiguous query-head groups per KV head, 1/sqrt(d) score scale, causal mask
 * by exclusion.
 *
 * Precision: `real` is float (the precision named for this oracle) or double
 * (build with -DORACLE_REAL=double); sums run in index order in `real`.
 * RoPE angles are always formed in double.  There is no blocking, fusion or
 * reordering: attention materialises the whole score matrix.
 *
 * OpenMP pragmas sit on outermost independent loops only.
 *
 * Pins (tests/test_oracle_*.py): linear vs a float64 library matmul; RMSNorm
 * closed forms; RoPE invariants; softmax sum/shift; attention vs an explicit
 * mask-matrix float64 evaluation and special cases; causal-prefix invariance;
 * cached decode == recompute; SwiGLU identities; zero-weight and composition
 * invariants of the layer and stage.  The paper prints no numeric value of a
 * block output, so absolute values beyond those pins are parity-unpinned.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#ifndef ORACLE_REAL
#define ORACLE_REAL float
#endif
typedef ORACLE_REAL real;

typedef struct {
  int hidden, n_q_heads, n_kv_heads, head_dim, ffn_dim;
  double rms_eps, rope_base;
} orc_shape;

typedef struct {
  const real *attn_norm_g; /* [hidden]               */
  const real *wq, *wk, *wv; /* [n_q*d,H] [n_kv*d,H] x2 */
  const real *wo;          /* [H, n_q*d]             */
  const real *ffn_norm_g;  /* [hidden]               */
  const real *w_gate, *w_up; /* [ffn,H]              */
  const real *w_down;      /* [H, ffn]               */
} orc_layer;

int orc_real_bytes(void) { return (int)sizeof(real); }

/* y[t,:] = x[t,:] * rsqrt(mean(x[t,:]^2) + eps) * g      (RMS Norm, Sec. III-A) */
void orc_rmsnorm(const real *x, const real *g, double eps, int T, int H, real *y) {
#pragma omp parallel for
  for (int t = 0; t < T; ++t) {
    real ss = 0;
    for (int i = 0; i < H; ++i) ss += x[(size_t)t * H + i] * x[(size_t)t * H + i];
    real r = (real)1 / (real)sqrt((double)(ss / (real)H + (real)eps));
    for (int i = 0; i < H; ++i) y[(size_t)t * H + i] = x[(size_t)t * H + i] * r * g[i];
  }
}

/* y[t,n] = sum_k x[t,k] W[n,k]      (bias-free projection, W row-major [out,in]) */
void orc_linear(const real *x, const real *W, int T, int K, int N, real *y) {
#pragma omp parallel for collapse(2)
  for (int t = 0; t < T; ++t)
    for (int n = 0; n < N; ++n) {
      real acc = 0;
      const real *xr = x + (size_t)t * K, *wr = W + (size_t)n * K;
      for (int k = 0; k < K; ++k) acc += xr[k] * wr[k];
      y[(size_t)t * N + n] = acc;
    }
}

/* Rotary position encoding, in place, z[t, head, d]; pair (i, i+d/2) of each head
 * turns by the angle pos[t] * base^(-2i/d). */
void orc_rope(real *z, const int *pos, int T, int n_heads, int d, double base) {
  int half = d / 2;
#pragma omp parallel for
  for (int t = 0; t < T; ++t)
    for (int h = 0; h < n_heads; ++h) {
      real *v = z + ((size_t)t * n_heads + h) * d;
      for (int i = 0; i < half; ++i) {
        double theta = pow(base, -2.0 * (double)i / (double)d);
        double ang = (double)pos[t] * theta;
        real c = (real)cos(ang), s = (real)sin(ang);
        real a = v[i], b = v[i + half];
        v[i] = a * c - b * s;
        v[i + half] = b * c + a * s;
      }
    }
}

/* softmax over s[0..n): subtract the maximum, exponentiate, divide by the sum */
void orc_softmax(real *s, int n) {
  real m = s[0];
  for (int j = 1; j < n; ++j) if (s[j] > m) m = s[j];
  real sum = 0;
  for (int j = 0; j < n; ++j) { s[j] = (real)exp((double)(s[j] - m)); sum += s[j]; }
  for (int j = 0; j < n; ++j) s[j] /= sum;
}

/* Causal grouped-query attention by brute force.
 *   q   [n_rows, n_q, d]   query row r sits at position q_pos[r]
 *   K,V [n_keys, n_kv, d]  key j sits at position j
 *   out [n_rows, n_q, d]
 * Query head h reads KV head h / (n_q/n_kv).  Row r sees keys j <= q_pos[r]
 * (q_pos[r] < n_keys required).  The whole [n_rows, n_keys] score matrix of a
 * head is materialised; `probs` (may be NULL) receives all of them as
 * [n_q, n_rows, n_keys] with masked entries 0. */
void orc_attention(const real *q, const int *q_pos, int n_rows, const real *K, const real *V,
                   int n_keys, int n_q, int n_kv, int d, real *out, real *probs) {
  int group = n_q / n_kv;
  real scale = (real)(1.0 / sqrt((double)d));
#pragma omp parallel for
  for (int h = 0; h < n_q; ++h) {
    int kh = h / group;
    real *S = (real *)malloc(sizeof(real) * (size_t)n_rows * (size_t)n_keys);
    for (int r = 0; r < n_rows; ++r)
      for (int j = 0; j < n_keys; ++j) {
        real acc = 0;
        const real *qv = q + ((size_t)r * n_q + h) * d;
        const real *kv = K + ((size_t)j * n_kv + kh) * d;
        for (int i = 0; i < d; ++i) acc += qv[i] * kv[i];
        S[(size_t)r * n_keys + j] = acc * scale;
      }
    for (int r = 0; r < n_rows; ++r) {
      int visible = q_pos[r] + 1;
      real *row = S + (size_t)r * n_keys;
      orc_softmax(row, visible);
      for (int j = visible; j < n_keys; ++j) row[j] = 0;
      real *o = out + ((size_t)r * n_q + h) * d;
      for (int i = 0; i < d; ++i) {
        real acc = 0;
        for (int j = 0; j < visible; ++j) acc += row[j] * V[((size_t)j * n_kv + kh) * d + i];
        o[i] = acc;
      }
    }
    if (probs) memcpy(probs + (size_t)h * n_rows * n_keys, S, sizeof(real) * (size_t)n_rows * n_keys);
    free(S);
  }
}

/* m[t,i] = silu(gate[t,i]) * up[t,i],   silu(z) = z / (1 + exp(-z)) */
void orc_swiglu(const real *gate, const real *up, size_t n, real *m) {
  for (size_t i = 0; i < n; ++i) {
    real z = gate[i];
    m[i] = z / ((real)1 + (real)exp((double)-z)) * up[i];
  }
}

/* One decoder block over S new tokens of ONE request, at positions
 * pos0 .. pos0+S-1.  Kc, Vc [cap, n_kv*d] hold the post-RoPE keys and the values
 * of positions < pos0 and receive the new ones (prefill: pos0 = 0; cached
 * decode: S = 1, pos0 = tokens already cached).  Keys and values are formed for
 * every new token; everything after that only for the rows listed in `rows`
 * (indices into 0..S-1, n_rows of them; rows == NULL means all S rows).
 * out [n_rows, H]. */
void orc_layer_forward(const orc_shape *c, const orc_layer *w, const real *x, int S, int pos0,
                       real *Kc, real *Vc, const int *rows, int n_rows, real *out) {
  int H = c->hidden, d = c->head_dim, nq = c->n_q_heads, nkv = c->n_kv_heads, I = c->ffn_dim;
  int qd = nq * d, kvd = nkv * d;
  int *all = NULL;
  if (!rows) {
    all = (int *)malloc(sizeof(int) * (size_t)S);
    for (int i = 0; i < S; ++i) all[i] = i;
    rows = all; n_rows = S;
  }
  real *u = (real *)malloc(sizeof(real) * (size_t)S * H);
  int *pos = (int *)malloc(sizeof(int) * (size_t)S);
  for (int t = 0; t < S; ++t) pos[t] = pos0 + t;

  /* pre-attention norm; keys and values of every new token into the cache */
  orc_rmsnorm(x, w->attn_norm_g, c->rms_eps, S, H, u);
  orc_linear(u, w->wk, S, H, kvd, Kc + (size_t)pos0 * kvd);
  orc_linear(u, w->wv, S, H, kvd, Vc + (size_t)pos0 * kvd);
  orc_rope(Kc + (size_t)pos0 * kvd, pos, S, nkv, d, c->rope_base);

  /* selected rows */
  real *xs = (real *)malloc(sizeof(real) * (size_t)n_rows * H);
  real *us = (real *)malloc(sizeof(real) * (size_t)n_rows * H);
  int *ps = (int *)malloc(sizeof(int) * (size_t)n_rows);
  for (int r = 0; r < n_rows; ++r) {
    memcpy(xs + (size_t)r * H, x + (size_t)rows[r] * H, sizeof(real) * H);
    memcpy(us + (size_t)r * H, u + (size_t)rows[r] * H, sizeof(real) * H);
    ps[r] = pos0 + rows[r];
  }
  real *q = (real *)malloc(sizeof(real) * (size_t)n_rows * qd);
  real *a = (real *)malloc(sizeof(real) * (size_t)n_rows * qd);
  orc_linear(us, w->wq, n_rows, H, qd, q);
  orc_rope(q, ps, n_rows, nq, d, c->rope_base);
  orc_attention(q, ps, n_rows, Kc, Vc, pos0 + S, nq, nkv, d, a, NULL);

  /* attention output projection + residual */
  real *hres = (real *)malloc(sizeof(real) * (size_t)n_rows * H);
  orc_linear(a, w->wo, n_rows, qd, H, hres);
  for (size_t i = 0; i < (size_t)n_rows * H; ++i) hres[i] = xs[i] + hres[i];

  /* pre-FFN norm, SwiGLU feed-forward, residual */
  real *r2 = us; /* reuse */
  orc_rmsnorm(hres, w->ffn_norm_g, c->rms_eps, n_rows, H, r2);
  real *gt = (real *)malloc(sizeof(real) * (size_t)n_rows * I);
  real *up = (real *)malloc(sizeof(real) * (size_t)n_rows * I);
  orc_linear(r2, w->w_gate, n_rows, H, I, gt);
  orc_linear(r2, w->w_up, n_rows, H, I, up);
  orc_swiglu(gt, up, (size_t)n_rows * I, gt);
  orc_linear(gt, w->w_down, n_rows, I, H, out);
  for (size_t i = 0; i < (size_t)n_rows * H; ++i) out[i] = hres[i] + out[i];

  free(u); free(pos); free(xs); free(us); free(ps); free(q); free(a); free(hres);
  free(gt); free(up); free(all);
}

/* A stage: blocks 0..n_layers-1 of `layers` (the caller passes the slice
 * [l_start, l_end) of the model, Eq. 6) applied in order (Eq. 1) to a packed
 * batch: request b contributes seq_lens[b] consecutive rows of x, at positions
 * pos0[b] .. pos0[b]+seq_lens[b]-1.  The cache slab is
 * [n_layers][batch][cap][n_kv*d] for K and for V.  out has the shape of x. */
void orc_stage_forward(const orc_shape *c, const orc_layer *layers, int n_layers, const real *x,
                       const int *seq_lens, const int *pos0, int batch, real *Kslab, real *Vslab,
                       int cap, real *out) {
  int H = c->hidden, kvd = c->n_kv_heads * c->head_dim;
  size_t T = 0;
  for (int b = 0; b < batch; ++b) T += (size_t)seq_lens[b];
  real *cur = (real *)malloc(sizeof(real) * T * H);
  real *nxt = (real *)malloc(sizeof(real) * T * H);
  memcpy(cur, x, sizeof(real) * T * H);
  for (int l = 0; l < n_layers; ++l) {
    size_t row0 = 0;
    for (int b = 0; b < batch; ++b) {
      size_t off = ((size_t)l * batch + b) * (size_t)cap * kvd;
      orc_layer_forward(c, &layers[l], cur + row0 * H, seq_lens[b], pos0[b], Kslab + off,
                        Vslab + off, NULL, 0, nxt + row0 * H);
      row0 += (size_t)seq_lens[b];
    }
    real *t = cur; cur = nxt; nxt = t;
  }
  memcpy(out, cur, sizeof(real) * T * H);
  free(cur); free(nxt);
}
