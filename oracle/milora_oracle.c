/*
 * MiLoRA routed-LoRA hot path: reference oracle (TEST INFRASTRUCTURE ONLY).
 *
 * A plain, slow, fp64 CPU statement of what the path computes, written from
 * the paper's definitions so that it can be checked against them by eye.
 * It shares no code with the GPU library and must never be called from the
 * product path; only the test-suite, the smoke check and the benchmark's
 * reported CPU baseline use it.
 *
 * Conventions (paper, Sec. 3.1): row vectors, x' = x W + x W^A W^B + b
 * (Eq. 1) with W in R^{d1 x d2}, W^A in R^{d1 x r}, W^B in R^{r x d2}.
 * Storage handed to this file:
 *   base weight  W  : [d2][d1]  (the mathematical W transposed, d1 contiguous)
 *   W^A ("A")       : [d1][r]   row-major, exactly as Eq. 1 writes it
 *   W^B ("B")       : [r][d2]   row-major
 *   router W_r      : [T][7][d] (column j of the paper's d x 7 matrix is a
 *                     contiguous d-vector), one per tenant (Eq. 3)
 * Sites (N_mod = 7, Sec. 3.1): 0 q, 1 k, 2 v, 3 o, 4 gate, 5 up, 6 down.
 * Every floating-point input is read in its stored precision and widened
 * exactly to double; nothing is ever rounded back.
 *
 * Every function here is pinned by tests that do not re-use its own formula
 * (closed forms, numpy's matmul on merged weights, invariants, the paper's
 * printed parameter counts); none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_BF16 = 0, ORC_F32 = 1, ORC_F64 = 2 };
enum { ORC_POOL_MEAN = 0, ORC_POOL_LAST = 1, ORC_POOL_MAX = 2, ORC_POOL_SELFATTN = 3 };
enum { ORC_ACT_IDENTITY = 0, ORC_ACT_TANH = 1, ORC_ACT_RELU = 2, ORC_ACT_GELU = 3, ORC_ACT_RATIONAL = 4 };
enum { ORC_OK = 0, ORC_EINVAL = -1, ORC_ERANGE = -2 };
enum { ORC_NMOD = 7 };
enum { ORC_FLAG_RMSNORM = 1 };

/* Widen element i of a stored array to double (exact for all three types). */
static double ld(const void *p, int dtype, int64_t i) {
  if (dtype == ORC_F64) return ((const double *)p)[i];
  if (dtype == ORC_F32) return (double)((const float *)p)[i];
  uint32_t bits = (uint32_t)((const uint16_t *)p)[i] << 16; /* bf16 = top half of an fp32 */
  float f;
  memcpy(&f, &bits, sizeof f);
  return (double)f;
}

/* Input and output width of site m in a layer with hidden d and FFN width F (Sec. 3.1). */
void orc_site_dims(int site, int d, int F, int *d1, int *d2) {
  *d1 = (site == 6) ? F : d;
  *d2 = (site == 4 || site == 5) ? F : d;
}

/*
 * Parameter counts the paper prints for LLaMA-2 7B (Table 1; Sec. 4.3
 * hyper-parameter paragraph): LoRA of rank r on all seven sites of L layers,
 * one d x 7 router per layer without bias, and the largest set that can be
 * active when one expert per layer is on.
 * out[0] = LoRA parameters, out[1] = router parameters, out[2] = max activated.
 */
void orc_param_counts(int d, int F, int L, int r, int64_t *out) {
  int64_t per_layer = 0, biggest = 0;
  for (int m = 0; m < ORC_NMOD; ++m) {
    int d1, d2;
    orc_site_dims(m, d, F, &d1, &d2);
    int64_t p = (int64_t)r * (d1 + d2);
    per_layer += p;
    if (p > biggest) biggest = p;
  }
  out[0] = (int64_t)L * per_layer;
  out[1] = (int64_t)L * d * ORC_NMOD;
  out[2] = (int64_t)L * biggest + out[1];
}

/* ---- Pooler (Eq. 2 and the list that follows it; App. C for self-attention) ---- */
/*
 * h_b = Pooler(H restricted to request b's valid tokens).  H is [M_tok][d];
 * request b owns rows seq_start[b] .. seq_start[b]+seq_len[b]-1.
 * w_sa: [T][d] query vector of the self-attention pooler (App. C), or NULL.
 */
int orc_pool(const void *H, int dtype, int64_t M_tok, int d, const int32_t *seq_start,
             const int32_t *seq_len, int B, int pool_kind, const void *w_sa,
             const int32_t *tenant_id, int T, double *h) {
  for (int b = 0; b < B; ++b) {
    int64_t s = seq_start[b], n = seq_len[b];
    if (n <= 0 || s < 0 || s + n > M_tok) return ORC_ERANGE;
    double *hb = h + (int64_t)b * d;
    if (pool_kind == ORC_POOL_LAST) {
      for (int i = 0; i < d; ++i) hb[i] = ld(H, dtype, (s + n - 1) * d + i);
    } else if (pool_kind == ORC_POOL_MEAN) {
      for (int i = 0; i < d; ++i) {
        double acc = 0.0;
        for (int64_t t = 0; t < n; ++t) acc += ld(H, dtype, (s + t) * d + i);
        hb[i] = acc / (double)n;
      }
    } else if (pool_kind == ORC_POOL_MAX) {
      for (int i = 0; i < d; ++i) {
        double mx = ld(H, dtype, s * d + i);
        for (int64_t t = 1; t < n; ++t) {
          double v = ld(H, dtype, (s + t) * d + i);
          if (v > mx) mx = v;
        }
        hb[i] = mx;
      }
    } else if (pool_kind == ORC_POOL_SELFATTN) {
      /* U = H w_sa, A = softmax over tokens, p = A^T H (App. C). */
      if (!w_sa || !tenant_id) return ORC_EINVAL;
      int t_id = tenant_id[b];
      if (t_id < 0 || t_id >= T) return ORC_ERANGE;
      double *u = (double *)malloc(sizeof(double) * (size_t)n);
      if (!u) return ORC_EINVAL;
      double umax = -INFINITY;
      for (int64_t t = 0; t < n; ++t) {
        double acc = 0.0;
        for (int i = 0; i < d; ++i)
          acc += ld(H, dtype, (s + t) * d + i) * ld(w_sa, dtype, (int64_t)t_id * d + i);
        u[t] = acc;
        if (acc > umax) umax = acc;
      }
      double Z = 0.0;
      for (int64_t t = 0; t < n; ++t) {
        u[t] = exp(u[t] - umax);
        Z += u[t];
      }
      for (int i = 0; i < d; ++i) {
        double acc = 0.0;
        for (int64_t t = 0; t < n; ++t) acc += (u[t] / Z) * ld(H, dtype, (s + t) * d + i);
        hb[i] = acc;
      }
      free(u);
    } else {
      return ORC_EINVAL;
    }
  }
  return ORC_OK;
}

/* ---- Router activation g (text before Eq. 3; rational form: Sec. 3.4) ---- */
/*
 * coef: for ORC_ACT_RATIONAL, 12 doubles a_0..a_6, b_1..b_5 of
 * Ra(x) = (sum_j a_j x^j) / (1 + |sum_i b_i x^i|); ignored otherwise.
 */
int orc_activation(double *z, int64_t n, int act_kind, const double *coef) {
  for (int64_t i = 0; i < n; ++i) {
    double x = z[i];
    switch (act_kind) {
      case ORC_ACT_IDENTITY: break;
      case ORC_ACT_TANH: z[i] = tanh(x); break;
      case ORC_ACT_RELU: z[i] = x > 0.0 ? x : 0.0; break;
      case ORC_ACT_GELU: z[i] = 0.5 * x * (1.0 + erf(x / sqrt(2.0))); break;
      case ORC_ACT_RATIONAL: {
        if (!coef) return ORC_EINVAL;
        double num = 0.0, den = 0.0, p = 1.0;
        for (int j = 0; j <= 6; ++j) {
          num += coef[j] * p;
          p *= x;
        }
        p = x;
        for (int k = 1; k <= 5; ++k) {
          den += coef[6 + k] * p;
          p *= x;
        }
        z[i] = num / (1.0 + fabs(den));
        break;
      }
      default: return ORC_EINVAL;
    }
  }
  return ORC_OK;
}

/* ---- Router linear, softmax and top-1 (Eq. 3) ---- */
/* logits[b][j] = sum_i z[b][i] * W_r^{tenant(b)}[i][j];  no bias. */
int orc_router_logits(const double *z, int B, int d, const void *Wr, int dtype,
                      const int32_t *tenant_id, int T, double *logits) {
  for (int b = 0; b < B; ++b) {
    int t = tenant_id[b];
    if (t < 0 || t >= T) return ORC_ERANGE;
    for (int j = 0; j < ORC_NMOD; ++j) {
      double acc = 0.0;
      for (int i = 0; i < d; ++i)
        acc += z[(int64_t)b * d + i] * ld(Wr, dtype, ((int64_t)t * ORC_NMOD + j) * d + i);
      logits[b * ORC_NMOD + j] = acc;
    }
  }
  return ORC_OK;
}

void orc_softmax7(const double *logit, double *prob) {
  double mx = logit[0], Z = 0.0;
  for (int j = 1; j < ORC_NMOD; ++j)
    if (logit[j] > mx) mx = logit[j];
  for (int j = 0; j < ORC_NMOD; ++j) {
    prob[j] = exp(logit[j] - mx);
    Z += prob[j];
  }
  for (int j = 0; j < ORC_NMOD; ++j) prob[j] /= Z;
}

/*
 * Top-1 of the softmax: the expert with the largest probability, the lowest
 * index winning an exact tie.  Because softmax is increasing, the choice is
 * taken on the logits (a test checks both give the same index).  gap[b] is
 * the distance between the two largest logits, which parity tests use to
 * leave out prompts whose choice a rounding error could flip.
 */
void orc_select(const double *logits, int B, uint8_t *route, double *gap) {
  for (int b = 0; b < B; ++b) {
    const double *l = logits + b * ORC_NMOD;
    int best = 0;
    for (int j = 1; j < ORC_NMOD; ++j)
      if (l[j] > l[best]) best = j;
    double second = -INFINITY;
    for (int j = 0; j < ORC_NMOD; ++j)
      if (j != best && l[j] > second) second = l[j];
    route[b] = (uint8_t)best;
    if (gap) gap[b] = l[best] - second;
  }
}

/*
 * A route byte names the sites whose LoRA a request uses: 0..6 = that one site (top-1, the reading the
 * printed parameter counts fix); 0x80 | mask with bit m of the 7-bit mask set for every chosen site m
 * (top-k with k > 1: the experiments' text mentions k = 3; the sites' LoRA terms are added without
 * weights, since the gate of Eq. 3 is never connected to Eq. 1 in the paper); 255 = none.
 */
int orc_route_has(uint8_t route, int site) {
  if (route < ORC_NMOD) return route == site;
  if (route == 255 || !(route & 0x80)) return 0;
  return (route >> site) & 1;
}

/*
 * Top-k of the softmax for k in 1..6, again taken on the logits: the k largest, an exact tie going to the
 * lower index.  k = 1 writes the site index like orc_select, k > 1 the mask form.  gap[b] is the distance
 * between the k-th and the (k+1)-th largest logit (what a rounding error would have to bridge to change the
 * chosen set).
 */
int orc_select_topk(const double *logits, int B, int k, uint8_t *route, double *gap) {
  if (k < 1 || k >= ORC_NMOD) return ORC_EINVAL;
  for (int b = 0; b < B; ++b) {
    const double *l = logits + b * ORC_NMOD;
    int taken[ORC_NMOD] = {0};
    int last = -1;
    for (int q = 0; q < k; ++q) {
      int best = -1;
      for (int j = 0; j < ORC_NMOD; ++j)
        if (!taken[j] && (best < 0 || l[j] > l[best])) best = j;
      taken[best] = 1;
      last = best;
    }
    double next = -INFINITY;
    unsigned mask = 0;
    for (int j = 0; j < ORC_NMOD; ++j) {
      if (taken[j]) mask |= 1u << j;
      else if (l[j] > next) next = l[j];
    }
    route[b] = k == 1 ? (uint8_t)last : (uint8_t)(0x80u | mask);
    if (gap) gap[b] = l[last] - next;
  }
  return ORC_OK;
}

/* The whole prompt-aware router of one layer: pool, g, linear, top-1. */
int orc_route(const void *H, int dtype, int64_t M_tok, int d, const int32_t *seq_start,
              const int32_t *seq_len, const int32_t *tenant_id, int B, int T, const void *Wr,
              int pool_kind, int act_kind, const void *w_sa, const double *act_coef,
              uint8_t *route, double *logits, double *gap, double *h_out) {
  double *h = (double *)malloc(sizeof(double) * (size_t)B * d);
  if (!h) return ORC_EINVAL;
  int rc = orc_pool(H, dtype, M_tok, d, seq_start, seq_len, B, pool_kind, w_sa, tenant_id, T, h);
  if (rc == ORC_OK && h_out) memcpy(h_out, h, sizeof(double) * (size_t)B * d);
  if (rc == ORC_OK) rc = orc_activation(h, (int64_t)B * d, act_kind, act_coef);
  if (rc == ORC_OK) rc = orc_router_logits(h, B, d, Wr, dtype, tenant_id, T, logits);
  if (rc == ORC_OK) orc_select(logits, B, route, gap);
  free(h);
  return rc;
}

/* ---- Routed LoRA linear (Eq. 1 with the layer-level expert gate of Sec. 3.3) ---- */
/*
 * For each requested row m (all M rows when rows == NULL), with
 * b = row_to_req ? row_to_req[m] : m and t = tenant_id[b]:
 *   y = x W + bias + [route[b] == site] * (x A_{t,site}) B_{t,site}
 * A_ptrs / B_ptrs: [T*7] host pointers, entry t*7+site; rank[t] = r_t.
 * X has its own dtype so that a chain of layers can stay in double.
 */
int orc_routed_linear(const void *X, int x_dtype, int64_t M, int d1, int d2,
                      const int32_t *row_to_req, const void *W, const void *bias, int w_dtype,
                      const void *const *A_ptrs, const void *const *B_ptrs, const int32_t *rank,
                      int T, int site, const int32_t *tenant_id, const uint8_t *route, int B,
                      const int64_t *rows, int64_t n_rows, double *Y) {
  if (site < 0 || site >= ORC_NMOD) return ORC_EINVAL;
  if (!row_to_req && !rows && M != B) return ORC_EINVAL;
  int64_t n = rows ? n_rows : M;
  int rc = ORC_OK;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t q = 0; q < n; ++q) {
    int64_t m = rows ? rows[q] : q;
    if (m < 0 || m >= M) { rc = ORC_ERANGE; continue; }
    int64_t b = row_to_req ? row_to_req[m] : m;
    if (b < 0 || b >= B) { rc = ORC_ERANGE; continue; }
    double *y = Y + q * d2;
    for (int j = 0; j < d2; ++j) {
      double acc = 0.0;
      for (int i = 0; i < d1; ++i) acc += ld(X, x_dtype, m * d1 + i) * ld(W, w_dtype, (int64_t)j * d1 + i);
      if (bias) acc += ld(bias, w_dtype, j);
      y[j] = acc;
    }
    if (!orc_route_has(route[b], site)) continue;
    int t = tenant_id[b];
    if (t < 0 || t >= T) { rc = ORC_ERANGE; continue; }
    int r = rank[t];
    const void *A = A_ptrs[t * ORC_NMOD + site], *Bm = B_ptrs[t * ORC_NMOD + site];
    double *tv = (double *)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
    for (int c = 0; c < r; ++c) {
      double acc = 0.0;
      for (int i = 0; i < d1; ++i) acc += ld(X, x_dtype, m * d1 + i) * ld(A, w_dtype, (int64_t)i * r + c);
      tv[c] = acc;
    }
    for (int j = 0; j < d2; ++j) {
      double acc = 0.0;
      for (int c = 0; c < r; ++c) acc += tv[c] * ld(Bm, w_dtype, (int64_t)c * d2 + j);
      y[j] += acc;
    }
    free(tv);
  }
  return rc;
}

/*
 * Cross-check form: every request evaluates the LoRA branch of this site and
 * scales it by gate[b][site], a real number.  With gate = one-hot(route) this
 * is the dense seven-way mixture that top-1 routing must reproduce.
 */
int orc_routed_linear_dense(const void *X, int x_dtype, int64_t M, int d1, int d2,
                            const int32_t *row_to_req, const void *W, const void *bias,
                            int w_dtype, const void *const *A_ptrs, const void *const *B_ptrs,
                            const int32_t *rank, int T, int site, const int32_t *tenant_id,
                            const double *gate, int B, double *Y) {
  if (site < 0 || site >= ORC_NMOD) return ORC_EINVAL;
  for (int64_t m = 0; m < M; ++m) {
    int64_t b = row_to_req ? row_to_req[m] : m;
    if (b < 0 || b >= B) return ORC_ERANGE;
    int t = tenant_id[b];
    if (t < 0 || t >= T) return ORC_ERANGE;
    int r = rank[t];
    const void *A = A_ptrs[t * ORC_NMOD + site], *Bm = B_ptrs[t * ORC_NMOD + site];
    for (int j = 0; j < d2; ++j) {
      double base = 0.0, delta = 0.0;
      for (int i = 0; i < d1; ++i) base += ld(X, x_dtype, m * d1 + i) * ld(W, w_dtype, (int64_t)j * d1 + i);
      for (int c = 0; c < r; ++c) {
        double tc = 0.0;
        for (int i = 0; i < d1; ++i) tc += ld(X, x_dtype, m * d1 + i) * ld(A, w_dtype, (int64_t)i * r + c);
        delta += tc * ld(Bm, w_dtype, (int64_t)c * d2 + j);
      }
      Y[m * d2 + j] = base + (bias ? ld(bias, w_dtype, j) : 0.0) + gate[b * ORC_NMOD + site] * delta;
    }
  }
  return ORC_OK;
}

/* ---- One decode step through the seven linears of a layer ---- */
static void rmsnorm_rows(const double *x, int B, int d, double *out) {
  for (int b = 0; b < B; ++b) {
    double ss = 0.0;
    for (int i = 0; i < d; ++i) ss += x[(int64_t)b * d + i] * x[(int64_t)b * d + i];
    double inv = 1.0 / sqrt(ss / d + 1e-5);
    for (int i = 0; i < d; ++i) out[(int64_t)b * d + i] = x[(int64_t)b * d + i] * inv;
  }
}

/*
 * The paper fixes the seven routed linears (Sec. 3.1, Fig. 1) and nothing of
 * what lies between them at decode time; the glue below is the smallest that
 * chains them at their true shapes:
 *   q,k,v = L_q(n1(x)), L_k(n1(x)), L_v(n1(x))
 *   a     = attn_out if given, else v   (causal attention over a context of one token)
 *   h     = x + L_o(a)
 *   g,u   = L_gate(n2(h)), L_up(n2(h));   m = silu(g) * u
 *   y     = h + L_down(m)
 * n1, n2 = weightless RMS normalisation (eps 1e-5) when ORC_FLAG_RMSNORM is
 * set, identity otherwise.  Everything stays in double.
 * W: 7 pointers, W[m] stored [d2][d1].  qkv (nullable): [B][3d].
 */
int orc_layer_decode(const void *x, int x_dtype, int B, int d, int F, const void *const *W,
                     int w_dtype, const void *const *A_ptrs, const void *const *B_ptrs,
                     const int32_t *rank, int T, const int32_t *tenant_id, const uint8_t *route,
                     int flags, const void *attn_out, double *y, double *qkv) {
  size_t nd = (size_t)B * d, nF = (size_t)B * F;
  double *xd = malloc(sizeof(double) * nd), *xn = malloc(sizeof(double) * nd);
  double *q = malloc(sizeof(double) * nd), *k = malloc(sizeof(double) * nd);
  double *v = malloc(sizeof(double) * nd), *a = malloc(sizeof(double) * nd);
  double *h = malloc(sizeof(double) * nd), *hn = malloc(sizeof(double) * nd);
  double *g = malloc(sizeof(double) * nF), *u = malloc(sizeof(double) * nF);
  double *o = malloc(sizeof(double) * nd), *dn = malloc(sizeof(double) * nd);
  int rc = ORC_OK;
  for (size_t i = 0; i < nd; ++i) xd[i] = ld(x, x_dtype, (int64_t)i);
  if (flags & ORC_FLAG_RMSNORM) rmsnorm_rows(xd, B, d, xn); else memcpy(xn, xd, sizeof(double) * nd);
#define LIN(site, in, d1, d2, out)                                                              \
  if (rc == ORC_OK)                                                                             \
    rc = orc_routed_linear(in, ORC_F64, B, d1, d2, NULL, W[site], NULL, w_dtype, A_ptrs, B_ptrs, \
                           rank, T, site, tenant_id, route, B, NULL, 0, out)
  LIN(0, xn, d, d, q);
  LIN(1, xn, d, d, k);
  LIN(2, xn, d, d, v);
  if (attn_out) for (size_t i = 0; i < nd; ++i) a[i] = ld(attn_out, x_dtype, (int64_t)i);
  else memcpy(a, v, sizeof(double) * nd);
  LIN(3, a, d, d, o);
  for (size_t i = 0; i < nd; ++i) h[i] = xd[i] + o[i];
  if (flags & ORC_FLAG_RMSNORM) rmsnorm_rows(h, B, d, hn); else memcpy(hn, h, sizeof(double) * nd);
  LIN(4, hn, d, F, g);
  LIN(5, hn, d, F, u);
  for (size_t i = 0; i < nF; ++i) g[i] = g[i] / (1.0 + exp(-g[i])) * u[i]; /* silu(g) * u */
  LIN(6, g, F, d, dn);
#undef LIN
  for (size_t i = 0; i < nd; ++i) y[i] = h[i] + dn[i];
  if (qkv)
    for (int b = 0; b < B; ++b)
      for (int i = 0; i < d; ++i) {
        qkv[(size_t)b * 3 * d + i] = q[(size_t)b * d + i];
        qkv[(size_t)b * 3 * d + d + i] = k[(size_t)b * d + i];
        qkv[(size_t)b * 3 * d + 2 * d + i] = v[(size_t)b * d + i];
      }
  free(xd); free(xn); free(q); free(k); free(v); free(a); free(h); free(hn);
  free(g); free(u); free(o); free(dn);
  return rc;
}
