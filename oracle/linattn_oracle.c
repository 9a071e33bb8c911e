/*
 * linattn_oracle.c -- plain, slow, obviously-correct CPU oracle (fp64).
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call, link or
 * import this file; it exists so that the GPU library has something
 * independent to be compared with.  It shares no code with the GPU path.
 *
 * What it computes, per (batch, head) independently, for a head of dimension
 * d and a token sequence of length L:
 *
 *   causal kernelised linear attention (Sec. 3 "Linear Attentions": the
 *   similarity is factored as phi(Q) phi(K)^T, which lets the product be
 *   re-associated as phi(Q) (phi(K)^T V)), restricted so that token t only
 *   uses tokens i <= t (Sec. 4.1: the query at step t meets the cumulative
 *   sum over i = 1..t of the key/value products), row-normalised by the
 *   matching cumulative sum of phi(K), plus a causally masked depthwise
 *   convolution over the sequence axis of V (Sec. 4.1, "masked DWConv"),
 *   added to the attention output.
 *
 *   Speculative verification (Sec. 4.2): k draft tokens are scored at once
 *   from one running state; each draft may see the verified past and the
 *   drafts before it, never a later one, and the convolution window of draft
 *   j is the verified history followed by drafts <= j (the paper's example:
 *   kernel 3 at step t1 must cover {t0, t1}).
 *
 *   The three-branch form of Sec. 4.1 as its text states it (grouped linear
 *   attention over the groups before a token's own, softmax attention inside the
 *   group, masked DWConv, weight alpha), for a whole sequence
 *   (oracle_prefill_grouped) and token by token with the state that generation
 *   carries (oracle_verify_grouped).
 *
 * Readings where the paper is silent (all are stated in the design notes of
 * the repository): phi(x) = elu(x)+1; the row normaliser; eps added to the
 * denominator; out = Y + U with no mixing weight; conv weights [H, d, Kc]
 * with tap j multiplying v_{t-j}; zero left padding at sequence start.
 *
 * Layouts (all contiguous, host memory, double):
 *   q, k, v, out : [B, H, L, d]          w    : [H, d, Kc]
 *   S            : [B, H, d, d]  S[i][c] = sum_t phi(k_t)[i] * v_t[c]
 *   z            : [B, H, d]     z[i]    = sum_t phi(k_t)[i]
 *   hist         : [B, H, Kc-1, d]  the last Kc-1 value rows, oldest first
 * NULL for an incoming S/z/hist means zeros (start of a sequence); NULL for an
 * outgoing one means "not wanted".
 *
 * Two prefill forms are given on purpose: the brute-force masked quadratic
 * form (the definition) and the token-by-token recurrence.  They are written
 * separately and the tests require them to agree.
 *
 * Pins (tests/test_oracle_pins.py): first-token identity, running mean for
 * K == 0, weighted running mean for Q == 0 and for d == 1, constant V,
 * linearity in V, exact rational brute force on a tiny case, conv against a
 * library grouped convolution, the paper's conv-window example, causality
 * under perturbation, chunk/split invariance, verify == k decode steps; for the
 * grouped form of Sec. 4.1: one group = a library softmax attention, one-token groups =
 * the token-level form shifted by one token, a closed-form example, shift invariance
 * of the logits, the weight alpha, splits at group boundaries, causality; token steps
 * of that form reproduce the whole-sequence form, commit counts across group
 * boundaries, blindness to rows beyond the count.
 * No function here is "parity unpinned" with respect to those properties; the
 * paper prints no numeric output of the operator, so there is no printed
 * value to compare with.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

/* phi(x) = elu(x) + 1 : x + 1 for x > 0, exp(x) otherwise (continuous at 0). */
/* The feature map.  0: elu(x) + 1 (the default of this build).  1: max(x, 0), the
 * "ReLU" linear attention that the paper lists among the existing linear
 * attentions it evaluates (Sec. 3, "Comprehensive Evaluation"); with it the
 * denominator can vanish, so callers pass eps > 0.  The choice is a property of
 * the loaded library (one setting for all calls that follow). */
static int g_feature_map = 0;
void oracle_set_feature_map(int kind) { g_feature_map = kind; }
double oracle_phi(double x) {
  if (g_feature_map == 1) return x > 0.0 ? x : 0.0;
  return x > 0.0 ? x + 1.0 : exp(x);
}

static double dot(const double *a, const double *b, int n) {
  double s = 0.0;
  for (int i = 0; i < n; ++i) s += a[i] * b[i];
  return s;
}

/* Row s of the value sequence extended to the left by the history:
 * s >= 0 -> v[s];  -(Kc-1) <= s < 0 -> hist[Kc-1+s];  nothing else exists. */
static const double *vext_row(const double *v, const double *hist, int Kc,
                              int d, int s) {
  if (s >= 0) return v + (size_t)s * d;
  if (hist && s >= -(Kc - 1)) return hist + (size_t)(Kc - 1 + s) * d;
  return NULL; /* zero padding */
}

/* One head: u[t][c] = sum_{j<Kc} w[c][j] * vext[t-j][c]   (Sec. 4.1) */
static void conv_head(int L, int d, int Kc, const double *v, const double *w,
                      const double *hist, double *u) {
  for (int t = 0; t < L; ++t)
    for (int c = 0; c < d; ++c) {
      double acc = 0.0;
      for (int j = 0; j < Kc; ++j) {
        const double *row = vext_row(v, hist, Kc, d, t - j);
        if (row) acc += w[(size_t)c * Kc + j] * row[c];
      }
      u[(size_t)t * d + c] = acc;
    }
}

/* New history = last Kc-1 rows of (old history ++ first n rows of v). */
static void hist_after(int n, int d, int Kc, const double *v,
                       const double *hist_in, double *hist_out) {
  int Hn = Kc - 1;
  double *tmp = (double *)malloc(sizeof(double) * (size_t)(Hn > 0 ? Hn : 1) * d);
  for (int r = 0; r < Hn; ++r) {
    int s = n - Hn + r; /* index into the extended sequence */
    const double *row = vext_row(v, hist_in, Kc, d, s);
    for (int c = 0; c < d; ++c) tmp[(size_t)r * d + c] = row ? row[c] : 0.0;
  }
  memcpy(hist_out, tmp, sizeof(double) * (size_t)Hn * d);
  free(tmp);
}

void oracle_causal_conv(int B, int H, int L, int d, int Kc, const double *v,
                        const double *w, const double *hist, double *u) {
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * H; ++bh) {
    int h = bh % H;
    conv_head(L, d, Kc, v + (size_t)bh * L * d, w + (size_t)h * d * Kc,
              hist ? hist + (size_t)bh * (Kc - 1) * d : NULL,
              u + (size_t)bh * L * d);
  }
}

/* ---- definition: brute-force masked quadratic form, one head ------------ */
static void quadratic_head(int L, int d, int Kc, double eps, const double *q,
                           const double *k, const double *v, const double *w,
                           const double *S0, const double *z0,
                           const double *hist0, double *out, double *S1,
                           double *z1, double *hist1) {
  double *fq = (double *)malloc(sizeof(double) * (size_t)L * d);
  double *fk = (double *)malloc(sizeof(double) * (size_t)L * d);
  double *u = (double *)malloc(sizeof(double) * (size_t)L * d);
  double *num = (double *)malloc(sizeof(double) * (size_t)d);
  for (size_t e = 0; e < (size_t)L * d; ++e) {
    fq[e] = oracle_phi(q[e]);
    fk[e] = oracle_phi(k[e]);
  }
  conv_head(L, d, Kc, v, w, hist0, u);
  for (int t = 0; t < L; ++t) {
    const double *fqt = fq + (size_t)t * d;
    double den = eps;
    for (int c = 0; c < d; ++c) num[c] = 0.0;
    /* the part that comes from before this call: phi(q_t)^T S0, phi(q_t).z0 */
    if (S0)
      for (int i = 0; i < d; ++i)
        for (int c = 0; c < d; ++c) num[c] += fqt[i] * S0[(size_t)i * d + c];
    if (z0) den += dot(fqt, z0, d);
    /* A[t][i] = phi(q_t).phi(k_i) for i <= t, nothing for i > t */
    for (int i = 0; i <= t; ++i) {
      double a = dot(fqt, fk + (size_t)i * d, d);
      den += a;
      for (int c = 0; c < d; ++c) num[c] += a * v[(size_t)i * d + c];
    }
    for (int c = 0; c < d; ++c)
      out[(size_t)t * d + c] = num[c] / den + u[(size_t)t * d + c];
  }
  if (S1) {
    for (int i = 0; i < d; ++i)
      for (int c = 0; c < d; ++c) {
        double s = S0 ? S0[(size_t)i * d + c] : 0.0;
        for (int t = 0; t < L; ++t)
          s += fk[(size_t)t * d + i] * v[(size_t)t * d + c];
        S1[(size_t)i * d + c] = s;
      }
  }
  if (z1) {
    for (int i = 0; i < d; ++i) {
      double s = z0 ? z0[i] : 0.0;
      for (int t = 0; t < L; ++t) s += fk[(size_t)t * d + i];
      z1[i] = s;
    }
  }
  if (hist1) hist_after(L, d, Kc, v, hist0, hist1);
  free(fq); free(fk); free(u); free(num);
}

/* ---- one recurrent step on a mutable head state (Sec. 4.1 cumulative sum):
 *   S += phi(k) v^T ; z += phi(k) ; Y = S^T phi(q) / (z.phi(q) + eps)
 *   U from (hist ++ v) ; out = Y + U ; hist <- shifted by one row           */
static void step_head(int d, int Kc, double eps, const double *q,
                      const double *k, const double *v, const double *w,
                      double *S, double *z, double *hist, double *out) {
  double *fq = (double *)malloc(sizeof(double) * (size_t)d);
  for (int i = 0; i < d; ++i) {
    double fk = oracle_phi(k[i]);
    fq[i] = oracle_phi(q[i]);
    z[i] += fk;
    for (int c = 0; c < d; ++c) S[(size_t)i * d + c] += fk * v[c];
  }
  double den = dot(fq, z, d) + eps;
  for (int c = 0; c < d; ++c) {
    double num = 0.0;
    for (int i = 0; i < d; ++i) num += fq[i] * S[(size_t)i * d + c];
    double u = w[(size_t)c * Kc + 0] * v[c];
    for (int j = 1; j < Kc; ++j) /* tap j looks j rows back: hist row Kc-1-j */
      u += w[(size_t)c * Kc + j] * hist[(size_t)(Kc - 1 - j) * d + c];
    out[c] = num / den + u;
  }
  for (int r = 0; r + 1 < Kc - 1; ++r)
    memcpy(hist + (size_t)r * d, hist + (size_t)(r + 1) * d, sizeof(double) * d);
  if (Kc > 1) memcpy(hist + (size_t)(Kc - 2) * d, v, sizeof(double) * d);
  free(fq);
}

static void load_state(int d, int Kc, const double *S0, const double *z0,
                       const double *h0, double *S, double *z, double *h) {
  size_t nS = (size_t)d * d, nh = (size_t)(Kc - 1) * d;
  if (S0) memcpy(S, S0, sizeof(double) * nS); else memset(S, 0, sizeof(double) * nS);
  if (z0) memcpy(z, z0, sizeof(double) * d); else memset(z, 0, sizeof(double) * d);
  if (h0) memcpy(h, h0, sizeof(double) * nh); else memset(h, 0, sizeof(double) * nh);
}

int oracle_prefill_quadratic(int B, int H, int L, int d, int Kc, double eps,
                             const double *q, const double *k, const double *v,
                             const double *w, const double *S0,
                             const double *z0, const double *hist0,
                             double *out, double *S1, double *z1,
                             double *hist1) {
  if (B < 0 || H < 1 || L < 0 || d < 1 || Kc < 1) return 1;
  size_t nS = (size_t)d * d, nh = (size_t)(Kc - 1) * d;
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * H; ++bh) {
    int h = bh % H;
    size_t o = (size_t)bh * L * d;
    quadratic_head(L, d, Kc, eps, q + o, k + o, v + o, w + (size_t)h * d * Kc,
                   S0 ? S0 + bh * nS : NULL, z0 ? z0 + (size_t)bh * d : NULL,
                   hist0 ? hist0 + bh * nh : NULL, out + o,
                   S1 ? S1 + bh * nS : NULL, z1 ? z1 + (size_t)bh * d : NULL,
                   hist1 ? hist1 + bh * nh : NULL);
  }
  return 0;
}

int oracle_prefill_recurrent(int B, int H, int L, int d, int Kc, double eps,
                             const double *q, const double *k, const double *v,
                             const double *w, const double *S0,
                             const double *z0, const double *hist0,
                             double *out, double *S1, double *z1,
                             double *hist1) {
  if (B < 0 || H < 1 || L < 0 || d < 1 || Kc < 1) return 1;
  size_t nS = (size_t)d * d, nh = (size_t)(Kc - 1) * d;
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * H; ++bh) {
    int h = bh % H;
    size_t o = (size_t)bh * L * d;
    double *S = (double *)malloc(sizeof(double) * nS);
    double *z = (double *)malloc(sizeof(double) * (size_t)d);
    double *hs = (double *)malloc(sizeof(double) * (nh ? nh : 1));
    load_state(d, Kc, S0 ? S0 + bh * nS : NULL, z0 ? z0 + (size_t)bh * d : NULL,
               hist0 ? hist0 + bh * nh : NULL, S, z, hs);
    for (int t = 0; t < L; ++t)
      step_head(d, Kc, eps, q + o + (size_t)t * d, k + o + (size_t)t * d,
                v + o + (size_t)t * d, w + (size_t)h * d * Kc, S, z, hs,
                out + o + (size_t)t * d);
    if (S1) memcpy(S1 + bh * nS, S, sizeof(double) * nS);
    if (z1) memcpy(z1 + (size_t)bh * d, z, sizeof(double) * d);
    if (hist1) memcpy(hist1 + bh * nh, hs, sizeof(double) * nh);
    free(S); free(z); free(hs);
  }
  return 0;
}

/* ---- the augmented attention of Sec. 4.1 as the text states it, one head ----
 * The sequence is cut into consecutive groups of C tokens (the last one may be
 * short).  Three branches are summed for every token t of a group:
 *   grouped linear attention: the query meets the key/value sums of the groups
 *     BEFORE its own (plus whatever state came in); nothing of its own group --
 *     the sums advance once per group, not once per token:
 *         G_t = phi(q_t)^T S / (phi(q_t).z + eps),   S, z as they stood before the group;
 *   local attention: softmax attention (Sec. 3, Eq. 1: logits q.k / sqrt(d)) over
 *     the tokens of its own group that are not later than t (the model is
 *     autoregressive; a token never sees a later one):
 *         A_t = sum_i softmax_i(q_t.k_i / sqrt(d)) v_i,  i in the group, i <= t;
 *   masked depthwise convolution of V, as in the other forms:  U_t.
 *   out_t = alpha * G_t + A_t + U_t   (alpha weighs the grouped against the local branch).
 * A grouped branch whose denominator is exactly zero (no token and no state before
 * the group, eps = 0) contributes nothing.  The state handed back is the same running
 * sum over all L tokens as in the other forms. */
static void grouped_head(int L, int d, int Kc, int C, double eps, double alpha,
                         const double *q, const double *k, const double *v,
                         const double *w, const double *S0, const double *z0,
                         const double *hist0, double *out, double *S1,
                         double *z1, double *hist1) {
  size_t nS = (size_t)d * d, nh = (size_t)(Kc - 1) * d;
  double *S = (double *)malloc(sizeof(double) * nS);
  double *z = (double *)malloc(sizeof(double) * (size_t)d);
  double *hs = (double *)malloc(sizeof(double) * (nh ? nh : 1));
  double *u = (double *)malloc(sizeof(double) * ((size_t)L * d + 1));
  double *fq = (double *)malloc(sizeof(double) * (size_t)d);
  double *logit = (double *)malloc(sizeof(double) * (size_t)(C > 0 ? C : 1));
  load_state(d, Kc, S0, z0, hist0, S, z, hs);
  conv_head(L, d, Kc, v, w, hist0, u);
  const double inv_sqrt_d = 1.0 / sqrt((double)d);
  for (int g0 = 0; g0 < L; g0 += C) {
    int g1 = g0 + C < L ? g0 + C : L;
    for (int t = g0; t < g1; ++t) {
      const double *qt = q + (size_t)t * d;
      for (int i = 0; i < d; ++i) fq[i] = oracle_phi(qt[i]);
      /* grouped branch: S and z have not seen any token of this group */
      double gden = dot(fq, z, d) + eps;
      /* local branch: logits of the group's tokens up to t, largest one taken out first */
      double top = -INFINITY;
      for (int i = g0; i <= t; ++i) {
        logit[i - g0] = dot(qt, k + (size_t)i * d, d) * inv_sqrt_d;
        if (logit[i - g0] > top) top = logit[i - g0];
      }
      double mass = 0.0;
      for (int i = g0; i <= t; ++i) {
        logit[i - g0] = exp(logit[i - g0] - top);
        mass += logit[i - g0];
      }
      for (int c = 0; c < d; ++c) {
        double gnum = 0.0, loc = 0.0;
        for (int i = 0; i < d; ++i) gnum += fq[i] * S[(size_t)i * d + c];
        for (int i = g0; i <= t; ++i) loc += logit[i - g0] * v[(size_t)i * d + c];
        double glob = gden != 0.0 ? gnum / gden : 0.0;
        out[(size_t)t * d + c] = alpha * glob + loc / mass + u[(size_t)t * d + c];
      }
    }
    /* only now do the group's keys and values enter the sums */
    for (int t = g0; t < g1; ++t)
      for (int i = 0; i < d; ++i) {
        double fk = oracle_phi(k[(size_t)t * d + i]);
        z[i] += fk;
        for (int c = 0; c < d; ++c) S[(size_t)i * d + c] += fk * v[(size_t)t * d + c];
      }
  }
  if (S1) memcpy(S1, S, sizeof(double) * nS);
  if (z1) memcpy(z1, z, sizeof(double) * (size_t)d);
  if (hist1) hist_after(L, d, Kc, v, hist0, hist1);
  free(S); free(z); free(hs); free(u); free(fq); free(logit);
}

int oracle_prefill_grouped(int B, int H, int L, int d, int Kc, int C, double eps,
                           double alpha, const double *q, const double *k,
                           const double *v, const double *w, const double *S0,
                           const double *z0, const double *hist0, double *out,
                           double *S1, double *z1, double *hist1) {
  if (B < 0 || H < 1 || L < 0 || d < 1 || Kc < 1 || C < 1) return 1;
  size_t nS = (size_t)d * d, nh = (size_t)(Kc - 1) * d;
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * H; ++bh) {
    int h = bh % H;
    size_t o = (size_t)bh * L * d;
    grouped_head(L, d, Kc, C, eps, alpha, q + o, k + o, v + o,
                 w + (size_t)h * d * Kc, S0 ? S0 + bh * nS : NULL,
                 z0 ? z0 + (size_t)bh * d : NULL, hist0 ? hist0 + bh * nh : NULL,
                 out + o, S1 ? S1 + bh * nS : NULL, z1 ? z1 + (size_t)bh * d : NULL,
                 hist1 ? hist1 + bh * nh : NULL);
  }
  return 0;
}

/* ---- gradient of the three-branch form, one head (training: Sec. 5.3 times a training
 * step, forward and backward, of FLASH with this block in groups of 256) ----
 * For a loss  Lo = sum_{t,c} dout[t][c] * out[t][c] + sum dS1 * S1 + sum dz1 * z1  the
 * derivatives with respect to every input of grouped_head, by the chain rule through
 * that function's own steps taken in reverse.  With P_g = (S, z) before group g:
 *   P_{g+1} = P_g + sum_{t in g} (phi(k_t) v_t^T, phi(k_t)), so the gradient D_g with respect
 *   to P_g is D_{g+1} plus what the queries of group g contribute;
 *   grouped branch of token t (group g):  G = alpha * N / D,  N = S^T phi(q_t),  D = phi(q_t).z + eps
 *       dN = alpha * dout_t / D,   dD = -alpha * (N . dout_t) / D^2,
 *       d phi(q_t) = S dN + z dD,   dS += phi(q_t) dN^T,   dz += phi(q_t) dD;
 *   local branch:  A = sum_i p_i v_i,  p = softmax(l),  l_i = q_t.k_i / sqrt(d):
 *       dv_i += p_i dout_t,   dp_i = dout_t . v_i,   dl_i = p_i (dp_i - sum_j p_j dp_j),
 *       dq_t += sum_i dl_i k_i / sqrt(d),   dk_i += dl_i q_t / sqrt(d);
 *   a token i of group g entered P_{g+1}:  d phi(k_i) = D_{g+1}.S v_i + D_{g+1}.z,
 *       dv_i += D_{g+1}.S^T phi(k_i);
 *   phi'(x) = 1 for x > 0, else exp(x)  (ReLU map: 1 for x > 0, else 0);
 *   conv:  out[t][c] has the term w[c][j] * vext[t-j][c].
 * dq, dk, dv are written; dw (this head's [d][Kc]) is ADDED to (the weights are shared
 * by the batch rows); dS0, dz0, dhist0 may be NULL (not wanted). */
static double dphi(double x) {
  if (g_feature_map == 1) return x > 0.0 ? 1.0 : 0.0;
  return x > 0.0 ? 1.0 : exp(x);
}

static void grouped_backward_head(int L, int d, int Kc, int C, double eps, double alpha,
                                  const double *q, const double *k, const double *v,
                                  const double *w, const double *S0, const double *z0,
                                  const double *hist0, const double *dout,
                                  const double *dS1, const double *dz1, double *dq,
                                  double *dk, double *dv, double *dw, double *dS0,
                                  double *dz0, double *dhist0) {
  size_t nS = (size_t)d * d;
  int ng = (L + C - 1) / C;
  /* the sums as they stood before every group (and after the last one) */
  double *Sg = (double *)calloc((size_t)(ng + 1) * nS, sizeof(double));
  double *zg = (double *)calloc((size_t)(ng + 1) * d, sizeof(double));
  if (S0) memcpy(Sg, S0, sizeof(double) * nS);
  if (z0) memcpy(zg, z0, sizeof(double) * (size_t)d);
  for (int g = 0; g < ng; ++g) {
    double *Sn = Sg + (size_t)(g + 1) * nS, *zn = zg + (size_t)(g + 1) * d;
    memcpy(Sn, Sg + (size_t)g * nS, sizeof(double) * nS);
    memcpy(zn, zg + (size_t)g * d, sizeof(double) * (size_t)d);
    int g0 = g * C, g1 = g0 + C < L ? g0 + C : L;
    for (int t = g0; t < g1; ++t)
      for (int i = 0; i < d; ++i) {
        double fk = oracle_phi(k[(size_t)t * d + i]);
        zn[i] += fk;
        for (int c = 0; c < d; ++c) Sn[(size_t)i * d + c] += fk * v[(size_t)t * d + c];
      }
  }
  double *DS = (double *)calloc(nS, sizeof(double));   /* gradient w.r.t. the sums after the current group */
  double *DZ = (double *)calloc((size_t)d, sizeof(double));
  double *gS = (double *)malloc(sizeof(double) * nS);  /* what the current group's queries add to it */
  double *gz = (double *)malloc(sizeof(double) * (size_t)d);
  double *fq = (double *)malloc(sizeof(double) * (size_t)d);
  double *gnum = (double *)malloc(sizeof(double) * (size_t)d);
  double *dnum = (double *)malloc(sizeof(double) * (size_t)d);
  double *p = (double *)malloc(sizeof(double) * (size_t)(C > 0 ? C : 1));
  double *dp = (double *)malloc(sizeof(double) * (size_t)(C > 0 ? C : 1));
  if (dS1) memcpy(DS, dS1, sizeof(double) * nS);
  if (dz1) memcpy(DZ, dz1, sizeof(double) * (size_t)d);
  memset(dq, 0, sizeof(double) * (size_t)L * d);
  memset(dk, 0, sizeof(double) * (size_t)L * d);
  memset(dv, 0, sizeof(double) * (size_t)L * d);
  const double inv_sqrt_d = 1.0 / sqrt((double)d);
  for (int g = ng - 1; g >= 0; --g) {
    int g0 = g * C, g1 = g0 + C < L ? g0 + C : L;
    const double *S = Sg + (size_t)g * nS, *z = zg + (size_t)g * d;
    /* the group's keys and values entered the sums that every later group read */
    for (int t = g0; t < g1; ++t)
      for (int i = 0; i < d; ++i) {
        double kti = k[(size_t)t * d + i], fk = oracle_phi(kti);
        double dfk = DZ[i];
        for (int c = 0; c < d; ++c) {
          dfk += DS[(size_t)i * d + c] * v[(size_t)t * d + c];
          dv[(size_t)t * d + c] += fk * DS[(size_t)i * d + c];
        }
        dk[(size_t)t * d + i] += dfk * dphi(kti);
      }
    memset(gS, 0, sizeof(double) * nS);
    memset(gz, 0, sizeof(double) * (size_t)d);
    for (int t = g0; t < g1; ++t) {
      const double *qt = q + (size_t)t * d, *dot_ = dout + (size_t)t * d;
      /* grouped branch */
      for (int i = 0; i < d; ++i) fq[i] = oracle_phi(qt[i]);
      double gden = dot(fq, z, d) + eps;
      if (gden != 0.0) {
        double nd = 0.0;
        for (int c = 0; c < d; ++c) {
          double a = 0.0;
          for (int i = 0; i < d; ++i) a += fq[i] * S[(size_t)i * d + c];
          gnum[c] = a;
          dnum[c] = alpha * dot_[c] / gden;
          nd += a * dot_[c];
        }
        double dden = -alpha * nd / (gden * gden);
        for (int i = 0; i < d; ++i) {
          double dfq = z[i] * dden;
          for (int c = 0; c < d; ++c) {
            dfq += S[(size_t)i * d + c] * dnum[c];
            gS[(size_t)i * d + c] += fq[i] * dnum[c];
          }
          gz[i] += fq[i] * dden;
          dq[(size_t)t * d + i] += dfq * dphi(qt[i]);
        }
      }
      /* local branch: the softmax weights of the group's tokens up to t, as in the forward */
      double top = -INFINITY, mass = 0.0;
      for (int i = g0; i <= t; ++i) {
        p[i - g0] = dot(qt, k + (size_t)i * d, d) * inv_sqrt_d;
        if (p[i - g0] > top) top = p[i - g0];
      }
      for (int i = g0; i <= t; ++i) {
        p[i - g0] = exp(p[i - g0] - top);
        mass += p[i - g0];
      }
      double pbar = 0.0;
      for (int i = g0; i <= t; ++i) {
        p[i - g0] /= mass;
        dp[i - g0] = dot(dot_, v + (size_t)i * d, d);
        pbar += p[i - g0] * dp[i - g0];
      }
      for (int i = g0; i <= t; ++i) {
        double dl = p[i - g0] * (dp[i - g0] - pbar);
        for (int f = 0; f < d; ++f) {
          dq[(size_t)t * d + f] += dl * k[(size_t)i * d + f] * inv_sqrt_d;
          dk[(size_t)i * d + f] += dl * qt[f] * inv_sqrt_d;
          dv[(size_t)i * d + f] += p[i - g0] * dot_[f];
        }
      }
    }
    for (size_t e = 0; e < nS; ++e) DS[e] += gS[e];
    for (int i = 0; i < d; ++i) DZ[i] += gz[i];
  }
  if (dS0) memcpy(dS0, DS, sizeof(double) * nS);
  if (dz0) memcpy(dz0, DZ, sizeof(double) * (size_t)d);
  /* masked DWConv: out[t][c] += w[c][j] * vext[t-j][c] */
  if (dhist0) memset(dhist0, 0, sizeof(double) * (size_t)(Kc - 1) * d);
  for (int t = 0; t < L; ++t)
    for (int c = 0; c < d; ++c)
      for (int j = 0; j < Kc; ++j) {
        int s2 = t - j;
        double go = dout[(size_t)t * d + c];
        if (s2 >= 0) {
          dv[(size_t)s2 * d + c] += w[(size_t)c * Kc + j] * go;
          dw[(size_t)c * Kc + j] += go * v[(size_t)s2 * d + c];
        } else if (hist0 && s2 >= -(Kc - 1)) {
          if (dhist0) dhist0[(size_t)(Kc - 1 + s2) * d + c] += w[(size_t)c * Kc + j] * go;
          dw[(size_t)c * Kc + j] += go * hist0[(size_t)(Kc - 1 + s2) * d + c];
        }
      }
  free(Sg); free(zg); free(DS); free(DZ); free(gS); free(gz); free(fq); free(gnum);
  free(dnum); free(p); free(dp);
}

/* dw: [H, d, Kc], summed over the batch rows.  dS1, dz1 (gradient flowing into the state
 * handed back) and S0, z0, hist0 may be NULL (zeros); dS0, dz0, dhist0 may be NULL. */
int oracle_prefill_grouped_backward(int B, int H, int L, int d, int Kc, int C, double eps,
                                    double alpha, const double *q, const double *k,
                                    const double *v, const double *w, const double *S0,
                                    const double *z0, const double *hist0,
                                    const double *dout, const double *dS1,
                                    const double *dz1, double *dq, double *dk, double *dv,
                                    double *dw, double *dS0, double *dz0, double *dhist0) {
  if (B < 0 || H < 1 || L < 0 || d < 1 || Kc < 1 || C < 1) return 1;
  size_t nS = (size_t)d * d, nh = (size_t)(Kc - 1) * d, nw = (size_t)d * Kc;
  double *dw_bh = (double *)calloc((size_t)(B * H > 0 ? B * H : 1) * nw, sizeof(double));
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * H; ++bh) {
    int h = bh % H;
    size_t o = (size_t)bh * L * d;
    grouped_backward_head(L, d, Kc, C, eps, alpha, q + o, k + o, v + o, w + (size_t)h * nw,
                          S0 ? S0 + bh * nS : NULL, z0 ? z0 + (size_t)bh * d : NULL,
                          hist0 ? hist0 + bh * nh : NULL, dout + o,
                          dS1 ? dS1 + bh * nS : NULL, dz1 ? dz1 + (size_t)bh * d : NULL,
                          dq + o, dk + o, dv + o, dw_bh + (size_t)bh * nw,
                          dS0 ? dS0 + bh * nS : NULL, dz0 ? dz0 + (size_t)bh * d : NULL,
                          dhist0 ? dhist0 + bh * nh : NULL);
  }
  memset(dw, 0, sizeof(double) * (size_t)H * nw);
  for (int bh = 0; bh < B * H; ++bh)
    for (size_t e = 0; e < nw; ++e) dw[(size_t)(bh % H) * nw + e] += dw_bh[(size_t)bh * nw + e];
  free(dw_bh);
  return 0;
}

/* Verification of kk draft tokens (Sec. 4.2): defined as kk recurrent steps
 * taken one after the other from the SAME incoming state; all kk outputs are
 * produced; the state handed back is the one reached after the first
 * n_commit[b] steps (drafts beyond that were rejected).  n_commit == NULL
 * means every draft is kept.  S, z, hist are updated in place. */
int oracle_verify(int B, int H, int kk, int d, int Kc, double eps,
                  const double *q, const double *k, const double *v,
                  const double *w, double *S, double *z, double *hist,
                  const int *n_commit, double *out) {
  if (B < 0 || H < 1 || kk < 0 || d < 1 || Kc < 1) return 1;
  if (n_commit)
    for (int b = 0; b < B; ++b)
      if (n_commit[b] < 0 || n_commit[b] > kk) return 2;
  size_t nS = (size_t)d * d, nh = (size_t)(Kc - 1) * d;
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * H; ++bh) {
    int b = bh / H, h = bh % H;
    int n = n_commit ? n_commit[b] : kk;
    size_t o = (size_t)bh * kk * d;
    double *Sw = (double *)malloc(sizeof(double) * nS);
    double *zw = (double *)malloc(sizeof(double) * (size_t)d);
    double *hw = (double *)malloc(sizeof(double) * (nh ? nh : 1));
    load_state(d, Kc, S + bh * nS, z + (size_t)bh * d,
               nh ? hist + bh * nh : NULL, Sw, zw, hw);
    for (int j = 0; j < kk; ++j) {
      step_head(d, Kc, eps, q + o + (size_t)j * d, k + o + (size_t)j * d,
                v + o + (size_t)j * d, w + (size_t)h * d * Kc, Sw, zw, hw,
                out + o + (size_t)j * d);
      if (j + 1 == n) { /* state after the last accepted draft */
        memcpy(S + bh * nS, Sw, sizeof(double) * nS);
        memcpy(z + (size_t)bh * d, zw, sizeof(double) * d);
        if (nh) memcpy(hist + bh * nh, hw, sizeof(double) * nh);
      }
    }
    free(Sw); free(zw); free(hw);
  }
  return 0;
}

/* ---- generation with the three-branch form (Sec. 4.1 block, Sec. 3 decode phase) ----
 * One token at a time, per head.  What is carried between tokens: S and z over the
 * COMPLETED groups only, the conv history, and the raw key and value rows of the
 * current, still incomplete group (kwin, vwin: [C][d], rows 0..fill-1 in use;
 * fill is a property of the batch row).  A step with (q, k, v):
 *   the token joins its group (row fill of the window);
 *   grouped branch from S, z (none of the current group is in them);
 *   local branch: softmax over the window rows 0..fill (the token itself included);
 *   conv over (hist ++ v);  out = alpha * grouped + local + conv;
 *   if the group is now complete (C rows) its keys and values enter S and z and the
 *   window starts again from row 0.
 * This is the same function of the token sequence as grouped_head: a sequence fed
 * token by token from an empty state gives grouped_head's outputs. */
static void grouped_step_head(int d, int Kc, int C, double eps, double alpha,
                              const double *q, const double *k, const double *v,
                              const double *w, double *S, double *z, double *hist,
                              double *kwin, double *vwin, int *fill, double *out) {
  double *fq = (double *)malloc(sizeof(double) * (size_t)d);
  double *wt = (double *)malloc(sizeof(double) * (size_t)C);
  int n = *fill;
  memcpy(kwin + (size_t)n * d, k, sizeof(double) * (size_t)d);
  memcpy(vwin + (size_t)n * d, v, sizeof(double) * (size_t)d);
  for (int i = 0; i < d; ++i) fq[i] = oracle_phi(q[i]);
  double gden = dot(fq, z, d) + eps;
  const double inv_sqrt_d = 1.0 / sqrt((double)d);
  double top = -INFINITY, mass = 0.0;
  for (int r = 0; r <= n; ++r) {
    wt[r] = dot(q, kwin + (size_t)r * d, d) * inv_sqrt_d;
    if (wt[r] > top) top = wt[r];
  }
  for (int r = 0; r <= n; ++r) {
    wt[r] = exp(wt[r] - top);
    mass += wt[r];
  }
  for (int c = 0; c < d; ++c) {
    double gnum = 0.0, loc = 0.0;
    for (int i = 0; i < d; ++i) gnum += fq[i] * S[(size_t)i * d + c];
    for (int r = 0; r <= n; ++r) loc += wt[r] * vwin[(size_t)r * d + c];
    double u = w[(size_t)c * Kc + 0] * v[c];
    for (int j = 1; j < Kc; ++j) u += w[(size_t)c * Kc + j] * hist[(size_t)(Kc - 1 - j) * d + c];
    out[c] = alpha * (gden != 0.0 ? gnum / gden : 0.0) + loc / mass + u;
  }
  for (int r = 0; r + 1 < Kc - 1; ++r)
    memcpy(hist + (size_t)r * d, hist + (size_t)(r + 1) * d, sizeof(double) * d);
  if (Kc > 1) memcpy(hist + (size_t)(Kc - 2) * d, v, sizeof(double) * d);
  n += 1;
  if (n == C) { /* the group is complete: it becomes part of the sums */
    for (int r = 0; r < C; ++r)
      for (int i = 0; i < d; ++i) {
        double fk = oracle_phi(kwin[(size_t)r * d + i]);
        z[i] += fk;
        for (int c = 0; c < d; ++c) S[(size_t)i * d + c] += fk * vwin[(size_t)r * d + c];
      }
    n = 0;
  }
  *fill = n;
  free(fq); free(wt);
}

/* kk draft tokens per head with the three-branch form: kk steps as above from the
 * same incoming state; all kk outputs are produced; the state handed back (S, z,
 * hist, kwin, vwin, fill, all updated in place) is the one reached after the first
 * n_commit[b] steps (NULL: all kk).  fill: [B], each in 0..C-1.  Window rows at or
 * beyond fill are not read and, unless a kept draft lands on them, not written. */
int oracle_verify_grouped(int B, int H, int kk, int d, int Kc, int C, double eps,
                          double alpha, const double *q, const double *k,
                          const double *v, const double *w, double *S, double *z,
                          double *hist, double *kwin, double *vwin, int *fill,
                          const int *n_commit, double *out) {
  if (B < 0 || H < 1 || kk < 0 || d < 1 || Kc < 1 || C < 1) return 1;
  for (int b = 0; b < B; ++b) {
    if (n_commit && (n_commit[b] < 0 || n_commit[b] > kk)) return 2;
    if (fill[b] < 0 || fill[b] >= C) return 3;
  }
  size_t nS = (size_t)d * d, nh = (size_t)(Kc - 1) * d, nw = (size_t)C * d;
  int *fill_after = (int *)malloc(sizeof(int) * (size_t)(B > 0 ? B : 1));
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * H; ++bh) {
    int b = bh / H, h = bh % H;
    int n = n_commit ? n_commit[b] : kk;
    size_t o = (size_t)bh * kk * d;
    double *Sw = (double *)malloc(sizeof(double) * nS);
    double *zw = (double *)malloc(sizeof(double) * (size_t)d);
    double *hw = (double *)malloc(sizeof(double) * (nh ? nh : 1));
    double *kw = (double *)malloc(sizeof(double) * nw);
    double *vw = (double *)malloc(sizeof(double) * nw);
    int fw = fill[b];
    load_state(d, Kc, S + bh * nS, z + (size_t)bh * d, nh ? hist + bh * nh : NULL, Sw, zw, hw);
    memcpy(kw, kwin + bh * nw, sizeof(double) * nw);
    memcpy(vw, vwin + bh * nw, sizeof(double) * nw);
    for (int j = 0; j < kk; ++j) {
      grouped_step_head(d, Kc, C, eps, alpha, q + o + (size_t)j * d, k + o + (size_t)j * d,
                        v + o + (size_t)j * d, w + (size_t)h * d * Kc, Sw, zw, hw, kw, vw, &fw,
                        out + o + (size_t)j * d);
      if (j + 1 == n) { /* state after the last accepted draft */
        memcpy(S + bh * nS, Sw, sizeof(double) * nS);
        memcpy(z + (size_t)bh * d, zw, sizeof(double) * d);
        if (nh) memcpy(hist + bh * nh, hw, sizeof(double) * nh);
        memcpy(kwin + bh * nw, kw, sizeof(double) * nw);
        memcpy(vwin + bh * nw, vw, sizeof(double) * nw);
        if (h == 0) fill_after[b] = fw;
      }
    }
    if (n == 0 && h == 0) fill_after[b] = fill[b];
    free(Sw); free(zw); free(hw); free(kw); free(vw);
  }
  for (int b = 0; b < B; ++b) fill[b] = fill_after[b];
  free(fill_after);
  return 0;
}

/* One generated token: a verification of a single draft that is always kept. */
/*
 * Tree-structured verification (Sec. 4.2, "Proposed Solution").  The n candidate
 * tokens of one speculation step form a tree that hangs off the verified
 * sequence: parent[i] < i is the candidate that precedes candidate i in time,
 * -1 if candidate i directly follows the verified sequence.  Candidates of the
 * same time step are siblings; they do not see each other.  Candidate i may
 * use the verified state and the candidates on its own root path (its
 * ancestors and itself), and its convolution window is that path read
 * backwards in time, continuing into the verified history (the paper's
 * example: with kernel 3 the candidate at step t1 covers {t0, t1}, not the
 * unchosen candidate of step t1 that happens to be stored next to it).
 *
 * Written out from that definition: for every candidate the visible tokens
 * are listed (path[0] = the candidate itself, path[1] = its parent, ...) and
 * every sum is taken over that list.  accept[b] names the candidate whose root
 * path becomes part of the verified sequence of batch row b (-1: none); the
 * state is advanced by exactly the tokens of that path, oldest first.
 * parent is shared by all batch rows and heads (the tree shape of a
 * speculation step is fixed in advance).
 */
int oracle_verify_tree(int B, int H, int n, int d, int Kc, double eps,
                       const double *q, const double *k, const double *v,
                       const int *parent, const double *w, double *S, double *z,
                       double *hist, const int *accept, double *out) {
  if (B < 0 || H < 1 || n < 0 || d < 1 || Kc < 1) return 1;
  for (int i = 0; i < n; ++i)
    if (parent[i] < -1 || parent[i] >= i) return 2;
  if (accept)
    for (int b = 0; b < B; ++b)
      if (accept[b] < -1 || accept[b] >= n) return 2;
  size_t nS = (size_t)d * d, nh = (size_t)(Kc - 1) * d;
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < B * H; ++bh) {
    int b = bh / H, h = bh % H;
    size_t o = (size_t)bh * n * d;
    const double *qh = q + o, *kh = k + o, *vh = v + o, *wh = w + (size_t)h * d * Kc;
    double *Sh = S + bh * nS, *zh = z + (size_t)bh * d;
    double *hh = nh ? hist + bh * nh : NULL;
    double *fq = (double *)malloc(sizeof(double) * (size_t)(n ? n : 1) * d);
    double *fk = (double *)malloc(sizeof(double) * (size_t)(n ? n : 1) * d);
    int *path = (int *)malloc(sizeof(int) * (size_t)(n ? n : 1));
    for (size_t e = 0; e < (size_t)n * d; ++e) {
      fq[e] = oracle_phi(qh[e]);
      fk[e] = oracle_phi(kh[e]);
    }
    for (int i = 0; i < n; ++i) {
      int len = 0;
      for (int a = i; a >= 0; a = parent[a]) path[len++] = a;
      const double *fqi = fq + (size_t)i * d;
      double den = eps;
      for (int f = 0; f < d; ++f) den += fqi[f] * zh[f];
      for (int c = 0; c < d; ++c) {
        double acc = 0.0;
        for (int f = 0; f < d; ++f) acc += fqi[f] * Sh[(size_t)f * d + c];
        out[o + (size_t)i * d + c] = acc; /* numerator so far: the verified state */
      }
      for (int m = 0; m < len; ++m) {
        int a = path[m];
        double sim = 0.0;
        for (int f = 0; f < d; ++f) sim += fqi[f] * fk[(size_t)a * d + f];
        den += sim;
        for (int c = 0; c < d; ++c) out[o + (size_t)i * d + c] += sim * vh[(size_t)a * d + c];
      }
      for (int c = 0; c < d; ++c) {
        double u = 0.0;
        for (int t = 0; t < Kc; ++t) {
          /* t steps back in time from candidate i: on the path, else (t - len + 1) rows into the history */
          double x = t < len ? vh[(size_t)path[t] * d + c]
                             : hh[(size_t)(Kc - 1 - (t - len + 1)) * d + c];
          u += wh[(size_t)c * Kc + t] * x;
        }
        out[o + (size_t)i * d + c] = out[o + (size_t)i * d + c] / den + u;
      }
    }
    int acc_node = accept ? accept[b] : -1;
    if (acc_node >= 0) {
      int len = 0;
      for (int a = acc_node; a >= 0; a = parent[a]) path[len++] = a;
      for (int m = len - 1; m >= 0; --m) { /* oldest first */
        int a = path[m];
        for (int f = 0; f < d; ++f) {
          double x = fk[(size_t)a * d + f];
          zh[f] += x;
          for (int c = 0; c < d; ++c) Sh[(size_t)f * d + c] += x * vh[(size_t)a * d + c];
        }
      }
      if (nh) { /* last Kc-1 rows of (history ++ accepted path) */
        double *nw = (double *)malloc(sizeof(double) * nh);
        for (int r = 0; r < Kc - 1; ++r) {
          int back = Kc - 1 - r; /* 1 = newest */
          const double *src = back <= len ? vh + (size_t)path[back - 1] * d
                                          : hh + (size_t)(Kc - 1 - (back - len)) * d;
          memcpy(nw + (size_t)r * d, src, sizeof(double) * d);
        }
        memcpy(hh, nw, sizeof(double) * nh);
        free(nw);
      }
    }
    free(fq); free(fk); free(path);
  }
  return 0;
}

int oracle_decode(int B, int H, int d, int Kc, double eps, const double *q,
                  const double *k, const double *v, const double *w, double *S,
                  double *z, double *hist, double *out) {
  return oracle_verify(B, H, 1, d, Kc, eps, q, k, v, w, S, z, hist, NULL, out);
}

/* Number of threads the parallel loops above will use (for reporting). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
void oracle_set_num_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int oracle_num_threads(void) { return 1; }
void oracle_set_num_threads(int n) { (void)n; }
#endif
