/*
 * fp64 CPU oracle for the routed FFN of SPT (arXiv 2312.10365), forward and backward.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call this; it shares no
 * code with the HIP kernels.  It is deliberately plain: one token at a time, one
 * hidden unit at a time, sums taken in index order in double precision.
 *
 * What it computes (paper section 4.2 "Dynamic routing", Eq. 4, Algorithm 4):
 *   route     x_R = x W_R (+ b_R), activate the k blocks with the largest key, where
 *             key = logit rounded once to fp32 (or its absolute value when flags bit0
 *             is set: the literal "largest magnitude" reading).  Equal keys: the lower
 *             block index wins.  Ids are returned ascending.
 *   bucket    Algorithm 4's per-block token selection written as one stable counting
 *             sort of the (token, slot) pairs by block id.
 *   forward   Eq. 4 restricted to the activated blocks:
 *             y_t = sum_{b in S(t)} W2[b]^T act(W1[b] x_t); block outputs ADD (Alg. 4's
 *             assignment is only right for one block per token) and carry no gate.
 *   backward  the derivative of the above with the routing held fixed.
 *
 * Storage: W1[N][Bs][d], W2[N][Bs][d] hold, per block, Bs adjacent hidden units: row u
 * of W1[b] is the inner-projection weight vector of unit b*Bs+u, row u of W2[b] its
 * outer-projection weight vector.  Inputs arrive as float (exact widenings of bf16 /
 * fp32 values); all arithmetic is double.
 *
 * Pins: see tests/test_oracle_pins.py (dense FFN with k=N through numpy matmul, masked
 * dense FFN + autograd, finite differences, brute-force loops, full-sort top-k,
 * activation closed forms, bucket invariants).  No function here is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ACT_GELU 0
#define ACT_RELU 1

int spt_oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* GELU(z) = z Phi(z), Phi the standard normal CDF (erf form). */
static double act_fn(double z, int act) {
  if (act == ACT_RELU) return z > 0.0 ? z : 0.0;
  return 0.5 * z * (1.0 + erf(z * M_SQRT1_2));
}

/* d/dz GELU(z) = Phi(z) + z phi(z), phi the standard normal density. */
static double act_grad(double z, int act) {
  if (act == ACT_RELU) return z > 0.0 ? 1.0 : 0.0;
  const double inv_sqrt_2pi = 0.39894228040143267794;
  return 0.5 * (1.0 + erf(z * M_SQRT1_2)) + z * inv_sqrt_2pi * exp(-0.5 * z * z);
}

void spt_oracle_act(const double* z, int64_t n, int act, double* out, double* grad) {
  for (int64_t i = 0; i < n; ++i) {
    if (out) out[i] = act_fn(z[i], act);
    if (grad) grad[i] = act_grad(z[i], act);
  }
}

/* Route network (section 4.2): L[t][b] = sum_i X[t][i] W_r[i][b] + b_r[b], i ascending. */
void spt_oracle_router_logits(const float* X, const float* W_r, const float* b_r,
                              int T, int d, int N, double* L) {
#pragma omp parallel for schedule(static)
  for (int t = 0; t < T; ++t) {
    double* Lt = L + (size_t)t * N;
    for (int b = 0; b < N; ++b) Lt[b] = 0.0;
    for (int i = 0; i < d; ++i) {
      const double x = (double)X[(size_t)t * d + i];
      const float* w = W_r + (size_t)i * N;
      for (int b = 0; b < N; ++b) Lt[b] += x * (double)w[b];
    }
    if (b_r)
      for (int b = 0; b < N; ++b) Lt[b] += (double)b_r[b];
  }
}

static int cmp_desc(const void* a, const void* b) {
  const double x = *(const double*)a, y = *(const double*)b;
  return (x < y) - (x > y);
}

/* Top-k of the fp32 keys; ties to the lower index; ids ascending.
 * margin[t] = (k-th largest) - ((k+1)-th largest) of the fp64 keys, +inf when k == N. */
void spt_oracle_topk(const double* L, int T, int N, int k, int flags,
                     int32_t* idx, double* margin) {
#pragma omp parallel
  {
    float* key = (float*)malloc(sizeof(float) * (size_t)N);
    double* key64 = (double*)malloc(sizeof(double) * (size_t)N);
    char* taken = (char*)malloc((size_t)N);
#pragma omp for schedule(static)
    for (int t = 0; t < T; ++t) {
      const double* Lt = L + (size_t)t * N;
      for (int b = 0; b < N; ++b) {
        const float l32 = (float)Lt[b];
        key[b] = (flags & 1) ? fabsf(l32) : l32;
        key64[b] = (flags & 1) ? fabs(Lt[b]) : Lt[b];
        taken[b] = 0;
      }
      for (int r = 0; r < k; ++r) {
        int best = -1;
        for (int b = 0; b < N; ++b) {
          if (taken[b]) continue;
          if (best < 0 || key[b] > key[best]) best = b; /* strict: lower index keeps ties */
        }
        taken[best] = 1;
      }
      int j = 0;
      for (int b = 0; b < N; ++b)
        if (taken[b]) idx[(size_t)t * k + j++] = b;
      if (margin) {
        if (k >= N) {
          margin[t] = INFINITY;
        } else {
          qsort(key64, (size_t)N, sizeof(double), cmp_desc);
          margin[t] = key64[k - 1] - key64[k];
        }
      }
    }
    free(key);
    free(key64);
    free(taken);
  }
}

/* Stable counting sort of pairs p = t*k + j by block id idx[p].
 * offsets[b] = number of pairs with a smaller block id; perm[q] = pair at sorted
 * position q; inv[perm[q]] = q. */
void spt_oracle_bucket(const int32_t* idx, int T, int N, int k,
                       int32_t* offsets, int32_t* perm, int32_t* inv) {
  const int64_t P = (int64_t)T * k;
  int64_t* cursor = (int64_t*)calloc((size_t)N + 1, sizeof(int64_t));
  for (int64_t p = 0; p < P; ++p) cursor[idx[p] + 1]++;
  for (int b = 0; b < N; ++b) cursor[b + 1] += cursor[b];
  for (int b = 0; b <= N; ++b) offsets[b] = (int32_t)cursor[b];
  for (int64_t p = 0; p < P; ++p) {
    const int64_t q = cursor[idx[p]]++;
    perm[q] = (int32_t)p;
    inv[p] = (int32_t)q;
  }
  free(cursor);
}

/* Forward for the listed tokens (tokens == NULL: tokens 0..nt-1).
 * Y[nt][d]; Hpre[nt][k][Bs] (pre-activation, token-major pair order), may be NULL. */
void spt_oracle_ffn_fwd(const float* X, const float* W1, const float* W2, const int32_t* idx,
                        int T, int d, int N, int Bs, int k, int act,
                        const int32_t* tokens, int nt, double* Y, double* Hpre) {
  (void)T; (void)N;
#pragma omp parallel for schedule(dynamic, 1)
  for (int s = 0; s < nt; ++s) {
    const int t = tokens ? tokens[s] : s;
    const float* x = X + (size_t)t * d;
    double* y = Y + (size_t)s * d;
    for (int c = 0; c < d; ++c) y[c] = 0.0;
    for (int j = 0; j < k; ++j) {
      const int b = idx[(size_t)t * k + j];
      for (int u = 0; u < Bs; ++u) {
        const float* w1 = W1 + ((size_t)b * Bs + u) * d;
        const float* w2 = W2 + ((size_t)b * Bs + u) * d;
        double hpre = 0.0;
        for (int i = 0; i < d; ++i) hpre += (double)w1[i] * (double)x[i];
        if (Hpre) Hpre[((size_t)s * k + j) * Bs + u] = hpre;
        const double h = act_fn(hpre, act);
        for (int c = 0; c < d; ++c) y[c] += h * (double)w2[c];
      }
    }
  }
}

/* Input gradient for the listed tokens: dX[nt][d]; dHpre[nt][k][Bs] may be NULL. */
void spt_oracle_ffn_bwd_dx(const float* X, const float* W1, const float* W2, const float* dY,
                           const int32_t* idx, int T, int d, int N, int Bs, int k, int act,
                           const int32_t* tokens, int nt, double* dX, double* dHpre) {
  (void)T; (void)N;
#pragma omp parallel for schedule(dynamic, 1)
  for (int s = 0; s < nt; ++s) {
    const int t = tokens ? tokens[s] : s;
    const float* x = X + (size_t)t * d;
    const float* dy = dY + (size_t)t * d;
    double* dx = dX + (size_t)s * d;
    for (int i = 0; i < d; ++i) dx[i] = 0.0;
    for (int j = 0; j < k; ++j) {
      const int b = idx[(size_t)t * k + j];
      for (int u = 0; u < Bs; ++u) {
        const float* w1 = W1 + ((size_t)b * Bs + u) * d;
        const float* w2 = W2 + ((size_t)b * Bs + u) * d;
        double hpre = 0.0, dh = 0.0;
        for (int i = 0; i < d; ++i) hpre += (double)w1[i] * (double)x[i];
        for (int c = 0; c < d; ++c) dh += (double)w2[c] * (double)dy[c];
        const double g = dh * act_grad(hpre, act);
        if (dHpre) dHpre[((size_t)s * k + j) * Bs + u] = g;
        for (int i = 0; i < d; ++i) dx[i] += (double)w1[i] * g;
      }
    }
  }
}

/* Weight gradients for the listed blocks (blocks == NULL: blocks 0..nb-1):
 * dW1[nb][Bs][d] = sum_t dhpre_u(t) x_t,  dW2[nb][Bs][d] = sum_t h_u(t) dy_t over the
 * tokens that activate the block, t ascending.  Blocks nobody activates stay zero. */
void spt_oracle_ffn_bwd_dw(const float* X, const float* W1, const float* W2, const float* dY,
                           const int32_t* idx, int T, int d, int N, int Bs, int k, int act,
                           const int32_t* blocks, int nb, double* dW1, double* dW2) {
  (void)N;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int s = 0; s < nb; ++s) {
    for (int u = 0; u < Bs; ++u) {
      const int b = blocks ? blocks[s] : s;
      const float* w1 = W1 + ((size_t)b * Bs + u) * d;
      const float* w2 = W2 + ((size_t)b * Bs + u) * d;
      double* g1 = dW1 + ((size_t)s * Bs + u) * d;
      double* g2 = dW2 + ((size_t)s * Bs + u) * d;
      for (int i = 0; i < d; ++i) { g1[i] = 0.0; g2[i] = 0.0; }
      for (int t = 0; t < T; ++t) {
        int hit = 0;
        for (int j = 0; j < k; ++j) hit |= (idx[(size_t)t * k + j] == b);
        if (!hit) continue;
        const float* x = X + (size_t)t * d;
        const float* dy = dY + (size_t)t * d;
        double hpre = 0.0, dh = 0.0;
        for (int i = 0; i < d; ++i) hpre += (double)w1[i] * (double)x[i];
        for (int c = 0; c < d; ++c) dh += (double)w2[c] * (double)dy[c];
        const double h = act_fn(hpre, act);
        const double g = dh * act_grad(hpre, act);
        for (int i = 0; i < d; ++i) g1[i] += g * (double)x[i];
        for (int c = 0; c < d; ++c) g2[c] += h * (double)dy[c];
      }
    }
  }
}

/* ---------------------------------------------------------------------------------------
 * Low-rank adapted routed FFN (paper section 2.2: a projection Y = XW becomes
 * Y = X(W + BC) with W frozen and the rank-r factors B, C trained; section 4.2 routing on
 * top).  The paper does not spell out how the adapters meet the block pruning; the reading
 * taken here: each projection matrix of Eq. 4 is replaced by W + BC as a whole and THEN
 * restricted to the activated blocks, i.e. a pruned hidden unit loses its adapter part too.
 *   inner:  hpre(b,u) = W1[b][u] . x  +  sum_rho C1[rho][b*Bs+u] * (sum_i A1[i][rho] x[i])
 *   outer:  y[c] = sum_{b in S(t)} sum_u h(b,u) * ( W2[b][u][c] + sum_rho B2[b*Bs+u][rho] C2[rho][c] )
 * Adapter storage (row-major): A1[d][r], C1[r][D], B2[D][r], C2[r][d], D = N*Bs.
 * Evaluated one token, one hidden unit at a time, in double.
 * Pins: tests/test_oracle_pins.py (numpy masked-dense FFN on explicitly merged W + BC,
 * torch autograd of it for all five gradients, r = 0 / zero adapters reduce to the base
 * functions above, finite differences). */
void spt_oracle_lora_fwd(const float* X, const float* W1, const float* W2, const float* A1,
                         const float* C1, const float* B2, const float* C2, const int32_t* idx,
                         int T, int d, int N, int Bs, int k, int r, int act,
                         const int32_t* tokens, int nt, double* Y, double* Hpre) {
  (void)T;
  const size_t D = (size_t)N * Bs;
#pragma omp parallel
  {
    double* up = (double*)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
    double* v = (double*)malloc(sizeof(double) * (size_t)(r > 0 ? r : 1));
#pragma omp for schedule(dynamic, 1)
    for (int s = 0; s < nt; ++s) {
      const int t = tokens ? tokens[s] : s;
      const float* x = X + (size_t)t * d;
      double* y = Y + (size_t)s * d;
      for (int c = 0; c < d; ++c) y[c] = 0.0;
      for (int rho = 0; rho < r; ++rho) {
        double a = 0.0;
        for (int i = 0; i < d; ++i) a += (double)x[i] * (double)A1[(size_t)i * r + rho];
        up[rho] = a;
        v[rho] = 0.0;
      }
      for (int j = 0; j < k; ++j) {
        const int b = idx[(size_t)t * k + j];
        for (int u = 0; u < Bs; ++u) {
          const size_t unit = (size_t)b * Bs + u;
          const float* w1 = W1 + unit * d;
          const float* w2 = W2 + unit * d;
          double hpre = 0.0;
          for (int i = 0; i < d; ++i) hpre += (double)w1[i] * (double)x[i];
          for (int rho = 0; rho < r; ++rho) hpre += (double)C1[(size_t)rho * D + unit] * up[rho];
          if (Hpre) Hpre[((size_t)s * k + j) * Bs + u] = hpre;
          const double h = act_fn(hpre, act);
          for (int c = 0; c < d; ++c) y[c] += h * (double)w2[c];
          for (int rho = 0; rho < r; ++rho) v[rho] += h * (double)B2[unit * r + rho];
        }
      }
      for (int rho = 0; rho < r; ++rho)
        for (int c = 0; c < d; ++c) y[c] += v[rho] * (double)C2[(size_t)rho * d + c];
    }
    free(up);
    free(v);
  }
}

/* Gradients of the above with W1, W2 frozen and the routing fixed, over ALL tokens:
 * dX[T][d], dA1[d][r], dC1[r][D], dB2[D][r], dC2[r][d].  Each thread sums the adapter
 * gradients of its tokens; the per-thread sums are then added in thread order. */
void spt_oracle_lora_bwd(const float* X, const float* W1, const float* W2, const float* A1,
                         const float* C1, const float* B2, const float* C2, const float* dY,
                         const int32_t* idx, int T, int d, int N, int Bs, int k, int r, int act,
                         double* dX, double* dA1, double* dC1, double* dB2, double* dC2) {
  const size_t D = (size_t)N * Bs;
  const size_t nA = (size_t)d * r, nC = (size_t)r * D;
  const size_t per = 2 * nA + 2 * nC; /* dA1 | dC1 | dB2 | dC2 */
  int nth = 1;
#ifdef _OPENMP
  nth = omp_get_max_threads();
#endif
  double* scratch = (double*)calloc((size_t)nth * per + 1, sizeof(double));
#pragma omp parallel
  {
    int me = 0;
#ifdef _OPENMP
    me = omp_get_thread_num();
#endif
    double* gA1 = scratch + (size_t)me * per;
    double* gC1 = gA1 + nA;
    double* gB2 = gC1 + nC;
    double* gC2 = gB2 + nC;
    const int rr = r > 0 ? r : 1;
    double* up = (double*)malloc(sizeof(double) * (size_t)rr);
    double* v = (double*)malloc(sizeof(double) * (size_t)rr);
    double* g = (double*)malloc(sizeof(double) * (size_t)rr);
    double* rs = (double*)malloc(sizeof(double) * (size_t)rr);
#pragma omp for schedule(dynamic, 1)
    for (int t = 0; t < T; ++t) {
      const float* x = X + (size_t)t * d;
      const float* dy = dY + (size_t)t * d;
      double* dx = dX + (size_t)t * d;
      for (int i = 0; i < d; ++i) dx[i] = 0.0;
      for (int rho = 0; rho < r; ++rho) {
        double a = 0.0, c2 = 0.0;
        for (int i = 0; i < d; ++i) a += (double)x[i] * (double)A1[(size_t)i * r + rho];
        for (int c = 0; c < d; ++c) c2 += (double)C2[(size_t)rho * d + c] * (double)dy[c];
        up[rho] = a;
        g[rho] = c2;
        v[rho] = 0.0;
        rs[rho] = 0.0;
      }
      for (int j = 0; j < k; ++j) {
        const int b = idx[(size_t)t * k + j];
        for (int u = 0; u < Bs; ++u) {
          const size_t unit = (size_t)b * Bs + u;
          const float* w1 = W1 + unit * d;
          const float* w2 = W2 + unit * d;
          double hpre = 0.0, dh = 0.0;
          for (int i = 0; i < d; ++i) hpre += (double)w1[i] * (double)x[i];
          for (int rho = 0; rho < r; ++rho) hpre += (double)C1[(size_t)rho * D + unit] * up[rho];
          for (int c = 0; c < d; ++c) dh += (double)w2[c] * (double)dy[c];
          for (int rho = 0; rho < r; ++rho) dh += (double)B2[unit * r + rho] * g[rho];
          const double h = act_fn(hpre, act);
          const double gh = dh * act_grad(hpre, act);
          for (int i = 0; i < d; ++i) dx[i] += (double)w1[i] * gh;
          for (int rho = 0; rho < r; ++rho) {
            rs[rho] += (double)C1[(size_t)rho * D + unit] * gh;
            v[rho] += h * (double)B2[unit * r + rho];
            gC1[(size_t)rho * D + unit] += up[rho] * gh;
            gB2[unit * r + rho] += h * g[rho];
          }
        }
      }
      for (int rho = 0; rho < r; ++rho) {
        for (int i = 0; i < d; ++i) {
          dx[i] += (double)A1[(size_t)i * r + rho] * rs[rho];
          gA1[(size_t)i * r + rho] += (double)x[i] * rs[rho];
        }
        for (int c = 0; c < d; ++c) gC2[(size_t)rho * d + c] += v[rho] * (double)dy[c];
      }
    }
    free(up);
    free(v);
    free(g);
    free(rs);
  }
  for (size_t e = 0; e < nA; ++e) { dA1[e] = 0.0; dC2[e] = 0.0; }
  for (size_t e = 0; e < nC; ++e) { dC1[e] = 0.0; dB2[e] = 0.0; }
  for (int th = 0; th < nth; ++th) {
    const double* gA1 = scratch + (size_t)th * per;
    const double* gC1 = gA1 + nA;
    const double* gB2 = gC1 + nC;
    const double* gC2 = gB2 + nC;
    for (size_t e = 0; e < nA; ++e) { dA1[e] += gA1[e]; dC2[e] += gC2[e]; }
    for (size_t e = 0; e < nC; ++e) { dC1[e] += gC1[e]; dB2[e] += gB2[e]; }
  }
  free(scratch);
}
