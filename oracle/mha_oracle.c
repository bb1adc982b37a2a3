/*
 * fp64 CPU oracle for the sparse multi-head attention of SPT (arXiv 2312.10365): section 4.1
 * (PQ sparsification, Eq. 6, Algorithm 1), section 5.1 (Algorithms 2 and 3, CSR with fixed row
 * length).  TEST INFRASTRUCTURE ONLY: nothing on the product path may call this and it shares
 * no code with the HIP kernels.
 *
 * Layout: "sequences" are (batch, head) pairs, s = batch * H + head; Q, K, V are [S][n][dh].
 * Codebooks C[H][M][E][dp] with dp = dh / M are shared by the queries and keys of a head (Eq. 6
 * compares codeword indices, which only means something under shared codebooks).
 *
 * Readings where the paper is silent or its listing cannot be run as printed:
 *  - PQ assignment (Alg. 2 lines 2-3): squared Euclidean distance, ties to the lower index.
 *  - Quantisation error (Alg. 2 lines 4-5): the Euclidean (not squared) distance to the chosen
 *    codeword, the quantity cdist measures; the codebook adjustment that consumes it is an
 *    optimiser step outside this path.
 *  - Top-L selection (Alg. 3): the bucket sort keeps, per score, the first L - 1 keys in index
 *    order (its write pointer stops at the last of L slots, which later arrivals overwrite and
 *    which is never read back), so a score class contributes at most L - 1 keys.
 *  - Reading the buckets back: the printed step to the next lower bucket would read an unwritten
 *    slot whenever that bucket is empty; here empty classes are skipped and, if every class is
 *    exhausted before L keys are found, the remaining entries are -1 (masked out of the softmax).
 *  - No causal or padding mask (none is mentioned); logits are scale * q.k with the scale an
 *    argument (the paper's softmax has no scale: scale = 1).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* codes[v][m] = argmin_e || x[v][m*dp .. ] - C[head(v)][m][e] ||^2; margin[v][m] = second
 * smallest distance minus the smallest (how safe the argmin is); err[v][m] = the quantisation
 * error of Alg. 2 lines 4-5: the Euclidean distance between the sub-vector and the codeword it was
 * given (what the codebook adjustment consumes). */
void mha_oracle_pq_assign(const float* X, const float* C, int S, int H, int n, int dh, int M, int E,
                          uint8_t* codes, double* margin, double* err) {
  const int dp = dh / M;
#pragma omp parallel for schedule(static)
  for (int64_t v = 0; v < (int64_t)S * n; ++v) {
    const int head = (int)((v / n) % H);
    const float* x = X + (size_t)v * dh;
    for (int m = 0; m < M; ++m) {
      double best = INFINITY, second = INFINITY;
      int arg = 0;
      for (int e = 0; e < E; ++e) {
        const float* c = C + (((size_t)head * M + m) * E + e) * dp;
        double dist = 0.0;
        for (int j = 0; j < dp; ++j) {
          const double df = (double)x[m * dp + j] - (double)c[j];
          dist += df * df;
        }
        if (dist < best) { second = best; best = dist; arg = e; }
        else if (dist < second) second = dist;
      }
      codes[(size_t)v * M + m] = (uint8_t)arg;
      if (margin) margin[(size_t)v * M + m] = second - best;
      if (err) err[(size_t)v * M + m] = sqrt(best);
    }
  }
}

/* Top-L selection (section 5.1, Algorithm 3) for every query of every sequence, written from what
 * the algorithm produces rather than from its bucket arrays: the keys of the sequence are ranked
 * by their Eq. 6 score against the query (number of codebooks in which both have the same
 * codeword), highest score first and, within a score, lowest key index first; a score class
 * contributes at most its first L - 1 keys (the sort's buckets have L slots of which the last is
 * a scratch slot that is never read back); the first L keys of that ranking are the row, and
 * rows that run out of keys end in -1.  idx[S][n][L]. */
void mha_oracle_topl(const uint8_t* cq, const uint8_t* ck, int S, int n, int M, int L, int32_t* idx) {
#pragma omp parallel
  {
    int* score = (int*)malloc(sizeof(int) * (size_t)n);
#pragma omp for schedule(static)
    for (int64_t qv = 0; qv < (int64_t)S * n; ++qv) {
      const int s = (int)(qv / n);
      const uint8_t* q = cq + (size_t)qv * M;
      for (int j = 0; j < n; ++j) {
        const uint8_t* kk = ck + ((size_t)s * n + j) * M;
        int same = 0;
        for (int m = 0; m < M; ++m) same += (q[m] == kk[m]);
        score[j] = same;
      }
      int32_t* out = idx + (size_t)qv * L;
      int filled = 0;
      for (int level = M; level >= 0 && filled < L; --level) {
        int from_class = 0;
        for (int j = 0; j < n && filled < L && from_class < L - 1; ++j)
          if (score[j] == level) { out[filled++] = j; ++from_class; }
      }
      while (filled < L) out[filled++] = -1;
    }
    free(score);
  }
}

/* Sparse attention forward over the selected keys (Alg. 1 lines 4-5):
 * A[v][l] = softmax_l(scale * q_v . k_{idx[v][l]}) over the valid entries, Y[v] = sum_l A[v][l] v_{idx}. */
void mha_oracle_attn_fwd(const float* Q, const float* K, const float* V, const int32_t* idx, int S,
                         int n, int dh, int L, double scale, double* A, double* Y) {
#pragma omp parallel for schedule(static)
  for (int64_t v = 0; v < (int64_t)S * n; ++v) {
    const int s = (int)(v / n);
    const float* q = Q + (size_t)v * dh;
    const int32_t* ix = idx + (size_t)v * L;
    double* a = A + (size_t)v * L;
    double mx = -INFINITY;
    for (int l = 0; l < L; ++l) {
      if (ix[l] < 0) { a[l] = -INFINITY; continue; }
      const float* kk = K + ((size_t)s * n + ix[l]) * dh;
      double dot = 0.0;
      for (int c = 0; c < dh; ++c) dot += (double)q[c] * (double)kk[c];
      a[l] = scale * dot;
      if (a[l] > mx) mx = a[l];
    }
    double sum = 0.0;
    for (int l = 0; l < L; ++l) { a[l] = (ix[l] < 0) ? 0.0 : exp(a[l] - mx); sum += a[l]; }
    double* y = Y + (size_t)v * dh;
    for (int c = 0; c < dh; ++c) y[c] = 0.0;
    for (int l = 0; l < L; ++l) {
      a[l] = (sum > 0.0) ? a[l] / sum : 0.0;
      if (ix[l] < 0) continue;
      const float* vv = V + ((size_t)s * n + ix[l]) * dh;
      for (int c = 0; c < dh; ++c) y[c] += a[l] * (double)vv[c];
    }
  }
}

/* Backward of the above with the selection fixed: dQ, dK, dV [S][n][dh]. */
void mha_oracle_attn_bwd(const float* Q, const float* K, const float* V, const float* dY,
                         const int32_t* idx, const double* A, int S, int n, int dh, int L, double scale,
                         double* dQ, double* dK, double* dV) {
  memset(dK, 0, sizeof(double) * (size_t)S * n * dh);
  memset(dV, 0, sizeof(double) * (size_t)S * n * dh);
#pragma omp parallel for schedule(static)
  for (int s = 0; s < S; ++s) {  /* a sequence's keys are only touched by its own queries */
    double* da = (double*)malloc(sizeof(double) * (size_t)L);
    for (int i = 0; i < n; ++i) {
      const size_t v = (size_t)s * n + i;
      const float* q = Q + v * dh;
      const float* dy = dY + v * dh;
      const int32_t* ix = idx + v * L;
      const double* a = A + v * L;
      double dotsum = 0.0;
      for (int l = 0; l < L; ++l) {
        da[l] = 0.0;
        if (ix[l] < 0) continue;
        const float* vv = V + ((size_t)s * n + ix[l]) * dh;
        for (int c = 0; c < dh; ++c) da[l] += (double)dy[c] * (double)vv[c];
        dotsum += a[l] * da[l];
      }
      double* dq = dQ + v * dh;
      for (int c = 0; c < dh; ++c) dq[c] = 0.0;
      for (int l = 0; l < L; ++l) {
        if (ix[l] < 0) continue;
        const size_t kv = (size_t)s * n + ix[l];
        const double ds = a[l] * (da[l] - dotsum) * scale;
        const float* kk = K + kv * dh;
        for (int c = 0; c < dh; ++c) {
          dq[c] += ds * (double)kk[c];
          dK[kv * dh + c] += ds * (double)q[c];
          dV[kv * dh + c] += a[l] * (double)dy[c];
        }
      }
    }
    free(da);
  }
}
