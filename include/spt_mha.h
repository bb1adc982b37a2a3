/*
 * C ABI of the sparse multi-head attention of SPT (arXiv 2312.10365): section 4.1 ("Sparse MHA":
 * PQ sparsification, Eq. 6, Algorithm 1) and section 5.1 (Algorithm 2 "PQ quantization",
 * Algorithm 3 "top-L selection", CSR with a fixed row length L).  Part of libspt.so.
 *
 * A "sequence" is one (batch, head) pair, s = batch * H + head.  Q, K, V, dY, Y, dQ, dK, dV are
 * device pointers to bf16 [S][n][dh], row-major.  Every call validates on the host, enqueues on
 * `stream` (a hipStream_t), never synchronises, never allocates; outputs are overwritten.
 * Return codes are those of spt.h (SPT_OK, SPT_ERR_ARG, SPT_ERR_UNSUPPORTED, SPT_ERR_WORKSPACE,
 * SPT_ERR_HIP).  Supported: dh in {64, 128}, dp = dh / M = 8 (the paper's codeword dimension),
 * E <= 16 codewords (the paper's codebook size), 1 <= L <= 256, L <= n <= 4096.
 */
#ifndef SPT_MHA_H
#define SPT_MHA_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int32_t S;    /* sequences = batch * heads */
  int32_t H;    /* heads: sequence s uses the codebooks of head s % H */
  int32_t n;    /* tokens per sequence */
  int32_t dh;   /* head dimension */
  int32_t M;    /* codebooks per head (dh / M dimensions each) */
  int32_t E;    /* codewords per codebook */
  int32_t L;    /* keys kept per query */
  float scale;  /* logits are scale * q.k (the paper's softmax has none: 1.0f) */
} spt_mha_shape_t;

/* Algorithm 2, lines 2-3, fused: codes[v][m] = index of the codeword of codebook m (of the
 * vector's head) nearest in squared Euclidean distance to sub-vector m of X[v]; ties go to the
 * lower index.  X: bf16 [S][n][dh]; C: fp32 [H][M][E][dh/M]; codes: uint8 [S][n][M].  The
 * distance is evaluated in fp32.  Lines 4-5: err (fp32 [S][n][M], or NULL on the mini-batches that
 * skip them -- the paper adjusts the codebooks every 20th) receives the quantisation error, the
 * Euclidean distance between the sub-vector and the codeword it was given; the codebook
 * adjustment that consumes it is an optimiser step outside this library. */
int spt_mha_pq_assign(const spt_mha_shape_t* shape, const void* X, const float* C, uint8_t* codes,
                      float* err, void* stream);

/* Algorithm 3 with the score of Eq. 6 (number of codebooks in which query and key share the
 * codeword), for every query: idx[v][0..L) = the keys it keeps, int32 positions inside the
 * sequence, -1 where the buckets ran dry.  Semantics of the listing, made explicit: keys are
 * visited in index order; a bucket keeps its first L-1 arrivals readable (its last slot is
 * overwritten by every later arrival and never read); buckets are read from score M down,
 * empty ones skipped.  cq, ck: uint8 [S][n][M] from spt_mha_pq_assign (8-byte aligned, every
 * code below 16); idx: int32 [S][n][L].
 * This idx IS the CSR column array of section 5.1 (row pointer 0, L, 2L, ...). */
int spt_mha_topl(const spt_mha_shape_t* shape, const uint8_t* cq, const uint8_t* ck, int32_t* idx,
                 void* stream);

/* Algorithm 1, lines 4-5 (SDDMM, softmax over the kept keys, SpMM), one pass:
 * A[v][l] = softmax_l(scale * Q[v] . K[idx[v][l]]) over the entries with idx >= 0 (0 elsewhere),
 * Y[v] = sum_l A[v][l] V[idx[v][l]].  A: fp32 [S][n][L] (kept for the backward pass).  An idx
 * entry outside [0, n) counts as -1; a row must not name the same key twice (spt_mha_topl never
 * does). */
int spt_mha_attn_fwd(const spt_mha_shape_t* shape, const void* Q, const void* K, const void* V,
                     const int32_t* idx, float* A, void* Y, void* stream);

/* Backward of spt_mha_attn_fwd with the selection held fixed: dQ, dK, dV (bf16 [S][n][dh]) from
 * dY.  Deterministic: a key's gradient is summed over the queries that kept it in an order that
 * depends on idx alone (no floating-point atomics).  ws: spt_mha_workspace_bytes(shape) bytes. */
int spt_mha_attn_bwd(const spt_mha_shape_t* shape, const void* Q, const void* K, const void* V,
                     const void* dY, const int32_t* idx, const float* A, void* dQ, void* dK, void* dV,
                     void* ws, size_t ws_bytes, void* stream);

/* Bytes of workspace spt_mha_attn_bwd needs (0 for an unsupported shape). */
size_t spt_mha_workspace_bytes(const spt_mha_shape_t* shape);

#ifdef __cplusplus
}
#endif
#endif /* SPT_MHA_H */
