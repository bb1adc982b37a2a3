/*
 * libspt -- routed feed-forward network of SPT (arXiv 2312.10365) on one MI355X (gfx950).
 *
 * C ABI.  Every pointer below is a DEVICE pointer unless it says "host".  The library
 * never allocates, frees or keeps a pointer: inputs, outputs and workspace belong to the
 * caller.  Every call validates its arguments on the host, then only enqueues kernels on
 * `stream` (a hipStream_t passed as void*; NULL = the default stream) and returns without
 * synchronising.  Outputs are overwritten, never accumulated into.  Same inputs give
 * bit-identical outputs on every run (no floating-point atomics anywhere).
 *
 * Notation (paper section 4.2 -> here): T tokens; d embedding width; the D = N*Bs hidden
 * units of the FFN are organised into N groups ("blocks") of Bs adjacent units (the
 * paper's G groups of D/G rows); each token activates k of them (the paper's G').
 * A "pair" is one (token, activated block): p = t*k + j, P = T*k pairs.
 *
 * Layouts, all row-major and dense:
 *   X, dY, Y, dX   bf16 [T, d]
 *   W_r            fp32 [d, N]        route network, x_R = x W_R
 *   W1             bf16 [N, Bs, d]    row u of block b = inner-projection weights of hidden
 *                                     unit b*Bs+u (a column of Eq. 4's W_I)
 *   W2             bf16 [N, Bs, d]    row u of block b = outer-projection weights of the
 *                                     same unit (a row of Eq. 4's W_O)
 *   idx            int32 [T, k]       activated block ids per token, ascending
 *   offsets        int32 [N+1]        bucket b owns sorted positions offsets[b]..offsets[b+1]
 *   perm           int32 [P]          sorted position -> pair id
 *   inv            int32 [P]          pair id -> sorted position
 *   Hsave          bf16 [P, Bs]       pre-activation of every pair, in sorted (bucket) order
 *   dW1, dW2       fp32 [N, Bs, d]
 *
 * Supported sizes: d % 64 == 0, Bs % 32 == 0, 1 <= k <= N <= 1024; the pair count T*k and the
 * hidden width N*Bs must each fit int32 (tensor elements are addressed with 64-bit offsets, so
 * T*k*d may exceed it).  Other sizes return SPT_ERR_UNSUPPORTED (a size the kernels do not
 * cover) or SPT_ERR_ARG (a size that makes no sense), and nothing is launched.
 */
#ifndef SPT_H
#define SPT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
  int32_t T, d, N, Bs, k;
  int32_t act;   /* SPT_ACT_GELU: z*Phi(z), erf form.  SPT_ACT_RELU: Eq. 4's activation */
  int32_t flags; /* SPT_FLAG_ABS_LOGIT: route on |logit| ("largest magnitude" read literally) */
} spt_shape_t;

#define SPT_ACT_GELU 0
#define SPT_ACT_RELU 1
#define SPT_FLAG_ABS_LOGIT 1

#define SPT_OK 0
#define SPT_ERR_ARG (-1)         /* null or misaligned pointer, T<1, k<1, k>N, size overflow   */
#define SPT_ERR_UNSUPPORTED (-2) /* d%64, Bs%32, N>1024, unknown act or flag bit               */
#define SPT_ERR_WORKSPACE (-3)   /* ws_bytes smaller than spt_workspace_bytes() says           */
#define SPT_ERR_HIP (-4)         /* a launch failed; the HIP error is left for hipGetLastError */
#define SPT_ERR_LIMIT (-5)       /* spt_bucket_tokens_noalloc only: shape beyond its fixed scratch */
/* On any error nothing has been launched except for SPT_ERR_HIP, where earlier kernels of
 * the same call may already be queued. */

#define SPT_WS_BUCKET 0
#define SPT_WS_FWD 1
#define SPT_WS_BWD 2
#define SPT_WS_ROUTER 3
#define SPT_WS_LORA_FWD 4
#define SPT_WS_LORA_BWD 5
#define SPT_WS_BALANCE 6
#define SPT_WS_SCHEDULE 7   /* the buffer spt_build_schedule fills */

/* Bytes of caller-provided device workspace a call needs (`which` = SPT_WS_*).
 * Returns 0 for an invalid shape.  Workspace needs 256-byte alignment. */
size_t spt_workspace_bytes(const spt_shape_t* shape, int which);

/* Route network and block selection (section 4.2, "Dynamic routing").
 * logit[t][b] = sum_i X[t][i]*W_r[i][b] + b_r[b], accumulated in fp64 and rounded once to
 * fp32; key = logit (or |logit| with SPT_FLAG_ABS_LOGIT); the k blocks with the largest
 * keys are activated, equal keys resolved in favour of the lower block id; ids are written
 * ascending.  Inputs must be finite.
 *   X      in   bf16 [T,d]
 *   W_r    in   fp32 [d,N]
 *   b_r    in   fp32 [N] or NULL (no bias)
 *   idx    out  int32 [T,k]
 *   logits out  fp32 [T,N] or NULL (diagnostic copy of the fp32 logits)
 *   ws: spt_workspace_bytes(shape, SPT_WS_ROUTER) bytes (holds the logits between the two
 *       kernels; not touched when `logits` is given).                               */
int spt_router_topk(const spt_shape_t* shape, const void* X, const float* W_r,
                    const float* b_r, int32_t* idx, float* logits, void* ws, size_t ws_bytes,
                    void* stream);

/* Token batching by activated block (Algorithm 4's per-block token selection done once
 * for all blocks): stable counting sort of the pairs p = t*k+j by idx[p].
 * Every idx value must lie in [0,N) and each token's ids must be distinct; ids out of
 * range are ignored by the histogram and leave perm/inv entries unwritten.
 *   idx in int32 [T,k];  offsets out [N+1];  perm out [P];  inv out [P]
 *   ws: spt_workspace_bytes(shape, SPT_WS_BUCKET) bytes.                              */
int spt_bucket_tokens(const spt_shape_t* shape, const int32_t* idx, int32_t* offsets,
                      int32_t* perm, int32_t* inv, void* ws, size_t ws_bytes, void* stream);

/* spt_bucket_tokens for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same inputs, outputs and results as spt_bucket_tokens; the per-chunk histogram
 * table lives in a fixed 1 MiB array inside the library instead (one copy per GPU, held until
 * the process ends), so the call allocates nothing and takes no workspace.
 * Limit: ceil(T / 128) * N <= 262144 table entries (e.g. T = 262144 tokens with N = 128
 * blocks); larger shapes return SPT_ERR_LIMIT and launch nothing.
 * All calls on one GPU share that array: calls that overlap in time on the same GPU (two
 * streams, two threads) race; calls on one stream, or otherwise ordered, are safe.  Nothing
 * needs clearing between calls (the first kernel of a call writes every entry the others read). */
int spt_bucket_tokens_noalloc(const spt_shape_t* shape, const int32_t* idx, int32_t* offsets,
                              int32_t* perm, int32_t* inv, void* stream);

/* Forward (Eq. 4 restricted to activated blocks; Algorithm 4 with block outputs added):
 *   y_t = sum_{b in S(t)} W2[b]^T act(W1[b] x_t)
 * Per bucket: gather-fused up-projection GEMM (bf16 MFMA, fp32 accumulate) + activation, then
 * the down-projection.  Blocks of at most 128 units: the down-projection kernel keeps the fp32
 * sum of a token's block outputs in LDS, adds them in ascending block order and rounds once to
 * bf16 (no per-pair rows in memory).  Wider blocks: the down-projection writes one bf16 row per
 * pair and a second kernel adds each token's k rows in fp32, in fixed order, through `inv`.
 * offsets/perm/inv may come from spt_bucket_tokens or from any source that satisfies the
 * same invariants (sorted by block, stable).
 *   Y     out bf16 [T,d]
 *   Hsave out bf16 [P,Bs] pre-activations in bucket order, or NULL when no backward follows
 *   ws: spt_workspace_bytes(shape, SPT_WS_FWD) bytes.                                 */
int spt_routed_ffn_fwd(const spt_shape_t* shape, const void* X, const void* W1, const void* W2,
                       const int32_t* offsets, const int32_t* perm, const int32_t* inv,
                       void* Y, void* Hsave, void* ws, size_t ws_bytes, void* stream);

/* Backward with the routing held fixed (derivative of the forward above):
 *   dh_b = W2[b] dy_t;  dhpre_b = dh_b * act'(hpre_b);  dx_t = sum_b W1[b]^T dhpre_b
 *   dW1[b] = sum_t dhpre_b(t) x_t^T;   dW2[b] = sum_t h_b(t) dy_t^T
 * Blocks that no token activates get all-zero gradients.  Hsave is the forward's output.
 *   dX out bf16 [T,d];  dW1, dW2 out fp32 [N,Bs,d]
 *   ws: spt_workspace_bytes(shape, SPT_WS_BWD) bytes.                                 */
int spt_routed_ffn_bwd(const spt_shape_t* shape, const void* X, const void* W1, const void* W2,
                       const void* dY, const int32_t* offsets, const int32_t* perm,
                       const int32_t* inv, const void* Hsave, void* dX, float* dW1, float* dW2,
                       void* ws, size_t ws_bytes, void* stream);

/* The launch tables of the two calls above (row tiles per XCD, the token id of every sorted
 * position, the runs of every token range, the pieces of the weight-gradient GEMMs) are a function
 * of (shape, offsets, perm) alone.  spt_routed_ffn_fwd and spt_routed_ffn_bwd each build them in
 * their own workspace; a caller that runs both on one bucketing -- a training step, Algorithm 4
 * followed by its derivative -- can build them once:
 *   spt_build_schedule(shape, offsets, perm, sched, sched_bytes, stream)
 *   spt_routed_ffn_fwd_sched(... as spt_routed_ffn_fwd ..., sched, sched_bytes)
 *   spt_routed_ffn_bwd_sched(... as spt_routed_ffn_bwd ..., sched, sched_bytes)
 * sched: device buffer of spt_workspace_bytes(shape, SPT_WS_SCHEDULE) bytes, 256-byte aligned,
 * caller-owned, written by spt_build_schedule only and read by the other two; it stays valid
 * for as long as offsets and perm are unchanged.  Results are bit-identical to the plain calls.
 * A schedule built for other offsets/perm gives wrong results without an error (the tables are
 * not checked against the bucketing); a sched_bytes that is too small is SPT_ERR_WORKSPACE. */
int spt_build_schedule(const spt_shape_t* shape, const int32_t* offsets, const int32_t* perm,
                       void* sched, size_t sched_bytes, void* stream);
int spt_routed_ffn_fwd_sched(const spt_shape_t* shape, const void* X, const void* W1, const void* W2,
                             const int32_t* offsets, const int32_t* perm, const int32_t* inv,
                             void* Y, void* Hsave, void* ws, size_t ws_bytes, const void* sched,
                             size_t sched_bytes, void* stream);
int spt_routed_ffn_bwd_sched(const spt_shape_t* shape, const void* X, const void* W1, const void* W2,
                             const void* dY, const int32_t* offsets, const int32_t* perm,
                             const int32_t* inv, const void* Hsave, void* dX, float* dW1,
                             float* dW2, void* ws, size_t ws_bytes, const void* sched,
                             size_t sched_bytes, void* stream);

/* Low-rank adapted routed FFN (paper section 2.2, "Fine-tuning Transformer": a projection
 * Y = XW is trained as Y = X(W + BC) with W frozen and B, C of rank r; section 4.2 routing on
 * top).  Each projection matrix of Eq. 4 is replaced by W + BC as a whole and then restricted
 * to the activated blocks:
 *   hpre(b,u) = W1[b][u] . x + sum_rho C1[rho][b*Bs+u] (A1^T x)[rho]
 *   y         = sum_{b in S(t)} sum_u act(hpre(b,u)) ( W2[b][u] + sum_rho B2[b*Bs+u][rho] C2[rho] )
 * Adapters, device pointers, bf16, row-major: A1[d][r], C1[r][N*Bs], B2[N*Bs][r], C2[r][d];
 * 1 <= r <= 32.
 * Everything else as spt_routed_ffn_fwd: same offsets/perm/inv, same Y; Hsave[T*k][Bs] holds the
 * pre-activations INCLUDING the adapter term and may be NULL when no backward pass follows.
 * ws: spt_workspace_bytes(shape, SPT_WS_LORA_FWD) bytes. */
int spt_lora_ffn_fwd(const spt_shape_t* shape, int r, const void* X, const void* W1, const void* W2,
                     const void* A1, const void* C1, const void* B2, const void* C2,
                     const int32_t* offsets, const int32_t* perm, const int32_t* inv, void* Y,
                     void* Hsave, void* ws, size_t ws_bytes, void* stream);

/* Backward of spt_lora_ffn_fwd with W1, W2 frozen and the routing fixed (the fine-tuning setting
 * of section 2.2: only the adapters are trained, so no dW1 / dW2 is formed).  Inputs as the
 * forward plus dY[T][d] bf16 and the Hsave the forward wrote.  Outputs, all overwritten:
 * dX[T][d] bf16 and the adapter gradients in fp32, shaped like the adapters:
 * dA1[d][r], dC1[r][N*Bs], dB2[N*Bs][r], dC2[r][d].  Deterministic (fixed summation order).
 * ws: spt_workspace_bytes(shape, SPT_WS_LORA_BWD) bytes. */
int spt_lora_ffn_bwd(const spt_shape_t* shape, int r, const void* X, const void* W1, const void* W2,
                     const void* A1, const void* C1, const void* B2, const void* C2, const void* dY,
                     const int32_t* offsets, const int32_t* perm, const int32_t* inv,
                     const void* Hsave, void* dX, float* dA1, float* dC1, float* dB2, float* dC2,
                     void* ws, size_t ws_bytes, void* stream);

/* Load-balancing loss of the route network and its gradient.  Section 4.2 ("Dynamic routing")
 * says the route network is trained with a load-balancing loss so that the weight groups have
 * similar activation rates, but prints no formula; the one implemented here is this build's
 * choice (the usual auxiliary loss of top-k routers):
 *   f_b    = share of the T*k (token, slot) pairs routed to block b (from offsets; a constant),
 *   p_t    = softmax over the N blocks of the token's logits,   pbar_b = mean_t p_t[b],
 *   loss   = N * sum_b f_b * pbar_b                              (1 for a uniform soft assignment),
 *   dW_r   = X^T dlogit,  db_r = sum_t dlogit[t],  dlogit[t][c] = (N/T) p_t[c] (f_c - sum_b f_b p_t[b]).
 * Inputs: X[T][d] bf16, logits[T][N] fp32 as written by spt_router_topk, offsets[N+1] from
 * spt_bucket_tokens.  Outputs (device, overwritten): loss[1], frac[N] = f (may be NULL),
 * dW_r[d][N] fp32, db_r[N] fp32 (may be NULL).  Signed-logit routing only (flags == 0).
 * ws: spt_workspace_bytes(shape, SPT_WS_BALANCE) bytes. */
int spt_router_balance(const spt_shape_t* shape, const void* X, const float* logits,
                       const int32_t* offsets, float* loss, float* frac, float* dW_r, float* db_r,
                       void* ws, size_t ws_bytes, void* stream);

/* Host string for an SPT_* code (static storage). */
const char* spt_strerror(int code);

/* Diagnostics, not part of the paper's path: per-kernel durations measured with HIP events
 * recorded on the caller's stream around every kernel the four calls above launch.
 * spt_profile_enable(1) starts recording every kernel slot, spt_profile_enable(2 + slot) that one
 * slot only (two events per launch of it and nothing else: the cheap way to time one kernel
 * inside a timed region), spt_profile_enable(0) stops (events are created on the host, lazily,
 * and recycled); spt_profile_read waits for the recorded events, adds up milliseconds and launch
 * counts per kernel slot into ms_sum[spt_profile_slots()] / launches[...] (host arrays), and
 * clears the records.  Not thread-safe; leave disabled in production. */
int spt_profile_enable(int on);
int spt_profile_slots(void);
const char* spt_profile_slot_name(int slot);
int spt_profile_read(float* ms_sum, int32_t* launches);

/* Diagnostics, not part of the paper's path: what this GPU sustains, measured, for the
 * benchmark to print beside the nominal peaks.  Both only enqueue on `stream`; the caller times
 * them (e.g. with events on that stream).
 * spt_calibrate_mfma: `workgroups` workgroups of four wavefronts, each wavefront issuing
 *   iters * 8 v_mfma_f32_32x32x16_bf16 on register-resident operands (no memory traffic):
 *   workgroups * 4 * iters * 8 * 32768 FLOP.  pattern 0: operands are small integers and ones;
 *   pattern 1: pseudo-random values in (-2, 2) (the bit-toggle rate of real data, which is what
 *   a power-limited chip sustains).  out: device, workgroups * 256 floats (sink).
 * spt_calibrate_stream: mode 0 copies `bytes` from src to dst, mode 1 only reads src (dst gets
 *   at most 16 bytes), mode 2 only writes dst.  Device pointers, 16-byte aligned, bytes % 16 == 0. */
int spt_calibrate_mfma(int iters, int workgroups, int pattern, float* out, void* stream);
int spt_calibrate_stream(const void* src, void* dst, size_t bytes, int mode, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SPT_H */
