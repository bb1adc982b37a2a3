// Host-side declarations shared by the translation units of libspt.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/spt.h"

namespace spt {

constexpr int kBucketChunkTokens = 128;  // tokens per workgroup in the bucketing pass

inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

hipError_t run_router_topk(const spt_shape_t& s, const void* X, const float* Wr, const float* br,
                           int32_t* idx, float* logits, hipStream_t st);
hipError_t run_bucket(const spt_shape_t& s, const int32_t* idx, int32_t* offsets, int32_t* perm,
                      int32_t* inv, int32_t* chunk_hist, hipStream_t st);
// Device address, on the current device, of the library's fixed bucketing scratch
// (kStaticBucketScratchInts int32: 1 MiB per GPU, held until the process ends).
constexpr size_t kStaticBucketScratchInts = 262144;
hipError_t bucket_static_scratch(int32_t** out);

// Device-built schedule tables shared by the forward and backward launches.
// One work item of the narrow-block weight-gradient GEMMs: the rows [lo, hi) of one bucket and
// where the product goes (dst < N: block dst of the gradient itself; dst >= N: staging slot
// dst - N, added to the block afterwards in slot order; dst < 0: unused table entry).
struct DwPiece { int32_t lo, hi, dst, pad; };
struct Schedule {
  int32_t* border;       // [N] buckets by size, largest first
  int32_t* kd_count;     // [8] row tiles of the K = d GEMMs per XCD
  void* kd_list;         // [8][kd_cap] (bucket, first row) in per-XCD run order
  int32_t* tok;          // [P] token id of every sorted position
  uint16_t* zero_row;    // 256 bytes of zeros (padding rows of the dW GEMMs' K dimension)
  int32_t* rstart;       // narrow blocks: per token range, the non-empty runs of bucket rows (ffn_scatter.hip)
  int kd_cap;
  // narrow blocks, backward: buckets cut into pieces of at most dw_rows rows (largest bucket first)
  DwPiece* dw_pieces;    // [dw_cap]
  int32_t* dw_xlist;     // [0] = number of buckets with staged pieces, then (bucket, first slot, end slot) triples
  int dw_cap, dw_rows;
};
struct FwdWorkspace {
  Schedule sched;
  uint16_t* Hact;        // bf16 activated hidden values per pair (narrow blocks: fragment order)
  uint16_t* part;        // [P,d] bf16 per-pair partial output rows (wide blocks only)
  size_t bytes;
};
struct BwdWorkspace {
  Schedule sched;
  uint16_t* Hact;   // act(Hsave) per pair  (narrow blocks: fragment order, ffn_common.hpp;
  uint16_t* dHpre;  // dHpre per pair        wide blocks: row-major [P,Bs])
  uint16_t* part;   // [P,d] per-pair partial dX rows (wide blocks only)
  float* dw_stage;  // [dw_cap - N][Bs][d] products of the pieces after a bucket's first (narrow blocks)
  size_t bytes;
};
FwdWorkspace plan_fwd(const spt_shape_t& s, void* ws);
// weight_grads = false: no tables or staging for the weight-gradient GEMMs (low-rank variant)
BwdWorkspace plan_bwd(const spt_shape_t& s, void* ws, bool weight_grads = true);

// Token-range-stationary K = Bs contraction of narrow blocks (down-projection, dX) with the
// per-token write-back folded in: R tokens x 64 columns per workgroup, nr ranges, nslab slabs.
struct ScatterPlan {
  int R, nr, nslab, smem;
  int cap;               // run records per range
  size_t runs_bytes;     // bytes of the [nr][cap] run records
  size_t counts_bytes;   // bytes of the per-range record counts
  size_t table_bytes;    // run records + counts + the dense [nr+1][N] table of run starts
};
ScatterPlan plan_scatter(const spt_shape_t& s);
// The dense table starts[r][b] (written by the schedule kernel) inside the run-table buffer.
int32_t* scatter_starts(const ScatterPlan& p, int32_t* table);
// Turns the dense table into the per-range lists of non-empty runs.
hipError_t run_scatter_ranges(const spt_shape_t& s, const ScatterPlan& p, int32_t* table, hipStream_t st);
// out[t][:] = sum_{b in S(t), ascending} Hin[pos(t,b)][:] W[b]  (+ Z[t][:] when Z is given)
hipError_t launch_scatter(const spt_shape_t& s, const ScatterPlan& p, const uint16_t* Hin, const uint16_t* W,
                          const int32_t* rstart, const int32_t* tok, uint16_t* out, const uint16_t* Z,
                          hipStream_t st);

// Arguments of the wide-block GEMM kernels (blocks of more than 128 hidden units).
struct WideArgs {
  const void* A;             // A-side operand (MFMA rows): W block, or the gathered activations
  const void* B;             // B-side operand: gathered activation rows, or H / dHpre
  const int32_t* offsets;
  const int32_t* kd_count;   // row tiles per XCD
  const void* kd_list;       // [8][cap] row tiles in per-XCD run order
  int cap;
  const int32_t* tok;
  const int32_t* border;
  const uint16_t* zero_row;
  int N, Bs, d;
  uint16_t* Hsave;           // written by the up-projection (may be null), read by dH
  uint16_t* Hact;
  uint16_t* dHpre;
  uint16_t* part;            // [P,d] row-major partial rows
  float* dW;
  const uint16_t* Xe;        // low-rank extension of the K = d GEMMs: [T][64] per token, or null
  const uint16_t* We;        //                                        [N*Bs][64] per hidden unit
};
enum WideOp { kWideUp = 0, kWideDH = 1, kWidePart = 2, kWideDW = 3 };
hipError_t launch_wide(int op, const spt_shape_t& s, const WideArgs& a, hipStream_t st);

// The schedule in a buffer of its own (the layout plan_bwd carves, weight-gradient tables included),
// filled once per bucketing by run_schedule; run_fwd / run_bwd given it as `prebuilt` skip building
// their own.
size_t schedule_bytes(const spt_shape_t& s);
Schedule plan_schedule(const spt_shape_t& s, void* buf);
hipError_t run_schedule(const spt_shape_t& s, const int32_t* offsets, const int32_t* perm, const Schedule& sc,
                        hipStream_t st);

hipError_t run_fwd(const spt_shape_t& s, const void* X, const void* W1, const void* W2,
                   const int32_t* offsets, const int32_t* perm, const int32_t* inv, void* Y,
                   void* Hsave, const FwdWorkspace& w, hipStream_t st, const Schedule* prebuilt = nullptr);
hipError_t run_bwd(const spt_shape_t& s, const void* X, const void* W1, const void* W2,
                   const void* dY, const int32_t* offsets, const int32_t* perm,
                   const int32_t* inv, const void* Hsave, void* dX, float* dW1, float* dW2,
                   const BwdWorkspace& w, hipStream_t st, const Schedule* prebuilt = nullptr);

// dW[b][u][c] = sum_{q in bucket b} Hin[q][u] * Act[tok[q]][c] (N buckets, Bs units, d columns):
// the narrow-block weight-gradient GEMM, also used with a 32/64-wide side by the adapter and
// router gradients.
// hin_frag: Hin is in the fragment order of the narrow-block hidden values (ffn_common.hpp).
hipError_t launch_dw(const uint16_t* Act, const uint16_t* Hin, bool hin_frag, const int32_t* offsets,
                     const int32_t* tok, const int32_t* border, const uint16_t* zero_row, int N,
                     int Bs, int d, float* dW, int slot, hipStream_t st);
// The same GEMM over a piece table (Schedule::dw_pieces) instead of whole buckets, followed by
// the fixed-order sum of the staged pieces into their blocks.
hipError_t launch_dw_pieces(const uint16_t* Act, const uint16_t* Hin, bool hin_frag, const Schedule& sc, int N,
                            int Bs, int d, float* dW, float* stage, int slot, hipStream_t st);

// Load-balancing loss of the route network and its gradient.
struct BalanceWorkspace {
  uint16_t* dl;        // [T][Npad] bf16 d loss / d logit
  float* part;         // [groups][2][N] partial sums of p and of dlogit
  float* gchunks;      // [chunks][Npad][d] gradient staging
  int32_t *c_off, *c_tok, *c_border;
  uint16_t* zero_row;
  int npad, groups, chunk, nchunks;
  size_t bytes;
};
BalanceWorkspace plan_balance(const spt_shape_t& s, void* ws);
hipError_t run_router_balance(const spt_shape_t& s, const void* X, const float* logits,
                              const int32_t* offsets, float* loss, float* frac, float* dWr, float* dbr,
                              const BalanceWorkspace& w, hipStream_t st);

// Low-rank adapted variant.  Workspace = the forward / backward
// workspace followed by zero-padded 32-wide adapter panels and the small intermediates.
struct LoraWorkspace {
  FwdWorkspace fwd;
  BwdWorkspace bwd;
  uint16_t *A1T, *C1T, *C1P, *B2T, *B2P, *C2P;  // [32][d] [D][64] [32][D] [32][D] [D][64] [32][d]
  uint16_t *A1P, *C2T;                          // [d][32] [d][32]: K-contiguous forms for lora_expand
  uint16_t* Z;                                  // [T][d] bf16: the low-rank term of an outer projection
  uint16_t *Upad, *Gpad;                        // [T][64] bf16 value | remainder: X A1, dY C2^T
  uint16_t* Sb;                                 // [T][32] bf16 rounded token sums
  float *Sp, *Sf;                               // [P][32] per pair, [T][32] per token
  float *gpad, *gchunks;                        // [pieces][Bs][64] and [chunks][32][d] gradient staging
  int32_t *c_off, *c_tok, *c_border;            // identity schedule over token chunks
  int32_t *p_first, *p_off, *p_id;              // buckets cut into pieces (see lora_pieces)
  int max_pieces;
  size_t bytes;
};
LoraWorkspace plan_lora(const spt_shape_t& s, void* ws, bool backward);
hipError_t run_lora_fwd(const spt_shape_t& s, int r, const void* X, const void* W1, const void* W2,
                        const void* A1, const void* C1, const void* B2, const void* C2,
                        const int32_t* offsets, const int32_t* perm, const int32_t* inv, void* Y,
                        void* Hsave, const LoraWorkspace& w, hipStream_t st);
hipError_t run_lora_bwd(const spt_shape_t& s, int r, const void* X, const void* W1, const void* W2,
                        const void* A1, const void* C1, const void* B2, const void* C2, const void* dY,
                        const int32_t* offsets, const int32_t* perm, const int32_t* inv,
                        const void* Hsave, void* dX, float* dA1, float* dC1, float* dB2, float* dC2,
                        const LoraWorkspace& w, hipStream_t st);
// One zero-padded bf16 panel: dst[a][b] (drows x dcols) = transpose ? src[b'][a] : src[a][b'],
// b' = dup ? b % 32 : b, zero outside src (srows x scols).
struct PadJob {
  const uint16_t* src;
  int srows, scols, transpose, dup;
  uint16_t* dst;
  int drows, dcols;
};
constexpr int kMaxPadJobs = 6;
struct PadJobs { PadJob job[kMaxPadJobs]; };
hipError_t lora_pad(const PadJobs& jobs, int njobs, hipStream_t st);
hipError_t lora_expand(const float* S, const uint16_t* MT, int T, int d, uint16_t* Z, hipStream_t st);
hipError_t lora_proj(const uint16_t* Act, const uint16_t* MT, int T, int d, uint16_t* S, hipStream_t st);
hipError_t lora_pair_gemm(const uint16_t* Hin, bool hin_frag, const uint16_t* WT, const int32_t* offsets, int N, int Bs,
                          int P, int act, float* Sp, hipStream_t st);
hipError_t lora_token_sum(const float* Sp, const int32_t* inv, int T, int k, float* Sf, uint16_t* Sb,
                          hipStream_t st);
hipError_t lora_chunks(int T, int chunk, int nchunks, int32_t* offsets, int32_t* tok, int32_t* border,
                       hipStream_t st);
hipError_t lora_pieces(const int32_t* offsets, int N, int piece, int max_pieces, int32_t* first,
                       int32_t* p_off, int32_t* p_id, hipStream_t st);
hipError_t lora_reduce_pieces(const float* src, const int32_t* first, int N, int Bs, int r, bool transpose,
                              float* out, hipStream_t st);
hipError_t lora_reduce(const float* src, int nchunks, int srows, int scols, bool transpose, bool fold,
                       float* out, int orows, int ocols, hipStream_t st);

}  // namespace spt
