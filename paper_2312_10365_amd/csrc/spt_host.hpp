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

// Device-built schedule tables shared by the forward and backward launches.
struct Schedule {
  int32_t* border;       // [N] buckets by size, largest first
  int32_t* kd_count;     // [8] row tiles of the K = d GEMMs per XCD
  void* kd_list;         // [8][kd_cap] (bucket, first row) in per-XCD run order
  int32_t* tok;          // [P] token id of every sorted position
  uint16_t* zero_row;    // 256 bytes of zeros (padding rows of the dW GEMMs' K dimension)
  int kd_cap;
};
struct FwdWorkspace {
  Schedule sched;
  uint16_t* Hact;        // [P,Bs] bf16 activated hidden values
  uint16_t* part;        // [P,d] bf16 per-pair partial output rows
  size_t bytes;
};
struct BwdWorkspace {
  Schedule sched;
  uint16_t* Hact;   // [P,Bs] act(Hsave)
  uint16_t* dHpre;  // [P,Bs]
  uint16_t* part;   // [P,d] per-pair partial dX rows
  size_t bytes;
};
FwdWorkspace plan_fwd(const spt_shape_t& s, void* ws);
BwdWorkspace plan_bwd(const spt_shape_t& s, void* ws);

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
};
enum WideOp { kWideUp = 0, kWideDH = 1, kWidePart = 2, kWideDW = 3 };
hipError_t launch_wide(int op, const spt_shape_t& s, const WideArgs& a, hipStream_t st);

hipError_t run_fwd(const spt_shape_t& s, const void* X, const void* W1, const void* W2,
                   const int32_t* offsets, const int32_t* perm, const int32_t* inv, void* Y,
                   void* Hsave, const FwdWorkspace& w, hipStream_t st);
hipError_t run_bwd(const spt_shape_t& s, const void* X, const void* W1, const void* W2,
                   const void* dY, const int32_t* offsets, const int32_t* perm,
                   const int32_t* inv, const void* Hsave, void* dX, float* dW1, float* dW2,
                   const BwdWorkspace& w, hipStream_t st);

}  // namespace spt
