// C ABI of libspt: argument validation and workspace carving; see include/spt.h.
#include <limits.h>

#include "spt_host.hpp"

using namespace spt;

namespace {

int check_shape(const spt_shape_t* s) {
  if (!s) return SPT_ERR_ARG;
  if (s->T < 1 || s->d < 1 || s->N < 1 || s->Bs < 1 || s->k < 1 || s->k > s->N) return SPT_ERR_ARG;
  if ((int64_t)s->T * s->k > INT_MAX || (int64_t)s->N * s->Bs > INT_MAX) return SPT_ERR_ARG;
  if (s->d % 64 != 0 || s->Bs % 32 != 0 || s->N > 1024) return SPT_ERR_UNSUPPORTED;
  if (s->act != SPT_ACT_GELU && s->act != SPT_ACT_RELU) return SPT_ERR_UNSUPPORTED;
  if (s->flags & ~SPT_FLAG_ABS_LOGIT) return SPT_ERR_UNSUPPORTED;
  return SPT_OK;
}

bool aligned(const void* p, size_t a) { return p && (reinterpret_cast<uintptr_t>(p) % a) == 0; }

size_t bucket_ws_bytes(const spt_shape_t& s) {
  const size_t nchunks = (s.T + kBucketChunkTokens - 1) / kBucketChunkTokens;
  return align256(nchunks * s.N * sizeof(int32_t));
}

}  // namespace

extern "C" {

size_t spt_workspace_bytes(const spt_shape_t* shape, int which) {
  if (check_shape(shape) != SPT_OK) return 0;
  switch (which) {
    case SPT_WS_BUCKET: return bucket_ws_bytes(*shape);
    case SPT_WS_FWD: return plan_fwd(*shape, nullptr).bytes;
    case SPT_WS_BWD: return plan_bwd(*shape, nullptr).bytes;
    case SPT_WS_ROUTER: return align256((size_t)shape->T * shape->N * sizeof(float));
    case SPT_WS_LORA_FWD: return plan_lora(*shape, nullptr, false).bytes;
    case SPT_WS_LORA_BWD: return plan_lora(*shape, nullptr, true).bytes;
    case SPT_WS_BALANCE: return plan_balance(*shape, nullptr).bytes;
    case SPT_WS_SCHEDULE: return schedule_bytes(*shape);
    default: return 0;
  }
}

int spt_router_topk(const spt_shape_t* shape, const void* X, const float* W_r, const float* b_r,
                    int32_t* idx, float* logits, void* ws, size_t ws_bytes, void* stream) {
  const int rc = check_shape(shape);
  if (rc != SPT_OK) return rc;
  if (!aligned(X, 16) || !aligned(W_r, 4) || !aligned(idx, 4)) return SPT_ERR_ARG;
  if ((b_r && !aligned(b_r, 4)) || (logits && !aligned(logits, 4))) return SPT_ERR_ARG;
  if (!logits) {
    if (!aligned(ws, 256)) return SPT_ERR_ARG;
    if (ws_bytes < align256((size_t)shape->T * shape->N * sizeof(float))) return SPT_ERR_WORKSPACE;
    logits = static_cast<float*>(ws);
  }
  const hipError_t e = run_router_topk(*shape, X, W_r, b_r, idx, logits, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? SPT_OK : SPT_ERR_HIP;
}

int spt_bucket_tokens(const spt_shape_t* shape, const int32_t* idx, int32_t* offsets, int32_t* perm,
                      int32_t* inv, void* ws, size_t ws_bytes, void* stream) {
  const int rc = check_shape(shape);
  if (rc != SPT_OK) return rc;
  if (!aligned(idx, 4) || !aligned(offsets, 4) || !aligned(perm, 4) || !aligned(inv, 4) ||
      !aligned(ws, 256))
    return SPT_ERR_ARG;
  if (ws_bytes < bucket_ws_bytes(*shape)) return SPT_ERR_WORKSPACE;
  const hipError_t e = run_bucket(*shape, idx, offsets, perm, inv, static_cast<int32_t*>(ws),
                                  static_cast<hipStream_t>(stream));
  return e == hipSuccess ? SPT_OK : SPT_ERR_HIP;
}

int spt_bucket_tokens_noalloc(const spt_shape_t* shape, const int32_t* idx, int32_t* offsets,
                              int32_t* perm, int32_t* inv, void* stream) {
  const int rc = check_shape(shape);
  if (rc != SPT_OK) return rc;
  if (!aligned(idx, 4) || !aligned(offsets, 4) || !aligned(perm, 4) || !aligned(inv, 4)) return SPT_ERR_ARG;
  if (bucket_ws_bytes(*shape) > kStaticBucketScratchInts * sizeof(int32_t)) return SPT_ERR_LIMIT;
  int32_t* scratch_ptr = nullptr;
  if (bucket_static_scratch(&scratch_ptr) != hipSuccess) return SPT_ERR_HIP;
  // every table entry the kernels read is written first by the histogram kernel of the same
  // call, so nothing has to be cleared between calls
  const hipError_t e = run_bucket(*shape, idx, offsets, perm, inv, scratch_ptr, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? SPT_OK : SPT_ERR_HIP;
}

int spt_routed_ffn_fwd_sched(const spt_shape_t* shape, const void* X, const void* W1, const void* W2,
                             const int32_t* offsets, const int32_t* perm, const int32_t* inv, void* Y,
                             void* Hsave, void* ws, size_t ws_bytes, const void* sched, size_t sched_bytes,
                             void* stream) {
  const int rc = check_shape(shape);
  if (rc != SPT_OK) return rc;
  if (!aligned(X, 16) || !aligned(W1, 16) || !aligned(W2, 16) || !aligned(Y, 16) ||
      !aligned(offsets, 4) || !aligned(perm, 4) || !aligned(inv, 4) || !aligned(ws, 256))
    return SPT_ERR_ARG;
  if (Hsave && !aligned(Hsave, 16)) return SPT_ERR_ARG;
  if (sched && !aligned(sched, 256)) return SPT_ERR_ARG;
  const FwdWorkspace w = plan_fwd(*shape, ws);
  if (ws_bytes < w.bytes) return SPT_ERR_WORKSPACE;
  Schedule pre;
  if (sched) {
    if (sched_bytes < schedule_bytes(*shape)) return SPT_ERR_WORKSPACE;
    pre = plan_schedule(*shape, const_cast<void*>(sched));
  }
  const hipError_t e = run_fwd(*shape, X, W1, W2, offsets, perm, inv, Y, Hsave, w,
                               static_cast<hipStream_t>(stream), sched ? &pre : nullptr);
  return e == hipSuccess ? SPT_OK : SPT_ERR_HIP;
}

int spt_routed_ffn_fwd(const spt_shape_t* shape, const void* X, const void* W1, const void* W2,
                       const int32_t* offsets, const int32_t* perm, const int32_t* inv, void* Y,
                       void* Hsave, void* ws, size_t ws_bytes, void* stream) {
  return spt_routed_ffn_fwd_sched(shape, X, W1, W2, offsets, perm, inv, Y, Hsave, ws, ws_bytes, nullptr, 0, stream);
}

int spt_routed_ffn_bwd_sched(const spt_shape_t* shape, const void* X, const void* W1, const void* W2,
                             const void* dY, const int32_t* offsets, const int32_t* perm,
                             const int32_t* inv, const void* Hsave, void* dX, float* dW1, float* dW2,
                             void* ws, size_t ws_bytes, const void* sched, size_t sched_bytes, void* stream) {
  const int rc = check_shape(shape);
  if (rc != SPT_OK) return rc;
  if (!aligned(X, 16) || !aligned(W1, 16) || !aligned(W2, 16) || !aligned(dY, 16) ||
      !aligned(Hsave, 16) || !aligned(dX, 16) || !aligned(dW1, 16) || !aligned(dW2, 16) ||
      !aligned(offsets, 4) || !aligned(perm, 4) || !aligned(inv, 4) || !aligned(ws, 256))
    return SPT_ERR_ARG;
  if (sched && !aligned(sched, 256)) return SPT_ERR_ARG;
  const BwdWorkspace w = plan_bwd(*shape, ws);
  if (ws_bytes < w.bytes) return SPT_ERR_WORKSPACE;
  Schedule pre;
  if (sched) {
    if (sched_bytes < schedule_bytes(*shape)) return SPT_ERR_WORKSPACE;
    pre = plan_schedule(*shape, const_cast<void*>(sched));
  }
  const hipError_t e = run_bwd(*shape, X, W1, W2, dY, offsets, perm, inv, Hsave, dX, dW1, dW2, w,
                               static_cast<hipStream_t>(stream), sched ? &pre : nullptr);
  return e == hipSuccess ? SPT_OK : SPT_ERR_HIP;
}

int spt_routed_ffn_bwd(const spt_shape_t* shape, const void* X, const void* W1, const void* W2,
                       const void* dY, const int32_t* offsets, const int32_t* perm,
                       const int32_t* inv, const void* Hsave, void* dX, float* dW1, float* dW2,
                       void* ws, size_t ws_bytes, void* stream) {
  return spt_routed_ffn_bwd_sched(shape, X, W1, W2, dY, offsets, perm, inv, Hsave, dX, dW1, dW2, ws, ws_bytes,
                                  nullptr, 0, stream);
}

int spt_build_schedule(const spt_shape_t* shape, const int32_t* offsets, const int32_t* perm, void* sched,
                       size_t sched_bytes, void* stream) {
  const int rc = check_shape(shape);
  if (rc != SPT_OK) return rc;
  if (!aligned(offsets, 4) || !aligned(perm, 4) || !aligned(sched, 256)) return SPT_ERR_ARG;
  if (sched_bytes < schedule_bytes(*shape)) return SPT_ERR_WORKSPACE;
  const hipError_t e = run_schedule(*shape, offsets, perm, plan_schedule(*shape, sched),
                                    static_cast<hipStream_t>(stream));
  return e == hipSuccess ? SPT_OK : SPT_ERR_HIP;
}

int spt_lora_ffn_fwd(const spt_shape_t* shape, int r, const void* X, const void* W1, const void* W2,
                     const void* A1, const void* C1, const void* B2, const void* C2,
                     const int32_t* offsets, const int32_t* perm, const int32_t* inv, void* Y,
                     void* Hsave, void* ws, size_t ws_bytes, void* stream) {
  const int rc = check_shape(shape);
  if (rc != SPT_OK) return rc;
  if (r < 1 || r > 32) return SPT_ERR_ARG;
  if (!aligned(X, 16) || !aligned(W1, 16) || !aligned(W2, 16) || !aligned(Y, 16) || !aligned(A1, 2) ||
      !aligned(C1, 2) || !aligned(B2, 2) || !aligned(C2, 2) || !aligned(offsets, 4) ||
      !aligned(perm, 4) || !aligned(inv, 4) || !aligned(ws, 256))
    return SPT_ERR_ARG;
  if (Hsave && !aligned(Hsave, 16)) return SPT_ERR_ARG;
  const LoraWorkspace w = plan_lora(*shape, ws, false);
  if (ws_bytes < w.bytes) return SPT_ERR_WORKSPACE;
  const hipError_t e = run_lora_fwd(*shape, r, X, W1, W2, A1, C1, B2, C2, offsets, perm, inv, Y, Hsave, w,
                                    static_cast<hipStream_t>(stream));
  return e == hipSuccess ? SPT_OK : SPT_ERR_HIP;
}

int spt_lora_ffn_bwd(const spt_shape_t* shape, int r, const void* X, const void* W1, const void* W2,
                     const void* A1, const void* C1, const void* B2, const void* C2, const void* dY,
                     const int32_t* offsets, const int32_t* perm, const int32_t* inv,
                     const void* Hsave, void* dX, float* dA1, float* dC1, float* dB2, float* dC2,
                     void* ws, size_t ws_bytes, void* stream) {
  const int rc = check_shape(shape);
  if (rc != SPT_OK) return rc;
  if (r < 1 || r > 32) return SPT_ERR_ARG;
  if (!aligned(X, 16) || !aligned(W1, 16) || !aligned(W2, 16) || !aligned(dY, 16) ||
      !aligned(Hsave, 16) || !aligned(dX, 16) || !aligned(A1, 2) || !aligned(C1, 2) || !aligned(B2, 2) ||
      !aligned(C2, 2) || !aligned(dA1, 4) || !aligned(dC1, 4) || !aligned(dB2, 4) || !aligned(dC2, 4) ||
      !aligned(offsets, 4) || !aligned(perm, 4) || !aligned(inv, 4) || !aligned(ws, 256))
    return SPT_ERR_ARG;
  const LoraWorkspace w = plan_lora(*shape, ws, true);
  if (ws_bytes < w.bytes) return SPT_ERR_WORKSPACE;
  const hipError_t e = run_lora_bwd(*shape, r, X, W1, W2, A1, C1, B2, C2, dY, offsets, perm, inv, Hsave, dX,
                                    dA1, dC1, dB2, dC2, w, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? SPT_OK : SPT_ERR_HIP;
}

int spt_router_balance(const spt_shape_t* shape, const void* X, const float* logits,
                       const int32_t* offsets, float* loss, float* frac, float* dW_r, float* db_r,
                       void* ws, size_t ws_bytes, void* stream) {
  const int rc = check_shape(shape);
  if (rc != SPT_OK) return rc;
  if (shape->flags != 0) return SPT_ERR_UNSUPPORTED;
  if (!aligned(X, 16) || !aligned(logits, 4) || !aligned(offsets, 4) || !aligned(loss, 4) ||
      !aligned(dW_r, 4) || !aligned(ws, 256))
    return SPT_ERR_ARG;
  if ((frac && !aligned(frac, 4)) || (db_r && !aligned(db_r, 4))) return SPT_ERR_ARG;
  const BalanceWorkspace w = plan_balance(*shape, ws);
  if (ws_bytes < w.bytes) return SPT_ERR_WORKSPACE;
  const hipError_t e = run_router_balance(*shape, X, logits, offsets, loss, frac, dW_r, db_r, w,
                                          static_cast<hipStream_t>(stream));
  return e == hipSuccess ? SPT_OK : SPT_ERR_HIP;
}

const char* spt_strerror(int code) {
  switch (code) {
    case SPT_OK: return "success";
    case SPT_ERR_ARG: return "invalid argument (null or misaligned pointer, or size out of range)";
    case SPT_ERR_UNSUPPORTED: return "unsupported shape, activation or flag";
    case SPT_ERR_WORKSPACE: return "workspace too small";
    case SPT_ERR_HIP: return "HIP launch failed";
    case SPT_ERR_LIMIT: return "size beyond the fixed scratch of the allocation-free entry point";
    default: return "unknown error code";
  }
}

}  // extern "C"
