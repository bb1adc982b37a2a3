// Optional per-kernel timing with HIP events on the caller's stream (diagnostic only).
// Disabled by default; when disabled a launch costs one predictable branch.
#pragma once
#include <hip/hip_runtime.h>

namespace spt {

enum KernelSlot {
  kSlotRouter = 0, kSlotTopk, kSlotBucketHist, kSlotBucketScan, kSlotBucketScatter, kSlotPlan,
  kSlotUp, kSlotDown, kSlotCombineY, kSlotDH, kSlotDW2, kSlotDW1, kSlotDXPart,
  kSlotCombineDX, kSlotLoraSmall, kSlotLoraGrad, kSlotBalance,
  kSlotMhaPq, kSlotMhaTopl, kSlotMhaFwd, kSlotMhaBwdQ, kSlotMhaTranspose, kSlotMhaBwdKV,
  kNumSlots
};

bool profile_on(int slot);
void profile_mark(int slot, bool begin, hipStream_t st);

struct ScopedKernelTimer {
  int slot; hipStream_t st; bool on;
  ScopedKernelTimer(int s, hipStream_t stream) : slot(s), st(stream), on(profile_on(s)) {
    if (on) profile_mark(slot, true, st);
  }
  ~ScopedKernelTimer() { if (on) profile_mark(slot, false, st); }
};

}  // namespace spt
