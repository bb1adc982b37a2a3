// Event bookkeeping behind spt_profile_enable / spt_profile_read (see include/spt.h).
#include "profile.hpp"

#include <vector>

#include "spt_host.hpp"

namespace spt {
namespace {

struct Record { int slot; hipEvent_t a, b; };
bool g_on = false;
int g_only = -1;                    // >= 0: record this slot only
std::vector<Record> g_records;      // used records
std::vector<hipEvent_t> g_pool;     // recycled events
hipEvent_t g_open[kNumSlots];

const char* kNames[kNumSlots] = {
    "router_logits", "topk", "bucket_hist", "bucket_scan", "bucket_scatter", "plan",
    "up_gemm", "down_gemm", "combine_y", "dh_gemm", "dw2_gemm", "dw1_gemm", "dx_gemm", "combine_dx", "lora_small", "lora_grad", "router_balance",
    "mha_pq_assign", "mha_topl", "mha_attn_fwd", "mha_attn_bwd_q", "mha_transpose", "mha_attn_bwd_kv"};

hipEvent_t take_event() {
  if (!g_pool.empty()) { hipEvent_t e = g_pool.back(); g_pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}

}  // namespace

bool profile_on(int slot) { return slot >= 0 && g_on && (g_only < 0 || g_only == slot); }

void profile_mark(int slot, bool begin, hipStream_t st) {
  hipEvent_t e = take_event();
  if (!e) return;
  (void)hipEventRecord(e, st);
  if (begin) { g_open[slot] = e; return; }
  g_records.push_back({slot, g_open[slot], e});
}

}  // namespace spt

using namespace spt;

extern "C" {

int spt_profile_enable(int on) {
  if (on >= 2 && on - 2 >= kNumSlots) return SPT_ERR_ARG;
  g_on = on != 0;
  g_only = on >= 2 ? on - 2 : -1;
  return SPT_OK;
}

int spt_profile_slots(void) { return kNumSlots; }

const char* spt_profile_slot_name(int slot) {
  return (slot >= 0 && slot < kNumSlots) ? kNames[slot] : "";
}

int spt_profile_read(float* ms_sum, int32_t* launches) {
  if (!ms_sum || !launches) return SPT_ERR_ARG;
  for (int s = 0; s < kNumSlots; ++s) { ms_sum[s] = 0.f; launches[s] = 0; }
  int rc = SPT_OK;
  for (const Record& r : g_records) {
    float ms = 0.f;
    if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess)
      rc = SPT_ERR_HIP;
    ms_sum[r.slot] += ms;
    launches[r.slot] += 1;
    g_pool.push_back(r.a);
    g_pool.push_back(r.b);
  }
  g_records.clear();
  return rc;
}

}  // extern "C"
