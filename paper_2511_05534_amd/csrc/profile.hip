#include "profile.h"

#include <atomic>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/flowmm_profile.h"

namespace flowmm {

namespace {

const char *const kNames[KID_COUNT] = {"meta_upload", "expand_modality", "score_stats", "score_combine",
                                       "score_colsum", "select", "match", "merge_csr", "merge_tasks",
                                       "merge_fold", "unit_plan", "unit_match", "unit_merge", "unit_flow_merge",
                                       "flow_exact", "decode_partial", "decode_combine", "cache_append",
                                       "cache_store_rows"};

struct Record { int id; hipEvent_t start, stop; };

std::atomic<unsigned> g_mask{0};  // bit per kernel id
std::mutex g_mu;
std::vector<Record> g_records;
std::vector<hipEvent_t> g_pool;

hipEvent_t get_event() {
  if (!g_pool.empty()) { hipEvent_t e = g_pool.back(); g_pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

}  // namespace

const char *kernel_name(int id) { return id >= 0 && id < KID_COUNT ? kNames[id] : "?"; }

ProfScope::ProfScope(hipStream_t stream, int id) : stream_(stream), slot_(-1) {
  if (!(g_mask.load(std::memory_order_relaxed) & (1u << id))) return;
  std::lock_guard<std::mutex> lk(g_mu);
  Record r{id, get_event(), get_event()};
  if (!r.start || !r.stop) return;
  (void)hipEventRecord(r.start, stream_);
  g_records.push_back(r);
  slot_ = (int)g_records.size() - 1;
}

ProfScope::~ProfScope() {
  if (slot_ < 0) return;
  std::lock_guard<std::mutex> lk(g_mu);
  (void)hipEventRecord(g_records[slot_].stop, stream_);
}

}  // namespace flowmm

using namespace flowmm;

extern "C" {

__attribute__((visibility("default"))) int flowmm_profile_kernel_count(void) { return KID_COUNT; }

__attribute__((visibility("default"))) const char *flowmm_profile_kernel_name(int id) { return kernel_name(id); }

__attribute__((visibility("default"))) void flowmm_profile_select(const char *names) {
  unsigned mask = 0;
  if (names && *names) {
    for (int i = 0; i < KID_COUNT; ++i) {
      if (!std::strcmp(names, "all")) { mask |= 1u << i; continue; }
      const char *p = std::strstr(names, kNames[i]);
      const size_t n = std::strlen(kNames[i]);
      while (p) {  // whole-word match inside a comma separated list
        const bool left = p == names || p[-1] == ',';
        const bool right = p[n] == '\0' || p[n] == ',';
        if (left && right) { mask |= 1u << i; break; }
        p = std::strstr(p + 1, kNames[i]);
      }
    }
  }
  g_mask.store(mask);
}

__attribute__((visibility("default"))) flowmm_status flowmm_profile_collect(double *total_ms, long long *launches) {
  std::lock_guard<std::mutex> lk(g_mu);
  for (int i = 0; i < KID_COUNT; ++i) { if (total_ms) total_ms[i] = 0.0; if (launches) launches[i] = 0; }
  flowmm_status st = FLOWMM_OK;
  for (Record &r : g_records) {
    float ms = 0.f;
    if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) {
      st = FLOWMM_EHIP;
    } else {
      if (total_ms) total_ms[r.id] += ms;
      if (launches) launches[r.id] += 1;
    }
    g_pool.push_back(r.start);
    g_pool.push_back(r.stop);
  }
  g_records.clear();
  return st;
}

}  // extern "C"
