// Optional per-kernel timing with HIP events on the launch stream (measurement support; off by
// default, and then a single relaxed atomic load per launch).
#pragma once
#include <hip/hip_runtime.h>

namespace flowmm {

enum KernelId {
  KID_META_UPLOAD = 0, KID_EXPAND_MODALITY, KID_SCORE_STATS, KID_SCORE_COMBINE, KID_SCORE_COLSUM,
  KID_SELECT, KID_MATCH, KID_MERGE_CSR, KID_MERGE_TASKS, KID_MERGE_FOLD,
  KID_UNIT_PLAN, KID_UNIT_MATCH, KID_UNIT_MERGE, KID_UNIT_FLOW_MERGE, KID_FLOW_EXACT, KID_DECODE_PARTIAL, KID_DECODE_COMBINE,
  KID_CACHE_APPEND, KID_CACHE_STORE_ROWS, KID_COUNT
};

const char *kernel_name(int id);

// Records an event before and after whatever is enqueued during its lifetime, if kernel `id` is selected.
class ProfScope {
 public:
  ProfScope(hipStream_t stream, int id);
  ~ProfScope();
 private:
  hipStream_t stream_;
  int slot_;
};

}  // namespace flowmm
