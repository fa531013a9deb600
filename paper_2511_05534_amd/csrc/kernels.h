// Host-side launchers of the gfx950 kernels.  Every launcher enqueues on ctx.stream and
// returns the hipError_t of the launch; none of them synchronises or allocates.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "layout.h"

namespace flowmm {

// LDS of a compute unit, and the most one workgroup may ask for (static plus dynamic)
constexpr size_t kLdsBytes = 160 * 1024;

// A kernel that wants more than 64 KB of dynamic LDS needs its cap raised first.  The cap belongs
// to the function (per device), not to a launch, so it is raised once per kernel and device to all the
// LDS there is beside the kernel's static share: no later call changes it, whatever shapes other
// host threads launch at the same time.
template <auto Kernel>
hipError_t allow_full_lds() {
  constexpr int kMaxDevices = 64;
  static std::atomic<bool> done[kMaxDevices];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev >= 0 && dev < kMaxDevices && done[dev].load(std::memory_order_acquire)) return hipSuccess;
  hipFuncAttributes at;
  if ((e = hipFuncGetAttributes(&at, reinterpret_cast<const void *>(Kernel))) != hipSuccess) return e;
  const size_t room = kLdsBytes > at.sharedSizeBytes ? kLdsBytes - at.sharedSizeBytes : 0;
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)room);
  if (e == hipSuccess && dev >= 0 && dev < kMaxDevices) done[dev].store(true, std::memory_order_release);
  return e;
}

struct Ctx {
  Shape sh;
  InlineMeta inl;  // valid when sh.unit_path
  hipStream_t stream;
  int layer0, layers;  // the unit-resident kernels work on layers [layer0, layer0 + layers) per launch
  // inputs
  const void *K, *V, *Q;
  // plan buffers
  float *importance, *rho;
  int *mode, *kept_idx, *assign, *n_dropped;
  // outputs
  void *K_out, *V_out;
  // workspace regions
  int *meta;
  uint8_t *mod;        // [T]                             modality of every packed token
  int *cls_order;      // [T]                             per sequence: text positions ascending, then image positions
  float2 *part_stats;  // [Lyr][Hkv][tiles_score][R_pad]  (max, sum exp2) of each row over a tile
  float *rowstat;      // [Lyr][Hkv][batch][R_pad]        max + log2(sum exp2) of each row, +inf for padding rows
  float *cross_part;   // [Lyr][Hq][tiles_score]          cross-modal mass of a head over a tile
  int *ev_list;        // [Lyr][Hkv][T]                   the tokens to be matched, per sequence in class order (text, then image)
  int *ev_n;           // [Lyr][Hkv][batch][2]            how many of either class (all in the first one in a cross-modal layer)
  int *pl_slot;        // [Lyr][Hkv][2*SBP]               eligible pivots per (sequence, token class): their slots, ascending
  int *pl_tok;         // [Lyr][Hkv][2*SBP]               their positions
  float *pl_w;         // [Lyr][Hkv][2*SBP]               1/norm of those pivots (0 for a zero row)
  int *pl_n;           // [Lyr][Hkv][batch][2]            list lengths, padded to multiples of 32
  uint4 *pack;         // [Lyr][Hkv][2*SBP][row chunks+1] their K rows, one chunk of padding after each
  int *seg_off;        // [Lyr][Hkv][SB + batch]          CSR offsets of the members of each slot
  int *members;        // [Lyr][Hkv][T]                   evicted tokens grouped by slot, ascending
  int4 *tasks;         // [Lyr][Hkv][tasks_total]         (slot, first member, count, partial index or -1); per sequence the
                       //                                 small ones from the front of its range, the others from the back
  int *n_tasks;        // [Lyr][Hkv][batch][2]            how many of either kind
  int4 *multi;         // [Lyr][Hkv][multi_total]         (slot, first partial, number of partials, members)
  int *n_multi;        // [Lyr][Hkv][batch]
  float *partials;     // [Lyr][Hkv][part_total][2][d]    fp32 partial row sums of K and V
  float *partial_w;    // [Lyr][Hkv][part_total]          weight sums of those partials (weighted merge)
};

// arguments of the exact (all-query) flow ratio that are not part of a plan
struct FlowExactArgs {
  const void *Q;                          // [Lyr][Hq][T][d] queries of every prompt token
  long long qs_layer, qs_head, qs_tok;    // strides in 16-byte chunks
  float *part;                            // [Lyr][Hq][qtiles_total] sum of the rows' cross-modal shares per query tile
  int qtiles_total;
  float *rho;                             // [Lyr][batch]
  int *mode;                              // [Lyr][batch]
};
hipError_t launch_flow_exact(const Ctx &c, const FlowExactArgs &a);

// arguments of the decode-step attention over the compacted cache
struct DecodeArgs {
  const void *q;               // [Lyr][Hq][batch][d]
  const void *K_c, *V_c;       // [Lyr][Hkv][SB][d] merged rows
  void *out;                   // [Lyr][Hq][batch][d]
  float *part;                 // [Lyr][Hq][batch][splits][d + 2] partial (weighted V, max, sum) per slot range
  int splits;                  // slot ranges per sequence
  int g0;                      // first query head (inside its kv group) of the current launch
};
int decode_splits(const Shape &sh);
hipError_t launch_decode_attention(const Ctx &c, const DecodeArgs &a);

// cache append (decode-time maintenance): one new K and V row per sequence, (layer, kv head) by (layer, kv head)
constexpr int kAppendSeqs = 64;  // sequences per launch (their target rows ride in the kernel arguments)
struct AppendArgs {
  void *K_c, *V_c;               // the cache, addressed through the strides below (16-byte chunks)
  const void *k_new, *v_new;     // [Lyr][Hkv][batch][d] contiguous
  long long ks_layer, ks_head, ks_tok;
  int nch, batch, b0;            // chunks per row; batch of the call; first sequence of this launch
  int row[kAppendSeqs];          // cache row (token index) that sequence b0 + i appends to
};
hipError_t launch_cache_append(const AppendArgs &a, int n_seqs, int Hkv, int n_layers, hipStream_t stream);

// rows of a dense [Lyr][Hkv][B][d] pair of tensors stored to cache rows [row0, row0 + B)
struct StoreRowsArgs {
  void *K_c, *V_c;
  const void *K_src, *V_src;
  long long ks_layer, ks_head, ks_tok;
  int nch, B, row0;
};
hipError_t launch_cache_store_rows(const StoreRowsArgs &a, int Hkv, int n_layers, hipStream_t stream);

constexpr int kMetaChunkWords = 960;
struct MetaChunk { int w[kMetaChunkWords]; };

hipError_t launch_meta_upload(const Ctx &c, const int *words, int n_words, bool expand_modality);
hipError_t launch_score(const Ctx &c);    // stats, combine, column sums
hipError_t launch_select(const Ctx &c);   // flow + top-B split
hipError_t launch_match(const Ctx &c);
hipError_t launch_merge(const Ctx &c);    // CSR build, task sums, combine

// unit-resident path (short prompts): one workgroup per (sequence, kv head, layer)
bool unit_path_fits(const Shape &sh);
// score, select and the cross-modal match of every unit; with_flow adds the launch that settles the
// layer strategies and matches the units of intra-modal layers again (the plan is then complete)
hipError_t launch_unit_plan(const Ctx &c, bool with_flow = true);
hipError_t launch_unit_flow_match(const Ctx &c);
// merge; with_flow: the same workgroups first do what launch_unit_flow_match does for their unit
hipError_t launch_unit_merge(const Ctx &c, bool with_flow = false);

// static LDS needs, used by the host to reject shapes that cannot be staged
size_t score_lds_bytes(const Shape &sh);
size_t merge_csr_lds_bytes(int max_budget);

}  // namespace flowmm
