// Host/device shared description of one flowmm call: the metadata block that the host packs
// into 32-bit words and a small kernel places at the head of the workspace, and the byte
// offsets of every scratch region behind it.
#pragma once
#include <stdint.h>

namespace flowmm {

// ---- metadata block (int32 words) -------------------------------------------------------
enum MetaWord {
  MW_BATCH = 0,
  MW_T,            // total packed tokens
  MW_SUMB,         // total kept tokens per (layer, kv head)
  MW_OFF_SEQ,      // word offset of the per-sequence records
  MW_OFF_SPANS,    // word offset of the spans (begin, end, modality), all sequences
  MW_N_SPANS,
  MW_OFF_CU_SCORE, // word offset of cu_runs_score[batch+1]: runs of key tiles of the score kernels
  MW_OFF_CU_MATCH, // word offset of cu_tiles_match[batch+1]
  MW_OFF_CU_TASK,  // word offset of cu_tasks[batch+1]   (upper bounds)
  MW_OFF_CU_MULTI, // word offset of cu_multi[batch+1]   (upper bounds)
  MW_OFF_CU_PART,  // word offset of cu_part[batch+1]    (upper bounds)
  MW_OFF_CU_BP,    // word offset of cu_bp[batch+1]      (budgets rounded up to 32, prefix sums)
  MW_ZERO16,       // four zero words (a 16-byte aligned chunk of zeros for padding loads)
  MW_OFF_CU_FLOWQ = 16,  // word offset of cu_flowq[batch+1] (query tiles of the exact flow ratio)
  MW_HEADER = 20
};

// per-sequence record
enum SeqWord {
  SW_TOK_OFF = 0,  // first packed token
  SW_L,
  SW_B,
  SW_KEPT_OFF,     // first slot of this sequence inside [SB]
  SW_TAU,          // float bits
  SW_SPAN_OFF,     // first span (index into spans)
  SW_N_SPANS,
  SW_WIN_HAS_IMG,  // 1 if any window row is an image token
  SW_N_TEXT,       // number of text tokens
  SW_WORDS = 12
};

// tiling constants shared by host sizing and kernels
// Eight waves with few registers each: two such workgroups fit a compute unit, so that one computes
// with two waves per SIMD (matrix and vector phases overlap) while the other waits for its keys.
constexpr int kScoreWaves = 8;
// 32-key groups a wave of the score kernels holds in registers (its MFMA operands)
constexpr int score_subs(bool bf16) { return bf16 ? 2 : 1; }
constexpr int score_tile_keys(bool bf16) { return kScoreWaves * 32 * score_subs(bf16); }  // keys per workgroup
// As in the score kernels: eight waves with few registers, two workgroups per compute unit
constexpr int kMatchWaves = 8;
// 32-token groups a wave of the match kernel holds in registers (its MFMA B operands)
constexpr int match_subs(bool bf16) { return bf16 ? 2 : 1; }
constexpr int match_tile_tokens(bool bf16) { return kMatchWaves * 32 * match_subs(bf16); }  // tokens per workgroup
// packed pivot rows staged in LDS at a time: 32 KB worth, 128 rows at most (nch = 16-byte chunks per row)
constexpr int match_tile_rows(int nch) { return 2048 / nch < 128 ? 2048 / nch : 128; }
constexpr int kFlowQueryTile = 256;                          // query rows per workgroup of the exact flow ratio
constexpr int kDecodeMaxSplits = 32;                         // slot ranges per sequence of the decode-step attention
// (32 members per task: 30 us of folding on the long 16k configuration against 15 with 128; the tasks kernel itself takes 2 % longer)
constexpr int kTaskChunk = 128;                               // members summed by one wave task
constexpr int kCsrWaves = 16;                                // waves of the CSR-building workgroup
constexpr int kFoldGroups = 4;                               // workgroups per (sequence, kv head, layer) that fold split slots

struct Shape {
  int n_layers, Hq, Hkv, G, d, bf16;
  int batch, T, SB, W, W_pad, R_pad, maxB, maxL, maxE, n_spans;
  int unit_path;  // 1: every unit is handled by one workgroup (unit_path.hip)
  int rows32;     // 1: the K rows of every sequence lie within 4 GiB of the sequence's first row (32-bit byte offsets)
  int invert_flow;     // 1: the misaligned strategy (cross-modal merging iff NOT rho > theta)
  int weighted_merge;  // 1: similarity-weighted mean instead of the uniform one
  int SBP;        // sum over sequences of the budget rounded up to a multiple of 32
  int tiles_score;  // runs of key tiles over all sequences: one score workgroup and one set of partials per run
  int score_tpw;    // key tiles per run (the last run of a sequence may be shorter)
  int tiles_match, tasks_total, multi_total, part_total, flowq_total;
  float scale_log2e, theta;
  long long ks_layer, ks_head, ks_tok;  // K/V strides in 16-byte chunks
  long long qs_layer, qs_head, qs_tok;  // Q strides in 16-byte chunks
};

// Metadata small enough to ride in the kernel arguments (the unit-resident kernels use only this,
// so short prompts need no upload launch): per-sequence records and the modality spans.
constexpr int kInlineSeqs = 8;
constexpr int kInlineSpans = 32;
struct InlineMeta {
  int tok_off[kInlineSeqs], L[kInlineSeqs], B[kInlineSeqs], kept_off[kInlineSeqs];
  float tau[kInlineSeqs];
  int span_off[kInlineSeqs + 1];  // spans of sequence b: [span_off[b], span_off[b+1])
  int span_end[kInlineSpans];     // exclusive end of each span, position local to its sequence
  unsigned span_is_image;         // bit j: span j holds image tokens
  unsigned win_has_img;           // bit b: some proxy token of sequence b is an image token
};

// byte offsets into the workspace (all multiples of 256)
struct Regions {
  size_t meta, mod, cls_order;                              // both calls
  size_t part_stats, rowstat, cross_part;                   // plan: score
  size_t decode_part;                                       // decode attention: [Lyr][Hq][batch][kDecodeMaxSplits][d+2]
  size_t flow_part;                                         // exact flow ratio: [Lyr][Hq][flowq_total]
  size_t pl_slot, pl_tok, pl_w, pl_n, pack, ev_list, ev_n;  // plan: match
  size_t seg_off, members, tasks, n_tasks, multi, n_multi, partials, partial_w;  // merge
  size_t plan_end, merge_end;
};

}  // namespace flowmm
