/*
 * flowmm.h - C ABI of the MI355X (gfx950) FlowMM prefill-time KV-cache merge.
 *
 * The library compresses the KV cache of a multimodal prompt right after prefill,
 * following FlowMM (arXiv 2511.05534), Method section:
 *   - flowmm_plan : scores every cached key with the attention of the last W prompt
 *     tokens (the proxy tokens; "Information Flow Guided Merging", importance equation),
 *     measures the layer's cross-modal interaction ratio rho and compares it with theta
 *     (same section, rho equation and threshold rule), picks the top-B pivots per KV head,
 *     and matches every non-pivot key to its most cosine-similar pivot whose importance
 *     does not exceed tau ("Sensitivity-Adaptive Token Matching", both equations); in an
 *     intra-modal layer (rho <= theta) only pivots of the token's own modality qualify.
 *   - flowmm_merge: folds every matched non-pivot K/V row into its pivot by a uniform mean
 *     (the paper's generic K_merged = f_merge(K, S), Preliminary) and writes a compacted cache.
 *
 * Conventions
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library allocates no
 *     device memory, never synchronises and launches only on the stream it is given.
 *   - Arrays inside flowmm_params are HOST pointers, read during the call only.
 *   - Tokens of a batch are packed: sequence b owns tokens [cu_seqlens[b], cu_seqlens[b+1]).
 *     "T" below is cu_seqlens[batch]; "SB" is the sum of budget_tokens.
 *   - K and V: element (layer l, kv head g, packed token t, channel c) lives at
 *     base + l*stride_layer + g*stride_head + t*stride_token + c   (elements, c contiguous).
 *     Q holds only the window rows: token index b*W + r is row r (prompt position L_b-W+r) of
 *     sequence b; heads are query heads; query head h reads KV head h / (Hq/Hkv).
 *   - Device pointers must be 16-byte aligned, strides multiples of 16 bytes.  The window queries
 *     of one (layer, kv head, sequence) must lie within 4 GiB of each other (FLOWMM_EUNSUPPORTED
 *     otherwise): (Hq/Hkv - 1)*q_stride_head + (W - 1)*q_stride_token + head_dim elements.
 *   - Errors in the arguments are found on the host before anything is launched; the call
 *     then returns a code and flowmm_last_error() describes it.  Nothing was enqueued.
 *   - Threads: every call is self-contained (no state is kept between calls beyond flags that say
 *     which kernels had their LDS limit raised on which device, set once and never changed), so
 *     host threads may call concurrently, each with its own stream, plan buffers, outputs and
 *     workspace.  Two calls that share a workspace or an output must be ordered by the caller
 *     (same stream, or events).  flowmm_last_error() is per thread.
 */
#ifndef FLOWMM_H
#define FLOWMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FLOWMM_OK = 0,
  FLOWMM_EINVAL = 1,       /* malformed argument (message says which) */
  FLOWMM_EUNSUPPORTED = 2, /* valid but not built: head_dim other than 64/128, ... */
  FLOWMM_EWORKSPACE = 3,   /* workspace_bytes smaller than flowmm_plan_sizes reports */
  FLOWMM_EHIP = 4          /* a HIP call failed (launch error, no device) */
} flowmm_status;

typedef enum { FLOWMM_F32 = 0, FLOWMM_BF16 = 1 } flowmm_dtype;

enum { FLOWMM_TEXT = 0, FLOWMM_IMAGE = 1 };
enum { FLOWMM_MODE_INTRA = 0, FLOWMM_MODE_CROSS = 1 };
/* Short bf16 prompts (every L <= 1024, (Hq/Hkv) * window padded to 32 <= 64, every B <= 256) are
 * handled by kernels that keep a whole (sequence, layer, kv head) inside one workgroup; this flag
 * sends them through the general multi-workgroup kernels instead (same results up to fp32
 * summation order; used by tests). */
enum { FLOWMM_FLAG_GENERIC_PATH = 1 };
/* Variants of the paper's component ablation (Effectiveness of Each Component), on the same
 * kernels.  Two of them need no flag: "without sensitivity-adaptive matching" is tau = +inf, and
 * "without information flow guidance" is a theta below 0 (always cross-modal) or above 1 (always
 * intra-modal).
 *   FLOWMM_FLAG_INVERT_FLOW    the strategy misaligned with the measured flow: a layer merges
 *                              cross-modally iff NOT rho > theta (mode reports what was done).
 *   FLOWMM_FLAG_WEIGHTED_MERGE f_merge / g_merge as a similarity-weighted mean:
 *                              out[slot] = (row[pivot] + sum_i w_i row[i]) / (1 + sum_i w_i),
 *                              w_i = max(u_i, 0), u_i the cosine between the keys of member i and
 *                              of the pivot (0 if either is a zero row); V rows take the weights
 *                              of their K rows.  Read by flowmm_merge and flowmm_plan_merge. */
enum { FLOWMM_FLAG_INVERT_FLOW = 2, FLOWMM_FLAG_WEIGHTED_MERGE = 4 };

/* Half-open token range [begin, end) local to its sequence, with its modality. */
typedef struct {
  int32_t begin, end, modality;
} flowmm_span;

typedef struct {
  int32_t n_layers, n_q_heads, n_kv_heads; /* n_q_heads % n_kv_heads == 0 */
  int32_t head_dim;                        /* 64 or 128 */
  int32_t dtype;                           /* flowmm_dtype of K, V, Q and of the outputs */
  int32_t batch;                           /* >= 1 */
  const int32_t *cu_seqlens;               /* host [batch+1], cu_seqlens[0] == 0, increasing */
  const int32_t *budget_tokens;            /* host [batch], W <= B_b <= L_b (tokens kept per KV head) */
  const flowmm_span *spans;                /* host, all sequences back to back */
  const int32_t *cu_spans;                 /* host [batch+1]; spans of b sorted, contiguous, covering [0,L_b) */
  int32_t window;                          /* W >= 1, W <= every L_b */
  float scale;                             /* logit scale; 0 means 1/sqrt(head_dim) */
  float theta;                             /* cross-modal merging iff rho > theta */
  const float *tau;                        /* host [batch]; pivot j is sensitive iff I_j > tau_b;
                                              +inf disables the gate, a negative value drops everything */
  int64_t k_stride_layer, k_stride_head, k_stride_token; /* elements; the same strides address V */
  int64_t q_stride_layer, q_stride_head, q_stride_token;
  int32_t flags;                           /* 0, or FLOWMM_FLAG_* bits */
} flowmm_params;

/* The plan: device buffers the caller allocates; flowmm_plan fills them, flowmm_merge reads
 * kept_idx and assign.  Sizes in bytes come from flowmm_plan_sizes, in this field order. */
typedef struct {
  float *importance;  /* [Lyr][Hkv][T]  proxy importance, normalised so each sequence sums to 1 */
  float *rho;         /* [Lyr][batch]   cross-modal interaction ratio */
  int32_t *mode;      /* [Lyr][batch]   FLOWMM_MODE_CROSS iff rho > theta */
  int32_t *kept_idx;  /* [Lyr][Hkv][SB] positions (local to the sequence) of the pivots, ascending;
                                        the pivots of sequence b start at sum_{b'<b} B_b' ("slot" = index there) */
  int32_t *assign;    /* [Lyr][Hkv][T]  pivot: its own slot; other tokens: matched slot, or -1 if no
                                        pivot is eligible (the token is then simply evicted) */
  int32_t *n_dropped; /* [Lyr][Hkv][batch] number of -1 entries */
} flowmm_plan_buffers;

/* Bytes of each plan buffer (6 values, field order above) and of the scratch workspace that
 * flowmm_plan / flowmm_merge need for these shapes.  Pure host computation. */
flowmm_status flowmm_plan_sizes(const flowmm_params *p, size_t plan_bytes[6], size_t *workspace_bytes);

/* Score, flow, select and match for all layers, heads and sequences.  K [Lyr][Hkv][T][d] and
 * Q_window [Lyr][Hq][batch*W][d] are read through the strides in p.  workspace: device scratch,
 * contents undefined afterwards.  stream: a hipStream_t (NULL = default stream). */
flowmm_status flowmm_plan(const flowmm_params *p, const void *K, const void *Q_window,
                          const flowmm_plan_buffers *plan, void *workspace, size_t workspace_bytes,
                          void *stream);

/* K_out, V_out [Lyr][Hkv][SB][d] contiguous, dtype of the inputs:
 *   out[slot] = (row[kept_idx[slot]] + sum of rows assigned to slot) / (1 + their number),
 * accumulated in fp32 in an order that depends only on the shapes and the plan (so a call is
 * reproducible; short prompts add in ascending token order, long ones by groups of rows and a fixed
 * tree, and the two can differ in the last bit of a result) and rounded to nearest-even; a pivot
 * nobody merges into is copied bit for bit.  Outputs must not overlap K or V. */
flowmm_status flowmm_merge(const flowmm_params *p, const flowmm_plan_buffers *plan, const void *K,
                           const void *V, void *K_out, void *V_out, void *workspace,
                           size_t workspace_bytes, void *stream);

/* flowmm_plan followed by flowmm_merge in one call, with the same arguments, results and rules:
 * the plan buffers are filled as flowmm_plan fills them and K_out, V_out as flowmm_merge does
 * from that plan (the whole method of the paper's Method section, score to merged cache).  The
 * caller who does not want to look at the plan in between saves the argument checks, one
 * metadata upload and, for short prompts, one kernel launch. */
flowmm_status flowmm_plan_merge(const flowmm_params *p, const void *K, const void *V, const void *Q_window,
                                const flowmm_plan_buffers *plan, void *K_out, void *V_out, void *workspace,
                                size_t workspace_bytes, void *stream);

/* flowmm_plan_merge for callers that cannot allocate device memory for a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * rules as flowmm_plan_merge, minus the workspace: the scratch lives in a device array that is part
 * of the library itself (flowmm_static_workspace_bytes() bytes, 64 MiB; every GPU the library runs
 * on holds it from the first use until the process ends).  The call makes no hipMalloc / hipFree and
 * calls no allocating library routine; inputs, plan buffers and outputs are still the caller's.
 * Shapes whose flowmm_plan_sizes workspace exceeds the array return FLOWMM_EWORKSPACE (nothing is
 * enqueued; the message gives both sizes).  All calls on one GPU share that GPU's array: calls that
 * overlap on one GPU (different streams without ordering, or different host threads) race; order them.
 * The kernels initialise every word of scratch they read, so what an earlier call left there does
 * not matter.  The first call on a device looks up the array's address on that device (which loads
 * the library's code there): make one call before capturing into a graph. */
size_t flowmm_static_workspace_bytes(void);
flowmm_status flowmm_plan_merge_static(const flowmm_params *p, const void *K, const void *V, const void *Q_window,
                                       const flowmm_plan_buffers *plan, void *K_out, void *V_out, void *stream);

/* The cross-modal interaction ratio with EVERY token of the prompt as a query: the rho^l equation
 * of the paper (Information Flow Guided Merging) evaluated literally over the causal prefill
 * attention, instead of the estimate from the last `window` queries that flowmm_plan uses.
 *   rho[l][b] = (1/Hq) sum_h (1/L_b) sum_r  (mass query r sends to keys of the other modality)
 *                                           / (total mass of query r),
 *   mode[l][b] = FLOWMM_MODE_CROSS iff rho > theta (inverted under FLOWMM_FLAG_INVERT_FLOW).
 * Q_full [Lyr][Hq][T][d]: the query of every packed token, dtype of K, read through the three
 * strides given here (elements; head_dim contiguous; 256 consecutive tokens of a head must lie
 * within 4 GiB, FLOWMM_EUNSUPPORTED otherwise).  K, p, workspace (size from
 * flowmm_plan_sizes), stream and the rules for errors as in flowmm_plan; window, budgets and tau
 * are validated but not used.  rho, mode: device, [Lyr][batch].  Cost grows with L^2: this is a
 * measurement, and a way to supply the strategy when the prefill can provide all queries. */
flowmm_status flowmm_flow_exact(const flowmm_params *p, const void *K, const void *Q_full,
                                int64_t qf_stride_layer, int64_t qf_stride_head, int64_t qf_stride_token,
                                float *rho, int32_t *mode, void *workspace, size_t workspace_bytes,
                                void *stream);

/* One decode step of attention over the compacted cache that flowmm_merge wrote (the attention
 * of the paper's Preliminary section, o = softmax(scale * q K^T) V, on the merged rows): for every
 * layer l, query head h and sequence b
 *   out[l][h][b] = sum_s softmax_s(scale * <q[l][h][b], K_c[l][kv(h)][s]>) V_c[l][kv(h)][s],
 * s over the B_b slots of sequence b.  q, out: device, [Lyr][Hq][batch][d] contiguous, dtype of the
 * cache; K_c, V_c: [Lyr][Hkv][SB][d] as flowmm_merge lays them out.  p as for the other calls (its
 * budgets give the slot ranges; spans, window and tau are validated but not used); workspace and
 * its size as reported by flowmm_plan_sizes.  Every merged row is read once. */
flowmm_status flowmm_decode_attention(const flowmm_params *p, const void *q, const void *K_c, const void *V_c,
                                      void *out, void *workspace, size_t workspace_bytes, void *stream);

/* ---- decode-time maintenance of the compacted cache --------------------------------------------
 * The paper's Preliminary section appends the key and value of every decoded token to the cache
 * (K_t = [K_{t-1}, k_t], V_t = [V_{t-1}, v_t]) and says nothing about what happens once a compressed
 * cache has grown past its budget again.  The reading built here: the cache of sequence b owns the
 * rows [cu_capacity[b], cu_capacity[b+1]) of K_c / V_c (capacity C_b >= its budget B_b, the same
 * range in every layer and kv head), of which the first lengths[b] are valid: the merged prompt rows,
 * then the decoded tokens in order.  flowmm_cache_append adds one token per sequence; when a
 * sequence's range is full the caller has flowmm_cache_remerge compress it back to B_b rows by the
 * very method of flowmm_plan_merge, with the cache's valid rows as the "prompt" and its last
 * `window` rows (the most recent tokens, whose queries the caller has kept) as the proxy tokens.
 * The re-merge is blind to modality: a row merged across modalities has none, decoded tokens are all
 * text, and the paper measures rho on prompt attention only; every row counts as one token of one
 * modality (so rho = 0 and the strategies coincide), and a merged row weighs like any other row.
 *
 * In both calls p describes the cache: n_layers, n_q_heads, n_kv_heads, head_dim, dtype, batch,
 * k_stride_* (the strides of K_c and V_c, elements), and for the re-merge budget_tokens, window,
 * scale, tau, q_stride_* and flags (FLOWMM_FLAG_GENERIC_PATH, FLOWMM_FLAG_WEIGHTED_MERGE);
 * cu_seqlens, spans, cu_spans and theta are not read.  cu_capacity (host, [batch+1], starts at 0,
 * increasing) and lengths (host, [batch], 0 <= lengths[b] <= C_b) are read during the call only. */

/* Cache-append equation: row cu_capacity[b] + lengths[b] of every (layer, kv head) of K_c / V_c
 * becomes k_new / v_new [Lyr][Hkv][batch][d] (device, contiguous, dtype of the cache).  The caller
 * then counts lengths[b] + 1.  FLOWMM_EINVAL if some sequence is full (re-merge it first); nothing
 * is enqueued then. */
flowmm_status flowmm_cache_append(const flowmm_params *p, const int32_t *cu_capacity, const int32_t *lengths,
                                  void *K_c, void *V_c, const void *k_new, const void *v_new, void *stream);

/* Sizes for flowmm_cache_remerge of sequence seq at the length given (at most its capacity): bytes of
 * the six plan buffers (field order of flowmm_plan_buffers, for one sequence of that many tokens)
 * and of the workspace (which also holds the merged rows until they are stored back). */
flowmm_status flowmm_cache_remerge_sizes(const flowmm_params *p, const int32_t *cu_capacity, int32_t seq,
                                         int32_t length, size_t plan_bytes[6], size_t *workspace_bytes);

/* Compress the lengths[seq] valid rows of sequence seq back to budget_tokens[seq] rows: score
 * (Q_window: the queries of the last `window` valid rows, [Lyr][Hq][window][d] through q_stride_*),
 * select, match and merge exactly as flowmm_plan_merge does for a single-modality prompt of
 * lengths[seq] tokens with tau[seq]; the merged rows replace rows [0, B) of the sequence's range
 * (ascending position, as always), the rows behind them are stale, and the caller sets
 * lengths[seq] = budget_tokens[seq].  plan receives the plan of this re-merge (positions are cache
 * rows relative to the start of the sequence's range).  Requires window <= lengths[seq] and
 * budget_tokens[seq] in [window, lengths[seq]]; other sequences are not touched. */
flowmm_status flowmm_cache_remerge(const flowmm_params *p, const int32_t *cu_capacity, const int32_t *lengths,
                                   int32_t seq, void *K_c, void *V_c, const void *Q_window,
                                   const flowmm_plan_buffers *plan, void *workspace, size_t workspace_bytes,
                                   void *stream);

/* Message of the last failing call on this thread (static storage, never NULL). */
const char *flowmm_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FLOWMM_H */
