// C ABI of the library (include/flowmm.h): host-side argument checking, workspace layout and
// kernel sequencing.  All arithmetic of the method runs in the kernels this file launches.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../include/flowmm.h"
#include "kernels.h"

namespace {

using namespace flowmm;

thread_local char g_err[512] = "";

flowmm_status fail(flowmm_status code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Layout {
  Shape sh;
  InlineMeta inl;
  Regions rg;
  std::vector<int32_t> words;
  size_t plan_bytes[6];
  size_t workspace_bytes;
  size_t kv_extent_bytes, q_extent_bytes;
};

constexpr size_t kLdsLimit = kLdsBytes;

flowmm_status build_layout(const flowmm_params *p, Layout &lo) {
  if (!p) return fail(FLOWMM_EINVAL, "params is NULL");
  if (p->n_layers < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1)
    return fail(FLOWMM_EINVAL, "n_layers, n_q_heads and n_kv_heads must be >= 1");
  if (p->n_q_heads % p->n_kv_heads != 0)
    return fail(FLOWMM_EINVAL, "n_q_heads (%d) is not a multiple of n_kv_heads (%d)", p->n_q_heads, p->n_kv_heads);
  if (p->dtype != FLOWMM_F32 && p->dtype != FLOWMM_BF16) return fail(FLOWMM_EINVAL, "dtype must be FLOWMM_F32 or FLOWMM_BF16");
  if (p->head_dim < 1) return fail(FLOWMM_EINVAL, "head_dim must be positive");
  if (p->head_dim != 64 && p->head_dim != 128)
    return fail(FLOWMM_EUNSUPPORTED, "head_dim %d is not built (64 and 128 are)", p->head_dim);
  if (p->batch < 1) return fail(FLOWMM_EINVAL, "batch must be >= 1");
  if (!p->cu_seqlens || !p->budget_tokens || !p->spans || !p->cu_spans || !p->tau)
    return fail(FLOWMM_EINVAL, "cu_seqlens, budget_tokens, spans, cu_spans and tau must not be NULL");
  if (p->window < 1) return fail(FLOWMM_EINVAL, "window must be >= 1");
  if (!(p->scale >= 0.f) || !std::isfinite(p->scale)) return fail(FLOWMM_EINVAL, "scale must be finite and >= 0");
  if (std::isnan(p->theta)) return fail(FLOWMM_EINVAL, "theta is NaN");
  if (p->flags & ~(FLOWMM_FLAG_GENERIC_PATH | FLOWMM_FLAG_INVERT_FLOW | FLOWMM_FLAG_WEIGHTED_MERGE))
    return fail(FLOWMM_EINVAL, "unknown bits in flags");
  if (p->cu_seqlens[0] != 0 || p->cu_spans[0] != 0) return fail(FLOWMM_EINVAL, "cu_seqlens[0] and cu_spans[0] must be 0");

  const int es = p->dtype == FLOWMM_BF16 ? 2 : 4;
  const int epc = 16 / es;  // elements per 16-byte chunk
  const int64_t strides[6] = {p->k_stride_layer, p->k_stride_head, p->k_stride_token,
                              p->q_stride_layer, p->q_stride_head, p->q_stride_token};
  for (int i = 0; i < 6; ++i)
    if (strides[i] < 0 || strides[i] % epc != 0)
      return fail(FLOWMM_EINVAL, "strides must be non-negative multiples of 16 bytes (%d elements)", epc);
  if (p->k_stride_token < p->head_dim || p->q_stride_token < p->head_dim)
    return fail(FLOWMM_EINVAL, "token strides must be at least head_dim");
  // the kernels address the window queries of one (layer, kv head, sequence) with 32-bit byte offsets
  if (((int64_t)(p->n_q_heads / p->n_kv_heads - 1) * p->q_stride_head + (int64_t)(p->window - 1) * p->q_stride_token +
       p->head_dim) * es >= (int64_t)1 << 32)
    return fail(FLOWMM_EUNSUPPORTED, "the window queries of one kv head span 4 GiB or more");

  Shape &sh = lo.sh;
  sh.n_layers = p->n_layers; sh.Hq = p->n_q_heads; sh.Hkv = p->n_kv_heads; sh.G = sh.Hq / sh.Hkv;
  sh.d = p->head_dim; sh.bf16 = p->dtype == FLOWMM_BF16; sh.batch = p->batch; sh.W = p->window;
  sh.W_pad = (sh.W + 31) / 32 * 32;
  sh.R_pad = sh.G * sh.W_pad;
  const float scale = p->scale > 0.f ? p->scale : 1.0f / std::sqrt((float)p->head_dim);
  sh.scale_log2e = scale * 1.4426950408889634f;
  sh.theta = p->theta;
  sh.invert_flow = (p->flags & FLOWMM_FLAG_INVERT_FLOW) != 0;
  sh.weighted_merge = (p->flags & FLOWMM_FLAG_WEIGHTED_MERGE) != 0;
  sh.ks_layer = p->k_stride_layer / epc; sh.ks_head = p->k_stride_head / epc; sh.ks_tok = p->k_stride_token / epc;
  sh.qs_layer = p->q_stride_layer / epc; sh.qs_head = p->q_stride_head / epc; sh.qs_tok = p->q_stride_token / epc;

  const int batch = p->batch;
  const int match_tile = match_tile_tokens(sh.bf16), score_tile = score_tile_keys(sh.bf16);
  // key tiles a score workgroup walks over (it stages the query rows once per run): as many as leave
  // every compute unit a few workgroups
  int tpw = 1;
  {
    long long tiles = 0;
    for (int b = 0; b < batch; ++b) {
      const long long L = (long long)p->cu_seqlens[b + 1] - p->cu_seqlens[b];
      if (L > 0) tiles += (L + score_tile - 1) / score_tile;
    }
    tiles *= (long long)p->n_layers * p->n_kv_heads;
    while (tpw < 8 && tiles / (2 * tpw) >= 4 * 256) tpw *= 2;
  }
  sh.score_tpw = tpw;
  std::vector<int32_t> cu_score(batch + 1, 0), cu_match(batch + 1, 0), cu_task(batch + 1, 0),
      cu_multi(batch + 1, 0), cu_part(batch + 1, 0), cu_bp(batch + 1, 0), cu_flowq(batch + 1, 0);
  std::vector<int32_t> seq((size_t)batch * SW_WORDS, 0);
  int64_t sumB = 0;
  int maxB = 0, maxL = 0, maxE = 0;
  sh.rows32 = 1;
  for (int b = 0; b < batch; ++b) {
    const int64_t L64 = (int64_t)p->cu_seqlens[b + 1] - p->cu_seqlens[b];
    if (L64 < 1) return fail(FLOWMM_EINVAL, "cu_seqlens must be strictly increasing (sequence %d)", b);
    const int L = (int)L64, B = p->budget_tokens[b];
    if (p->window > L) return fail(FLOWMM_EINVAL, "window %d exceeds the length %d of sequence %d", p->window, L, b);
    if (B < p->window || B > L)
      return fail(FLOWMM_EINVAL, "budget %d of sequence %d is outside [window=%d, length=%d]", B, b, p->window, L);
    if (std::isnan(p->tau[b])) return fail(FLOWMM_EINVAL, "tau[%d] is NaN", b);
    const int s0 = p->cu_spans[b], s1 = p->cu_spans[b + 1];
    if (s1 <= s0) return fail(FLOWMM_EINVAL, "sequence %d has no spans", b);
    int pos = 0, win_img = 0, n_text = 0;
    for (int j = s0; j < s1; ++j) {
      const flowmm_span &sp = p->spans[j];
      if (sp.begin != pos || sp.end <= sp.begin)
        return fail(FLOWMM_EINVAL, "spans of sequence %d are not sorted, non-empty and contiguous (span %d)", b, j - s0);
      if (sp.modality != FLOWMM_TEXT && sp.modality != FLOWMM_IMAGE)
        return fail(FLOWMM_EINVAL, "span %d of sequence %d has modality %d", j - s0, b, sp.modality);
      if (sp.modality == FLOWMM_IMAGE && sp.end > L - p->window) win_img = 1;
      if (sp.modality == FLOWMM_TEXT) n_text += sp.end - sp.begin;
      pos = sp.end;
    }
    if (pos != L) return fail(FLOWMM_EINVAL, "spans of sequence %d cover [0,%d), not [0,%d)", b, pos, L);
    const int E = L - B;
    if (((int64_t)(L - 1) * p->k_stride_token + p->head_dim) * es >= (int64_t)1 << 32) sh.rows32 = 0;
    cu_score[b + 1] = cu_score[b] + ((L + score_tile - 1) / score_tile + tpw - 1) / tpw;
    // an intra-modal layer matches text and image tokens in separate tiles: one tile more at most
    cu_match[b + 1] = cu_match[b] + (L + match_tile - 1) / match_tile + 1;
    cu_bp[b + 1] = cu_bp[b] + (B + 31) / 32 * 32;
    cu_flowq[b + 1] = cu_flowq[b] + (L + kFlowQueryTile - 1) / kFlowQueryTile;
    cu_task[b + 1] = cu_task[b] + B + E / kTaskChunk + 1;
    cu_multi[b + 1] = cu_multi[b] + E / (kTaskChunk + 1) + 1;
    cu_part[b + 1] = cu_part[b] + 2 * (E / kTaskChunk) + 2;
    int32_t *r = &seq[(size_t)b * SW_WORDS];
    r[SW_TOK_OFF] = p->cu_seqlens[b]; r[SW_L] = L; r[SW_B] = B; r[SW_KEPT_OFF] = (int32_t)sumB;
    std::memcpy(&r[SW_TAU], &p->tau[b], 4);
    r[SW_SPAN_OFF] = s0; r[SW_N_SPANS] = s1 - s0; r[SW_WIN_HAS_IMG] = win_img; r[SW_N_TEXT] = n_text;
    sumB += B;
    if (B > maxB) maxB = B;
    if (L > maxL) maxL = L;
    if (E > maxE) maxE = E;
  }
  const int64_t T = p->cu_seqlens[batch];
  const int n_spans = p->cu_spans[batch];
  const int64_t units = (int64_t)sh.n_layers * sh.Hkv;
  if (units * T >= (int64_t)1 << 40) return fail(FLOWMM_EUNSUPPORTED, "cache too large");
  sh.T = (int)T; sh.SB = (int)sumB; sh.maxB = maxB; sh.maxL = maxL; sh.maxE = maxE; sh.n_spans = n_spans;
  sh.unit_path = !(p->flags & FLOWMM_FLAG_GENERIC_PATH) && unit_path_fits(sh);
  std::memset(&lo.inl, 0, sizeof(lo.inl));
  if (sh.unit_path) {
    for (int b = 0; b <= batch; ++b) cu_score[b] = b;  // one score tile per sequence
    InlineMeta &m = lo.inl;
    for (int b = 0; b < batch; ++b) {
      const int32_t *r = &seq[(size_t)b * SW_WORDS];
      m.tok_off[b] = r[SW_TOK_OFF]; m.L[b] = r[SW_L]; m.B[b] = r[SW_B]; m.kept_off[b] = r[SW_KEPT_OFF];
      m.tau[b] = p->tau[b];
      m.span_off[b] = p->cu_spans[b];
      if (r[SW_WIN_HAS_IMG]) m.win_has_img |= 1u << b;
    }
    m.span_off[batch] = n_spans;
    for (int j = 0; j < n_spans; ++j) {
      m.span_end[j] = p->spans[j].end;
      if (p->spans[j].modality == FLOWMM_IMAGE) m.span_is_image |= 1u << j;
    }
  }
  sh.tiles_score = cu_score[batch]; sh.tiles_match = cu_match[batch];
  sh.tasks_total = cu_task[batch]; sh.multi_total = cu_multi[batch]; sh.part_total = cu_part[batch];
  sh.SBP = cu_bp[batch];
  sh.flowq_total = cu_flowq[batch];
  if (score_lds_bytes(sh) > kLdsLimit)
    return fail(FLOWMM_EUNSUPPORTED, "(n_q_heads/n_kv_heads) x window = %d query rows per kv head do not fit in LDS", sh.R_pad);
  if (merge_csr_lds_bytes(maxB) > kLdsLimit)
    return fail(FLOWMM_EUNSUPPORTED, "budget %d per sequence is beyond what the merge kernel stages (32768)", maxB);
  if ((int64_t)sh.Hq > 1024) return fail(FLOWMM_EUNSUPPORTED, "more than 1024 query heads");

  // metadata words
  std::vector<int32_t> &w = lo.words;
  w.assign(MW_HEADER, 0);
  auto append = [&](const std::vector<int32_t> &v) { const int off = (int)w.size(); w.insert(w.end(), v.begin(), v.end()); return off; };
  w[MW_BATCH] = batch; w[MW_T] = sh.T; w[MW_SUMB] = sh.SB; w[MW_N_SPANS] = n_spans;
  w[MW_OFF_SEQ] = append(seq);
  {
    std::vector<int32_t> sp((size_t)n_spans * 3);
    for (int j = 0; j < n_spans; ++j) { sp[3 * j] = p->spans[j].begin; sp[3 * j + 1] = p->spans[j].end; sp[3 * j + 2] = p->spans[j].modality; }
    const int off = append(sp);
    w[MW_OFF_SPANS] = off;
  }
  w[MW_OFF_CU_SCORE] = append(cu_score);
  w[MW_OFF_CU_MATCH] = append(cu_match);
  w[MW_OFF_CU_TASK] = append(cu_task);
  w[MW_OFF_CU_MULTI] = append(cu_multi);
  w[MW_OFF_CU_PART] = append(cu_part);
  w[MW_OFF_CU_BP] = append(cu_bp);
  w[MW_OFF_CU_FLOWQ] = append(cu_flowq);

  // plan buffers
  lo.plan_bytes[0] = (size_t)units * T * 4;
  lo.plan_bytes[1] = (size_t)sh.n_layers * batch * 4;
  lo.plan_bytes[2] = (size_t)sh.n_layers * batch * 4;
  lo.plan_bytes[3] = (size_t)units * sumB * 4;
  lo.plan_bytes[4] = (size_t)units * T * 4;
  lo.plan_bytes[5] = (size_t)units * batch * 4;

  // workspace regions: metadata first, then the plan and the merge scratch share the rest
  Regions &rg = lo.rg;
  size_t off = 0;
  rg.meta = off; off += align256(w.size() * 4);
  rg.mod = off; off += align256((size_t)T);
  rg.cls_order = off; off += align256((size_t)T * 4);
  const size_t shared0 = off;
  rg.part_stats = off; off += align256((size_t)units * sh.tiles_score * sh.R_pad * sizeof(float2));
  rg.rowstat = off; off += align256((size_t)units * batch * sh.R_pad * sizeof(float2));
  rg.cross_part = off; off += align256((size_t)sh.n_layers * sh.Hq * sh.tiles_score * 4);
  rg.decode_part = off; off += align256((size_t)sh.n_layers * sh.Hq * batch * kDecodeMaxSplits * (sh.d + 2) * 4);
  rg.flow_part = off; off += align256((size_t)sh.n_layers * sh.Hq * sh.flowq_total * 4);
  if (!sh.unit_path) {
    rg.pl_slot = off; off += align256((size_t)units * 2 * sh.SBP * 4);
    rg.pl_tok = off; off += align256((size_t)units * 2 * sh.SBP * 4);
    rg.pl_w = off; off += align256((size_t)units * 2 * sh.SBP * 4);
    rg.pl_n = off; off += align256((size_t)units * batch * 2 * 4);
    rg.pack = off; off += align256((size_t)units * 2 * sh.SBP * (sh.d * es + 16));
    rg.ev_list = off; off += align256((size_t)units * T * 4);
    rg.ev_n = off; off += align256((size_t)units * batch * 2 * 4);
  } else {
    rg.pl_slot = rg.pl_tok = rg.pl_w = rg.pl_n = rg.pack = rg.ev_list = rg.ev_n = off;
  }
  rg.plan_end = off;
  off = shared0;
  rg.seg_off = off; off += align256((size_t)units * (sumB + batch) * 4);
  rg.members = off; off += align256((size_t)units * T * 4);
  rg.tasks = off; off += align256((size_t)units * sh.tasks_total * sizeof(int4));
  rg.n_tasks = off; off += align256((size_t)units * batch * 2 * 4);
  rg.multi = off; off += align256((size_t)units * sh.multi_total * sizeof(int4));
  rg.n_multi = off; off += align256((size_t)units * batch * 4);
  rg.partials = off; off += align256((size_t)units * sh.part_total * 2 * sh.d * 4);
  rg.partial_w = off; off += align256((size_t)units * sh.part_total * 4);
  rg.merge_end = off;
  lo.workspace_bytes = rg.plan_end > rg.merge_end ? rg.plan_end : rg.merge_end;

  lo.kv_extent_bytes = ((size_t)(sh.n_layers - 1) * p->k_stride_layer + (size_t)(sh.Hkv - 1) * p->k_stride_head +
                        (size_t)(T - 1) * p->k_stride_token + sh.d) * es;
  lo.q_extent_bytes = ((size_t)(sh.n_layers - 1) * p->q_stride_layer + (size_t)(sh.Hq - 1) * p->q_stride_head +
                       (size_t)((int64_t)batch * sh.W - 1) * p->q_stride_token + sh.d) * es;
  return FLOWMM_OK;
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }

bool overlaps(const void *a, size_t na, const void *b, size_t nb) {
  const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
  return a0 < b0 + nb && b0 < a0 + na;
}

flowmm_status check_plan_buffers(const flowmm_plan_buffers *plan) {
  if (!plan) return fail(FLOWMM_EINVAL, "plan is NULL");
  const void *ptrs[6] = {plan->importance, plan->rho, plan->mode, plan->kept_idx, plan->assign, plan->n_dropped};
  static const char *names[6] = {"importance", "rho", "mode", "kept_idx", "assign", "n_dropped"};
  for (int i = 0; i < 6; ++i) {
    if (!ptrs[i]) return fail(FLOWMM_EINVAL, "plan->%s is NULL", names[i]);
    if (reinterpret_cast<uintptr_t>(ptrs[i]) & 3) return fail(FLOWMM_EINVAL, "plan->%s is not 4-byte aligned", names[i]);
  }
  return FLOWMM_OK;
}

void fill_ctx(Ctx &c, const Layout &lo, const flowmm_plan_buffers *plan, void *workspace, void *stream) {
  std::memset(&c, 0, sizeof(c));
  c.sh = lo.sh;
  c.inl = lo.inl;
  c.stream = reinterpret_cast<hipStream_t>(stream);
  c.layer0 = 0;
  c.layers = lo.sh.n_layers;
  c.importance = plan->importance; c.rho = plan->rho; c.mode = plan->mode;
  c.kept_idx = plan->kept_idx; c.assign = plan->assign; c.n_dropped = plan->n_dropped;
  char *ws = reinterpret_cast<char *>(workspace);
  c.meta = reinterpret_cast<int *>(ws + lo.rg.meta);
  c.mod = reinterpret_cast<uint8_t *>(ws + lo.rg.mod);
  c.part_stats = reinterpret_cast<float2 *>(ws + lo.rg.part_stats);
  c.rowstat = reinterpret_cast<float *>(ws + lo.rg.rowstat);
  c.cross_part = reinterpret_cast<float *>(ws + lo.rg.cross_part);
  c.cls_order = reinterpret_cast<int *>(ws + lo.rg.cls_order);
  c.pl_slot = reinterpret_cast<int *>(ws + lo.rg.pl_slot);
  c.pl_tok = reinterpret_cast<int *>(ws + lo.rg.pl_tok);
  c.pl_w = reinterpret_cast<float *>(ws + lo.rg.pl_w);
  c.pl_n = reinterpret_cast<int *>(ws + lo.rg.pl_n);
  c.pack = reinterpret_cast<uint4 *>(ws + lo.rg.pack);
  c.ev_list = reinterpret_cast<int *>(ws + lo.rg.ev_list);
  c.ev_n = reinterpret_cast<int *>(ws + lo.rg.ev_n);
  c.seg_off = reinterpret_cast<int *>(ws + lo.rg.seg_off);
  c.members = reinterpret_cast<int *>(ws + lo.rg.members);
  c.tasks = reinterpret_cast<int4 *>(ws + lo.rg.tasks);
  c.n_tasks = reinterpret_cast<int *>(ws + lo.rg.n_tasks);
  c.multi = reinterpret_cast<int4 *>(ws + lo.rg.multi);
  c.n_multi = reinterpret_cast<int *>(ws + lo.rg.n_multi);
  c.partials = reinterpret_cast<float *>(ws + lo.rg.partials);
  c.partial_w = reinterpret_cast<float *>(ws + lo.rg.partial_w);
}

flowmm_status hip_fail(hipError_t e, const char *what) {
  return fail(FLOWMM_EHIP, "%s: %s", what, hipGetErrorString(e));
}

}  // namespace

#define FLOWMM_API __attribute__((visibility("default")))

extern "C" {

FLOWMM_API const char *flowmm_last_error(void) { return g_err; }

FLOWMM_API flowmm_status flowmm_plan_sizes(const flowmm_params *p, size_t plan_bytes[6], size_t *workspace_bytes) {
  Layout lo;
  const flowmm_status st = build_layout(p, lo);
  if (st != FLOWMM_OK) return st;
  if (plan_bytes) for (int i = 0; i < 6; ++i) plan_bytes[i] = lo.plan_bytes[i];
  if (workspace_bytes) *workspace_bytes = lo.workspace_bytes;
  return FLOWMM_OK;
}

FLOWMM_API flowmm_status flowmm_plan(const flowmm_params *p, const void *K, const void *Q_window,
                          const flowmm_plan_buffers *plan, void *workspace, size_t workspace_bytes,
                          void *stream) {
  Layout lo;
  flowmm_status st = build_layout(p, lo);
  if (st != FLOWMM_OK) return st;
  if (!K || !Q_window || !workspace) return fail(FLOWMM_EINVAL, "K, Q_window and workspace must not be NULL");
  if (misaligned(K) || misaligned(Q_window) || misaligned(workspace))
    return fail(FLOWMM_EINVAL, "K, Q_window and workspace must be 16-byte aligned");
  if ((st = check_plan_buffers(plan)) != FLOWMM_OK) return st;
  if (workspace_bytes < lo.workspace_bytes)
    return fail(FLOWMM_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, lo.workspace_bytes);
  Ctx c;
  fill_ctx(c, lo, plan, workspace, stream);
  c.K = K; c.Q = Q_window;
  hipError_t e;
  if (c.sh.unit_path) {
    if ((e = launch_unit_plan(c)) != hipSuccess) return hip_fail(e, "unit-resident plan kernels");
    return FLOWMM_OK;
  }
  if ((e = launch_meta_upload(c, lo.words.data(), (int)lo.words.size(), true)) != hipSuccess) return hip_fail(e, "metadata upload");
  if ((e = launch_score(c)) != hipSuccess) return hip_fail(e, "score kernels");
  if ((e = launch_select(c)) != hipSuccess) return hip_fail(e, "select kernel");
  if ((e = launch_match(c)) != hipSuccess) return hip_fail(e, "match kernel");
  return FLOWMM_OK;
}

}  // extern "C"

namespace {

flowmm_status check_merge_args(const Layout &lo, const void *K, const void *V, void *K_out, void *V_out) {
  if (!K || !V || !K_out || !V_out) return fail(FLOWMM_EINVAL, "K, V, K_out and V_out must not be NULL");
  if (misaligned(K) || misaligned(V) || misaligned(K_out) || misaligned(V_out))
    return fail(FLOWMM_EINVAL, "K, V, K_out and V_out must be 16-byte aligned");
  const size_t out_bytes = (size_t)lo.sh.n_layers * lo.sh.Hkv * lo.sh.SB * lo.sh.d * (lo.sh.bf16 ? 2 : 4);
  const void *ins[2] = {K, V};
  void *outs[2] = {K_out, V_out};
  for (int i = 0; i < 2; ++i)
    for (int j = 0; j < 2; ++j)
      if (overlaps(outs[i], out_bytes, ins[j], lo.kv_extent_bytes))
        return fail(FLOWMM_EINVAL, "outputs must not overlap K or V (in-place compaction is not supported)");
  if (overlaps(K_out, out_bytes, V_out, out_bytes)) return fail(FLOWMM_EINVAL, "K_out and V_out overlap");
  return FLOWMM_OK;
}


// ---- the whole method in one enqueue, on a workspace that has already been found large enough ----
flowmm_status check_plan_merge_args(const Layout &lo, const void *K, const void *V, const void *Q_window,
                                    const flowmm_plan_buffers *plan, void *K_out, void *V_out) {
  flowmm_status st;
  if (!Q_window) return fail(FLOWMM_EINVAL, "Q_window must not be NULL");
  if (misaligned(Q_window)) return fail(FLOWMM_EINVAL, "Q_window must be 16-byte aligned");
  if ((st = check_merge_args(lo, K, V, K_out, V_out)) != FLOWMM_OK) return st;
  return check_plan_buffers(plan);
}

flowmm_status plan_merge_in(const Layout &lo, const void *K, const void *V, const void *Q_window,
                            const flowmm_plan_buffers *plan, void *K_out, void *V_out, void *workspace, void *stream) {
  Ctx c;
  fill_ctx(c, lo, plan, workspace, stream);
  c.K = K; c.V = V; c.Q = Q_window; c.K_out = K_out; c.V_out = V_out;
  hipError_t e;
  if (c.sh.unit_path) {
    if ((e = launch_unit_plan(c, false)) != hipSuccess) return hip_fail(e, "unit-resident plan kernel");
    if ((e = launch_unit_merge(c, true)) != hipSuccess) return hip_fail(e, "unit-resident flow and merge kernel");
    return FLOWMM_OK;
  }
  // the metadata block sits in front of the scratch that the plan and the merge kernels share, so one upload serves both
  if ((e = launch_meta_upload(c, lo.words.data(), (int)lo.words.size(), true)) != hipSuccess) return hip_fail(e, "metadata upload");
  if ((e = launch_score(c)) != hipSuccess) return hip_fail(e, "score kernels");
  if ((e = launch_select(c)) != hipSuccess) return hip_fail(e, "select kernel");
  if ((e = launch_match(c)) != hipSuccess) return hip_fail(e, "match kernel");
  if ((e = launch_merge(c)) != hipSuccess) return hip_fail(e, "merge kernels");
  return FLOWMM_OK;
}

// ---- scratch for callers that cannot allocate ------------------------------------------------------
// Device memory the library itself owns: every GPU it runs on holds this array from the first use
// until the process ends.  Host code never uses the array's name as an address: the name is a
// host-side stand-in, and each device has its own copy at its own address, looked up once per
// device (with that device current) and kept.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

flowmm_status static_scratch(void **out) {
  constexpr int kMaxDevices = 64;
  static std::atomic<void *> ptr_of[kMaxDevices];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(FLOWMM_EUNSUPPORTED, "device ordinal %d beyond %d", dev, kMaxDevices - 1);
  void *ptr = ptr_of[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if ((e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch))) != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    if (!ptr || (reinterpret_cast<uintptr_t>(ptr) & 255)) return fail(FLOWMM_EHIP, "the scratch array has no usable device address");
    ptr_of[dev].store(ptr, std::memory_order_release);
  }
  *out = ptr;
  return FLOWMM_OK;
}

}  // namespace

extern "C" {

FLOWMM_API flowmm_status flowmm_merge(const flowmm_params *p, const flowmm_plan_buffers *plan, const void *K,
                           const void *V, void *K_out, void *V_out, void *workspace,
                           size_t workspace_bytes, void *stream) {
  Layout lo;
  flowmm_status st = build_layout(p, lo);
  if (st != FLOWMM_OK) return st;
  if (!workspace || misaligned(workspace)) return fail(FLOWMM_EINVAL, "workspace must be a 16-byte aligned device pointer");
  if ((st = check_merge_args(lo, K, V, K_out, V_out)) != FLOWMM_OK) return st;
  if ((st = check_plan_buffers(plan)) != FLOWMM_OK) return st;
  if (workspace_bytes < lo.workspace_bytes)
    return fail(FLOWMM_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, lo.workspace_bytes);
  Ctx c;
  fill_ctx(c, lo, plan, workspace, stream);
  c.K = K; c.V = V; c.K_out = K_out; c.V_out = V_out;
  hipError_t e;
  if (c.sh.unit_path) {
    if ((e = launch_unit_merge(c)) != hipSuccess) return hip_fail(e, "unit-resident merge kernel");
    return FLOWMM_OK;
  }
  if ((e = launch_meta_upload(c, lo.words.data(), (int)lo.words.size(), false)) != hipSuccess) return hip_fail(e, "metadata upload");
  if ((e = launch_merge(c)) != hipSuccess) return hip_fail(e, "merge kernels");
  return FLOWMM_OK;
}

FLOWMM_API flowmm_status flowmm_plan_merge(const flowmm_params *p, const void *K, const void *V, const void *Q_window,
                                const flowmm_plan_buffers *plan, void *K_out, void *V_out, void *workspace,
                                size_t workspace_bytes, void *stream) {
  Layout lo;
  flowmm_status st = build_layout(p, lo);
  if (st != FLOWMM_OK) return st;
  if (!workspace) return fail(FLOWMM_EINVAL, "workspace must not be NULL");
  if (misaligned(workspace)) return fail(FLOWMM_EINVAL, "workspace must be 16-byte aligned");
  if ((st = check_plan_merge_args(lo, K, V, Q_window, plan, K_out, V_out)) != FLOWMM_OK) return st;
  if (workspace_bytes < lo.workspace_bytes)
    return fail(FLOWMM_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, lo.workspace_bytes);
  return plan_merge_in(lo, K, V, Q_window, plan, K_out, V_out, workspace, stream);
}

FLOWMM_API size_t flowmm_static_workspace_bytes(void) { return kStaticScratchBytes; }

FLOWMM_API flowmm_status flowmm_plan_merge_static(const flowmm_params *p, const void *K, const void *V,
                                       const void *Q_window, const flowmm_plan_buffers *plan, void *K_out,
                                       void *V_out, void *stream) {
  Layout lo;
  flowmm_status st = build_layout(p, lo);
  if (st != FLOWMM_OK) return st;
  if (lo.workspace_bytes > kStaticScratchBytes)
    return fail(FLOWMM_EWORKSPACE,
                "these shapes need %zu bytes of scratch, the library's own scratch array holds %zu: "
                "use flowmm_plan_merge with a workspace of the caller's",
                lo.workspace_bytes, kStaticScratchBytes);
  if ((st = check_plan_merge_args(lo, K, V, Q_window, plan, K_out, V_out)) != FLOWMM_OK) return st;
  void *ws = nullptr;
  if ((st = static_scratch(&ws)) != FLOWMM_OK) return st;  // the first HIP call: everything above is host-only
  return plan_merge_in(lo, K, V, Q_window, plan, K_out, V_out, ws, stream);
}

FLOWMM_API flowmm_status flowmm_flow_exact(const flowmm_params *p, const void *K, const void *Q_full,
                                int64_t qf_stride_layer, int64_t qf_stride_head, int64_t qf_stride_token,
                                float *rho, int32_t *mode, void *workspace, size_t workspace_bytes, void *stream) {
  Layout lo;
  flowmm_status st = build_layout(p, lo);
  if (st != FLOWMM_OK) return st;
  if (!K || !Q_full || !rho || !mode || !workspace) return fail(FLOWMM_EINVAL, "K, Q_full, rho, mode and workspace must not be NULL");
  if (misaligned(K) || misaligned(Q_full) || misaligned(workspace))
    return fail(FLOWMM_EINVAL, "K, Q_full and workspace must be 16-byte aligned");
  if ((reinterpret_cast<uintptr_t>(rho) | reinterpret_cast<uintptr_t>(mode)) & 3)
    return fail(FLOWMM_EINVAL, "rho and mode must be 4-byte aligned");
  const int epc = lo.sh.bf16 ? 8 : 4;
  const int64_t strides[3] = {qf_stride_layer, qf_stride_head, qf_stride_token};
  for (int i = 0; i < 3; ++i)
    if (strides[i] < 0 || strides[i] % epc != 0)
      return fail(FLOWMM_EINVAL, "strides must be non-negative multiples of 16 bytes (%d elements)", epc);
  if (qf_stride_token < lo.sh.d) return fail(FLOWMM_EINVAL, "token strides must be at least head_dim");
  // a tile of kFlowQueryTile query rows is addressed with 32-bit byte offsets
  if (((int64_t)(kFlowQueryTile - 1) * qf_stride_token + lo.sh.d) * (lo.sh.bf16 ? 2 : 4) >= (int64_t)1 << 32)
    return fail(FLOWMM_EUNSUPPORTED, "256 query rows span 4 GiB or more");
  if (workspace_bytes < lo.workspace_bytes)
    return fail(FLOWMM_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, lo.workspace_bytes);
  flowmm_plan_buffers none;
  std::memset(&none, 0, sizeof(none));
  Ctx c;
  fill_ctx(c, lo, &none, workspace, stream);
  c.K = K;
  FlowExactArgs a;
  a.Q = Q_full;
  a.qs_layer = qf_stride_layer / epc; a.qs_head = qf_stride_head / epc; a.qs_tok = qf_stride_token / epc;
  a.part = reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) + lo.rg.flow_part);
  a.qtiles_total = lo.sh.flowq_total;
  a.rho = rho; a.mode = mode;
  hipError_t e;
  if ((e = launch_meta_upload(c, lo.words.data(), (int)lo.words.size(), true)) != hipSuccess) return hip_fail(e, "metadata upload");
  if ((e = launch_flow_exact(c, a)) != hipSuccess) return hip_fail(e, "exact flow-ratio kernels");
  return FLOWMM_OK;
}

FLOWMM_API flowmm_status flowmm_decode_attention(const flowmm_params *p, const void *q, const void *K_c, const void *V_c,
                                      void *out, void *workspace, size_t workspace_bytes, void *stream) {
  Layout lo;
  flowmm_status st = build_layout(p, lo);
  if (st != FLOWMM_OK) return st;
  if (!q || !K_c || !V_c || !out || !workspace) return fail(FLOWMM_EINVAL, "q, K_c, V_c, out and workspace must not be NULL");
  if (misaligned(q) || misaligned(K_c) || misaligned(V_c) || misaligned(out) || misaligned(workspace))
    return fail(FLOWMM_EINVAL, "q, K_c, V_c, out and workspace must be 16-byte aligned");
  if (workspace_bytes < lo.workspace_bytes)
    return fail(FLOWMM_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, lo.workspace_bytes);
  flowmm_plan_buffers none;
  std::memset(&none, 0, sizeof(none));
  Ctx c;
  fill_ctx(c, lo, &none, workspace, stream);
  DecodeArgs a;
  a.q = q; a.K_c = K_c; a.V_c = V_c; a.out = out;
  a.part = reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) + lo.rg.decode_part);
  a.splits = decode_splits(lo.sh);
  a.g0 = 0;
  hipError_t e;
  if ((e = launch_meta_upload(c, lo.words.data(), (int)lo.words.size(), false)) != hipSuccess) return hip_fail(e, "metadata upload");
  if ((e = launch_decode_attention(c, a)) != hipSuccess) return hip_fail(e, "decode attention kernels");
  return FLOWMM_OK;
}

}  // extern "C"

namespace {

// The single-sequence, single-modality call that a re-merge of one sequence of the cache amounts to.
struct RemergeCall {
  flowmm_params one;
  int32_t cu[2], budget[1], cu_spans[2];
  flowmm_span span[1];
  float tau[1];
  Layout lo;
  size_t out_bytes, tmp_k, tmp_v, total_bytes;  // merged rows wait behind the ordinary scratch
};

flowmm_status check_cache_ranges(const flowmm_params *p, const int32_t *cu_capacity) {
  if (!p) return fail(FLOWMM_EINVAL, "params is NULL");
  if (!cu_capacity) return fail(FLOWMM_EINVAL, "cu_capacity must not be NULL");
  if (p->batch < 1) return fail(FLOWMM_EINVAL, "batch must be >= 1");
  if (cu_capacity[0] != 0) return fail(FLOWMM_EINVAL, "cu_capacity[0] must be 0");
  for (int b = 0; b < p->batch; ++b)
    if (cu_capacity[b + 1] <= cu_capacity[b]) return fail(FLOWMM_EINVAL, "cu_capacity must be strictly increasing (sequence %d)", b);
  return FLOWMM_OK;
}

flowmm_status build_remerge(const flowmm_params *p, const int32_t *cu_capacity, int32_t seq, int32_t length, RemergeCall &rc) {
  flowmm_status st = check_cache_ranges(p, cu_capacity);
  if (st != FLOWMM_OK) return st;
  if (seq < 0 || seq >= p->batch) return fail(FLOWMM_EINVAL, "sequence %d is outside the batch of %d", seq, p->batch);
  if (!p->budget_tokens || !p->tau) return fail(FLOWMM_EINVAL, "budget_tokens and tau must not be NULL");
  const int cap = cu_capacity[seq + 1] - cu_capacity[seq];
  if (length < 1 || length > cap) return fail(FLOWMM_EINVAL, "length %d of sequence %d is outside [1, capacity=%d]", length, seq, cap);
  rc.one = *p;
  rc.cu[0] = 0; rc.cu[1] = length;
  rc.budget[0] = p->budget_tokens[seq];
  rc.tau[0] = p->tau[seq];
  rc.span[0].begin = 0; rc.span[0].end = length; rc.span[0].modality = FLOWMM_TEXT;
  rc.cu_spans[0] = 0; rc.cu_spans[1] = 1;
  rc.one.batch = 1;
  rc.one.cu_seqlens = rc.cu; rc.one.budget_tokens = rc.budget; rc.one.spans = rc.span; rc.one.cu_spans = rc.cu_spans;
  rc.one.tau = rc.tau;
  rc.one.theta = -1.0f;  // one modality: rho = 0 and both strategies admit the same pivots
  if (p->flags & ~(FLOWMM_FLAG_GENERIC_PATH | FLOWMM_FLAG_INVERT_FLOW | FLOWMM_FLAG_WEIGHTED_MERGE))
    return fail(FLOWMM_EINVAL, "unknown bits in flags");
  rc.one.flags = p->flags & (FLOWMM_FLAG_GENERIC_PATH | FLOWMM_FLAG_WEIGHTED_MERGE);
  if ((st = build_layout(&rc.one, rc.lo)) != FLOWMM_OK) return st;
  const Shape &sh = rc.lo.sh;
  rc.out_bytes = (size_t)sh.n_layers * sh.Hkv * sh.SB * sh.d * (sh.bf16 ? 2 : 4);
  rc.tmp_k = align256(rc.lo.workspace_bytes);
  rc.tmp_v = rc.tmp_k + align256(rc.out_bytes);
  rc.total_bytes = rc.tmp_v + align256(rc.out_bytes);
  return FLOWMM_OK;
}

}  // namespace

extern "C" {

FLOWMM_API flowmm_status flowmm_cache_append(const flowmm_params *p, const int32_t *cu_capacity, const int32_t *lengths,
                                  void *K_c, void *V_c, const void *k_new, const void *v_new, void *stream) {
  flowmm_status st = check_cache_ranges(p, cu_capacity);
  if (st != FLOWMM_OK) return st;
  if (!lengths) return fail(FLOWMM_EINVAL, "lengths must not be NULL");
  if (p->n_layers < 1 || p->n_kv_heads < 1) return fail(FLOWMM_EINVAL, "n_layers and n_kv_heads must be >= 1");
  if (p->dtype != FLOWMM_F32 && p->dtype != FLOWMM_BF16) return fail(FLOWMM_EINVAL, "dtype must be FLOWMM_F32 or FLOWMM_BF16");
  if (p->head_dim != 64 && p->head_dim != 128) return fail(FLOWMM_EUNSUPPORTED, "head_dim %d is not built (64 and 128 are)", p->head_dim);
  const int es = p->dtype == FLOWMM_BF16 ? 2 : 4, epc = 16 / es;
  const int64_t strides[3] = {p->k_stride_layer, p->k_stride_head, p->k_stride_token};
  for (int i = 0; i < 3; ++i)
    if (strides[i] < 0 || strides[i] % epc != 0)
      return fail(FLOWMM_EINVAL, "strides must be non-negative multiples of 16 bytes (%d elements)", epc);
  if (p->k_stride_token < p->head_dim) return fail(FLOWMM_EINVAL, "token strides must be at least head_dim");
  if (!K_c || !V_c || !k_new || !v_new) return fail(FLOWMM_EINVAL, "K_c, V_c, k_new and v_new must not be NULL");
  if (misaligned(K_c) || misaligned(V_c) || misaligned(k_new) || misaligned(v_new))
    return fail(FLOWMM_EINVAL, "K_c, V_c, k_new and v_new must be 16-byte aligned");
  for (int b = 0; b < p->batch; ++b) {
    const int cap = cu_capacity[b + 1] - cu_capacity[b];
    if (lengths[b] < 0 || lengths[b] > cap) return fail(FLOWMM_EINVAL, "lengths[%d] = %d is outside [0, capacity=%d]", b, lengths[b], cap);
    if (lengths[b] == cap) return fail(FLOWMM_EINVAL, "the cache of sequence %d is full (%d rows): re-merge it before appending", b, cap);
  }
  AppendArgs a;
  a.K_c = K_c; a.V_c = V_c; a.k_new = k_new; a.v_new = v_new;
  a.ks_layer = p->k_stride_layer / epc; a.ks_head = p->k_stride_head / epc; a.ks_tok = p->k_stride_token / epc;
  a.nch = p->head_dim * es / 16; a.batch = p->batch;
  for (int b0 = 0; b0 < p->batch; b0 += kAppendSeqs) {
    const int n = p->batch - b0 < kAppendSeqs ? p->batch - b0 : kAppendSeqs;
    a.b0 = b0;
    for (int i = 0; i < n; ++i) a.row[i] = cu_capacity[b0 + i] + lengths[b0 + i];
    const hipError_t e = launch_cache_append(a, n, p->n_kv_heads, p->n_layers, reinterpret_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "cache append kernel");
  }
  return FLOWMM_OK;
}

FLOWMM_API flowmm_status flowmm_cache_remerge_sizes(const flowmm_params *p, const int32_t *cu_capacity, int32_t seq,
                                         int32_t length, size_t plan_bytes[6], size_t *workspace_bytes) {
  RemergeCall rc;
  const flowmm_status st = build_remerge(p, cu_capacity, seq, length, rc);
  if (st != FLOWMM_OK) return st;
  if (plan_bytes) for (int i = 0; i < 6; ++i) plan_bytes[i] = rc.lo.plan_bytes[i];
  if (workspace_bytes) *workspace_bytes = rc.total_bytes;
  return FLOWMM_OK;
}

FLOWMM_API flowmm_status flowmm_cache_remerge(const flowmm_params *p, const int32_t *cu_capacity, const int32_t *lengths,
                                   int32_t seq, void *K_c, void *V_c, const void *Q_window,
                                   const flowmm_plan_buffers *plan, void *workspace, size_t workspace_bytes,
                                   void *stream) {
  if (!lengths) return fail(FLOWMM_EINVAL, "lengths must not be NULL");
  if (!p || seq < 0 || seq >= p->batch) return fail(FLOWMM_EINVAL, "params is NULL or the sequence is outside the batch");
  RemergeCall rc;
  flowmm_status st = build_remerge(p, cu_capacity, seq, lengths[seq], rc);
  if (st != FLOWMM_OK) return st;
  if (!K_c || !V_c) return fail(FLOWMM_EINVAL, "K_c and V_c must not be NULL");
  if (!workspace) return fail(FLOWMM_EINVAL, "workspace must not be NULL");
  if (misaligned(workspace)) return fail(FLOWMM_EINVAL, "workspace must be 16-byte aligned");
  if (workspace_bytes < rc.total_bytes)
    return fail(FLOWMM_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, rc.total_bytes);
  const int es = rc.lo.sh.bf16 ? 2 : 4;
  const size_t seq_off = (size_t)cu_capacity[seq] * (size_t)p->k_stride_token * es;
  char *Ks = reinterpret_cast<char *>(K_c) + seq_off, *Vs = reinterpret_cast<char *>(V_c) + seq_off;
  char *ws = reinterpret_cast<char *>(workspace);
  void *tmp_k = ws + rc.tmp_k, *tmp_v = ws + rc.tmp_v;
  // the merged rows are written behind the scratch first (the merge reads rows that the result will overwrite)
  if ((st = check_plan_merge_args(rc.lo, Ks, Vs, Q_window, plan, tmp_k, tmp_v)) != FLOWMM_OK) return st;
  if ((st = plan_merge_in(rc.lo, Ks, Vs, Q_window, plan, tmp_k, tmp_v, workspace, stream)) != FLOWMM_OK) return st;
  StoreRowsArgs a;
  a.K_c = Ks; a.V_c = Vs; a.K_src = tmp_k; a.V_src = tmp_v;
  const int epc = 16 / es;
  a.ks_layer = p->k_stride_layer / epc; a.ks_head = p->k_stride_head / epc; a.ks_tok = p->k_stride_token / epc;
  a.nch = rc.lo.sh.d * es / 16; a.B = rc.lo.sh.SB; a.row0 = 0;
  const hipError_t e = launch_cache_store_rows(a, rc.lo.sh.Hkv, rc.lo.sh.n_layers, reinterpret_cast<hipStream_t>(stream));
  if (e != hipSuccess) return hip_fail(e, "cache store kernel");
  return FLOWMM_OK;
}

}  // extern "C"
