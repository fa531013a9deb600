// Places the host-packed metadata words at the head of the workspace (they travel as kernel
// arguments, so no host memory has to outlive the call and nothing synchronises) and expands
// the modality spans into one byte per packed token.
#include "device_common.h"
#include "kernels.h"
#include "profile.h"

namespace flowmm {

namespace {

__global__ __launch_bounds__(256) void meta_upload_kernel(MetaChunk chunk, int *dst, int n) {
  for (int i = threadIdx.x; i < n; i += 256) dst[i] = chunk.w[i];
}

// one workgroup per span: the modality byte of its tokens, and their places in the sequence's
// class order (all text positions ascending, then all image positions ascending)
__device__ __forceinline__ void expand_span(const int *meta, uint8_t *mod, int *cls_order) {
  const int batch = meta[MW_BATCH];
  const int *spans = meta + meta[MW_OFF_SPANS] + 3 * blockIdx.x;
  // owner sequence: the one whose span range contains this span
  int b = 0;
  for (int i = 0; i < batch; ++i) {
    const int *r = meta + meta[MW_OFF_SEQ] + i * SW_WORDS;
    if ((int)blockIdx.x >= r[SW_SPAN_OFF] && (int)blockIdx.x < r[SW_SPAN_OFF] + r[SW_N_SPANS]) b = i;
  }
  const int *rec = meta + meta[MW_OFF_SEQ] + b * SW_WORDS;
  const int tok_off = rec[SW_TOK_OFF];
  const uint8_t m = (uint8_t)spans[2];
  int before = m ? rec[SW_N_TEXT] : 0;  // tokens of this class in earlier spans of the sequence
  for (int j = rec[SW_SPAN_OFF]; j < (int)blockIdx.x; ++j) {
    const int *sp = meta + meta[MW_OFF_SPANS] + 3 * j;
    if (sp[2] == m) before += sp[1] - sp[0];
  }
  for (int i = spans[0] + threadIdx.x; i < spans[1]; i += 256) {
    mod[tok_off + i] = m;
    cls_order[tok_off + before + i - spans[0]] = i;
  }
}

__global__ __launch_bounds__(256) void expand_modality_kernel(const int *meta, uint8_t *mod, int *cls_order) {
  expand_span(meta, mod, cls_order);
}

// Both in one launch when the metadata fits one kernel-argument block: every workgroup reads the
// words from its arguments (nothing waits for the copy in the workspace), workgroup 0 also writes them.
__global__ __launch_bounds__(256) void meta_upload_expand_kernel(MetaChunk chunk, int *dst, int n, uint8_t *mod,
                                                                 int *cls_order) {
  if (blockIdx.x == 0)
    for (int i = threadIdx.x; i < n; i += 256) dst[i] = chunk.w[i];
  expand_span(chunk.w, mod, cls_order);
}

}  // namespace

hipError_t launch_meta_upload(const Ctx &c, const int *words, int n_words, bool expand_modality) {
  if (expand_modality && n_words <= kMetaChunkWords && words[MW_N_SPANS] > 0) {
    MetaChunk chunk;
    for (int i = 0; i < n_words; ++i) chunk.w[i] = words[i];
    ProfScope ps(c.stream, KID_META_UPLOAD);
    meta_upload_expand_kernel<<<words[MW_N_SPANS], 256, 0, c.stream>>>(chunk, c.meta, n_words, c.mod, c.cls_order);
    return hipGetLastError();
  }
  for (int off = 0; off < n_words; off += kMetaChunkWords) {
    MetaChunk chunk;
    const int n = n_words - off < kMetaChunkWords ? n_words - off : kMetaChunkWords;
    for (int i = 0; i < n; ++i) chunk.w[i] = words[off + i];
    ProfScope ps(c.stream, KID_META_UPLOAD);
    meta_upload_kernel<<<1, 256, 0, c.stream>>>(chunk, c.meta + off, n);
  }
  if (expand_modality) {
    ProfScope ps(c.stream, KID_EXPAND_MODALITY);
    expand_modality_kernel<<<words[MW_N_SPANS], 256, 0, c.stream>>>(c.meta, c.mod, c.cls_order);
  }
  return hipGetLastError();
}

}  // namespace flowmm
