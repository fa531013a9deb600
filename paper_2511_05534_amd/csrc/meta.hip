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

// one workgroup per span
__global__ __launch_bounds__(256) void expand_modality_kernel(const int *meta, uint8_t *mod) {
  const int batch = meta[MW_BATCH];
  const int *spans = meta + meta[MW_OFF_SPANS] + 3 * blockIdx.x;
  // owner sequence: the one whose span range contains this span
  int b = 0;
  for (int i = 0; i < batch; ++i) {
    const int *r = meta + meta[MW_OFF_SEQ] + i * SW_WORDS;
    if ((int)blockIdx.x >= r[SW_SPAN_OFF] && (int)blockIdx.x < r[SW_SPAN_OFF] + r[SW_N_SPANS]) b = i;
  }
  const int tok_off = (meta + meta[MW_OFF_SEQ] + b * SW_WORDS)[SW_TOK_OFF];
  const uint8_t m = (uint8_t)spans[2];
  for (int i = spans[0] + threadIdx.x; i < spans[1]; i += 256) mod[tok_off + i] = m;
}

}  // namespace

hipError_t launch_meta_upload(const Ctx &c, const int *words, int n_words, bool expand_modality) {
  for (int off = 0; off < n_words; off += kMetaChunkWords) {
    MetaChunk chunk;
    const int n = n_words - off < kMetaChunkWords ? n_words - off : kMetaChunkWords;
    for (int i = 0; i < n; ++i) chunk.w[i] = words[off + i];
    ProfScope ps(c.stream, KID_META_UPLOAD);
    meta_upload_kernel<<<1, 256, 0, c.stream>>>(chunk, c.meta + off, n);
  }
  if (expand_modality) {
    ProfScope ps(c.stream, KID_EXPAND_MODALITY);
    expand_modality_kernel<<<words[MW_N_SPANS], 256, 0, c.stream>>>(c.meta, c.mod);
  }
  return hipGetLastError();
}

}  // namespace flowmm
