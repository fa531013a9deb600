// Steps "flow" and "select".
//   flow  : rho = mean over query heads of the share of proxy attention that lands on tokens
//           of the other modality; the layer merges across modalities iff rho > theta
//           (FlowMM, Information Flow Guided Merging: rho equation and threshold rule).
//   select: the B most important tokens of each KV head form the pivot set, the rest are
//           merged into it (same section, top-B rule).  The proxy tokens themselves are always
//           pivots.  Ties go to the lower position, pivots are listed in ascending position.
// One workgroup per (sequence, kv head, layer).  The B-th largest importance is found by a
// 4-pass radix select on the float bit patterns (importances are non-negative, so the bits
// order like the values); a block-wide ordered scan then compacts the pivots.
#include "device_common.h"
#include "kernels.h"
#include "profile.h"
#include "select_core.h"

namespace flowmm {

namespace {

constexpr int kThreads = 1024;

__global__ __launch_bounds__(kThreads) void select_kernel(Ctx c) {
  __shared__ SelectScratch<kThreads> scratch;
  __shared__ float lds_head[kThreads];
  const Shape &sh = c.sh;
  const int b = blockIdx.x, gkv = blockIdx.y, l = blockIdx.z;
  const SeqInfo s = load_seq(c.meta, b);

  // ---- flow (one workgroup per sequence and layer does it) ------------------------------
  if (gkv == 0) {
    const int *cu = c.meta + c.meta[MW_OFF_CU_SCORE];
    const int x0 = cu[b], x1 = cu[b + 1];
    for (int h0 = 0; h0 < sh.Hq; h0 += kThreads) {
      const int h = h0 + threadIdx.x;
      if (h < sh.Hq) {
        const float *cp = c.cross_part + (long long)(l * sh.Hq + h) * sh.tiles_score;
        float v = 0.f;
        for (int x = x0; x < x1; ++x) v += cp[x];
        lds_head[threadIdx.x] = v / (float)sh.W;  // share of this head's proxy attention
      }
      __syncthreads();
      if (threadIdx.x == 0) {
        float acc = h0 == 0 ? 0.f : c.rho[l * sh.batch + b];
        const int nh = min(kThreads, sh.Hq - h0);
        for (int i = 0; i < nh; ++i) acc += lds_head[i];
        c.rho[l * sh.batch + b] = acc;
      }
      __syncthreads();
    }
    if (threadIdx.x == 0) {
      const float rho = c.rho[l * sh.batch + b] / (float)sh.Hq;
      c.rho[l * sh.batch + b] = rho;
      c.mode[l * sh.batch + b] = rho > sh.theta ? 1 : 0;
    }
  }
  if (threadIdx.x == 0) c.n_dropped[(l * sh.Hkv + gkv) * sh.batch + b] = 0;

  // ---- top-B split -----------------------------------------------------------------------------
  const unsigned *imp = reinterpret_cast<const unsigned *>(c.importance) +
                        (long long)(l * sh.Hkv + gkv) * sh.T + s.tok_off;
  int *kept = c.kept_idx + (long long)(l * sh.Hkv + gkv) * sh.SB + s.kept_off;
  int *assign = c.assign + (long long)(l * sh.Hkv + gkv) * sh.T + s.tok_off;
  select_top_b<kThreads>(imp, s.L, sh.W, s.B, kept, assign, scratch);
}

}  // namespace

hipError_t launch_select(const Ctx &c) {
  ProfScope ps(c.stream, KID_SELECT);
  select_kernel<<<dim3(c.sh.batch, c.sh.Hkv, c.sh.n_layers), kThreads, 0, c.stream>>>(c);
  return hipGetLastError();
}

}  // namespace flowmm
