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

namespace flowmm {

namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;

// exclusive prefix sum over the workgroup, in thread order; *total receives the block sum
__device__ __forceinline__ int block_exclusive_scan(int v, int *lds_wave /*[kWaves+1]*/, int *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int u = __shfl_up(inc, o, 64);
    if (lane >= o) inc += u;
  }
  __syncthreads();  // lds_wave may still be read from a previous call
  if (lane == 63) lds_wave[wave] = inc;
  __syncthreads();
  if (wave == 0) {
    int w = lane < kWaves ? lds_wave[lane] : 0;
    int winc = w;
#pragma unroll
    for (int o = 1; o < kWaves; o <<= 1) {
      const int u = __shfl_up(winc, o, 64);
      if (lane >= o) winc += u;
    }
    if (lane < kWaves) lds_wave[lane] = winc - w;
    if (lane == kWaves - 1) lds_wave[kWaves] = winc;
  }
  __syncthreads();
  *total = lds_wave[kWaves];
  return lds_wave[wave] + inc - v;
}

__global__ __launch_bounds__(kThreads) void select_kernel(Ctx c) {
  __shared__ int hist[256];
  __shared__ int lds_wave[kWaves + 1];
  __shared__ unsigned sh_prefix;
  __shared__ int sh_remaining;
  __shared__ float lds_head[kThreads];
  const Shape &sh = c.sh;
  const int b = blockIdx.x, gkv = blockIdx.y, l = blockIdx.z;
  const SeqInfo s = load_seq(c.meta, b);
  const int lane = threadIdx.x & 63;

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

  // ---- B-th largest importance among the non-proxy tokens ---------------------------------
  const unsigned *imp = reinterpret_cast<const unsigned *>(c.importance) +
                        (long long)(l * sh.Hkv + gkv) * sh.T + s.tok_off;
  const int nbody = s.L - sh.W;
  const int need = s.B - sh.W;  // pivots still to choose among the body tokens
  unsigned thr = 0xffffffffu;   // nothing in the body exceeds or equals this
  int need_eq = 0;
  if (need > 0) {
    unsigned prefix = 0, mask = 0;
    int remaining = need;
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      if (threadIdx.x < 256) hist[threadIdx.x] = 0;
      __syncthreads();
      for (int i0 = 0; i0 < nbody; i0 += kThreads) {
        const int i = i0 + threadIdx.x;
        const unsigned k = i < nbody ? imp[i] : 0u;
        const bool act = i < nbody && (k & mask) == prefix;
        const int dg = (k >> shift) & 255;
        const unsigned long long am = __ballot(act);
        if (am) {
          const int first = __ffsll((long long)am) - 1;
          const int d0 = __shfl(dg, first, 64);
          if (__ballot(act && dg == d0) == am) {
            if (lane == first) atomicAdd(&hist[d0], __popcll(am));
          } else if (act) {
            atomicAdd(&hist[dg], 1);
          }
        }
      }
      __syncthreads();
      // bins in descending order: thread t looks at bin 255 - t
      const int cnt = threadIdx.x < 256 ? hist[255 - threadIdx.x] : 0;
      int total;
      const int before = block_exclusive_scan(cnt, lds_wave, &total);
      if (threadIdx.x < 256 && before < remaining && remaining <= before + cnt) {
        sh_prefix = prefix | ((unsigned)(255 - threadIdx.x) << shift);
        sh_remaining = remaining - before;
      }
      __syncthreads();
      prefix = sh_prefix;
      remaining = sh_remaining;
      mask |= 255u << shift;
    }
    thr = prefix;
    need_eq = remaining;  // how many tokens equal to the threshold are still pivots
  }

  // ---- ordered compaction -------------------------------------------------------------------
  int *kept = c.kept_idx + (long long)(l * sh.Hkv + gkv) * sh.SB + s.kept_off;
  int *assign = c.assign + (long long)(l * sh.Hkv + gkv) * sh.T + s.tok_off;
  int gt_carry = 0, eq_carry = 0;
  for (int i0 = 0; i0 < s.L; i0 += kThreads) {
    const int i = i0 + threadIdx.x;
    int gt = 0, eq = 0;
    if (i < s.L) {
      if (i >= nbody) {
        gt = 1;
      } else {
        const unsigned k = imp[i];
        gt = k > thr;
        eq = k == thr;
      }
    }
    int total;
    const int before = block_exclusive_scan(gt | (eq << 16), lds_wave, &total);
    const int gt_before = gt_carry + (before & 0xffff);
    const int eq_before = eq_carry + (before >> 16);
    if (i < s.L) {
      const bool is_kept = gt || (eq && eq_before < need_eq);
      const int slot = gt_before + min(eq_before, need_eq);
      if (is_kept) kept[slot] = i;
      assign[i] = is_kept ? slot : -2;  // -2: to be matched
    }
    gt_carry += total & 0xffff;
    eq_carry += total >> 16;
  }
}

}  // namespace

hipError_t launch_select(const Ctx &c) {
  ProfScope ps(c.stream, KID_SELECT);
  select_kernel<<<dim3(c.sh.batch, c.sh.Hkv, c.sh.n_layers), kThreads, 0, c.stream>>>(c);
  return hipGetLastError();
}

}  // namespace flowmm
