// Step "match": every non-pivot key goes to the pivot with the largest cosine similarity
// among the pivots that are not highly sensitive (importance <= tau) and, in an intra-modal
// layer, share its modality (FlowMM, Sensitivity-Adaptive Token Matching: cosine equation and
// thresholded argmax; the intra/cross rule of Information Flow Guided Merging).
//
// The similarity matrix is never stored.  A workgroup owns 256 tokens (64 per wave, held as
// MFMA operands in registers straight from HBM) and walks over the pivots in LDS-staged
// tiles of 128 rows; each 32x32 block of dot products is scaled by the pivot's 1/norm, masked
// by eligibility and folded into a running (best value, best slot) per token.  The token's own
// norm is a positive factor common to all its candidates and is left out of the comparison.
#include "device_common.h"
#include "kernels.h"
#include "profile.h"

namespace flowmm {

namespace {

constexpr int kThreads = kMatchWaves * 64;
constexpr int kSub = kMatchTokPerWave / 32;

template <bool BF16, int D>
__global__ __launch_bounds__(kThreads) void match_kernel(Ctx c) {
  constexpr int NCH = Cfg<BF16, D>::NCH, NF = Cfg<BF16, D>::NF;
  __shared__ uint4 lds_piv[kPivotTile * (NCH + 1)];
  __shared__ float lds_w[kPivotTile];         // 1/norm of the pivot (0 for a zero row)
  __shared__ float lds_bias[2][kPivotTile];   // [token modality][pivot]: 0 eligible, -inf not
  const Shape &sh = c.sh;
  const int *meta = c.meta;
  const int *cu = meta + meta[MW_OFF_CU_MATCH];
  const int x = blockIdx.x, gkv = blockIdx.y, l = blockIdx.z;
  const int b = find_seq(cu, meta[MW_BATCH], x);
  const int tile = x - cu[b];
  const SeqInfo s = load_seq(meta, b);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 31, half = lane >> 5;
  const int tok0 = tile * kMatchTile + wave * kMatchTokPerWave;
  const long long unit = (long long)l * sh.Hkv + gkv;

  const uint4 *K = reinterpret_cast<const uint4 *>(c.K) + (long long)l * sh.ks_layer +
                   (long long)gkv * sh.ks_head + (long long)s.tok_off * sh.ks_tok;
  const uint8_t *mod = c.mod + s.tok_off;
  const float *imp = c.importance + unit * sh.T + s.tok_off;
  const int *kept = c.kept_idx + unit * sh.SB + s.kept_off;
  int *assign = c.assign + unit * sh.T + s.tok_off;
  const int mode_cross = c.mode[l * sh.batch + b];

  // this wave's tokens as B operands
  uint4 kf[kSub][NF];
  int tok[kSub], tokmod[kSub];
#pragma unroll
  for (int sub = 0; sub < kSub; ++sub) {
    tok[sub] = tok0 + sub * 32 + n;
    const int tc = tok[sub] < s.L ? tok[sub] : s.L - 1;
    tokmod[sub] = mod[tc];
    const uint4 *row = K + (long long)tc * sh.ks_tok + half;
#pragma unroll
    for (int f = 0; f < NF; ++f) kf[sub][f] = row[2 * f];
  }
  float best[kSub];
  int best_slot[kSub];
#pragma unroll
  for (int sub = 0; sub < kSub; ++sub) { best[sub] = -INFINITY; best_slot[sub] = -1; }

  for (int p0 = 0; p0 < s.B; p0 += kPivotTile) {
    const int np = min(kPivotTile, s.B - p0);
    __syncthreads();  // previous tile fully consumed
    // stage pivot rows, their inverse norms and eligibility
    constexpr int kRowsPerPass = kThreads / NCH;
    for (int r0 = 0; r0 < kPivotTile; r0 += kRowsPerPass) {
      const int pr = r0 + threadIdx.x / NCH, ch = threadIdx.x % NCH;
      uint4 v = make_uint4(0, 0, 0, 0);
      int ptok = 0;
      if (pr < np) {
        ptok = kept[p0 + pr];
        v = K[(long long)ptok * sh.ks_tok + ch];
      }
      lds_piv[pr * (NCH + 1) + ch] = v;
      float ss = chunk_sumsq<BF16>(v);
#pragma unroll
      for (int o = NCH / 2; o >= 1; o >>= 1) ss += __shfl_xor(ss, o, 64);
      if (ch == 0) {
        const bool real = pr < np;
        const bool sensitive = real && imp[ptok] > s.tau;
        const int pm = real ? mod[ptok] : 0;
        lds_w[pr] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
        const bool ok = real && !sensitive;
        lds_bias[0][pr] = ok && (mode_cross || pm == 0) ? 0.f : -INFINITY;
        lds_bias[1][pr] = ok && (mode_cross || pm == 1) ? 0.f : -INFINITY;
      }
    }
    __syncthreads();
    const int nblk = (np + 31) >> 5;
    for (int pb = 0; pb < nblk; ++pb) {
      f32x16_t acc[kSub];
#pragma unroll
      for (int sub = 0; sub < kSub; ++sub)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[sub][i] = 0.f;
      const uint4 *prow = lds_piv + (pb * 32 + n) * (NCH + 1) + half;
#pragma unroll
      for (int f = 0; f < NF; ++f) {
        const uint4 pf = prow[2 * f];
#pragma unroll
        for (int sub = 0; sub < kSub; ++sub) mma_chunk<BF16>(acc[sub], pf, kf[sub][f]);  // [pivot][token]
      }
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int pr = pb * 32 + acc_row(i, half);
        const float w = lds_w[pr];
#pragma unroll
        for (int sub = 0; sub < kSub; ++sub) {
          const float u = fmaf(acc[sub][i], w, lds_bias[tokmod[sub]][pr]);
          if (u > best[sub]) { best[sub] = u; best_slot[sub] = p0 + pr; }  // ascending slots: first maximum stays
        }
      }
    }
  }
  // the two half-waves saw disjoint pivot rows of the same token
  int dropped = 0;
#pragma unroll
  for (int sub = 0; sub < kSub; ++sub) {
    const float ob = __shfl_xor(best[sub], 32, 64);
    const int os = __shfl_xor(best_slot[sub], 32, 64);
    if (ob > best[sub] || (ob == best[sub] && (unsigned)os < (unsigned)best_slot[sub])) {
      best[sub] = ob;
      best_slot[sub] = os;
    }
    if (half == 0 && tok[sub] < s.L && assign[tok[sub]] == -2) {
      assign[tok[sub]] = best_slot[sub];
      dropped += best_slot[sub] < 0;
    }
  }
  dropped = wave_sum_int(dropped);
  if (lane == 0 && dropped) atomicAdd(&c.n_dropped[unit * sh.batch + b], dropped);
}

template <bool BF16, int D>
hipError_t launch_match_t(const Ctx &c) {
  ProfScope ps(c.stream, KID_MATCH);
  match_kernel<BF16, D><<<dim3(c.sh.tiles_match, c.sh.Hkv, c.sh.n_layers), kThreads, 0, c.stream>>>(c);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_match(const Ctx &c) {
  if (c.sh.bf16) return c.sh.d == 128 ? launch_match_t<true, 128>(c) : launch_match_t<true, 64>(c);
  return c.sh.d == 128 ? launch_match_t<false, 128>(c) : launch_match_t<false, 64>(c);
}

}  // namespace flowmm
