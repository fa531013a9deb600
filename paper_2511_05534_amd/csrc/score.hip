// Step "score": attention of the proxy (window) queries over all cached keys, reduced to the
// proxy importance of every key and to each query head's cross-modal attention mass
// (FlowMM, Information Flow Guided Merging: importance equation and the A_{v->t}, A_{t->v}
// sums; attention as in the Preliminary section).
//
// The logits tile of a workgroup never leaves registers.  Keys are split across workgroups,
// so the softmax needs every row's global (max, sum): pass 1 writes those per tile, a small
// pass 2 folds them per row, pass 3 recomputes the tile's logits and reduces the normalised
// probabilities over the query rows.  Both heavy passes read K once, straight from HBM into
// MFMA operand registers (one 16-byte chunk per lane and k step).
#include "device_common.h"
#include "kernels.h"
#include "profile.h"

namespace flowmm {

namespace {

constexpr int kThreads = kScoreWaves * 64;
constexpr int kSub = kScoreKeysPerWave / 32;

struct TileCtx {
  int b, tile, x, gkv, l, wave, lane, n, half, key0;  // key0: first key of this wave
  SeqInfo s;
};

__device__ __forceinline__ TileCtx tile_ctx(const Ctx &c) {
  TileCtx t;
  const int *meta = c.meta;
  const int batch = meta[MW_BATCH];
  const int *cu = meta + meta[MW_OFF_CU_SCORE];
  t.x = blockIdx.x;
  t.b = find_seq(cu, batch, t.x);
  t.tile = t.x - cu[t.b];
  t.gkv = blockIdx.y;
  t.l = blockIdx.z;
  t.s = load_seq(meta, t.b);
  t.wave = threadIdx.x >> 6;
  t.lane = threadIdx.x & 63;
  t.n = t.lane & 31;
  t.half = t.lane >> 5;
  t.key0 = t.tile * kScoreTile + t.wave * kScoreKeysPerWave;
  return t;
}

// Stage the R_pad query rows of this (sequence, layer, kv head) into LDS, row stride NCH+1
// chunks (the odd stride keeps the 16-byte fragment reads of 16 consecutive rows on distinct
// banks).  Rows beyond W inside a head's padded block are zero.
template <bool BF16, int D>
__device__ __forceinline__ void stage_queries(const Ctx &c, const TileCtx &t, uint4 *ldsq) {
  constexpr int NCH = Cfg<BF16, D>::NCH;
  const Shape &sh = c.sh;
  const uint4 *Q = reinterpret_cast<const uint4 *>(c.Q) + (long long)t.l * sh.qs_layer;
  for (int idx = threadIdx.x; idx < sh.R_pad * NCH; idx += kThreads) {
    const int row = idx / NCH, ch = idx - row * NCH;
    const int g = row / sh.W_pad, r = row - g * sh.W_pad;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r < sh.W)
      v = Q[(long long)(t.gkv * sh.G + g) * sh.qs_head + (long long)(t.b * sh.W + r) * sh.qs_tok + ch];
    ldsq[row * (NCH + 1) + ch] = v;
  }
}

template <bool BF16, int D>
__device__ __forceinline__ void load_keys(const Ctx &c, const TileCtx &t, uint4 (&kf)[kSub][Cfg<BF16, D>::NF]) {
  constexpr int NF = Cfg<BF16, D>::NF;
  const Shape &sh = c.sh;
  const uint4 *K = reinterpret_cast<const uint4 *>(c.K) + (long long)t.l * sh.ks_layer +
                   (long long)t.gkv * sh.ks_head;
#pragma unroll
  for (int sub = 0; sub < kSub; ++sub) {
    int key = t.key0 + sub * 32 + t.n;
    key = key < t.s.L ? key : t.s.L - 1;
    const uint4 *row = K + (long long)(t.s.tok_off + key) * sh.ks_tok + t.half;
#pragma unroll
    for (int f = 0; f < NF; ++f) kf[sub][f] = row[2 * f];
  }
}

// ---- pass 1: per-tile row statistics ---------------------------------------------------
template <bool BF16, int D>
__global__ __launch_bounds__(kThreads) void score_stats_kernel(Ctx c) {
  constexpr int NCH = Cfg<BF16, D>::NCH, NF = Cfg<BF16, D>::NF;
  extern __shared__ uint4 lds[];
  const Shape &sh = c.sh;
  const TileCtx t = tile_ctx(c);
  uint4 *ldsq = lds;
  float2 *lds_stats = reinterpret_cast<float2 *>(lds + sh.R_pad * (NCH + 1));  // [waves][R_pad]

  uint4 kf[kSub][NF];
  load_keys<BF16, D>(c, t, kf);
  stage_queries<BF16, D>(c, t, ldsq);
  __syncthreads();

  const int RB = sh.R_pad >> 5;
  const float cl = sh.scale_log2e;
  for (int rb = 0; rb < RB; ++rb) {
    f32x16_t acc[kSub];
#pragma unroll
    for (int sub = 0; sub < kSub; ++sub)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[sub][i] = 0.f;
    const uint4 *qrow = ldsq + (rb * 32 + t.n) * (NCH + 1) + t.half;
#pragma unroll
    for (int f = 0; f < NF; ++f) {
      const uint4 qf = qrow[2 * f];
#pragma unroll
      for (int sub = 0; sub < kSub; ++sub) mma_chunk<BF16>(acc[sub], kf[sub][f], qf);  // [key][query row]
    }
    const int row = rb * 32 + t.n;
    const int r = row % sh.W_pad;
    const int limit = r < sh.W ? t.s.L - sh.W + r : -1;  // last key this query may see
    float m = -INFINITY;
#pragma unroll
    for (int sub = 0; sub < kSub; ++sub)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = t.key0 + sub * 32 + acc_row(i, t.half);
        const float v = key <= limit ? acc[sub][i] * cl : -INFINITY;
        acc[sub][i] = v;
        m = fmaxf(m, v);
      }
    float z = 0.f;
    if (m > -INFINITY) {
#pragma unroll
      for (int sub = 0; sub < kSub; ++sub)
#pragma unroll
        for (int i = 0; i < 16; ++i) z += fast_exp2(acc[sub][i] - m);
    }
    const float m2 = __shfl_xor(m, 32, 64), z2 = __shfl_xor(z, 32, 64);
    stat_combine(m, z, m2, z2);
    if (t.half == 0) lds_stats[t.wave * sh.R_pad + row] = make_float2(m, z);
  }
  __syncthreads();
  float2 *out = c.part_stats + ((long long)(t.l * sh.Hkv + t.gkv) * sh.tiles_score + t.x) * sh.R_pad;
  for (int row = threadIdx.x; row < sh.R_pad; row += kThreads) {
    float2 a = lds_stats[row];
#pragma unroll
    for (int w = 1; w < kScoreWaves; ++w) {
      const float2 o = lds_stats[w * sh.R_pad + row];
      stat_combine(a.x, a.y, o.x, o.y);
    }
    out[row] = a;
  }
}

// ---- pass 2: fold the tiles of a sequence ----------------------------------------------
__global__ __launch_bounds__(256) void score_combine_kernel(Ctx c) {
  const Shape &sh = c.sh;
  const int b = blockIdx.x, gkv = blockIdx.y, l = blockIdx.z;
  const int *cu = c.meta + c.meta[MW_OFF_CU_SCORE];
  const int x0 = cu[b], x1 = cu[b + 1];
  const float2 *in = c.part_stats + (long long)(l * sh.Hkv + gkv) * sh.tiles_score * sh.R_pad;
  float2 *out = c.rowstat + ((long long)(l * sh.Hkv + gkv) * sh.batch + b) * sh.R_pad;
  for (int row = threadIdx.x; row < sh.R_pad; row += 256) {
    float m = -INFINITY, z = 0.f;
    for (int x = x0; x < x1; ++x) {
      const float2 o = in[(long long)x * sh.R_pad + row];
      stat_combine(m, z, o.x, o.y);
    }
    out[row] = z > 0.f ? make_float2(m, 1.0f / z) : make_float2(0.f, 0.f);
  }
}

// ---- pass 3: normalised probabilities reduced over the query rows ------------------------
template <bool BF16, int D>
__global__ __launch_bounds__(kThreads) void score_colsum_kernel(Ctx c) {
  constexpr int NCH = Cfg<BF16, D>::NCH, NF = Cfg<BF16, D>::NF;
  extern __shared__ uint4 lds[];
  const Shape &sh = c.sh;
  const TileCtx t = tile_ctx(c);
  uint4 *ldsq = lds;
  float2 *lds_rs = reinterpret_cast<float2 *>(lds + sh.R_pad * (NCH + 1));  // [R_pad]
  float *lds_rowimg = reinterpret_cast<float *>(lds_rs + sh.R_pad);          // [W_pad]
  float *lds_cross = lds_rowimg + sh.W_pad;                                  // [waves][G]

  uint4 kf[kSub][NF];
  load_keys<BF16, D>(c, t, kf);
  stage_queries<BF16, D>(c, t, ldsq);
  const float2 *rs = c.rowstat + ((long long)(t.l * sh.Hkv + t.gkv) * sh.batch + t.b) * sh.R_pad;
  for (int row = threadIdx.x; row < sh.R_pad; row += kThreads) lds_rs[row] = rs[row];
  const uint8_t *mod = c.mod + t.s.tok_off;
  for (int r = threadIdx.x; r < sh.W_pad; r += kThreads)
    lds_rowimg[r] = (r < sh.W && mod[t.s.L - sh.W + r]) ? 1.f : 0.f;
  int keymod[kSub], key[kSub];
#pragma unroll
  for (int sub = 0; sub < kSub; ++sub) {
    key[sub] = t.key0 + sub * 32 + t.n;
    keymod[sub] = mod[key[sub] < t.s.L ? key[sub] : t.s.L - 1];
  }
  __syncthreads();

  const int RB = sh.R_pad >> 5;
  const int blocks_per_head = sh.W_pad >> 5;
  const float cl = sh.scale_log2e;
  const bool win_img = t.s.win_has_img != 0;
  float colsum[kSub], cross_acc = 0.f;
#pragma unroll
  for (int sub = 0; sub < kSub; ++sub) colsum[sub] = 0.f;

  for (int rb = 0; rb < RB; ++rb) {
    f32x16_t acc[kSub];
#pragma unroll
    for (int sub = 0; sub < kSub; ++sub)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[sub][i] = 0.f;
    const uint4 *qrow = ldsq + (rb * 32 + t.n) * (NCH + 1) + t.half;
#pragma unroll
    for (int f = 0; f < NF; ++f) {
      const uint4 qf = qrow[2 * f];
#pragma unroll
      for (int sub = 0; sub < kSub; ++sub) mma_chunk<BF16>(acc[sub], qf, kf[sub][f]);  // [query row][key]
    }
    const int rbase = (rb % blocks_per_head) * 32;  // first window row of this block
    float bs[kSub], bsi[kSub];
#pragma unroll
    for (int sub = 0; sub < kSub; ++sub) bs[sub] = bsi[sub] = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int ri = acc_row(i, t.half);
      const float2 st = lds_rs[rb * 32 + ri];           // (max, 1/sum); (0, 0) for padding rows
      const int r = rbase + ri;
      const int limit = r < sh.W ? t.s.L - sh.W + r : -1;
      const float wimg = win_img ? lds_rowimg[r] : 0.f;
#pragma unroll
      for (int sub = 0; sub < kSub; ++sub) {
        const float p = key[sub] <= limit ? fast_exp2(acc[sub][i] * cl - st.x) * st.y : 0.f;
        bs[sub] += p;
        bsi[sub] = fmaf(p, wimg, bsi[sub]);
      }
    }
#pragma unroll
    for (int sub = 0; sub < kSub; ++sub) {
      colsum[sub] += bs[sub];
      // mass sent to the other modality: image keys seen by text rows, text keys by image rows
      cross_acc += keymod[sub] ? bs[sub] - bsi[sub] : bsi[sub];
    }
    if ((rb + 1) % blocks_per_head == 0) {
      const float v = wave_sum(cross_acc);
      if (t.lane == 0) lds_cross[t.wave * sh.G + rb / blocks_per_head] = v;
      cross_acc = 0.f;
    }
  }
  const float inv_rows = 1.0f / (float)(sh.G * sh.W);
  float *imp = c.importance + (long long)(t.l * sh.Hkv + t.gkv) * sh.T + t.s.tok_off;
#pragma unroll
  for (int sub = 0; sub < kSub; ++sub) {
    const float tot = colsum[sub] + __shfl_xor(colsum[sub], 32, 64);
    if (t.half == 0 && key[sub] < t.s.L) imp[key[sub]] = tot * inv_rows;
  }
  __syncthreads();
  for (int g = threadIdx.x; g < sh.G; g += kThreads) {
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < kScoreWaves; ++w) v += lds_cross[w * sh.G + g];
    c.cross_part[(long long)(t.l * sh.Hq + t.gkv * sh.G + g) * sh.tiles_score + t.x] = v;
  }
}

template <bool BF16, int D>
hipError_t launch_score_t(const Ctx &c) {
  constexpr int NCH = Cfg<BF16, D>::NCH;
  const Shape &sh = c.sh;
  const size_t q_bytes = (size_t)sh.R_pad * (NCH + 1) * 16;
  const size_t lds1 = q_bytes + (size_t)kScoreWaves * sh.R_pad * sizeof(float2);
  const size_t lds3 = q_bytes + (size_t)sh.R_pad * sizeof(float2) + (size_t)sh.W_pad * 4 +
                      (size_t)kScoreWaves * sh.G * 4;
  hipError_t e;
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(score_stats_kernel<BF16, D>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds1);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(score_colsum_kernel<BF16, D>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds3);
  if (e != hipSuccess) return e;
  const dim3 grid(sh.tiles_score, sh.Hkv, sh.n_layers);
  {
    ProfScope ps(c.stream, KID_SCORE_STATS);
    score_stats_kernel<BF16, D><<<grid, kThreads, lds1, c.stream>>>(c);
  }
  {
    ProfScope ps(c.stream, KID_SCORE_COMBINE);
    score_combine_kernel<<<dim3(sh.batch, sh.Hkv, sh.n_layers), 256, 0, c.stream>>>(c);
  }
  {
    ProfScope ps(c.stream, KID_SCORE_COLSUM);
    score_colsum_kernel<BF16, D><<<grid, kThreads, lds3, c.stream>>>(c);
  }
  return hipGetLastError();
}

}  // namespace

size_t score_lds_bytes(const Shape &sh) {
  const int nch = sh.d * (sh.bf16 ? 2 : 4) / 16;
  return (size_t)sh.R_pad * (nch + 1) * 16 + (size_t)kScoreWaves * sh.R_pad * sizeof(float2) +
         (size_t)sh.W_pad * 4 + (size_t)kScoreWaves * sh.G * 4;
}

hipError_t launch_score(const Ctx &c) {
  if (c.sh.bf16) return c.sh.d == 128 ? launch_score_t<true, 128>(c) : launch_score_t<true, 64>(c);
  return c.sh.d == 128 ? launch_score_t<false, 128>(c) : launch_score_t<false, 64>(c);
}

}  // namespace flowmm
