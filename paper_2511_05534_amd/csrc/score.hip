// Step "score": attention of the proxy (window) queries over all cached keys, reduced to the
// proxy importance of every key and to each query head's cross-modal attention mass
// (FlowMM, Information Flow Guided Merging: importance equation and the A_{v->t}, A_{t->v}
// sums; attention as in the Preliminary section).
//
// The logits tile of a workgroup never leaves registers.  Keys are split across workgroups,
// so the softmax needs every row's global (max, sum): pass 1 writes those per tile, a small
// pass 2 folds them per row into one offset c = max + log2(sum), pass 3 recomputes the tile's
// logits and reduces exp2(logit - c) over the query rows.  Both heavy passes read K once,
// straight from HBM into MFMA operand registers (one 16-byte chunk per lane and k step, 32*KS
// keys per wave); the query rows of the (sequence, kv head, layer) arrive in LDS by direct
// global->LDS loads and every fragment read from there feeds KS matrix instructions.
// Only the tiles that reach into the window (or past the end of the sequence) pay for the
// causal mask; only sequences whose window holds image tokens pay for per-row modality weights.
#include "device_common.h"
#include "kernels.h"
#include "profile.h"
#include "score_core.h"

namespace flowmm {

namespace {

constexpr int kThreads = kScoreWaves * 64;

struct TileCtx {
  int b, tile, x, gkv, l, wave, lane, n, half, key0;  // key0: first key of this wave in the current tile
  int tile_end;                                       // the run covers tiles [tile, tile_end) of sequence b
  bool masked;                                        // some key of the current tile is hidden from some window row
  SeqInfo s;
};

// Workgroups are handed to the eight XCDs in turn; all runs of a (layer, kv head) go to one
// XCD so that its query rows sit in one L2.  Returns false for the padding workgroups.
template <int TILE>
__device__ __forceinline__ bool tile_ctx(const Ctx &c, TileCtx &t) {
  const Shape &sh = c.sh;
  const int *meta = c.meta;
  const int xcd = blockIdx.x & 7, k = blockIdx.x >> 3;
  const int ul = k / sh.tiles_score;
  t.x = k - ul * sh.tiles_score;
  const int unit = ul * 8 + xcd;
  if (unit >= sh.n_layers * sh.Hkv) return false;
  t.l = unit / sh.Hkv;
  t.gkv = unit - t.l * sh.Hkv;
  const int *cu = meta + meta[MW_OFF_CU_SCORE];
  t.b = find_seq(cu, meta[MW_BATCH], t.x);
  t.s = load_seq(meta, t.b);
  t.tile = (t.x - cu[t.b]) * sh.score_tpw;
  t.tile_end = min(t.tile + sh.score_tpw, (t.s.L + TILE - 1) / TILE);
  t.wave = threadIdx.x >> 6;
  t.lane = threadIdx.x & 63;
  t.n = t.lane & 31;
  t.half = t.lane >> 5;
  t.key0 = t.tile * TILE + t.wave * (TILE / kScoreWaves);
  t.masked = (t.tile + 1) * TILE > t.s.L - sh.W;
  return true;
}

// position the context on tile `tile` of the run
template <int TILE>
__device__ __forceinline__ void set_tile(const Ctx &c, TileCtx &t, int tile) {
  t.tile = tile;
  t.key0 = tile * TILE + t.wave * (TILE / kScoreWaves);
  t.masked = (tile + 1) * TILE > t.s.L - c.sh.W;
}

// Request the R_pad query rows of this (sequence, layer, kv head) into LDS, row stride NCH+1
// chunks (the odd stride keeps the 16-byte fragment reads of 16 consecutive rows on distinct
// banks).  Rows beyond W inside a head's padded block, and the padding chunk of every row, come
// from 16 zero bytes in the metadata block.
template <bool BF16, int D>
__device__ __forceinline__ void stage_queries(const Ctx &c, const TileCtx &t, uint4 *ldsq) {
  constexpr int NCH = Cfg<BF16, D>::NCH, RS = NCH + 1;
  const Shape &sh = c.sh;
  const uint4 *Q = reinterpret_cast<const uint4 *>(c.Q) + (long long)t.l * sh.qs_layer +
                   (long long)(t.gkv * sh.G) * sh.qs_head + (long long)(t.b * sh.W) * sh.qs_tok;
  const int total = sh.R_pad * RS;
  // chunk q of the LDS image is chunk ch of row r of head g; q advances by the workgroup size per
  // trip, so (g, r, ch) are carried along instead of being divided out again
  constexpr int kRowStep = kThreads / RS, kChStep = kThreads % RS;
  int q = t.wave * 64 + t.lane;
  int row = q / RS, ch = q - row * RS;
  int g = row / sh.W_pad, r = row - g * sh.W_pad;
  for (int q0 = t.wave * 64; q0 < total; q0 += kThreads) {
    if (q0 + t.lane < total) {
      if (r < sh.W && ch < NCH)
        load_to_lds<16>(Q, (unsigned)(g * sh.qs_head + r * sh.qs_tok + ch) * 16u, ldsq + q0);
      else
        ldsq[q0 + t.lane] = make_uint4(0, 0, 0, 0);  // padding rows and the padding chunk of every row
    }
    ch += kChStep;
    r += kRowStep;
    if (ch >= RS) { ch -= RS; ++r; }
    while (r >= sh.W_pad) { r -= sh.W_pad; ++g; }
  }
}

template <bool BF16, int D, int KS>
__device__ __forceinline__ void load_keys(const Ctx &c, const TileCtx &t, uint4 (&kf)[KS][Cfg<BF16, D>::NF]) {
  constexpr int NF = Cfg<BF16, D>::NF;
  const Shape &sh = c.sh;
  const uint4 *K = reinterpret_cast<const uint4 *>(c.K) + (long long)t.l * sh.ks_layer +
                   (long long)t.gkv * sh.ks_head;
#pragma unroll
  for (int sub = 0; sub < KS; ++sub) {
    int key = t.key0 + sub * 32 + t.n;
    key = key < t.s.L ? key : t.s.L - 1;
    const uint4 *row = K + (long long)(t.s.tok_off + key) * sh.ks_tok + t.half;
#pragma unroll
    for (int f = 0; f < NF; ++f) kf[sub][f] = row[2 * f];
  }
}

// ---- pass 1: per-tile row statistics ---------------------------------------------------
template <bool BF16, int D, int KS, bool MASKED>
__device__ __forceinline__ void stats_body(const Ctx &c, const TileCtx &t, const uint4 (&kf)[KS][Cfg<BF16, D>::NF],
                                           const uint4 *ldsq, float *lds_stats) {
  constexpr int NF = Cfg<BF16, D>::NF, RS = Cfg<BF16, D>::NCH + 1;
  constexpr int AHEAD = NF < 2 ? NF : 2;
  const Shape &sh = c.sh;
  const int RB = sh.R_pad >> 5;
  const float cl = sh.scale_log2e;
  const char *qbase = reinterpret_cast<const char *>(ldsq) + (t.n * RS + t.half) * 16;
  uint4 pf[AHEAD];
#pragma unroll
  for (int f = 0; f < AHEAD; ++f) pf[f] = *reinterpret_cast<const uint4 *>(qbase + 32 * f);
  for (int rb = 0; rb < RB; ++rb) {
    f32x16_t acc[KS];
    block_products<BF16, D, KS, true, AHEAD>(acc, kf, pf, qbase + rb * (32 * RS * 16), rb + 1 < RB);  // [key][query row]
    const int row = rb * 32 + t.n;
    float m = -INFINITY, z = 0.f;
    if constexpr (MASKED) {
      const int r = row % sh.W_pad;
      const int limit = r < sh.W ? t.s.L - sh.W + r : -1;  // last key this query may see
#pragma unroll
      for (int sub = 0; sub < KS; ++sub)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = t.key0 + sub * 32 + acc_row(i, t.half);
          acc[sub][i] = key <= limit ? acc[sub][i] : -INFINITY;
          m = fmaxf(m, acc[sub][i]);
        }
      if (m > -INFINITY) {
        const float mc = m * cl;
#pragma unroll
        for (int sub = 0; sub < KS; ++sub)
#pragma unroll
          for (int i = 0; i < 16; ++i) z += fast_exp2(fmaf(acc[sub][i], cl, -mc));
      }
      m *= cl;
    } else {
#pragma unroll
      for (int sub = 0; sub < KS; ++sub)
#pragma unroll
        for (int i = 0; i < 16; i += 2) m = fmaxf(fmaxf(m, acc[sub][i]), acc[sub][i + 1]);
      m *= cl;  // cl > 0: the largest logit is the largest product
#pragma unroll
      for (int sub = 0; sub < KS; ++sub)
#pragma unroll
        for (int i = 0; i < 16; ++i) z += fast_exp2(fmaf(acc[sub][i], cl, -m));
    }
    const float m2 = __shfl_xor(m, 32, 64), z2 = __shfl_xor(z, 32, 64);
    stat_combine(m, z, m2, z2);
    // log2 of the row's sum of 2^logit over this wave's keys so far in the run: the pair (that, 1)
    // stands for (m, z); the slot belongs to this lane, earlier tiles of the run left their sum there
    if (t.half == 0) {
      float *slot = lds_stats + t.wave * sh.R_pad + row;
      float m0 = *slot, z0 = m0 == -INFINITY ? 0.f : 1.f;
      stat_combine(m0, z0, m, z);
      *slot = z0 > 0.f ? m0 + __builtin_amdgcn_logf(z0) : -INFINITY;
    }
  }
}

// RUN: the workgroup may have several tiles (a loop around the tile costs a few registers that the
// one-tile kernel, which small workloads get, does not have to spill)
template <bool BF16, int D, bool RUN>
__global__ __launch_bounds__(kThreads, 4) void score_stats_kernel(Ctx c) {
  constexpr int NCH = Cfg<BF16, D>::NCH, NF = Cfg<BF16, D>::NF, KS = score_subs(BF16);
  extern __shared__ uint4 lds[];
  const Shape &sh = c.sh;
  TileCtx t;
  if (!tile_ctx<score_tile_keys(BF16)>(c, t)) return;
  uint4 *ldsq = lds;
  float *lds_stats = reinterpret_cast<float *>(lds + sh.R_pad * (NCH + 1));  // [waves][R_pad]
  uint4 kf[KS][NF];
  load_keys<BF16, D, KS>(c, t, kf);  // the long way first (HBM); the query rows come from L2
  stage_queries<BF16, D>(c, t, ldsq);
  for (int row = t.lane; row < sh.R_pad; row += 64) lds_stats[t.wave * sh.R_pad + row] = -INFINITY;
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  // the run's tiles one after the other on the same query rows; the workgroup that shares the compute
  // unit computes while this one waits for its next keys
  const int tile_end = RUN ? t.tile_end : t.tile + 1;
  for (int tile = t.tile; tile < tile_end; ++tile) {
    if (tile != t.tile) {
      set_tile<score_tile_keys(BF16)>(c, t, tile);
      load_keys<BF16, D, KS>(c, t, kf);
    }
    if (t.key0 < t.s.L) {  // waves past the end of the sequence have nothing to add
      if (t.masked) stats_body<BF16, D, KS, true>(c, t, kf, ldsq, lds_stats);
      else stats_body<BF16, D, KS, false>(c, t, kf, ldsq, lds_stats);
    }
  }
  __syncthreads();
  float2 *out = c.part_stats + ((long long)(t.l * sh.Hkv + t.gkv) * sh.tiles_score + t.x) * sh.R_pad;
  for (int row = threadIdx.x; row < sh.R_pad; row += kThreads) {
    float2 a = make_float2(lds_stats[row], 1.f);
    if (a.x == -INFINITY) a.y = 0.f;
#pragma unroll
    for (int w = 1; w < kScoreWaves; ++w) {
      const float o = lds_stats[w * sh.R_pad + row];
      stat_combine(a.x, a.y, o, o == -INFINITY ? 0.f : 1.f);
    }
    out[row] = a;
  }
}

// ---- pass 2: fold the tiles of a sequence ----------------------------------------------
__global__ __launch_bounds__(256) void score_combine_kernel(Ctx c) {
  const Shape &sh = c.sh;
  const int b = rotated_block_x(), gkv = blockIdx.y, l = blockIdx.z;
  const int *cu = c.meta + c.meta[MW_OFF_CU_SCORE];
  const int x0 = cu[b], x1 = cu[b + 1];
  const float2 *in = c.part_stats + (long long)(l * sh.Hkv + gkv) * sh.tiles_score * sh.R_pad;
  float *out = c.rowstat + ((long long)(l * sh.Hkv + gkv) * sh.batch + b) * sh.R_pad;
  for (int row = threadIdx.x; row < sh.R_pad; row += 256) {
    float m = -INFINITY, z = 0.f;
    if (row % sh.W_pad < sh.W) {
      for (int x = x0; x < x1; ++x) {
        const float2 o = in[(long long)x * sh.R_pad + row];
        stat_combine(m, z, o.x, o.y);
      }
    }
    // exp2(logit - c) is the normalised probability; padding rows get c = +inf, probability 0
    out[row] = z > 0.f ? m + __builtin_amdgcn_logf(z) : INFINITY;
  }
}

// ---- pass 3: normalised probabilities reduced over the query rows ------------------------
template <bool BF16, int D, int KS, bool MASKED, bool WIN_IMG>
__device__ __forceinline__ void colsum_body(const Ctx &c, const TileCtx &t, const uint4 (&kf)[KS][Cfg<BF16, D>::NF],
                                            const int (&keymod)[KS], const uint4 *ldsq, const float *lds_c,
                                            const float *lds_rowimg, float *lds_cross, float (&colsum)[KS]) {
  constexpr int NF = Cfg<BF16, D>::NF, RS = Cfg<BF16, D>::NCH + 1;
  constexpr int AHEAD = 1;  // registers are short here: one fragment in flight
  const Shape &sh = c.sh;
  const int RB = sh.R_pad >> 5;
  const int bph = sh.W_pad >> 5;  // row blocks per query head
  const float cl = sh.scale_log2e;
  const char *qbase = reinterpret_cast<const char *>(ldsq) + (t.n * RS + t.half) * 16;
  uint4 pf[AHEAD];
#pragma unroll
  for (int f = 0; f < AHEAD; ++f) pf[f] = *reinterpret_cast<const uint4 *>(qbase + 32 * f);
  float cross_acc = 0.f;
  int rbh = 0;  // row block inside the head
  for (int rb = 0; rb < RB; ++rb) {
    f32x16_t acc[KS];
    block_products<BF16, D, KS, false, AHEAD>(acc, kf, pf, qbase + rb * (32 * RS * 16), rb + 1 < RB);  // [query row][key]
    float bs[KS], bsi[KS];
#pragma unroll
    for (int sub = 0; sub < KS; ++sub) bs[sub] = bsi[sub] = 0.f;
    // rows 8g + 4 half + j of the block, j = 0..3 (the fences keep the compiler from fetching the
    // constants of all four groups up front: registers are short)
    const float *crow = lds_c + rb * 32 + 4 * t.half, *wrow = lds_rowimg + rbh * 32 + 4 * t.half;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 c4 = *reinterpret_cast<const float4 *>(crow + 8 * g);
      float4 w4 = make_float4(0.f, 0.f, 0.f, 0.f);
      if constexpr (WIN_IMG) w4 = *reinterpret_cast<const float4 *>(wrow + 8 * g);
      const float cr[4] = {c4.x, c4.y, c4.z, c4.w};
      const float wimg[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
      for (int sub = 0; sub < KS; ++sub) {
        const int key = t.key0 + sub * 32 + t.n;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float p = fast_exp2(fmaf(acc[sub][4 * g + j], cl, -cr[j]));
          if constexpr (MASKED) {
            // window row r sees keys up to L - W + r; padding rows already have probability 0
            const int r = rbh * 32 + 8 * g + 4 * t.half + j;
            p = key <= t.s.L - sh.W + r ? p : 0.f;
          }
          bs[sub] += p;
          if constexpr (WIN_IMG) bsi[sub] = fmaf(p, wimg[j], bsi[sub]);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int sub = 0; sub < KS; ++sub) {
      colsum[sub] += bs[sub];
      // mass sent to the other modality: image keys seen by text rows, text keys by image rows
      if constexpr (WIN_IMG) cross_acc += keymod[sub] ? bs[sub] - bsi[sub] : bsi[sub];
      else cross_acc += keymod[sub] ? bs[sub] : 0.f;
    }
    if (++rbh == bph) {
      rbh = 0;
      const float v = wave_sum(cross_acc);
      if (t.lane == 0) lds_cross[t.wave * sh.G + rb / bph] += v;  // over the tiles of the run
      cross_acc = 0.f;
    }
  }
}

template <bool BF16, int D, bool RUN>
__global__ __launch_bounds__(kThreads, 4) void score_colsum_kernel(Ctx c) {
  constexpr int NCH = Cfg<BF16, D>::NCH, NF = Cfg<BF16, D>::NF, KS = score_subs(BF16);
  extern __shared__ uint4 lds[];
  const Shape &sh = c.sh;
  TileCtx t;
  if (!tile_ctx<score_tile_keys(BF16)>(c, t)) return;
  uint4 *ldsq = lds;
  float *lds_c = reinterpret_cast<float *>(lds + sh.R_pad * (NCH + 1));  // [R_pad]
  float *lds_rowimg = lds_c + sh.R_pad;                                  // [W_pad]
  float *lds_cross = lds_rowimg + sh.W_pad;                              // [waves][G]

  uint4 kf[KS][NF];
  load_keys<BF16, D, KS>(c, t, kf);  // the long way first (HBM); the query rows come from L2
  stage_queries<BF16, D>(c, t, ldsq);
  const float *rs = c.rowstat + ((long long)(t.l * sh.Hkv + t.gkv) * sh.batch + t.b) * sh.R_pad;
  for (int row = threadIdx.x; row < sh.R_pad; row += kThreads) lds_c[row] = rs[row];
  const uint8_t *mod = c.mod + t.s.tok_off;
  for (int r = threadIdx.x; r < sh.W_pad; r += kThreads)
    lds_rowimg[r] = (r < sh.W && mod[t.s.L - sh.W + r]) ? 1.f : 0.f;
  for (int i = threadIdx.x; i < kScoreWaves * sh.G; i += kThreads) lds_cross[i] = 0.f;
  int keymod[KS];
#pragma unroll
  for (int sub = 0; sub < KS; ++sub) {
    const int key = t.key0 + sub * 32 + t.n;
    keymod[sub] = mod[key < t.s.L ? key : t.s.L - 1];
  }
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();

  // the run's tiles one after the other on the same query rows (see score_stats_kernel)
  const int tile_end = RUN ? t.tile_end : t.tile + 1;
  for (int tile = t.tile; tile < tile_end; ++tile) {
    if (tile != t.tile) {
      set_tile<score_tile_keys(BF16)>(c, t, tile);
      load_keys<BF16, D, KS>(c, t, kf);
#pragma unroll
      for (int sub = 0; sub < KS; ++sub) {
        const int key = t.key0 + sub * 32 + t.n;
        keymod[sub] = mod[key < t.s.L ? key : t.s.L - 1];
      }
    }
    if (t.key0 >= t.s.L) continue;  // this wave's keys lie past the end of the sequence
    float colsum[KS];
#pragma unroll
    for (int sub = 0; sub < KS; ++sub) colsum[sub] = 0.f;
    const bool win_img = t.s.win_has_img != 0;
    if (t.masked) {
      if (win_img) colsum_body<BF16, D, KS, true, true>(c, t, kf, keymod, ldsq, lds_c, lds_rowimg, lds_cross, colsum);
      else colsum_body<BF16, D, KS, true, false>(c, t, kf, keymod, ldsq, lds_c, lds_rowimg, lds_cross, colsum);
    } else {
      if (win_img) colsum_body<BF16, D, KS, false, true>(c, t, kf, keymod, ldsq, lds_c, lds_rowimg, lds_cross, colsum);
      else colsum_body<BF16, D, KS, false, false>(c, t, kf, keymod, ldsq, lds_c, lds_rowimg, lds_cross, colsum);
    }
    const float inv_rows = 1.0f / (float)(sh.G * sh.W);
    float *imp = c.importance + (long long)(t.l * sh.Hkv + t.gkv) * sh.T + t.s.tok_off;
#pragma unroll
    for (int sub = 0; sub < KS; ++sub) {
      const int key = t.key0 + sub * 32 + t.n;
      const float tot = colsum[sub] + __shfl_xor(colsum[sub], 32, 64);
      if (t.half == 0 && key < t.s.L) imp[key] = tot * inv_rows;
    }
  }
  __syncthreads();
  for (int g = threadIdx.x; g < sh.G; g += kThreads) {
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < kScoreWaves; ++w) v += lds_cross[w * sh.G + g];
    c.cross_part[(long long)(t.l * sh.Hq + t.gkv * sh.G + g) * sh.tiles_score + t.x] = v;
  }
}

template <bool BF16, int D, bool RUN>
hipError_t launch_score_t(const Ctx &c) {
  constexpr int NCH = Cfg<BF16, D>::NCH;
  const Shape &sh = c.sh;
  const size_t q_bytes = (size_t)sh.R_pad * (NCH + 1) * 16;
  const size_t lds1 = q_bytes + (size_t)kScoreWaves * sh.R_pad * sizeof(float);
  const size_t lds3 = q_bytes + (size_t)sh.R_pad * 4 + (size_t)sh.W_pad * 4 + (size_t)kScoreWaves * sh.G * 4;
  hipError_t e;
  e = allow_full_lds<score_stats_kernel<BF16, D, RUN>>();
  if (e != hipSuccess) return e;
  e = allow_full_lds<score_colsum_kernel<BF16, D, RUN>>();
  if (e != hipSuccess) return e;
  const int units = sh.n_layers * sh.Hkv;
  const long long grid = (long long)((units + 7) / 8) * 8 * sh.tiles_score;
  if (grid > 0x7fffffffLL) return hipErrorInvalidConfiguration;
  {
    ProfScope ps(c.stream, KID_SCORE_STATS);
    score_stats_kernel<BF16, D, RUN><<<dim3((unsigned)grid), kThreads, lds1, c.stream>>>(c);
  }
  {
    ProfScope ps(c.stream, KID_SCORE_COMBINE);
    score_combine_kernel<<<dim3(sh.batch, sh.Hkv, sh.n_layers), 256, 0, c.stream>>>(c);
  }
  {
    ProfScope ps(c.stream, KID_SCORE_COLSUM);
    score_colsum_kernel<BF16, D, RUN><<<dim3((unsigned)grid), kThreads, lds3, c.stream>>>(c);
  }
  return hipGetLastError();
}

template <bool BF16, int D>
hipError_t launch_score_r(const Ctx &c) {
  return c.sh.score_tpw > 1 ? launch_score_t<BF16, D, true>(c) : launch_score_t<BF16, D, false>(c);
}

}  // namespace

size_t score_lds_bytes(const Shape &sh) {
  const int nch = sh.d * (sh.bf16 ? 2 : 4) / 16;
  return (size_t)sh.R_pad * (nch + 1) * 16 + (size_t)kScoreWaves * sh.R_pad * sizeof(float) +
         (size_t)sh.W_pad * 4 + (size_t)kScoreWaves * sh.G * 4;
}

hipError_t launch_score(const Ctx &c) {
  if (c.sh.bf16) return c.sh.d == 128 ? launch_score_r<true, 128>(c) : launch_score_r<true, 64>(c);
  return c.sh.d == 128 ? launch_score_r<false, 128>(c) : launch_score_r<false, 64>(c);
}

}  // namespace flowmm
