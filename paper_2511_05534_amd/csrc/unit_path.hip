// Unit-resident path for short prompts (bf16, every L <= 1024, G*W_pad <= 64, every B <= 256,
// at most 8 sequences and 32 modality spans, whose description rides in the kernel arguments).
//
// When one (sequence, layer, kv head) unit fits on a compute unit, every step of a unit runs inside
// one workgroup and nothing but K, V and the results touches HBM:
//   unit_plan   : proxy attention -> importance, top-B split, cosine argmax as a cross-modal layer
//                 does; the unit's keys stay in registers throughout (K read once)
//   unit_match  : the layer's flow ratio and strategy (needs all its query heads, hence its own
//                 launch); units of intra-modal layers are split and matched again with the
//                 modality restriction, the others return at once
//   unit_merge  : counting sort + segment sums    (K and V read once)
// Three launches instead of eleven.  The arithmetic is the same as in the generic kernels
// (score.hip, select.hip, match.hip, merge.hip); see those files for the paper passages.
#include "device_common.h"
#include "kernels.h"
#include "profile.h"
#include "select_core.h"
#include "unit_merge_core.h"

namespace flowmm {

namespace {

constexpr bool kBF16 = true;

// ============================ score + select + match (cross-modal) ===========================
// One workgroup of WAVES (eight or twelve) waves per unit.  Wave w keeps the key tiles w, w+WAVES, ... (32 keys each) in
// registers for the whole kernel, in the layout every contraction here uses, so K is read from
// HBM once.  The logits are computed twice from those registers: once for the row statistics,
// once for the normalised column sums.  The pivots' rows go from the registers of the lanes that
// hold them to LDS, and the same registers are the token operands of the cosine contraction.
// Every fragment read from LDS (query rows, pivot rows) feeds one matrix instruction per tile of
// the wave.  The layer's strategy needs all its query heads and is not known here: this kernel
// matches as a cross-modal layer does; unit_match_kernel then settles the strategy and redoes the
// intra-modal layers.
constexpr int kPMaxWaves = 12;  // workgroups of 8 or 12 waves (12 * 154 registers still fit a compute unit)

struct PlanLds {  // byte offsets into the dynamic LDS block
  int q, stat, cval, rowimg, cross, keys, assign, kept, piv, w, bias, total_bytes;
};

__host__ __device__ inline PlanLds plan_lds_layout(int rows, int b_pad, int nch) {
  PlanLds m;
  int off = 0;
  m.q = off; off += rows * (nch + 1) * 16;
  m.piv = off; off += b_pad * (nch + 1) * 16;
  m.stat = off; off += kPMaxWaves * rows * 8;
  m.cval = off; off += rows * 4;
  m.rowimg = off; off += rows * 4;
  m.cross = off; off += 32 * 2 * 4;
  m.keys = off; off += 1024 * 4;
  m.assign = off; off += 1024 * 4;
  m.kept = off; off += b_pad * 4;
  m.w = off; off += b_pad * 4;
  m.bias = off; off += b_pad * 4;
  m.total_bytes = (off + 15) & ~15;
  return m;
}

template <int D, int RB, int NT, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void unit_plan_kernel(Ctx c, int b_pad) {
  constexpr int kPThreads = WAVES * 64, kPWaves = WAVES;
  using CF = Cfg<kBF16, D>;
  constexpr int NCH = CF::NCH, NF = CF::NF, RS = NCH + 1;
  constexpr int ROWS = RB * 32;
  extern __shared__ __align__(16) char lds_dyn[];
  const PlanLds lay = plan_lds_layout(ROWS, b_pad, NCH);
  uint4 *ldsq = reinterpret_cast<uint4 *>(lds_dyn + lay.q);            // [ROWS][RS] query rows
  uint4 *lds_piv = reinterpret_cast<uint4 *>(lds_dyn + lay.piv);       // [b_pad][RS] pivot rows
  float2 *lds_stat = reinterpret_cast<float2 *>(lds_dyn + lay.stat);   // [waves][ROWS] (max, sum exp2)
  float *lds_c = reinterpret_cast<float *>(lds_dyn + lay.cval);        // [ROWS] max + log2(sum)
  float *lds_rowimg = reinterpret_cast<float *>(lds_dyn + lay.rowimg); // [ROWS] 1 for an image proxy row
  float *lds_cross = reinterpret_cast<float *>(lds_dyn + lay.cross);   // [tiles][RB] cross-modal mass per key tile
  unsigned *lds_keys = reinterpret_cast<unsigned *>(lds_dyn + lay.keys);  // [1024] importance bits
  int *lds_assign = reinterpret_cast<int *>(lds_dyn + lay.assign);     // [1024] slot of a pivot, -2 otherwise
  int *lds_kept = reinterpret_cast<int *>(lds_dyn + lay.kept);         // [B]
  float *lds_w = reinterpret_cast<float *>(lds_dyn + lay.w);           // [b_pad] 1/norm (0 for a zero row)
  float *lds_bias = reinterpret_cast<float *>(lds_dyn + lay.bias);     // [b_pad] added to a candidate
  __shared__ SmallSelectScratch<kPThreads> scratch;
  __shared__ int sh_dropped;

  const Shape &sh = c.sh;
  const int b = rotated_block_x(), gkv = blockIdx.y, l = blockIdx.z + c.layer0;
  const SeqInfo s = inline_seq(c.inl, b);
  const int L = s.L;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 31, half = lane >> 5;
  const long long unit = (long long)l * sh.Hkv + gkv;

  // ---- every key of the unit into registers ----------------------------------------------------
  const uint4 *K = reinterpret_cast<const uint4 *>(c.K) + (long long)l * sh.ks_layer +
                   (long long)gkv * sh.ks_head + (long long)s.tok_off * sh.ks_tok;
  uint4 kf[NT][NF];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int key0 = (wave + kPWaves * j) * 32;
    if (key0 < L) {
      const uint4 *row = K + (long long)min(key0 + n, L - 1) * sh.ks_tok + half;
#pragma unroll
      for (int f = 0; f < NF; ++f) kf[j][f] = row[2 * f];
    } else {
#pragma unroll
      for (int f = 0; f < NF; ++f) kf[j][f] = make_uint4(0, 0, 0, 0);
    }
  }
  // the query rows (zero rows pad every head to a multiple of 32)
  {
    const uint4 *Q = reinterpret_cast<const uint4 *>(c.Q) + (long long)l * sh.qs_layer;
    for (int idx = threadIdx.x; idx < ROWS * NCH; idx += kPThreads) {
      const int row = idx / NCH, ch = idx - row * NCH;
      const int g = row / sh.W_pad, r = row - g * sh.W_pad;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (r < sh.W) v = Q[(long long)(gkv * sh.G + g) * sh.qs_head + (long long)(b * sh.W + r) * sh.qs_tok + ch];
      ldsq[row * RS + ch] = v;
    }
    for (int row = threadIdx.x; row < ROWS; row += kPThreads) {
      const int r = row % sh.W_pad;
      lds_rowimg[row] = (r < sh.W && inline_mod(c.inl, b, L - sh.W + r)) ? 1.f : 0.f;
    }
    if (threadIdx.x == 0) sh_dropped = 0;
  }
  __syncthreads();

  const float cl = sh.scale_log2e;
  const int wmask = sh.W_pad - 1;  // W_pad is 32 or 64 here
  const uint4 *qlane = ldsq + n * RS + half;  // this lane's first fragment of row block 0
  // ---- pass 1: row statistics; accumulator rows are keys, lane n owns query row rb*32+n ----------
  // Only the tiles that reach into the window (or past the end) pay for the causal mask.
  {
    float m[RB], z[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) { m[rb] = -INFINITY; z[rb] = 0.f; }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      f32x16_t acc[NT];
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
#pragma unroll
      for (int f = 0; f < NF; ++f) {
        const uint4 qf = qlane[rb * 32 * RS + 2 * f];
#pragma unroll
        for (int j = 0; j < NT; ++j) mma_chunk<kBF16>(acc[j], kf[j][f], qf);  // [key][query row]
      }
      const int r = (rb * 32 + n) & wmask;
      const int limit = r < sh.W ? L - sh.W + r : -1;  // last key this query may see
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int key0 = (wave + kPWaves * j) * 32;
        if (key0 >= L) continue;
        float tm = -INFINITY;
        if (key0 + 31 > L - sh.W) {
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            acc[j][i] = key0 + acc_row(i, half) <= limit ? acc[j][i] : -INFINITY;
            tm = fmaxf(tm, acc[j][i]);
          }
        } else {
#pragma unroll
          for (int i = 0; i < 16; i += 2) tm = fmaxf(fmaxf(tm, acc[j][i]), acc[j][i + 1]);
        }
        if (tm > -INFINITY) {
          const float M = fmaxf(m[rb], tm * cl);  // cl > 0: the largest logit is the largest product
          float zt = 0.f;
#pragma unroll
          for (int i = 0; i < 16; ++i) zt += fast_exp2(fmaf(acc[j][i], cl, -M));
          z[rb] = z[rb] * fast_exp2(m[rb] - M) + zt;
          m[rb] = M;
        }
      }
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const float m2 = __shfl_xor(m[rb], 32, 64), z2 = __shfl_xor(z[rb], 32, 64);
      stat_combine(m[rb], z[rb], m2, z2);
      if (half == 0) lds_stat[wave * ROWS + rb * 32 + n] = make_float2(m[rb], z[rb]);
    }
  }
  __syncthreads();
  if (threadIdx.x < ROWS) {
    float2 a = lds_stat[threadIdx.x];
#pragma unroll
    for (int w = 1; w < kPWaves; ++w) {
      const float2 o = lds_stat[w * ROWS + threadIdx.x];
      stat_combine(a.x, a.y, o.x, o.y);
    }
    // exp2(logit - c) is the normalised probability; padding rows get c = +inf, probability 0
    lds_c[threadIdx.x] = ((int)threadIdx.x & wmask) < sh.W && a.y > 0.f ? a.x + __builtin_amdgcn_logf(a.y) : INFINITY;
  }
  __syncthreads();

  // ---- pass 2: probabilities reduced over the query rows; rows are query rows, lane n owns key n --
  {
    const float inv_rows = 1.0f / (float)(sh.G * sh.W);
    float *imp = c.importance + unit * sh.T + s.tok_off;
    const bool win_img = s.win_has_img != 0;
    float colsum[NT];
    int keymod[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      colsum[j] = 0.f;
      keymod[j] = inline_mod(c.inl, b, min((wave + kPWaves * j) * 32 + n, L - 1));
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      f32x16_t acc[NT];
#pragma unroll
      for (int j = 0; j < NT; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
#pragma unroll
      for (int f = 0; f < NF; ++f) {
        const uint4 qf = qlane[rb * 32 * RS + 2 * f];
#pragma unroll
        for (int j = 0; j < NT; ++j) mma_chunk<kBF16>(acc[j], qf, kf[j][f]);  // [query row][key]
      }
      float cr[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 c4 = *reinterpret_cast<const float4 *>(lds_c + rb * 32 + 8 * g + 4 * half);
        cr[4 * g] = c4.x; cr[4 * g + 1] = c4.y; cr[4 * g + 2] = c4.z; cr[4 * g + 3] = c4.w;
      }
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int key0 = (wave + kPWaves * j) * 32;
        if (key0 >= L) continue;
        const int key = key0 + n;
        float bs = 0.f, bsi = 0.f;
        if (win_img || key0 + 31 > L - sh.W) {  // general form: causal mask, image rows in the window
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int row = rb * 32 + acc_row(i, half);
            float p = fast_exp2(fmaf(acc[j][i], cl, -cr[i]));  // padding rows: c = +inf, p = 0
            p = key <= L - sh.W + (row & wmask) ? p : 0.f;
            bs += p;
            bsi = fmaf(p, lds_rowimg[row], bsi);
          }
        } else {
#pragma unroll
          for (int i = 0; i < 16; ++i) bs += fast_exp2(fmaf(acc[j][i], cl, -cr[i]));
        }
        colsum[j] += bs;
        // mass on keys of the other modality: image keys seen by text rows, text keys by image rows
        const float cross = wave_sum(keymod[j] ? bs - bsi : bsi);
        if (lane == 0) lds_cross[(key0 >> 5) * RB + rb] = cross;
      }
    }
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int key = (wave + kPWaves * j) * 32 + n;
      const float tot = (colsum[j] + __shfl_xor(colsum[j], 32, 64)) * inv_rows;
      if (half == 0 && key < L) {
        imp[key] = tot;
        lds_keys[key] = __float_as_uint(tot);
      }
    }
  }
  __syncthreads();
  if (wave < sh.G) {
    // query head `wave` owns the row blocks [wave*W_pad/32, (wave+1)*W_pad/32); lane t adds tile t's
    // share, then a fixed tree over the lanes (the same for every shape of workgroup)
    const int bph = sh.W_pad >> 5;
    float v = 0.f;
    if (lane < ((L + 31) >> 5))
      for (int k = 0; k < bph; ++k) v += lds_cross[lane * RB + wave * bph + k];
    v = wave_sum(v);
    if (lane == 0) c.cross_part[(long long)(l * sh.Hq + gkv * sh.G + wave) * sh.tiles_score + b] = v;
  }

  // ---- top-B split ---------------------------------------------------------------------------------
  {
    unsigned keys4[4];  // every thread's four consecutive keys (threads past the end hold none)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int i = threadIdx.x * 4 + j;
      keys4[j] = i < L ? lds_keys[i] : 0u;
    }
    select_top_b_small<kPThreads>(keys4, L, sh.W, s.B, lds_kept, lds_assign, scratch);
    for (int idx = s.B * NCH + (int)threadIdx.x; idx < b_pad * NCH; idx += kPThreads)  // padding pivot rows
      lds_piv[(idx / NCH) * RS + idx % NCH] = make_uint4(0, 0, 0, 0);
  }
  __syncthreads();
  int *kept = c.kept_idx + unit * sh.SB + s.kept_off;
  for (int i = threadIdx.x; i < s.B; i += kPThreads) kept[i] = lds_kept[i];

  // ---- pivots: rows from the registers that hold them, then inverse norms and the sensitivity gate ----
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int tok = (wave + kPWaves * j) * 32 + n;
    const int slot = tok < L ? lds_assign[tok] : -2;
    if (slot >= 0) {
#pragma unroll
      for (int f = 0; f < NF; ++f) lds_piv[slot * RS + 2 * f + half] = kf[j][f];
    }
  }
  __syncthreads();
  for (int pr0 = 0; pr0 < b_pad; pr0 += kPThreads / NCH) {  // NCH lanes per row
    const int pr = pr0 + threadIdx.x / NCH, ch = threadIdx.x % NCH;
    float ss = pr < b_pad ? chunk_sumsq<kBF16>(lds_piv[pr * RS + ch]) : 0.f;
#pragma unroll
    for (int o = NCH / 2; o >= 1; o >>= 1) ss += __shfl_xor(ss, o, 64);
    if (ch == 0 && pr < b_pad) {
      const bool ok = pr < s.B && !(__uint_as_float(lds_keys[lds_kept[pr < s.B ? pr : 0]]) > s.tau);
      lds_w[pr] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
      // added to every candidate: keeps an eligible one a normal float, sinks the others
      lds_bias[pr] = ok ? 1e-30f : -3e38f;
    }
  }
  __syncthreads();

  // ---- match as a cross-modal layer does ---------------------------------------------------------------
  // Each candidate is cosine * |token| (+ bias); its low four mantissa bits are replaced by 15 - i,
  // i the row inside this lane's 16 rows of the block, so one running maximum carries the argmax.
  int *assign = c.assign + unit * sh.T + s.tok_off;
  const int nblk = b_pad >> 5;
  float best[NT];
  int best_blk[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) { best[j] = -INFINITY; best_blk[j] = 0; }
  const uint4 *plane = lds_piv + n * RS + half;
  for (int pb = 0; pb < nblk; ++pb) {
    f32x16_t acc[NT];
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
#pragma unroll
    for (int f = 0; f < NF; ++f) {
      const uint4 pf = plane[pb * 32 * RS + 2 * f];
#pragma unroll
      for (int j = 0; j < NT; ++j) mma_chunk<kBF16>(acc[j], pf, kf[j][f]);  // [pivot][token]
    }
    float wv[16], bv[16];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 w4 = *reinterpret_cast<const float4 *>(lds_w + pb * 32 + 8 * g + 4 * half);
      const float4 b4 = *reinterpret_cast<const float4 *>(lds_bias + pb * 32 + 8 * g + 4 * half);
      wv[4 * g] = w4.x; wv[4 * g + 1] = w4.y; wv[4 * g + 2] = w4.z; wv[4 * g + 3] = w4.w;
      bv[4 * g] = b4.x; bv[4 * g + 1] = b4.y; bv[4 * g + 2] = b4.z; bv[4 * g + 3] = b4.w;
    }
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      float m = -INFINITY;
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float p0 = __uint_as_float((__float_as_uint(fmaf(acc[j][i], wv[i], bv[i])) & ~15u) | (unsigned)(15 - i));
        const float p1 = __uint_as_float((__float_as_uint(fmaf(acc[j][i + 1], wv[i + 1], bv[i + 1])) & ~15u) | (unsigned)(14 - i));
        m = fmaxf(fmaxf(m, p0), p1);
      }
      if (m > best[j]) { best[j] = m; best_blk[j] = pb; }
    }
  }
  int dropped = 0;
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int tok = (wave + kPWaves * j) * 32 + n;
    int best_slot = best_blk[j] * 32 + acc_row(15 - (int)(__float_as_uint(best[j]) & 15u), half);
    const float ob = __shfl_xor(best[j], 32, 64);
    const int os = __shfl_xor(best_slot, 32, 64);
    float bj = best[j];
    if (ob > bj || (ob == bj && os < best_slot)) { bj = ob; best_slot = os; }
    if (!(bj > -1e38f)) best_slot = -1;  // no eligible pivot
    if (half == 0 && tok < L) {
      const int cur = lds_assign[tok];
      assign[tok] = cur == -2 ? best_slot : cur;  // a pivot keeps its own slot
      dropped += cur == -2 && best_slot < 0;
    }
  }
  dropped = wave_sum_int(dropped);
  if (lane == 0 && dropped) atomicAdd(&sh_dropped, dropped);
  __syncthreads();
  if (threadIdx.x == 0) c.n_dropped[unit * sh.batch + b] = sh_dropped;
}

// ============================ flow (+ select + match of intra-modal layers) ====================
constexpr int kF2Threads = 256;
constexpr int kF2Waves = kF2Threads / 64;

struct MatchLds {  // byte offsets into the dynamic LDS block
  int piv, w, bias, head, keys, assign, kept, total_bytes;
};

__host__ __device__ inline MatchLds match_lds_layout(int b_pad, int nch, int Hq, int maxL) {
  MatchLds m;
  int off = 0;
  m.piv = off; off += b_pad * (nch + 1) * 16;
  m.w = off; off += b_pad * 4;
  m.bias = off; off += 2 * b_pad * 4;
  m.head = off; off += Hq * 4;
  m.keys = off; off += maxL * 4;
  m.assign = off; off += maxL * 4;
  m.kept = off; off += b_pad * 4;
  m.total_bytes = (off + 15) & ~15;
  return m;
}

// All 256 threads of the workgroup of unit (b, gkv, l) call; lds_dyn: match_lds_layout bytes.
template <int D>
__device__ __forceinline__ void unit_flow_match_body(const Ctx &c, int b_pad, char *lds_dyn, int b, int gkv, int l) {
  using CF = Cfg<kBF16, D>;
  constexpr int NCH = CF::NCH, NF = CF::NF;
  const MatchLds lay = match_lds_layout(b_pad, NCH, c.sh.Hq, c.sh.maxL);
  uint4 *lds_piv = reinterpret_cast<uint4 *>(lds_dyn + lay.piv);     // [b_pad][NCH+1] pivot rows
  float *lds_w = reinterpret_cast<float *>(lds_dyn + lay.w);         // [b_pad] 1/norm (0 for a zero row)
  float *lds_bias = reinterpret_cast<float *>(lds_dyn + lay.bias);   // [2][b_pad] 0 eligible, -inf not
  float *lds_head = reinterpret_cast<float *>(lds_dyn + lay.head);   // [Hq]
  unsigned *lds_keys = reinterpret_cast<unsigned *>(lds_dyn + lay.keys);  // [L] importance bits
  int *lds_assign = reinterpret_cast<int *>(lds_dyn + lay.assign);   // [L] slot of a pivot, -2 otherwise
  int *lds_kept = reinterpret_cast<int *>(lds_dyn + lay.kept);       // [B]
  __shared__ SmallSelectScratch<kF2Threads> scratch;
  __shared__ float sh_rho;
  __shared__ int sh_dropped;

  const Shape &sh = c.sh;
  const SeqInfo s = inline_seq(c.inl, b);
  const int L = s.L;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 31, half = lane >> 5;
  const long long unit = (long long)l * sh.Hkv + gkv;
  const uint4 *K = reinterpret_cast<const uint4 *>(c.K) + (long long)l * sh.ks_layer +
                   (long long)gkv * sh.ks_head + (long long)s.tok_off * sh.ks_tok;
  const unsigned *imp = reinterpret_cast<const unsigned *>(c.importance) + unit * sh.T + s.tok_off;
  int *kept = c.kept_idx + unit * sh.SB + s.kept_off;
  int *assign = c.assign + unit * sh.T + s.tok_off;

  // flow: every workgroup of the layer folds the same numbers in the same order
  for (int h = threadIdx.x; h < sh.Hq; h += kF2Threads)
    lds_head[h] = c.cross_part[(long long)(l * sh.Hq + h) * sh.tiles_score + b] / (float)sh.W;
  if (threadIdx.x == 0) sh_dropped = 0;
  __syncthreads();
  if (threadIdx.x == 0) {
    float acc = 0.f;
    for (int h = 0; h < sh.Hq; ++h) acc += lds_head[h];
    const float rho = acc / (float)sh.Hq;
    sh_rho = rho;
    if (gkv == 0) {
      c.rho[l * sh.batch + b] = rho;
      c.mode[l * sh.batch + b] = (rho > sh.theta) != (sh.invert_flow != 0) ? 1 : 0;
    }
  }
  __syncthreads();
  const bool mode_cross = (sh_rho > sh.theta) != (sh.invert_flow != 0);
  if (mode_cross) return;  // unit_plan_kernel has matched this unit as a cross-modal layer does

  // intra-modal layer: the split again (same result) and the match restricted to the token's modality
  const int ntiles = (L + 31) >> 5;
  uint4 kf[NF];
  int t = wave;
  if (t < ntiles) {
    const uint4 *row = K + (long long)min(t * 32 + n, L - 1) * sh.ks_tok + half;
#pragma unroll
    for (int f = 0; f < NF; ++f) kf[f] = row[2 * f];
  }
  unsigned keys4[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int i = threadIdx.x * 4 + j;
    keys4[j] = i < L ? imp[i] : 0u;
    if (i < L) lds_keys[i] = keys4[j];
  }
  // top-B split (pivot list and pivot/non-pivot marks stay in LDS; the plan gets its copy below)
  select_top_b_small<kF2Threads>(keys4, L, sh.W, s.B, lds_kept, lds_assign, scratch);
  __syncthreads();
  for (int i = threadIdx.x; i < s.B; i += kF2Threads) kept[i] = lds_kept[i];

  // stage all pivots once: rows, inverse norms, eligibility per token modality
  constexpr int kRowsPerPass = kF2Threads / NCH;
  for (int r0 = 0; r0 < b_pad; r0 += kRowsPerPass) {
    const int pr = r0 + threadIdx.x / NCH, ch = threadIdx.x % NCH;
    uint4 v = make_uint4(0, 0, 0, 0);
    const bool real = pr < s.B;
    const int ptok = real ? lds_kept[pr] : 0;
    if (real) v = K[(long long)ptok * sh.ks_tok + ch];
    const int pm = real ? inline_mod(c.inl, b, ptok) : 0;
    if (pr < b_pad) lds_piv[pr * (NCH + 1) + ch] = v;
    float ss = chunk_sumsq<kBF16>(v);
#pragma unroll
    for (int o = NCH / 2; o >= 1; o >>= 1) ss += __shfl_xor(ss, o, 64);
    if (ch == 0 && pr < b_pad) {
      const bool ok = real && !(__uint_as_float(lds_keys[ptok]) > s.tau);
      lds_w[pr] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
      lds_bias[pr] = ok && (mode_cross || pm == 0) ? 0.f : -INFINITY;
      lds_bias[b_pad + pr] = ok && (mode_cross || pm == 1) ? 0.f : -INFINITY;
    }
  }
  __syncthreads();

  const int nblk = b_pad >> 5;
  int dropped = 0;
  for (; t < ntiles; t += kF2Waves) {
    const int tok = t * 32 + n;
    const int tc = min(tok, L - 1);
    const int cur = lds_assign[tc];
    const float *bias = lds_bias + (inline_mod(c.inl, b, tc) ? b_pad : 0);
    uint4 nxt[NF];
    if (t + kF2Waves < ntiles) {
      const uint4 *row = K + (long long)min((t + kF2Waves) * 32 + n, L - 1) * sh.ks_tok + half;
#pragma unroll
      for (int f = 0; f < NF; ++f) nxt[f] = row[2 * f];
    }
    float best = -INFINITY;
    int best_slot = -1;
    for (int pb = 0; pb < nblk; ++pb) {
      f32x16_t acc;
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[i] = 0.f;
      const uint4 *prow = lds_piv + (pb * 32 + n) * (NCH + 1) + half;
#pragma unroll
      for (int f = 0; f < NF; ++f) mma_chunk<kBF16>(acc, prow[2 * f], kf[f]);  // [pivot][token]
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int pr = pb * 32 + acc_row(i, half);
        const float u = fmaf(acc[i], lds_w[pr], bias[pr]);
        if (u > best) { best = u; best_slot = pr; }
      }
    }
    const float ob = __shfl_xor(best, 32, 64);
    const int os = __shfl_xor(best_slot, 32, 64);
    if (ob > best || (ob == best && (unsigned)os < (unsigned)best_slot)) { best = ob; best_slot = os; }
    if (half == 0 && tok < L) {
      assign[tok] = cur == -2 ? best_slot : cur;  // a pivot keeps its own slot
      dropped += cur == -2 && best_slot < 0;
    }
    if (t + kF2Waves < ntiles) {
#pragma unroll
      for (int f = 0; f < NF; ++f) kf[f] = nxt[f];
    }
  }
  dropped = wave_sum_int(dropped);
  if (lane == 0 && dropped) atomicAdd(&sh_dropped, dropped);
  __syncthreads();
  if (threadIdx.x == 0) c.n_dropped[unit * sh.batch + b] = sh_dropped;
}

template <int D>
__global__ __launch_bounds__(kF2Threads) void unit_match_kernel(Ctx c, int b_pad) {
  extern __shared__ __align__(16) char lds_dyn[];
  unit_flow_match_body<D>(c, b_pad, lds_dyn, rotated_block_x(), blockIdx.y, blockIdx.z + c.layer0);
}

// ============================ merge =========================================================
// Merge of one unit per workgroup (unit_merge_core.h).  U rows in flight per lane group.
// FLOW: the workgroup first settles its layer's strategy and, in an intra-modal layer, matches its
// unit again (what unit_match_kernel does), so that plan and merge take two launches, not three.
template <int D, int U, bool FLOW, bool WEIGHTED>
__global__ __launch_bounds__(kF3Threads) void unit_merge_kernel(Ctx c, int maxB, int maxE, int b_pad) {
  extern __shared__ __align__(16) int lds_i[];
  __shared__ long long lds_wave[kF3Waves + 1];
  __shared__ int sh_next;
  const Shape &sh = c.sh;
  const int b = rotated_block_x(), gkv = blockIdx.y, l = blockIdx.z + c.layer0;
  if constexpr (FLOW) {
    static_assert(kF2Threads == kF3Threads, "one workgroup runs both bodies");
    unit_flow_match_body<D>(c, b_pad, reinterpret_cast<char *>(lds_i), b, gkv, l);
    __syncthreads();  // the assignment written above is read below; the LDS block changes hands
  }
  const SeqInfo s = inline_seq(c.inl, b);
  const long long unit = (long long)l * sh.Hkv + gkv;
  unit_merge_body<D, U, WEIGHTED>(c, s, unit, l, gkv, c.assign + unit * sh.T + s.tok_off, c.kept_idx + unit * sh.SB + s.kept_off,
                        lds_i, maxB, maxE, lds_wave, &sh_next);
}

// ---- dispatch --------------------------------------------------------------------------------
size_t plan_lds_bytes(const Shape &sh, int b_pad) {
  return (size_t)plan_lds_layout(sh.R_pad, b_pad, sh.d * 2 / 16).total_bytes;
}

template <int D, int RB, int NT, int WAVES>
hipError_t launch_plan_k(const Ctx &c, int b_pad, size_t lds) {
  hipError_t e = allow_full_lds<unit_plan_kernel<D, RB, NT, WAVES>>();
  if (e != hipSuccess) return e;
  ProfScope ps(c.stream, KID_UNIT_PLAN);
  unit_plan_kernel<D, RB, NT, WAVES><<<dim3(c.sh.batch, c.sh.Hkv, c.layers), WAVES * 64, lds, c.stream>>>(c, b_pad);
  return hipGetLastError();
}

template <int D, int RB>
hipError_t launch_f1(const Ctx &c) {
  const int b_pad = (c.sh.maxB + 31) / 32 * 32;
  const size_t lds = plan_lds_bytes(c.sh, b_pad);
  // Key tiles per wave and waves per workgroup: the unit's keys must fit the registers of one
  // workgroup, and twelve waves with two tiles each need fewer registers per wave (three waves per
  // SIMD) than eight waves with three.
  const int tiles = (c.sh.maxL + 31) / 32;
  if (tiles <= 8) return launch_plan_k<D, RB, 1, 8>(c, b_pad, lds);
  if (tiles <= 12) return launch_plan_k<D, RB, 1, 12>(c, b_pad, lds);
  if (tiles <= 16) return launch_plan_k<D, RB, 2, 8>(c, b_pad, lds);
  if (tiles <= 24) return launch_plan_k<D, RB, 2, 12>(c, b_pad, lds);
  return launch_plan_k<D, RB, 4, 8>(c, b_pad, lds);
}

size_t match_lds_bytes(const Shape &sh, int b_pad) {
  return (size_t)match_lds_layout(b_pad, sh.d * 2 / 16, sh.Hq, sh.maxL).total_bytes;
}

template <int D>
hipError_t launch_f2(const Ctx &c) {
  const int b_pad = (c.sh.maxB + 31) / 32 * 32;
  const size_t lds = match_lds_bytes(c.sh, b_pad);
  hipError_t e = allow_full_lds<unit_match_kernel<D>>();
  if (e != hipSuccess) return e;
  ProfScope ps(c.stream, KID_UNIT_MATCH);
  unit_match_kernel<D><<<dim3(c.sh.batch, c.sh.Hkv, c.layers), kF2Threads, lds, c.stream>>>(c, b_pad);
  return hipGetLastError();
}

template <int D, int U, bool FLOW, bool WEIGHTED>
hipError_t launch_f3w(const Ctx &c) {
  const int b_pad = (c.sh.maxB + 31) / 32 * 32;
  size_t lds = (size_t)merge_lds_layout(c.sh.maxB, c.sh.maxE, D).total_bytes;
  if (FLOW && match_lds_bytes(c.sh, b_pad) > lds) lds = match_lds_bytes(c.sh, b_pad);
  hipError_t e = allow_full_lds<unit_merge_kernel<D, U, FLOW, WEIGHTED>>();
  if (e != hipSuccess) return e;
  ProfScope ps(c.stream, FLOW ? KID_UNIT_FLOW_MERGE : KID_UNIT_MERGE);
  unit_merge_kernel<D, U, FLOW, WEIGHTED><<<dim3(c.sh.batch, c.sh.Hkv, c.layers), kF3Threads, lds, c.stream>>>(
      c, c.sh.maxB, c.sh.maxE, b_pad);
  return hipGetLastError();
}

template <int D, int U, bool FLOW>
hipError_t launch_f3(const Ctx &c) {
  // the weighted variant keeps U = 4 rows in flight: its cosines need every row of a trip in registers
  return c.sh.weighted_merge ? launch_f3w<D, (U > 4 ? 4 : U), FLOW, true>(c) : launch_f3w<D, U, FLOW, false>(c);
}

}  // namespace

bool unit_path_fits(const Shape &sh) {
  if (!sh.bf16 || sh.maxL > 1024 || sh.R_pad > 64 || sh.maxB > 256 || sh.Hq > 4096) return false;
  if (sh.batch > kInlineSeqs || sh.n_spans > kInlineSpans) return false;  // metadata must fit the kernel arguments
  if (sh.ks_tok * 16 * 1024 >= (1ll << 32)) return false;  // the merge addresses a sequence's rows with 32-bit offsets
  const int b_pad = (sh.maxB + 31) / 32 * 32;
  if (match_lds_bytes(sh, b_pad) > 150 * 1024 || plan_lds_bytes(sh, b_pad) > 150 * 1024) return false;
  if ((size_t)merge_lds_layout(sh.maxB, sh.maxE, sh.d).total_bytes > 150 * 1024) return false;
  return true;
}

hipError_t launch_unit_flow_match(const Ctx &c) { return c.sh.d == 128 ? launch_f2<128>(c) : launch_f2<64>(c); }

hipError_t launch_unit_plan(const Ctx &c, bool with_flow) {  // score + select + cross-modal match, then flow + intra-modal layers
  const int rb = c.sh.R_pad / 32;
  hipError_t e;
  if (c.sh.d == 128) e = rb == 1 ? launch_f1<128, 1>(c) : launch_f1<128, 2>(c);
  else e = rb == 1 ? launch_f1<64, 1>(c) : launch_f1<64, 2>(c);
  if (e != hipSuccess || !with_flow) return e;
  return launch_unit_flow_match(c);
}

// with_flow: the launch also settles the layer strategies and rematches the intra-modal layers
// (then it takes the place of launch_unit_flow_match + launch_unit_merge after the plan kernel)
hipError_t launch_unit_merge(const Ctx &c, bool with_flow) {
  // Rows in flight per lane group: with four workgroups on every compute unit the kernel is bound
  // by memory bandwidth and more than two rows in flight only lengthen the queues (measured: 80 us
  // with 2, 102 us with 8 on 1024 units); a grid that leaves compute units short of workgroups is
  // bound by latency and wants many (20 us instead of 40 us per workgroup).
  const bool many = (long long)c.sh.batch * c.sh.Hkv * c.layers >= 4 * 256;
  if (c.sh.d == 128) {
    if (many) return with_flow ? launch_f3<128, 2, true>(c) : launch_f3<128, 2, false>(c);
    return with_flow ? launch_f3<128, 8, true>(c) : launch_f3<128, 8, false>(c);
  }
  if (many) return with_flow ? launch_f3<64, 2, true>(c) : launch_f3<64, 2, false>(c);
  return with_flow ? launch_f3<64, 8, true>(c) : launch_f3<64, 8, false>(c);
}

}  // namespace flowmm
