// The cross-modal interaction ratio with EVERY token of the prompt as a query: the rho^l equation
// of Information Flow Guided Merging taken literally,
//   rho^l = (1/H) sum_h (A_{v->t} + A_{t->v}) / A,   A_{v->t} = sum_{i in V} sum_{j in T} alpha_{i->j}, ...
// with alpha the causal prefill attention of head h (attention equation of the Preliminary
// section) and A the total mass (one per query row).  The proxy-window kernels estimate the same
// ratio from the last W queries only; this one needs the queries of the whole prompt.
//
// Flash-style: the attention matrix is never stored.  A workgroup owns 256 consecutive query
// rows of one (sequence, query head, layer), staged in LDS by direct global->LDS loads, and walks
// over the keys up to its last row; every wave takes 32*KS keys per step straight from global
// memory into MFMA operand registers (accumulator rows are keys, lane n owns query row n of each
// block of 32, so the running softmax statistics of a row live in one lane).  Per row it keeps
// the running maximum, the running sum of exp2 and the running sum over IMAGE keys only; the
// cross-modal mass of the row is the image part for a text query and the rest for an image
// query.  Groups of 32 keys of one modality (almost all) cost nothing extra, and only the steps
// that reach past the first query row of the tile pay for the causal mask.
#include "device_common.h"
#include "kernels.h"
#include "profile.h"
#include "score_core.h"

namespace flowmm {

namespace {

constexpr int kFThreads = 256;
constexpr int kFWaves = kFThreads / 64;
constexpr int kQT = kFlowQueryTile;  // query rows per workgroup
constexpr int kRB = kQT / 32;        // blocks of 32 query rows

template <bool BF16, int D>
__global__ __launch_bounds__(kFThreads, 2) void flow_exact_kernel(Ctx c, FlowExactArgs a) {
  using CF = Cfg<BF16, D>;
  constexpr int NCH = CF::NCH, NF = CF::NF, RS = NCH + 1;
  constexpr int KS = BF16 ? 2 : 1;  // groups of 32 keys a wave holds per step (its registers also carry the running statistics of 256 rows)
  constexpr int KT = kFWaves * 32 * KS;  // keys per step of the workgroup
  constexpr int AHEAD = NF < 3 ? NF : 3;
  extern __shared__ uint4 lds[];
  uint4 *ldsq = lds;                                                   // [kQT][RS] query rows
  // once the keys are done, the same space holds the statistics
  float4 *lds_stat = reinterpret_cast<float4 *>(lds);                  // [waves][kQT] (max, sum, image sum, -)
  float *lds_red = reinterpret_cast<float *>(lds_stat + kFWaves * kQT);  // [kQT] cross-modal share of each row

  const Shape &sh = c.sh;
  const int *meta = c.meta;
  const int x = blockIdx.x, h = blockIdx.y, l = blockIdx.z;
  const int *cu = meta + meta[MW_OFF_CU_FLOWQ];
  const int b = find_seq(cu, meta[MW_BATCH], x);
  const SeqInfo s = load_seq(meta, b);
  const int L = s.L;
  const int q0 = (x - cu[b]) * kQT;  // first query row (prompt position) of this tile
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 31, half = lane >> 5;
  const int gkv = h / sh.G;
  const uint8_t *mod = c.mod + s.tok_off;

  // ---- the query rows of the tile (zero rows past the end of the sequence) ---------------------------
  {
    const uint4 *Q = reinterpret_cast<const uint4 *>(a.Q) + (long long)l * a.qs_layer + (long long)h * a.qs_head +
                     (long long)(s.tok_off + q0) * a.qs_tok;
    const int total = kQT * RS;
    for (int qi0 = wave * 64; qi0 < total; qi0 += kFThreads) {
      const int qi = qi0 + lane;
      if (qi < total) {
        const int row = qi / RS, ch = qi - row * RS;
        if (q0 + row < L && ch < NCH) load_to_lds<16>(Q, (unsigned)(row * a.qs_tok + ch) * 16u, ldsq + qi0);
        else ldsq[qi] = make_uint4(0, 0, 0, 0);  // rows past the end, the padding chunk of every row
      }
    }
  }

  const uint4 *K = reinterpret_cast<const uint4 *>(c.K) + (long long)l * sh.ks_layer + (long long)gkv * sh.ks_head +
                   (long long)s.tok_off * sh.ks_tok;
  const float cl = sh.scale_log2e;
  const char *qbase = reinterpret_cast<const char *>(ldsq) + (n * RS + half) * 16;
  float m[kRB], z[kRB], zi[kRB];  // of query row rb*32+n over the keys this wave has seen
#pragma unroll
  for (int rb = 0; rb < kRB; ++rb) { m[rb] = -INFINITY; z[rb] = zi[rb] = 0.f; }

  const int last_q = min(q0 + kQT, L) - 1;  // last real query row of the tile: no key beyond it is visible
  bool staged = false;
  for (int k0 = 0; k0 <= last_q; k0 += KT) {
    const int key0 = k0 + wave * 32 * KS;  // first key of this wave in this step
    uint4 kf[KS][NF];
    unsigned kimg[KS];  // bit j: key key0 + sub*32 + j is an image token
#pragma unroll
    for (int sub = 0; sub < KS; ++sub) {
      const int key = min(key0 + sub * 32 + n, L - 1);
      const uint4 *row = K + (long long)key * sh.ks_tok + half;
#pragma unroll
      for (int f = 0; f < NF; ++f) kf[sub][f] = row[2 * f];
      kimg[sub] = (unsigned)__ballot(mod[key] != 0 && half == 0);
    }
    if (!staged) {  // the query rows must have landed before the first products
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
      staged = true;
    }
    if (key0 > last_q) continue;  // nothing this wave's keys can be seen by
    const bool masked = key0 + 32 * KS - 1 > q0;  // some key of the wave lies past the tile's first row

    uint4 pf[AHEAD];
#pragma unroll
    for (int f = 0; f < AHEAD; ++f) pf[f] = *reinterpret_cast<const uint4 *>(qbase + 32 * f);
#pragma unroll
    for (int rb = 0; rb < kRB; ++rb) {
      f32x16_t acc[KS];
      block_products<BF16, D, KS, true, AHEAD>(acc, kf, pf, qbase + rb * (32 * RS * 16), rb + 1 < kRB);  // [key][query row]
      const int qpos = q0 + rb * 32 + n;
      const int limit = qpos < L ? qpos : -1;  // causal: the query at qpos sees keys 0..qpos
      float tm = -INFINITY;
      if (masked) {
#pragma unroll
        for (int sub = 0; sub < KS; ++sub)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = key0 + sub * 32 + acc_row(i, half);
            acc[sub][i] = key <= limit ? acc[sub][i] : -INFINITY;
            tm = fmaxf(tm, acc[sub][i]);
          }
      } else {
#pragma unroll
        for (int sub = 0; sub < KS; ++sub)
#pragma unroll
          for (int i = 0; i < 16; i += 2) tm = fmaxf(fmaxf(tm, acc[sub][i]), acc[sub][i + 1]);
      }
      if (tm > -INFINITY) {
        const float M = fmaxf(m[rb], tm * cl);  // cl > 0: the largest logit is the largest product
        float zt = 0.f, zit = 0.f;
#pragma unroll
        for (int sub = 0; sub < KS; ++sub) {
          float zs = 0.f;
          if (kimg[sub] == 0u || kimg[sub] == 0xffffffffu) {  // one modality: the whole group goes one way
#pragma unroll
            for (int i = 0; i < 16; ++i) zs += fast_exp2(fmaf(acc[sub][i], cl, -M));
            zit += kimg[sub] ? zs : 0.f;
          } else {
            float zsi = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const float p = fast_exp2(fmaf(acc[sub][i], cl, -M));
              zs += p;
              zsi += (kimg[sub] >> acc_row(i, half)) & 1u ? p : 0.f;
            }
            zit += zsi;
          }
          zt += zs;
        }
        const float sc = fast_exp2(m[rb] - M);  // 0 for the first visible keys (m = -inf)
        z[rb] = z[rb] * sc + zt;
        zi[rb] = zi[rb] * sc + zit;
        m[rb] = M;
      }
    }
  }
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();  // nobody reads query rows any more (and they have landed, if no step was taken)

  // ---- fold the two half-waves, then the waves; the share of every row; the tile's sum -----------------
#pragma unroll
  for (int rb = 0; rb < kRB; ++rb) {
    const float m2 = __shfl_xor(m[rb], 32, 64), z2 = __shfl_xor(z[rb], 32, 64), zi2 = __shfl_xor(zi[rb], 32, 64);
    const float M = fmaxf(m[rb], m2);
    if (M > -INFINITY) {
      const float s1 = fast_exp2(m[rb] - M), s2 = fast_exp2(m2 - M);
      z[rb] = z[rb] * s1 + z2 * s2;
      zi[rb] = zi[rb] * s1 + zi2 * s2;
    }
    if (half == 0) lds_stat[wave * kQT + rb * 32 + n] = make_float4(M, z[rb], zi[rb], 0.f);
  }
  __syncthreads();
  for (int row = threadIdx.x; row < kQT; row += kFThreads) {
    float4 t = lds_stat[row];
#pragma unroll
    for (int w = 1; w < kFWaves; ++w) {
      const float4 o = lds_stat[w * kQT + row];
      const float M = fmaxf(t.x, o.x);
      if (M > -INFINITY) {
        const float s1 = fast_exp2(t.x - M), s2 = fast_exp2(o.x - M);
        t.y = t.y * s1 + o.y * s2;
        t.z = t.z * s1 + o.z * s2;
        t.x = M;
      }
    }
    float share = 0.f;  // mass this query sends to the other modality, as a fraction of its total mass
    if (q0 + row < L && t.y > 0.f) share = (mod[q0 + row] ? t.y - t.z : t.z) / t.y;
    lds_red[row] = share;
  }
  __syncthreads();
  for (int span = kQT / 2; span >= 1; span >>= 1) {  // fixed tree: the same sum on every run
    if ((int)threadIdx.x < span) lds_red[threadIdx.x] += lds_red[threadIdx.x + span];
    __syncthreads();
  }
  if (threadIdx.x == 0) a.part[((long long)l * sh.Hq + h) * a.qtiles_total + x] = lds_red[0];
}

// rho of every (layer, sequence): thread h adds the query tiles of head h in order, thread 0 then the heads in order
__global__ __launch_bounds__(256) void flow_exact_finish_kernel(Ctx c, FlowExactArgs a) {
  __shared__ float lds_head[256];
  const Shape &sh = c.sh;
  const int b = blockIdx.x, l = blockIdx.y;
  const int *cu = c.meta + c.meta[MW_OFF_CU_FLOWQ];
  const SeqInfo s = load_seq(c.meta, b);
  float acc = 0.f;
  for (int h0 = 0; h0 < sh.Hq; h0 += 256) {
    const int h = h0 + threadIdx.x;
    if (h < sh.Hq) {
      float hs = 0.f;
      for (int x = cu[b]; x < cu[b + 1]; ++x) hs += a.part[((long long)l * sh.Hq + h) * a.qtiles_total + x];
      lds_head[threadIdx.x] = hs / (float)s.L;
    }
    __syncthreads();
    if (threadIdx.x == 0)
      for (int i = 0; i < min(256, sh.Hq - h0); ++i) acc += lds_head[i];
    __syncthreads();
  }
  if (threadIdx.x != 0) return;
  const float rho = acc / (float)sh.Hq;
  a.rho[l * sh.batch + b] = rho;
  a.mode[l * sh.batch + b] = (rho > sh.theta) != (sh.invert_flow != 0) ? 1 : 0;
}

template <bool BF16, int D>
hipError_t launch_flow_exact_t(const Ctx &c, const FlowExactArgs &a) {
  constexpr int NCH = Cfg<BF16, D>::NCH;
  size_t lds = (size_t)kQT * (NCH + 1) * 16;  // the query rows; later the statistics in the same space
  const size_t lds_stats = (size_t)kFWaves * kQT * sizeof(float4) + (size_t)kQT * 4;
  if (lds_stats > lds) lds = lds_stats;
  hipError_t e = allow_full_lds<flow_exact_kernel<BF16, D>>();
  if (e != hipSuccess) return e;
  {
    ProfScope ps(c.stream, KID_FLOW_EXACT);
    flow_exact_kernel<BF16, D><<<dim3(a.qtiles_total, c.sh.Hq, c.sh.n_layers), kFThreads, lds, c.stream>>>(c, a);
  }
  flow_exact_finish_kernel<<<dim3(c.sh.batch, c.sh.n_layers), 256, 0, c.stream>>>(c, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_flow_exact(const Ctx &c, const FlowExactArgs &a) {
  if (c.sh.bf16) return c.sh.d == 128 ? launch_flow_exact_t<true, 128>(c, a) : launch_flow_exact_t<true, 64>(c, a);
  return c.sh.d == 128 ? launch_flow_exact_t<false, 128>(c, a) : launch_flow_exact_t<false, 64>(c, a);
}

}  // namespace flowmm
