// One decode step of attention over the compacted cache (attention-output equation of the paper's
// Preliminary section, o_t = softmax(q_t K^T / sqrt d) V, with K and V the merged rows that
// flowmm_merge wrote): the operation whose cost the paper's decoding-latency table follows as the
// budget shrinks.  Pure streaming: every merged K and V row is read once.
//
// A workgroup takes a range of slots of one (sequence, kv head, layer) for all G query heads of the
// group.  Lanes that together cover one row (16-byte chunks) form a group; a group walks over its
// rows U at a time (all loads of a trip issued before the first use), computes the G dot products
// of a row with shuffles inside the group, and keeps a running (max, sum, weighted V) per query
// head in the exp2 domain.  The groups of a wave, then the waves, are folded in a fixed order; a
// range that is the whole sequence writes the output, otherwise partials that a second kernel folds.
#include "device_common.h"
#include "kernels.h"
#include "profile.h"

namespace flowmm {

namespace {

constexpr int kDThreads = 256;
constexpr int kDWaves = kDThreads / 64;

// (m, z, acc) <- fold of two partial softmax states of the same query head
__device__ __forceinline__ void fold_state(float &m, float &z, float *acc, int n, float m2, float z2, const float *acc2) {
  const float M = fmaxf(m, m2);
  const float Ms = M == -INFINITY ? 0.f : M;
  const float s1 = fast_exp2(m - Ms), s2 = fast_exp2(m2 - Ms);
  z = z * s1 + z2 * s2;
  for (int e = 0; e < n; ++e) acc[e] = acc[e] * s1 + acc2[e] * s2;
  m = M;
}

// sum over the LPR lanes that share a row, left in every one of them.  Sixteen lanes are one DPP row:
// four rotate-and-add steps on the vector unit; other widths go through the lane permute.
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
  if constexpr (LPR == 16) {
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x128, 0xf, 0xf, false));  // row_ror:8
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x124, 0xf, 0xf, false));  // row_ror:4
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x122, 0xf, 0xf, false));  // row_ror:2
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x121, 0xf, 0xf, false));  // row_ror:1
  } else {
#pragma unroll
    for (int o = LPR / 2; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  }
  return v;
}

template <bool BF16, int D, int GP>
__global__ __launch_bounds__(kDThreads) void decode_partial_kernel(Ctx c, DecodeArgs a) {
  using CF = Cfg<BF16, D>;
  constexpr int LPR = CF::NCH, RPL = 64 / LPR, EPC = CF::kElemsPerChunk, U = 4;
  constexpr int kGroups = kDWaves * RPL;
  __shared__ float lds_state[kDWaves][GP][D + 2];  // per wave and head: acc[D], m, z

  const Shape &sh = c.sh;
  const int b = blockIdx.x / a.splits, split = blockIdx.x - b * a.splits;
  const int gkv = blockIdx.y, l = blockIdx.z;
  const SeqInfo sq = load_seq(c.meta, b);
  const int B = sq.B;
  const int per = (B + a.splits - 1) / a.splits;
  const int s0 = split * per, s1 = min(B, s0 + per);  // this workgroup's slots
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, rg = lane / LPR, ch = lane % LPR;
  const int gid = wave * RPL + rg;
  const long long unit = (long long)l * sh.Hkv + gkv;
  const uint4 *Kc = reinterpret_cast<const uint4 *>(a.K_c) + (unit * sh.SB + sq.kept_off) * LPR;
  const uint4 *Vc = reinterpret_cast<const uint4 *>(a.V_c) + (unit * sh.SB + sq.kept_off) * LPR;

  // this lane's channels of the G queries (heads past G are zero and never written)
  float q[GP][EPC];
#pragma unroll
  for (int g = 0; g < GP; ++g) {
    if (a.g0 + g < sh.G) {
      const long long qrow = ((long long)l * sh.Hq + gkv * sh.G + a.g0 + g) * sh.batch + b;
      chunk_to_floats<BF16>(reinterpret_cast<const uint4 *>(a.q)[qrow * LPR + ch], q[g]);
    } else {
#pragma unroll
      for (int e = 0; e < EPC; ++e) q[g][e] = 0.f;
    }
  }
  float m[GP], z[GP], acc[GP][EPC];
#pragma unroll
  for (int g = 0; g < GP; ++g) {
    m[g] = -INFINITY;
    z[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPC; ++e) acc[g][e] = 0.f;
  }

  const float cl = sh.scale_log2e;
  for (int r0 = s0 + gid; r0 < s1; r0 += kGroups * U) {
    uint4 kc[U], vc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int r = min(r0 + u * kGroups, s1 - 1);  // a trip past the end reads the last row again; its weight is 0
      kc[u] = Kc[(long long)r * LPR + ch];
      vc[u] = Vc[(long long)r * LPR + ch];
    }
    // the logits of the U rows for every head, then one rescale of the running state per head and trip
    float fv[U][EPC];
    float sl[GP][U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float fk[EPC];
      chunk_to_floats<BF16>(kc[u], fk);
      chunk_to_floats<BF16>(vc[u], fv[u]);
      const bool real = r0 + u * kGroups < s1;
#pragma unroll
      for (int g = 0; g < GP; ++g) {
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < EPC; ++e) dot = fmaf(fk[e], q[g][e], dot);
        dot = group_sum<LPR>(dot);
        sl[g][u] = real ? dot * cl : -INFINITY;
      }
    }
#pragma unroll
    for (int g = 0; g < GP; ++g) {
      float M = m[g];
#pragma unroll
      for (int u = 0; u < U; ++u) M = fmaxf(M, sl[g][u]);
      const float Ms = M == -INFINITY ? 0.f : M;
      const float sc = fast_exp2(m[g] - Ms);
      z[g] *= sc;
#pragma unroll
      for (int e = 0; e < EPC; ++e) acc[g][e] *= sc;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float p = fast_exp2(sl[g][u] - Ms);
        z[g] += p;
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[g][e] = fmaf(p, fv[u][e], acc[g][e]);
      }
      m[g] = M;
    }
  }

  // fold the row groups of the wave (fixed tree), then the waves (in order)
#pragma unroll
  for (int o = LPR; o < 64; o <<= 1) {
#pragma unroll
    for (int g = 0; g < GP; ++g) {
      const float m2 = __shfl_xor(m[g], o, 64), z2 = __shfl_xor(z[g], o, 64);
      float a2[EPC];
#pragma unroll
      for (int e = 0; e < EPC; ++e) a2[e] = __shfl_xor(acc[g][e], o, 64);
      fold_state(m[g], z[g], acc[g], EPC, m2, z2, a2);
    }
  }
  if (rg == 0) {
#pragma unroll
    for (int g = 0; g < GP; ++g) {
#pragma unroll
      for (int e = 0; e < EPC; ++e) lds_state[wave][g][ch * EPC + e] = acc[g][e];
      if (ch == 0) { lds_state[wave][g][D] = m[g]; lds_state[wave][g][D + 1] = z[g]; }
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < GP * D; idx += kDThreads) {
    const int g = idx / D, ci = idx - g * D;
    if (a.g0 + g >= sh.G) continue;
    float mm = lds_state[0][g][D], zz = lds_state[0][g][D + 1], av = lds_state[0][g][ci];
#pragma unroll
    for (int w = 1; w < kDWaves; ++w) fold_state(mm, zz, &av, 1, lds_state[w][g][D], lds_state[w][g][D + 1], &lds_state[w][g][ci]);
    const long long qrow = ((long long)l * sh.Hq + gkv * sh.G + a.g0 + g) * sh.batch + b;
    if (a.splits == 1) {
      const float o = av / zz;  // B >= 1: at least one row has been seen
      if constexpr (BF16) reinterpret_cast<uint16_t *>(a.out)[qrow * D + ci] = (uint16_t)float_to_bf16_bits(o);
      else reinterpret_cast<float *>(a.out)[qrow * D + ci] = o;
    } else {
      float *part = a.part + (qrow * a.splits + split) * (D + 2);
      part[ci] = av;
      if (ci == 0) { part[D] = mm; part[D + 1] = zz; }
    }
  }
}

// out[l][h][b] from the partial states of the slot ranges, in range order
template <bool BF16, int D>
__global__ __launch_bounds__(D) void decode_combine_kernel(Ctx c, DecodeArgs a) {
  const Shape &sh = c.sh;
  const long long qrow = ((long long)blockIdx.z * sh.Hq + blockIdx.y) * sh.batch + blockIdx.x;
  const int ci = threadIdx.x;
  const float *part = a.part + qrow * a.splits * (D + 2);
  float mm = part[D], zz = part[D + 1], av = part[ci];
  for (int sp = 1; sp < a.splits; ++sp) {
    const float *p2 = part + (long long)sp * (D + 2);
    fold_state(mm, zz, &av, 1, p2[D], p2[D + 1], &p2[ci]);
  }
  const float o = av / zz;
  if constexpr (BF16) reinterpret_cast<uint16_t *>(a.out)[qrow * D + ci] = (uint16_t)float_to_bf16_bits(o);
  else reinterpret_cast<float *>(a.out)[qrow * D + ci] = o;
}

template <bool BF16, int D, int GP>
hipError_t launch_partial(const Ctx &c, const DecodeArgs &a) {
  ProfScope ps(c.stream, KID_DECODE_PARTIAL);
  decode_partial_kernel<BF16, D, GP><<<dim3(c.sh.batch * a.splits, c.sh.Hkv, c.sh.n_layers), kDThreads, 0, c.stream>>>(c, a);
  return hipGetLastError();
}

template <bool BF16, int D>
hipError_t launch_decode_t(const Ctx &c, DecodeArgs a) {
  // query heads of a kv group in register-sized batches (one batch unless G > 8: the cache is then read once per batch)
  for (int g0 = 0; g0 < c.sh.G; g0 += 8) {
    a.g0 = g0;
    const int left = c.sh.G - g0;
    hipError_t e = left > 4 ? launch_partial<BF16, D, 8>(c, a)
                 : left > 2 ? launch_partial<BF16, D, 4>(c, a)
                 : left > 1 ? launch_partial<BF16, D, 2>(c, a) : launch_partial<BF16, D, 1>(c, a);
    if (e != hipSuccess) return e;
  }
  if (a.splits > 1) {
    ProfScope ps(c.stream, KID_DECODE_COMBINE);
    decode_combine_kernel<BF16, D><<<dim3(c.sh.batch, c.sh.Hq, c.sh.n_layers), D, 0, c.stream>>>(c, a);
  }
  return hipGetLastError();
}

}  // namespace

// slot ranges per sequence: enough workgroups to fill the chip, ranges of at least 64 slots
int decode_splits(const Shape &sh) {
  const long long units = (long long)sh.batch * sh.Hkv * sh.n_layers;
  long long want = (2048 + units - 1) / units;
  const long long most = (sh.maxB + 63) / 64;
  if (want > most) want = most;
  if (want > kDecodeMaxSplits) want = kDecodeMaxSplits;
  return want < 1 ? 1 : (int)want;
}

hipError_t launch_decode_attention(const Ctx &c, const DecodeArgs &a) {
  if (c.sh.bf16) return c.sh.d == 128 ? launch_decode_t<true, 128>(c, a) : launch_decode_t<true, 64>(c, a);
  return c.sh.d == 128 ? launch_decode_t<false, 128>(c, a) : launch_decode_t<false, 64>(c, a);
}

}  // namespace flowmm
