// Step "merge": fold every matched non-pivot K/V row into its pivot,
//   out[slot] = (row[pivot] + sum of member rows) / (1 + number of members),
// the uniform-weight instance of the paper's K_merged = f_merge(K, S), V_merged = g_merge(V, S)
// (FlowMM, Preliminary), writing a compacted cache in ascending pivot position.  On request the
// similarity-weighted mean instead (pivot weight 1, member weight max(cosine to the pivot's key, 0),
// computed here from the rows being merged): the variant of the paper's component ablation.
//
// Three kernels, no floating-point atomics, so results are bit-identical from run to run:
//   1. csr   : one workgroup per (sequence, kv head, layer) groups the evicted tokens by slot,
//              ascending inside each slot (a stable counting sort: every wave counts a fixed
//              token range per slot, a scan turns the counts into exact write cursors), and
//              cuts the slots into tasks of at most kTaskChunk members.
//   2. tasks : one wave per task streams its rows with 16-byte loads (a wave covers 64/NCH rows
//              per load), sums them in fp32 and either finishes the slot or leaves a partial.
//   3. fold  : slots with several tasks add up their partials in task order (a few workgroups per
//              (sequence, kv head, layer) walk over them).
#include "device_common.h"
#include "kernels.h"
#include "profile.h"

namespace flowmm {

namespace {

constexpr int kCsrThreads = kCsrWaves * 64;

__device__ __forceinline__ int block_exclusive_scan_1024(int v, int *lds_wave, int *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int u = __shfl_up(inc, o, 64);
    if (lane >= o) inc += u;
  }
  __syncthreads();
  if (lane == 63) lds_wave[wave] = inc;
  __syncthreads();
  if (wave == 0) {
    const int w = lane < kCsrWaves ? lds_wave[lane] : 0;
    int winc = w;
#pragma unroll
    for (int o = 1; o < kCsrWaves; o <<= 1) {
      const int u = __shfl_up(winc, o, 64);
      if (lane >= o) winc += u;
    }
    if (lane < kCsrWaves) lds_wave[lane] = winc - w;
    if (lane == kCsrWaves - 1) lds_wave[kCsrWaves] = winc;
  }
  __syncthreads();
  *total = lds_wave[kCsrWaves];
  return lds_wave[wave] + inc - v;
}

// lanes of the wave that hold the same slot as this lane (only meaningful where member)
__device__ __forceinline__ unsigned long long same_slot_mask(bool member, int slot, int nbits) {
  unsigned long long m = __ballot(member);
  for (int bit = 0; bit < nbits; ++bit) {
    const bool one = (slot >> bit) & 1;
    const unsigned long long bb = __ballot(member && one);
    m &= one ? bb : ~bb;
  }
  return m;
}

__global__ __launch_bounds__(kCsrThreads) void merge_csr_kernel(Ctx c, int nw_shift) {
  extern __shared__ int lds_tbl[];  // [B][NW] per-wave counts, later write cursors
  __shared__ int lds_wave[kCsrWaves + 1];
  const Shape &sh = c.sh;
  const int *meta = c.meta;
  const int b = blockIdx.x, gkv = blockIdx.y, l = blockIdx.z;
  const SeqInfo s = load_seq(meta, b);
  const long long unit = (long long)l * sh.Hkv + gkv;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int NW = 1 << nw_shift;  // waves that walk tokens (the table must fit in LDS)
  const int *assign = c.assign + unit * sh.T + s.tok_off;
  const int *kept = c.kept_idx + unit * sh.SB + s.kept_off;
  int *members = c.members + unit * sh.T + s.tok_off;
  int *seg_off = c.seg_off + unit * (sh.SB + sh.batch) + s.kept_off + b;
  const int task_base = (meta + meta[MW_OFF_CU_TASK])[b];
  const int multi_base = (meta + meta[MW_OFF_CU_MULTI])[b];
  const int part_base = (meta + meta[MW_OFF_CU_PART])[b];
  int4 *tasks = c.tasks + unit * sh.tasks_total + task_base;
  int4 *multi = c.multi + unit * sh.multi_total + multi_base;

  int nbits = 0;
  while ((1 << nbits) < s.B) ++nbits;
  const int range = ((s.L + NW - 1) / NW + 63) & ~63;  // tokens per walking wave
  const int r0 = wave * range, r1 = min(s.L, r0 + range);

  for (int i = threadIdx.x; i < s.B * NW; i += kCsrThreads) lds_tbl[i] = 0;
  __syncthreads();

  // pass 1: members of each slot inside each wave's token range
  if (wave < NW) {
    for (int i0 = r0; i0 < r1; i0 += 64) {
      const int i = i0 + lane;
      const int slot = i < r1 ? assign[i] : -1;
      const bool member = slot >= 0 && kept[slot] != i;
      const unsigned long long m = same_slot_mask(member, slot, nbits);
      if (member && (m & ((1ull << lane) - 1)) == 0) lds_tbl[slot * NW + wave] += __popcll(m);
    }
  }
  __syncthreads();

  // scan over slots: segment offsets, write cursors, task list
  int seg_carry = 0, task_carry = 0, multi_carry = 0, part_carry = 0;
  for (int s0 = 0; s0 < s.B; s0 += kCsrThreads) {
    const int slot = s0 + threadIdx.x;
    int n = 0;
    if (slot < s.B)
      for (int w = 0; w < NW; ++w) n += lds_tbl[slot * NW + w];
    const int nt = slot < s.B ? max(1, (n + kTaskChunk - 1) / kTaskChunk) : 0;
    const int is_multi = nt > 1;
    int tot_n, tot_t, tot_m, tot_p;
    const int seg = seg_carry + block_exclusive_scan_1024(n, lds_wave, &tot_n);
    const int tb = task_carry + block_exclusive_scan_1024(nt, lds_wave, &tot_t);
    const int mb = multi_carry + block_exclusive_scan_1024(is_multi, lds_wave, &tot_m);
    const int pb = part_carry + block_exclusive_scan_1024(is_multi ? nt : 0, lds_wave, &tot_p);
    if (slot < s.B) {
      seg_off[slot] = seg;
      int base = seg;
      for (int w = 0; w < NW; ++w) {
        const int t = lds_tbl[slot * NW + w];
        lds_tbl[slot * NW + w] = base;
        base += t;
      }
      for (int j = 0; j < nt; ++j)
        tasks[tb + j] = make_int4(slot, seg + j * kTaskChunk, min(kTaskChunk, n - j * kTaskChunk),
                                  is_multi ? part_base + pb + j : -1);
      if (is_multi) multi[mb] = make_int4(slot, part_base + pb, nt, n);
    }
    seg_carry += tot_n;
    task_carry += tot_t;
    multi_carry += tot_m;
    part_carry += tot_p;
  }
  if (threadIdx.x == 0) {
    seg_off[s.B] = seg_carry;
    c.n_tasks[unit * sh.batch + b] = task_carry;
    c.n_multi[unit * sh.batch + b] = multi_carry;
  }
  __syncthreads();

  // pass 2: write the members, ascending inside every slot
  if (wave < NW) {
    for (int i0 = r0; i0 < r1; i0 += 64) {
      const int i = i0 + lane;
      const int slot = i < r1 ? assign[i] : -1;
      const bool member = slot >= 0 && kept[slot] != i;
      const unsigned long long m = same_slot_mask(member, slot, nbits);
      const unsigned long long below = m & ((1ull << lane) - 1);
      if (member) {
        const int cur = lds_tbl[slot * NW + wave];
        members[cur + __popcll(below)] = i;
        if (below == 0) lds_tbl[slot * NW + wave] = cur + __popcll(m);
      }
    }
  }
}

// WEIGHTED: the similarity-weighted mean (the pivot counts 1, a member max(u, 0), u the cosine of
// its key to the pivot's key, 0 for a zero row; V rows take the weights of their K rows).
template <bool BF16, int D, bool WEIGHTED>
__global__ __launch_bounds__(256) void merge_tasks_kernel(Ctx c) {
  using CF = Cfg<BF16, D>;
  constexpr int LPR = CF::NCH;        // lanes that cover one row
  constexpr int RPL = 64 / LPR;       // rows a wave covers per load
  constexpr int EPC = CF::kElemsPerChunk;
  constexpr int U = 4;                // loads in flight per lane and tensor
  const Shape &sh = c.sh;
  const int *meta = c.meta;
  const int *cu = meta + meta[MW_OFF_CU_TASK];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int q = blockIdx.x * 4 + wave;
  if (q >= sh.tasks_total) return;
  const int gkv = blockIdx.y, l = blockIdx.z;
  const long long unit = (long long)l * sh.Hkv + gkv;
  const int b = find_seq(cu, meta[MW_BATCH], q);
  const int ql = q - cu[b];
  if (ql >= c.n_tasks[unit * sh.batch + b]) return;
  const SeqInfo s = load_seq(meta, b);
  const int4 task = c.tasks[unit * sh.tasks_total + q];  // (slot, first member, count, partial index)
  const int rg = lane / LPR, ch = lane % LPR;
  const long long head_off = (long long)l * sh.ks_layer + (long long)gkv * sh.ks_head + (long long)s.tok_off * sh.ks_tok;
  const uint4 *K = reinterpret_cast<const uint4 *>(c.K) + head_off;
  const uint4 *V = reinterpret_cast<const uint4 *>(c.V) + head_off;
  const int *members = c.members + unit * sh.T + s.tok_off + task.y;

  float ak[EPC], av[EPC];
#pragma unroll
  for (int e = 0; e < EPC; ++e) ak[e] = av[e] = 0.f;
  const bool single = task.w < 0;
  const int pivot_tok = c.kept_idx[unit * sh.SB + s.kept_off + task.x];
  float wsum = 0.f;        // weighted merge: weights this row group has added
  float pk[EPC], pss = 0.f;  // weighted merge: this lane's chunk of the pivot's key, its squared norm
  if constexpr (WEIGHTED) {
    chunk_to_floats<BF16>(K[(long long)pivot_tok * sh.ks_tok + ch], pk);
#pragma unroll
    for (int e = 0; e < EPC; ++e) pss = fmaf(pk[e], pk[e], pss);
#pragma unroll
    for (int o = LPR / 2; o >= 1; o >>= 1) pss += __shfl_xor(pss, o, 64);
  }
  if (single && rg == 0) {
    if constexpr (WEIGHTED) {
#pragma unroll
      for (int e = 0; e < EPC; ++e) ak[e] = pk[e];
      wsum = 1.f;
    } else {
      chunk_to_floats<BF16>(K[(long long)pivot_tok * sh.ks_tok + ch], ak);
    }
    chunk_to_floats<BF16>(V[(long long)pivot_tok * sh.ks_tok + ch], av);
  }
  for (int j0 = rg; j0 < task.z; j0 += RPL * U) {
    int tokv[U];
    uint4 kc[U], vc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = j0 + u * RPL;
      tokv[u] = j < task.z ? members[j] : -1;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (tokv[u] >= 0) {
        kc[u] = K[(long long)tokv[u] * sh.ks_tok + ch];
        vc[u] = V[(long long)tokv[u] * sh.ks_tok + ch];
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      // every lane takes part in the exchanges below, so rows past the end count as zero rows
      float fk[EPC], fv[EPC];
      const bool real = tokv[u] >= 0;
      if (real) {
        chunk_to_floats<BF16>(kc[u], fk);
        chunk_to_floats<BF16>(vc[u], fv);
      } else {
#pragma unroll
        for (int e = 0; e < EPC; ++e) fk[e] = fv[e] = 0.f;
      }
      if constexpr (WEIGHTED) {
        float dot = 0.f, ss = 0.f;
#pragma unroll
        for (int e = 0; e < EPC; ++e) { dot = fmaf(fk[e], pk[e], dot); ss = fmaf(fk[e], fk[e], ss); }
#pragma unroll
        for (int o = LPR / 2; o >= 1; o >>= 1) { dot += __shfl_xor(dot, o, 64); ss += __shfl_xor(ss, o, 64); }
        const float w = ss > 0.f && pss > 0.f ? fmaxf(dot / (sqrtf(ss) * sqrtf(pss)), 0.f) : 0.f;
        wsum += w;
#pragma unroll
        for (int e = 0; e < EPC; ++e) { ak[e] = fmaf(w, fk[e], ak[e]); av[e] = fmaf(w, fv[e], av[e]); }
      } else if (real) {
#pragma unroll
        for (int e = 0; e < EPC; ++e) { ak[e] += fk[e]; av[e] += fv[e]; }
      }
    }
  }
  // fold the row groups (fixed tree)
#pragma unroll
  for (int o = LPR; o < 64; o <<= 1) {
#pragma unroll
    for (int e = 0; e < EPC; ++e) {
      ak[e] += __shfl_xor(ak[e], o, 64);
      av[e] += __shfl_xor(av[e], o, 64);
    }
    if constexpr (WEIGHTED) wsum += __shfl_xor(wsum, o, 64);
  }
  if (rg != 0) return;
  if (single) {
    const float den = WEIGHTED ? wsum : (float)(1 + task.z);
#pragma unroll
    for (int e = 0; e < EPC; ++e) { ak[e] = ak[e] / den; av[e] = av[e] / den; }
    const long long orow = (unit * sh.SB + s.kept_off + task.x) * LPR + ch;
    reinterpret_cast<uint4 *>(c.K_out)[orow] = floats_to_chunk<BF16>(ak);
    reinterpret_cast<uint4 *>(c.V_out)[orow] = floats_to_chunk<BF16>(av);
  } else {
    float *p = c.partials + ((unit * sh.part_total + task.w) * 2) * D + ch * EPC;
#pragma unroll
    for (int e = 0; e < EPC; e += 4) {
      *reinterpret_cast<float4 *>(p + e) = make_float4(ak[e], ak[e + 1], ak[e + 2], ak[e + 3]);
      *reinterpret_cast<float4 *>(p + D + e) = make_float4(av[e], av[e + 1], av[e + 2], av[e + 3]);
    }
    if (WEIGHTED && ch == 0) c.partial_w[unit * sh.part_total + task.w] = wsum;
  }
}

// kFoldGroups workgroups per (sequence, kv head, layer) walk over its split slots, one wave per slot
template <bool BF16, int D, bool WEIGHTED>
__global__ __launch_bounds__(256) void merge_fold_kernel(Ctx c) {
  constexpr int EPC = Cfg<BF16, D>::kElemsPerChunk;
  constexpr int NCH = Cfg<BF16, D>::NCH;
  const Shape &sh = c.sh;
  const int *meta = c.meta;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int b = blockIdx.x / kFoldGroups;
  const int gkv = blockIdx.y, l = blockIdx.z;
  const long long unit = (long long)l * sh.Hkv + gkv;
  const int n_multi = c.n_multi[unit * sh.batch + b];
  const int q0 = (meta + meta[MW_OFF_CU_MULTI])[b];
  for (int qm = (blockIdx.x % kFoldGroups) * 4 + wave; qm < n_multi; qm += kFoldGroups * 4) {
    const int q = q0 + qm;
    const SeqInfo s = load_seq(meta, b);
    const int4 e4 = c.multi[unit * sh.multi_total + q];  // (slot, first partial, partials, members)
    const int pivot_tok = c.kept_idx[unit * sh.SB + s.kept_off + e4.x];
    const long long head_off = (long long)l * sh.ks_layer + (long long)gkv * sh.ks_head +
                               (long long)(s.tok_off + pivot_tok) * sh.ks_tok;
    float den = (float)(1 + e4.w);
    if constexpr (WEIGHTED) {
      den = 1.f;  // the pivot's own weight, then the partial sums in task order
      for (int pi = 0; pi < e4.z; ++pi) den += c.partial_w[unit * sh.part_total + e4.y + pi];
    }
    // lanes [0, NCH) fold K chunks, lanes [NCH, 2 NCH) fold V chunks
    for (int idx = lane; idx < 2 * NCH; idx += 64) {
      const int tensor = idx / NCH, ch = idx % NCH;
      const uint4 *src = reinterpret_cast<const uint4 *>(tensor ? c.V : c.K) + head_off;
      float acc[EPC];
      chunk_to_floats<BF16>(src[ch], acc);
      constexpr int U = 8;  // partials in flight; they are added in task order all the same
      for (int p0 = 0; p0 < e4.z; p0 += U) {
        float part[U][EPC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          if (p0 + u < e4.z) {
            const float *pp = c.partials + ((unit * sh.part_total + e4.y + p0 + u) * 2 + tensor) * D + ch * EPC;
#pragma unroll
            for (int e = 0; e < EPC; e += 4) {
              const float4 f4 = *reinterpret_cast<const float4 *>(pp + e);
              part[u][e] = f4.x; part[u][e + 1] = f4.y; part[u][e + 2] = f4.z; part[u][e + 3] = f4.w;
            }
          }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          if (p0 + u < e4.z) {
#pragma unroll
            for (int e = 0; e < EPC; ++e) acc[e] += part[u][e];
          }
        }
      }
#pragma unroll
      for (int e = 0; e < EPC; ++e) acc[e] = acc[e] / den;
      const long long orow = (unit * sh.SB + s.kept_off + e4.x) * NCH + ch;
      reinterpret_cast<uint4 *>(tensor ? c.V_out : c.K_out)[orow] = floats_to_chunk<BF16>(acc);
    }
  }
}

template <bool BF16, int D, bool WEIGHTED>
hipError_t launch_merge_w(const Ctx &c, int nw_shift, size_t lds) {
  const Shape &sh = c.sh;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(merge_csr_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  {
    ProfScope ps(c.stream, KID_MERGE_CSR);
    merge_csr_kernel<<<dim3(sh.batch, sh.Hkv, sh.n_layers), kCsrThreads, lds, c.stream>>>(c, nw_shift);
  }
  {
    ProfScope ps(c.stream, KID_MERGE_TASKS);
    merge_tasks_kernel<BF16, D, WEIGHTED><<<dim3((sh.tasks_total + 3) / 4, sh.Hkv, sh.n_layers), 256, 0, c.stream>>>(c);
  }
  {
    ProfScope ps(c.stream, KID_MERGE_FOLD);
    merge_fold_kernel<BF16, D, WEIGHTED><<<dim3(sh.batch * kFoldGroups, sh.Hkv, sh.n_layers), 256, 0, c.stream>>>(c);
  }
  return hipGetLastError();
}

template <bool BF16, int D>
hipError_t launch_merge_t(const Ctx &c, int nw_shift, size_t lds) {
  return c.sh.weighted_merge ? launch_merge_w<BF16, D, true>(c, nw_shift, lds) : launch_merge_w<BF16, D, false>(c, nw_shift, lds);
}

}  // namespace

// largest per-sequence budget decides how many waves may walk tokens: the [B][NW] table lives in LDS
static int merge_csr_wave_shift(int max_budget) {
  int shift = 4;  // 16 waves
  while (shift > 0 && (size_t)max_budget * (1u << shift) * 4 > 128u * 1024u) --shift;
  return shift;
}

size_t merge_csr_lds_bytes(int max_budget) {
  return (size_t)max_budget * (1u << merge_csr_wave_shift(max_budget)) * 4;
}

hipError_t launch_merge(const Ctx &c) {
  const int shift = merge_csr_wave_shift(c.sh.maxB);
  const size_t lds = merge_csr_lds_bytes(c.sh.maxB);
  if (c.sh.bf16)
    return c.sh.d == 128 ? launch_merge_t<true, 128>(c, shift, lds) : launch_merge_t<true, 64>(c, shift, lds);
  return c.sh.d == 128 ? launch_merge_t<false, 128>(c, shift, lds) : launch_merge_t<false, 64>(c, shift, lds);
}

}  // namespace flowmm
