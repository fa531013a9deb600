// Merge of one (sequence, layer, kv head) unit by one workgroup of 256 threads: the body shared by
// the stand-alone merge kernel and the kernels that merge right after matching.
//   out[slot] = (row[kept[slot]] + sum of the rows assigned to slot) / (1 + their number)
// for K and V (the merged cache K_merged = f_merge(K, S), V_merged = g_merge(V, S) of the paper's
// Preliminary section, with the uniform mean as the merge operator).
#pragma once
#include "device_common.h"
#include "kernels.h"
#include "select_core.h"

namespace flowmm {

// 16-byte chunk number `chunk` behind a wave-uniform base: the lane's part of the address is a 32-bit
// byte offset (the unit-resident path is only taken when a sequence's rows lie within 4 GiB), which
// spares the 64-bit multiply-add per row that a pointer per lane costs.
template <typename T>
__device__ __forceinline__ T chunk_at(const void *base, unsigned chunk) {
  return *reinterpret_cast<const T *>(reinterpret_cast<const char *>(base) + (size_t)(chunk * 16u));
}

constexpr int kF3Threads = 256;
constexpr int kF3Waves = kF3Threads / 64;
constexpr int kF3Chunks = 4;   // 64-token chunks a wave walks: ceil(1024 / 4 waves / 64)
constexpr int kUnitChunk = 64;  // members per task of a slot that is cut up (keeps the partial sums in LDS few)

struct MergeLds {  // element offsets (ints) into the dynamic LDS block
  int tbl, kept, copies, members, tasks, multi, partials, partial_w, total_bytes;
};

__host__ __device__ inline MergeLds merge_lds_layout(int maxB, int maxE, int d) {
  MergeLds m;
  int off = 0;
  m.tbl = off; off += maxB * kF3Waves;
  m.kept = off; off += maxB;
  m.copies = off; off += maxB;
  m.members = off; off += maxE + 1;
  off = (off + 3) & ~3;
  m.tasks = off; off += 4 * (maxB + maxE / kUnitChunk + 1);
  m.multi = off; off += 4 * (maxE / (kUnitChunk + 1) + 1);
  m.partials = off; off += (2 * (maxE / kUnitChunk) + 2) * 2 * d;
  m.partial_w = off; off += 2 * (maxE / kUnitChunk) + 2;  // weight sums of the partials (weighted merge)
  m.total_bytes = off * 4;
  return m;
}

__device__ __forceinline__ unsigned long long same_slot_lanes(bool member, int slot, int nbits) {
  unsigned long long m = __ballot(member);
  for (int bit = 0; bit < nbits; ++bit) {
    const bool one = (slot >> bit) & 1;
    const unsigned long long bb = __ballot(member && one);
    m &= one ? bb : ~bb;
  }
  return m;
}

// All 256 threads of the workgroup call.  assign: slot of every token of the unit (pivot: own slot,
// -1: dropped), global or LDS; kept_src: the pivot positions, ascending (global or LDS).
// One workgroup per unit.  A stable counting sort groups the evicted tokens by slot in LDS; then
// every group of LPR lanes (one 16-byte chunk per lane, so a group covers one row per load)
// works on its own: pivots nobody merges into are copied, U rows in flight per group; the other
// slots become tasks (a slot, or a chunk of at most kUnitChunk members of a larger slot) that a
// group adds up row after row, U row loads in flight, large chunks first; slots cut into several
// tasks are folded from their partial sums at the end.
// WEIGHTED: the similarity-weighted mean instead of the uniform one: the pivot counts 1, a member
// max(u, 0) with u the cosine of its key to the pivot's key (0 for a zero row), computed here from
// the rows that are being merged; V rows take the weights of their K rows.
template <int D, int U = 8, bool WEIGHTED = false>
__device__ __forceinline__ void unit_merge_body(const Ctx &c, const SeqInfo &s, long long unit, int l, int gkv,
                                                const int *assign, const int *kept_src, int *lds_i, int maxB,
                                                int maxE, long long *lds_wave, int *sh_next_p) {
  using CF = Cfg<true, D>;
  constexpr int LPR = CF::NCH, RPL = 64 / LPR, EPC = CF::kElemsPerChunk;
  constexpr bool kBF16 = true;
  const MergeLds lay = merge_lds_layout(maxB, maxE, D);
  int *tbl = lds_i + lay.tbl;          // [B][waves] members per wave range, later write cursors
  int *lds_kept = lds_i + lay.kept;    // [B] pivot positions
  int *copies = lds_i + lay.copies;    // slots without members
  int *members = lds_i + lay.members;  // evicted tokens grouped by slot, ascending
  int4 *tasks = reinterpret_cast<int4 *>(lds_i + lay.tasks);  // (slot, first member, members, partial or -1)
  int4 *multi = reinterpret_cast<int4 *>(lds_i + lay.multi);  // (slot, first partial, partials, members)
  float *partials = reinterpret_cast<float *>(lds_i + lay.partials);
  float *partial_w = reinterpret_cast<float *>(lds_i + lay.partial_w);
  int &sh_next = *sh_next_p;           // next task nobody has taken yet

  const Shape &sh = c.sh;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  constexpr int NW = kF3Waves;
  int nbits = 0;
  while ((1 << nbits) < s.B) ++nbits;
  const int range = ((s.L + NW - 1) / NW + 63) & ~63;  // <= 64 * kF3Chunks since L <= 1024
  const int r0 = wave * range, r1 = min(s.L, r0 + range);

  // this wave's assignments and the pivot list arrive in one round trip
  int slot_of[kF3Chunks];
#pragma unroll
  for (int k = 0; k < kF3Chunks; ++k) {
    const int i = r0 + k * 64 + lane;
    slot_of[k] = i < r1 ? assign[i] : -1;
  }
  for (int i = threadIdx.x; i < s.B; i += kF3Threads) lds_kept[i] = kept_src[i];
  for (int i = threadIdx.x; i < s.B * NW; i += kF3Threads) tbl[i] = 0;
  if (threadIdx.x == 0) sh_next = kF3Waves * (64 / CF::NCH);  // the first tasks go to the groups in order
  __syncthreads();
  // members of each slot inside each wave's token range
  unsigned long long same[kF3Chunks];
  bool member[kF3Chunks];
#pragma unroll
  for (int k = 0; k < kF3Chunks; ++k) {
    const int i = r0 + k * 64 + lane;
    member[k] = slot_of[k] >= 0 && lds_kept[slot_of[k]] != i;
    same[k] = same_slot_lanes(member[k], slot_of[k], nbits);
    if (member[k] && (same[k] & ((1ull << lane) - 1)) == 0) tbl[slot_of[k] * NW + wave] += __popcll(same[k]);
  }
  __syncthreads();
  int n_tasks, n_multi, n_copy;
  {  // one packed scan over the slots (B <= 256 <= threads): member offsets, multi-task slots,
     // their chunks, single-task slots and copy-only slots
    const int slot = threadIdx.x;
    int n = 0;
    if (slot < s.B)
      for (int w = 0; w < NW; ++w) n += tbl[slot * NW + w];
    const int nt = (n + kUnitChunk - 1) / kUnitChunk;  // 0: copy, 1: one task, more: chunks + fold
    const bool valid = slot < s.B;
    const long long packed = (long long)n | ((long long)(valid && nt > 1) << 16) |
                             ((long long)(nt > 1 ? nt : 0) << 24) | ((long long)(valid && nt == 1) << 36) |
                             ((long long)(valid && nt == 0) << 48);
    long long tot;
    const long long ex = block_exclusive_scan<kF3Threads, long long>(packed, lds_wave, &tot);
    const int sg = (int)(ex & 0xffff), mb = (int)((ex >> 16) & 0xff), pb = (int)((ex >> 24) & 0xfff),
              sb = (int)((ex >> 36) & 0xfff), cb = (int)((ex >> 48) & 0xfff);
    const int n_part = (int)((tot >> 24) & 0xfff);
    n_multi = (int)((tot >> 16) & 0xff);
    n_tasks = n_part + (int)((tot >> 36) & 0xfff);
    n_copy = (int)((tot >> 48) & 0xfff);
    if (valid) {
      int base = sg;
      for (int w = 0; w < NW; ++w) {
        const int t = tbl[slot * NW + w];
        tbl[slot * NW + w] = base;
        base += t;
      }
      if (nt == 0) {
        copies[cb] = slot;
      } else if (nt == 1) {
        tasks[n_part + sb] = make_int4(slot, sg, n, -1);  // after all the chunks of large slots
      } else {
        for (int j = 0; j < nt; ++j)
          tasks[pb + j] = make_int4(slot, sg + j * kUnitChunk, min(kUnitChunk, n - j * kUnitChunk), pb + j);
        multi[mb] = make_int4(slot, pb, nt, n);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kF3Chunks; ++k) {
    const unsigned long long below = same[k] & ((1ull << lane) - 1);
    if (member[k]) {
      const int cur = tbl[slot_of[k] * NW + wave];
      members[cur + __popcll(below)] = r0 + k * 64 + lane;
      if (below == 0) tbl[slot_of[k] * NW + wave] = cur + __popcll(same[k]);
    }
  }

  const int rg = lane / LPR, ch = lane % LPR;
  const long long head_off = (long long)l * sh.ks_layer + (long long)gkv * sh.ks_head + (long long)s.tok_off * sh.ks_tok;
  const uint4 *K = reinterpret_cast<const uint4 *>(c.K) + head_off;
  const uint4 *V = reinterpret_cast<const uint4 *>(c.V) + head_off;
  const unsigned kst = (unsigned)sh.ks_tok;
  uint4 *Ko = reinterpret_cast<uint4 *>(c.K_out) + (unit * sh.SB + s.kept_off) * LPR;
  uint4 *Vo = reinterpret_cast<uint4 *>(c.V_out) + (unit * sh.SB + s.kept_off) * LPR;
  constexpr int kGroups = kF3Waves * RPL;
  const int gid = wave * RPL + rg;

  // pivots nobody merges into: bit copies (needs no member list, so it runs before the barrier).
  // Full passes first: U rows per group with nothing conditional between the loads, so that they
  // are all in flight before the first store; then the rest one row at a time.  (The rows pass
  // through a native vector type: arrays of the uint4 class would be kept in scratch memory.)
  {
    typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
    u32x4_t *Koc = reinterpret_cast<u32x4_t *>(Ko), *Voc = reinterpret_cast<u32x4_t *>(Vo);
    int idx = gid;
    for (; idx + (U - 1) * kGroups < n_copy; idx += U * kGroups) {
      int slotv[U];
      u32x4_t kc[U], vc[U];
#pragma unroll
      for (int u = 0; u < U; ++u) slotv[u] = copies[idx + u * kGroups];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int tok = lds_kept[slotv[u]];
        kc[u] = chunk_at<u32x4_t>(K, (unsigned)tok * kst + ch);
        vc[u] = chunk_at<u32x4_t>(V, (unsigned)tok * kst + ch);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        Koc[(long long)slotv[u] * LPR + ch] = kc[u];
        Voc[(long long)slotv[u] * LPR + ch] = vc[u];
      }
    }
    for (; idx < n_copy; idx += kGroups) {
      const int slot = copies[idx];
      const int tok = lds_kept[slot];
      const u32x4_t kc = chunk_at<u32x4_t>(K, (unsigned)tok * kst + ch);
      const u32x4_t vc = chunk_at<u32x4_t>(V, (unsigned)tok * kst + ch);
      Koc[(long long)slot * LPR + ch] = kc;
      Voc[(long long)slot * LPR + ch] = vc;
    }
  }
  __syncthreads();

  // Every group works on its own task, one batch of U rows per trip of the loop, and takes the
  // next free task when it is done (large chunks come first in the list), so neither a long
  // task nor an unlucky share holds anybody up.  Who computes a task does not change its sum.
  int q = gid;
  bool have = q < n_tasks;
  int4 task = have ? tasks[q] : make_int4(0, 0, 0, 0);
  int j0 = 0;
  float ak[EPC], av[EPC];
  float wsum = 0.f;  // weighted merge: sum of the weights added so far
#pragma unroll
  for (int e = 0; e < EPC; ++e) ak[e] = av[e] = 0.f;
  while (__any(have)) {
    if (have) {
      // rows of this task: the pivot itself first if the task finishes its slot, then the members
      const int lead = task.w < 0 ? 1 : 0;
      const int nrows = task.z + lead;
      const int *mem = members + task.y - lead;
      const int pivot_tok = lds_kept[task.x];
      // The U row loads of a trip are unconditional (a lane past the end of its task reads its last
      // row again, from the cache) and a row past the end adds zeros, so that no branch
      // separates the loads and all of them are in flight at once.
      int tokv[U];
      uint4 kc[U], vc[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = min(j0 + u, nrows - 1);  // a task has at least one member: nrows - 1 >= lead
        const int tok = mem[max(j, lead)];
        tokv[u] = j < lead ? pivot_tok : tok;
      }
      uint4 pkc;
      if constexpr (WEIGHTED) pkc = K[(long long)pivot_tok * sh.ks_tok + ch];  // the cosines need the pivot's key
#pragma unroll
      for (int u = 0; u < U; ++u) {
        kc[u] = chunk_at<uint4>(K, (unsigned)tokv[u] * kst + ch);
        vc[u] = chunk_at<uint4>(V, (unsigned)tokv[u] * kst + ch);
      }
      if constexpr (WEIGHTED) {
        float pk[EPC], fk[U][EPC], dot[U], ss[U];
        chunk_to_floats<kBF16>(pkc, pk);
        float pss = 0.f;
#pragma unroll
        for (int e = 0; e < EPC; ++e) pss = fmaf(pk[e], pk[e], pss);
#pragma unroll
        for (int u = 0; u < U; ++u) {
          chunk_to_floats<kBF16>(kc[u], fk[u]);
          dot[u] = ss[u] = 0.f;
#pragma unroll
          for (int e = 0; e < EPC; ++e) { dot[u] = fmaf(fk[u][e], pk[e], dot[u]); ss[u] = fmaf(fk[u][e], fk[u][e], ss[u]); }
        }
#pragma unroll
        for (int o = LPR / 2; o >= 1; o >>= 1) {  // over the lanes that share the row
          pss += __shfl_xor(pss, o, 64);
#pragma unroll
          for (int u = 0; u < U; ++u) { dot[u] += __shfl_xor(dot[u], o, 64); ss[u] += __shfl_xor(ss[u], o, 64); }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          float fv[EPC];
          chunk_to_floats<kBF16>(vc[u], fv);
          const int j = j0 + u;
          float w = ss[u] > 0.f && pss > 0.f ? fmaxf(dot[u] / (sqrtf(ss[u]) * sqrtf(pss)), 0.f) : 0.f;
          w = j < lead ? 1.f : (j < nrows ? w : 0.f);
          wsum += w;
#pragma unroll
          for (int e = 0; e < EPC; ++e) { ak[e] = fmaf(w, fk[u][e], ak[e]); av[e] = fmaf(w, fv[e], av[e]); }
        }
      } else {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          float fk[EPC], fv[EPC];
          chunk_to_floats<kBF16>(kc[u], fk);
          chunk_to_floats<kBF16>(vc[u], fv);
          const bool real = j0 + u < nrows;
#pragma unroll
          for (int e = 0; e < EPC; ++e) { ak[e] += real ? fk[e] : 0.f; av[e] += real ? fv[e] : 0.f; }
        }
      }
      j0 += U;
      if (j0 >= nrows) {  // task finished: write its result, move to the next one of this group
        if (lead) {
          const float w = WEIGHTED ? 1.0f / wsum : 1.0f / (float)(1 + task.z);  // uniform merge weight 1/(1+n)
#pragma unroll
          for (int e = 0; e < EPC; ++e) { ak[e] *= w; av[e] *= w; }
          Ko[(long long)task.x * LPR + ch] = floats_to_chunk<kBF16>(ak);
          Vo[(long long)task.x * LPR + ch] = floats_to_chunk<kBF16>(av);
        } else {
          float *pp = partials + (long long)task.w * 2 * D + ch * EPC;
#pragma unroll
          for (int e = 0; e < EPC; ++e) { pp[e] = ak[e]; pp[D + e] = av[e]; }
          if (WEIGHTED && ch == 0) partial_w[task.w] = wsum;
        }
        int nq = 0;
        if (ch == 0) nq = atomicAdd(&sh_next, 1);
        q = __shfl(nq, rg * LPR, 64);
        have = q < n_tasks;
        if (have) task = tasks[q];
        j0 = 0;
        wsum = 0.f;
#pragma unroll
        for (int e = 0; e < EPC; ++e) ak[e] = av[e] = 0.f;
      }
    }
  }
  __syncthreads();
  // slots cut into several tasks: pivot row plus the partials in task order
  for (int qm = wave; qm < n_multi; qm += kF3Waves) {
    const int4 e4 = multi[qm];
    const int pivot_tok = lds_kept[e4.x];
    float w = 1.0f / (float)(1 + e4.w);
    if constexpr (WEIGHTED) {
      float tot = 1.f;  // the pivot's own weight, then the partial sums in task order
      for (int pi = 0; pi < e4.z; ++pi) tot += partial_w[e4.y + pi];
      w = 1.0f / tot;
    }
    if (lane < 2 * LPR) {
      const int tensor = lane / LPR, cch = lane % LPR;
      const uint4 *src = tensor ? V : K;
      float acc[EPC];
      chunk_to_floats<kBF16>(src[(long long)pivot_tok * sh.ks_tok + cch], acc);
      for (int pi = 0; pi < e4.z; ++pi) {
        const float *pp = partials + (long long)(e4.y + pi) * 2 * D + tensor * D + cch * EPC;
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[e] += pp[e];
      }
#pragma unroll
      for (int e = 0; e < EPC; ++e) acc[e] *= w;
      (tensor ? Vo : Ko)[(long long)e4.x * LPR + cch] = floats_to_chunk<kBF16>(acc);
    }
  }
}

}  // namespace flowmm
