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
constexpr int kCsrAhead = 4;   // rounds of 64 tokens a walking wave loads ahead
// Words of LDS in front of the counting table for the pivot positions of the longest budget (a whole number
// of 16-byte chunks), or 0 when table and positions together would not fit: the positions then stay in memory.
__host__ __device__ constexpr int csr_kept_words(int max_budget, int nw_shift) {
  return ((size_t)max_budget << nw_shift) * 4 + (size_t)max_budget * 4 <= 144u * 1024u ? (max_budget + 3) & ~3 : 0;
}
constexpr int kSmallTask = 4;  // a slot with fewer members is merged by one row group (pivot + members = loads in flight)

// Exclusive scan over the workgroup of a 64-bit value that packs several small counters (their
// sums must not carry into each other); *total gets the sum over all threads.
__device__ __forceinline__ unsigned long long block_exclusive_scan_packed(unsigned long long v, unsigned long long *lds_wave,
                                                                      unsigned long long *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned long long inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const unsigned long long u = __shfl_up(inc, o, 64);
    if (lane >= o) inc += u;
  }
  __syncthreads();
  if (lane == 63) lds_wave[wave] = inc;
  __syncthreads();
  if (wave == 0) {
    const unsigned long long w = lane < kCsrWaves ? lds_wave[lane] : 0ull;
    unsigned long long winc = w;
#pragma unroll
    for (int o = 1; o < kCsrWaves; o <<= 1) {
      const unsigned long long u = __shfl_up(winc, o, 64);
      if (lane >= o) winc += u;
    }
    if (lane < kCsrWaves) lds_wave[lane] = winc - w;
    if (lane == kCsrWaves - 1) lds_wave[kCsrWaves] = winc;
  }
  __syncthreads();
  *total = lds_wave[kCsrWaves];
  return lds_wave[wave] + inc - v;
}

// How many lower lanes of the wave hold the same slot as this lane, and how many lanes do in all (only
// meaningful where member).  One ballot per slot bit; the lanes that agree with this one on the bit
// are ballot XNOR (bit ? ~0 : 0), taken on the two halves of the wave mask.
__device__ __forceinline__ void same_slot_rank(bool member, int slot, int nbits, int &below, int &total) {
  const unsigned long long mm = __ballot(member);
  unsigned lo = (unsigned)mm, hi = (unsigned)(mm >> 32);
  for (int bit = 0; bit < nbits; ++bit) {
    const unsigned e = 0u - ((unsigned)(slot >> bit) & 1u);  // all ones where the bit is set
    const unsigned long long bb = __ballot(member && e != 0u);
    lo &= ~((unsigned)bb ^ e);
    hi &= ~((unsigned)(bb >> 32) ^ e);
  }
  below = __builtin_amdgcn_mbcnt_hi(hi, __builtin_amdgcn_mbcnt_lo(lo, 0u));
  total = __popc(lo) + __popc(hi);
}

// at most 64 registers: two workgroups of 16 waves then share a compute unit
// members_off: where (in ints from the start of the dynamic LDS) the member list is put together before it
// goes to memory in whole lines, or -1 to write it directly (scattered 4-byte stores: every one of them
// costs a 32-byte memory transaction)
__global__ __launch_bounds__(kCsrThreads, 8) void merge_csr_kernel(Ctx c, int nw_shift, int members_off) {
  // [NW][B] per-wave counts, later write cursors; the slot runs fastest, so that the slots of a wave's 64
  // tokens and the 1024 slots of a scan step fall on different banks
  // in front of it the pivot positions of the sequence (the test "is this token its slot's pivot" then
  // needs no second trip to memory behind the token's assignment)
  extern __shared__ int lds_csr[];
  __shared__ unsigned long long lds_wave[kCsrWaves + 1];
  const Shape &sh = c.sh;
  const int *meta = c.meta;
  const int b = rotated_block_x(), gkv = blockIdx.y, l = blockIdx.z;
  const SeqInfo s = load_seq(meta, b);
  const long long unit = (long long)l * sh.Hkv + gkv;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int NW = 1 << nw_shift;  // waves that walk tokens (the table must fit in LDS)
  const int *assign = c.assign + unit * sh.T + s.tok_off;
  const int *kept = c.kept_idx + unit * sh.SB + s.kept_off;
  int *members = c.members + unit * sh.T + s.tok_off;
  int *seg_off = c.seg_off + unit * (sh.SB + sh.batch) + s.kept_off + b;
  const int task_base = (meta + meta[MW_OFF_CU_TASK])[b];
  const int task_room = (meta + meta[MW_OFF_CU_TASK])[b + 1] - task_base;
  const int multi_base = (meta + meta[MW_OFF_CU_MULTI])[b];
  const int part_base = (meta + meta[MW_OFF_CU_PART])[b];
  int4 *tasks = c.tasks + unit * sh.tasks_total + task_base;
  int4 *multi = c.multi + unit * sh.multi_total + multi_base;

  int nbits = 0;
  while ((1 << nbits) < s.B) ++nbits;
  const int range = ((s.L + NW - 1) / NW + 63) & ~63;  // tokens per walking wave
  const int r0 = wave * range, r1 = min(s.L, r0 + range);

  const int kept_words = csr_kept_words(sh.maxB, nw_shift);
  int *lds_tbl = lds_csr + kept_words;
  const int *kept_near = kept_words ? lds_csr : kept;  // where the walks below look the pivot of a slot up
  if (kept_words)
    for (int i = threadIdx.x; i < s.B; i += kCsrThreads) lds_csr[i] = kept[i];
  for (int i = threadIdx.x; i < s.B * NW; i += kCsrThreads) lds_tbl[i] = 0;
  __syncthreads();

  // pass 1: members of each slot inside each wave's token range (kCsrAhead rounds of 64 tokens have
  // their two dependent loads in flight together)
  if (wave < NW) {
    for (int i0 = r0; i0 < r1; i0 += 64 * kCsrAhead) {
      int slotv[kCsrAhead], keptv[kCsrAhead];
#pragma unroll
      for (int u = 0; u < kCsrAhead; ++u) {
        const int i = i0 + 64 * u + lane;
        slotv[u] = i < r1 ? assign[i] : -1;
      }
#pragma unroll
      for (int u = 0; u < kCsrAhead; ++u) keptv[u] = slotv[u] >= 0 ? kept_near[slotv[u]] : -1;
#pragma unroll
      for (int u = 0; u < kCsrAhead; ++u) {
        if (i0 + 64 * u >= r1) break;
        const int i = i0 + 64 * u + lane, slot = slotv[u];
        // counting needs no order: the few lanes of a round that share a slot take their turns in the LDS
        if (slot >= 0 && keptv[u] != i) atomicAdd(&lds_tbl[wave * s.B + slot], 1);
      }
    }
  }
  __syncthreads();

  // scan over slots: segment offsets, write cursors, task list
  // A slot with fewer than kSmallTask members is a small task (a row group of the task kernel does it
  // alone); the small tasks fill the sequence's range of the table from the front, the others from the back.
  int seg_carry = 0, small_carry = 0, task_carry = 0, multi_carry = 0, part_carry = 0;
  for (int s0 = 0; s0 < s.B; s0 += kCsrThreads) {
    const int slot = s0 + threadIdx.x;
    int n = 0;
    if (slot < s.B)
      for (int w = 0; w < NW; ++w) n += lds_tbl[w * s.B + slot];
    const int nt = slot < s.B ? max(1, (n + kTaskChunk - 1) / kTaskChunk) : 0;
    const int is_multi = nt > 1;
    const int is_small = slot < s.B && n < kSmallTask;
    // two scans of packed counters: (members, small tasks) and (other tasks, partials, split slots), 21 bits each
    constexpr unsigned long long kF = (1ull << 21) - 1;
    unsigned long long tot_a, tot_b;
    const unsigned long long ea = block_exclusive_scan_packed((unsigned long long)n | ((unsigned long long)is_small << 32), lds_wave, &tot_a);
    const unsigned long long eb = block_exclusive_scan_packed(
        (unsigned long long)(is_small ? 0 : nt) | ((unsigned long long)(is_multi ? nt : 0) << 21) | ((unsigned long long)is_multi << 42),
        lds_wave, &tot_b);
    const int seg = seg_carry + (int)(ea & 0xffffffffull), sb = small_carry + (int)(ea >> 32);
    const int tb = task_carry + (int)(eb & kF), pb = part_carry + (int)((eb >> 21) & kF), mb = multi_carry + (int)(eb >> 42);
    const int tot_n = (int)(tot_a & 0xffffffffull), tot_s = (int)(tot_a >> 32);
    const int tot_t = (int)(tot_b & kF), tot_p = (int)((tot_b >> 21) & kF), tot_m = (int)(tot_b >> 42);
    if (slot < s.B) {
      seg_off[slot] = seg;
      int base = seg;
      for (int w = 0; w < NW; ++w) {
        const int t = lds_tbl[w * s.B + slot];
        lds_tbl[w * s.B + slot] = base;
        base += t;
      }
      if (is_small) tasks[sb] = make_int4(slot, seg, n, -1);
      else
        for (int j = 0; j < nt; ++j)
          tasks[task_room - 1 - (tb + j)] = make_int4(slot, seg + j * kTaskChunk, min(kTaskChunk, n - j * kTaskChunk),
                                                      is_multi ? part_base + pb + j : -1);
      if (is_multi) multi[mb] = make_int4(slot, part_base + pb, nt, n);
    }
    seg_carry += tot_n;
    small_carry += tot_s;
    task_carry += tot_t;
    multi_carry += tot_m;
    part_carry += tot_p;
  }
  if (threadIdx.x == 0) {
    seg_off[s.B] = seg_carry;
    c.n_tasks[(unit * sh.batch + b) * 2] = small_carry;
    c.n_tasks[(unit * sh.batch + b) * 2 + 1] = task_carry;
    c.n_multi[unit * sh.batch + b] = multi_carry;
  }
  __syncthreads();

  // pass 2: write the members, ascending inside every slot
  int *members_dst = members_off >= 0 ? lds_csr + members_off : members;
  if (wave < NW) {
    for (int i0 = r0; i0 < r1; i0 += 64 * kCsrAhead) {
      int slotv[kCsrAhead], keptv[kCsrAhead];
#pragma unroll
      for (int u = 0; u < kCsrAhead; ++u) {
        const int i = i0 + 64 * u + lane;
        slotv[u] = i < r1 ? assign[i] : -1;
      }
#pragma unroll
      for (int u = 0; u < kCsrAhead; ++u) keptv[u] = slotv[u] >= 0 ? kept_near[slotv[u]] : -1;
#pragma unroll
      for (int u = 0; u < kCsrAhead; ++u) {
        if (i0 + 64 * u >= r1) break;
        const int i = i0 + 64 * u + lane, slot = slotv[u];
        const bool member = slot >= 0 && keptv[u] != i;
        int below, total;
        same_slot_rank(member, slot, nbits, below, total);
        if (member) {
          const int cur = lds_tbl[wave * s.B + slot];
          members_dst[cur + below] = i;
          if (below == 0) lds_tbl[wave * s.B + slot] = cur + total;
        }
      }
    }
  }
  if (members_off >= 0) {
    __syncthreads();
    for (int i = threadIdx.x; i < seg_carry; i += kCsrThreads) members[i] = members_dst[i];
  }
}

// WEIGHTED: the similarity-weighted mean (the pivot counts 1, a member max(u, 0), u the cosine of
// its key to the pivot's key, 0 for a zero row; V rows take the weights of their K rows).
template <bool BF16, int D, bool WEIGHTED>
__global__ __launch_bounds__(256) void merge_tasks_kernel(Ctx c) {
  using CF = Cfg<BF16, D>;
  constexpr int LPR = CF::NCH;        // lanes that cover one row
  constexpr int RPL = 64 / LPR;       // rows a wave covers per load = row groups of a wave
  constexpr int EPC = CF::kElemsPerChunk;
  constexpr int U = 4;                // loads in flight per lane and tensor
  const Shape &sh = c.sh;
  const int *meta = c.meta;
  const int *cu = meta + meta[MW_OFF_CU_TASK];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  // One wave per entry of the task table.  Most slots have a few members or none: RPL such small
  // tasks (whole slot, at most U - 1 members) are done side by side by the row groups of a wave,
  // so the waves at the front of a sequence's range take RPL of them each; the waves at the back of
  // the range stream one larger task each; those in between have nothing to do.
  static_assert(U == kSmallTask, "a small task is the pivot and fewer than U members");
  const int w = blockIdx.x * 4 + wave;
  if (w >= sh.tasks_total) return;
  const int gkv = blockIdx.y, l = blockIdx.z;
  const long long unit = (long long)l * sh.Hkv + gkv;
  const int b = find_seq(cu, meta[MW_BATCH], w);
  const int wl = w - cu[b], room = cu[b + 1] - cu[b];
  const int n_small = c.n_tasks[(unit * sh.batch + b) * 2], n_big = c.n_tasks[(unit * sh.batch + b) * 2 + 1];
  const bool small_wave = wl * RPL < n_small;
  if (!small_wave && wl < room - n_big) return;
  const SeqInfo s = load_seq(meta, b);
  const int rg = lane / LPR, ch = lane % LPR;
  const long long head_off = (long long)l * sh.ks_layer + (long long)gkv * sh.ks_head + (long long)s.tok_off * sh.ks_tok;
  const uint4 *K = reinterpret_cast<const uint4 *>(c.K) + head_off;
  const uint4 *V = reinterpret_cast<const uint4 *>(c.V) + head_off;
  const int *kept = c.kept_idx + unit * sh.SB + s.kept_off;
  const int *seq_members = c.members + unit * sh.T + s.tok_off;
  uint4 *K_out = reinterpret_cast<uint4 *>(c.K_out) + (unit * sh.SB + s.kept_off) * LPR;
  uint4 *V_out = reinterpret_cast<uint4 *>(c.V_out) + (unit * sh.SB + s.kept_off) * LPR;
  const int4 *seq_tasks = c.tasks + unit * sh.tasks_total + cu[b];

  // ---- small tasks: the pivot's row and up to U - 1 member rows, summed in that order by one row group
  if (small_wave) {
    if (wl * RPL + rg >= n_small) return;
    const int4 mine = seq_tasks[wl * RPL + rg];  // (slot, first member, count, -1)
    int tokv[U];
    tokv[0] = kept[mine.x];
#pragma unroll
    for (int u = 1; u < U; ++u) tokv[u] = u <= mine.z ? seq_members[mine.y + u - 1] : -1;
    uint4 kc[U], vc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (tokv[u] >= 0) {
        kc[u] = K[(long long)tokv[u] * sh.ks_tok + ch];
        vc[u] = V[(long long)tokv[u] * sh.ks_tok + ch];
      }
    }
    float ak[EPC], av[EPC];
    chunk_to_floats<BF16>(kc[0], ak);
    chunk_to_floats<BF16>(vc[0], av);
    float den = (float)(1 + mine.z);
    if constexpr (WEIGHTED) {
      float pk[EPC], pss = 0.f;
#pragma unroll
      for (int e = 0; e < EPC; ++e) { pk[e] = ak[e]; pss = fmaf(pk[e], pk[e], pss); }
#pragma unroll
      for (int o = LPR / 2; o >= 1; o >>= 1) pss += __shfl_xor(pss, o, 64);
      den = 1.f;
#pragma unroll
      for (int u = 1; u < U; ++u) {
        // lanes of other row groups may be elsewhere: the exchanges stay inside this row group
        float fk[EPC], fv[EPC];
        const bool real = tokv[u] >= 0;
        if (real) {
          chunk_to_floats<BF16>(kc[u], fk);
          chunk_to_floats<BF16>(vc[u], fv);
        } else {
#pragma unroll
          for (int e = 0; e < EPC; ++e) fk[e] = fv[e] = 0.f;
        }
        float dot = 0.f, ss = 0.f;
#pragma unroll
        for (int e = 0; e < EPC; ++e) { dot = fmaf(fk[e], pk[e], dot); ss = fmaf(fk[e], fk[e], ss); }
#pragma unroll
        for (int o = LPR / 2; o >= 1; o >>= 1) { dot += __shfl_xor(dot, o, 64); ss += __shfl_xor(ss, o, 64); }
        const float w = ss > 0.f && pss > 0.f ? fmaxf(dot / (sqrtf(ss) * sqrtf(pss)), 0.f) : 0.f;
        den += w;
#pragma unroll
        for (int e = 0; e < EPC; ++e) { ak[e] = fmaf(w, fk[e], ak[e]); av[e] = fmaf(w, fv[e], av[e]); }
      }
    } else {
#pragma unroll
      for (int u = 1; u < U; ++u) {
        if (tokv[u] >= 0) {
          float fk[EPC], fv[EPC];
          chunk_to_floats<BF16>(kc[u], fk);
          chunk_to_floats<BF16>(vc[u], fv);
#pragma unroll
          for (int e = 0; e < EPC; ++e) { ak[e] += fk[e]; av[e] += fv[e]; }
        }
      }
    }
#pragma unroll
    for (int e = 0; e < EPC; ++e) { ak[e] = ak[e] / den; av[e] = av[e] / den; }
    K_out[(long long)mine.x * LPR + ch] = floats_to_chunk<BF16>(ak);
    V_out[(long long)mine.x * LPR + ch] = floats_to_chunk<BF16>(av);
    return;
  }

  // ---- a larger task: all row groups of the wave stream its rows
  {
    const int4 task = seq_tasks[wl];  // (slot, first member, count, partial index or -1)
    const int *members = seq_members + task.y;
    float ak[EPC], av[EPC];
#pragma unroll
    for (int e = 0; e < EPC; ++e) ak[e] = av[e] = 0.f;
    const bool single = task.w < 0;
    const int pivot_tok = kept[task.x];
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
      K_out[(long long)task.x * LPR + ch] = floats_to_chunk<BF16>(ak);
      V_out[(long long)task.x * LPR + ch] = floats_to_chunk<BF16>(av);
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
}

// kFoldGroups workgroups per (sequence, kv head, layer) walk over its split slots, one wave per slot
template <bool BF16, int D, bool WEIGHTED>
__global__ __launch_bounds__(256) void merge_fold_kernel(Ctx c) {
  constexpr int EPC = Cfg<BF16, D>::kElemsPerChunk;
  constexpr int NCH = Cfg<BF16, D>::NCH;
  const Shape &sh = c.sh;
  const int *meta = c.meta;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bx = rotated_block_x();
  const int b = bx / kFoldGroups;
  const int gkv = blockIdx.y, l = blockIdx.z;
  const long long unit = (long long)l * sh.Hkv + gkv;
  const int n_multi = c.n_multi[unit * sh.batch + b];
  const int q0 = (meta + meta[MW_OFF_CU_MULTI])[b];
  for (int qm = (bx % kFoldGroups) * 4 + wave; qm < n_multi; qm += kFoldGroups * 4) {
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
    // 2 NCH lanes cover the K and V chunks of the row; the wave's kParts such lane groups share the
    // slot's partials (consecutive ranges, in task order inside each; group 0 starts from the pivot's
    // row) and their sums are added in a fixed tree: the longest chain is 1/kParts of the slot's
    constexpr int kParts = 64 / (2 * NCH);
    {
      const int part_id = lane / (2 * NCH), idx = lane % (2 * NCH);
      const int tensor = idx / NCH, ch = idx % NCH;
      const uint4 *src = reinterpret_cast<const uint4 *>(tensor ? c.V : c.K) + head_off;
      float acc[EPC];
      if (part_id == 0) {
        chunk_to_floats<BF16>(src[ch], acc);
      } else {
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[e] = 0.f;
      }
      const int per = (e4.z + kParts - 1) / kParts;
      const int pbeg = part_id * per, pend = min(e4.z, pbeg + per);
      constexpr int U = 8;  // partials in flight; they are added in task order all the same
      for (int p0 = pbeg; p0 < pend; p0 += U) {
        float part[U][EPC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          if (p0 + u < pend) {
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
          if (p0 + u < pend) {
#pragma unroll
            for (int e = 0; e < EPC; ++e) acc[e] += part[u][e];
          }
        }
      }
#pragma unroll
      for (int o = 2 * NCH; o < 64; o <<= 1)
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[e] += __shfl_xor(acc[e], o, 64);
      if (part_id == 0) {
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[e] = acc[e] / den;
        const long long orow = (unit * sh.SB + s.kept_off + e4.x) * NCH + ch;
        reinterpret_cast<uint4 *>(tensor ? c.V_out : c.K_out)[orow] = floats_to_chunk<BF16>(acc);
      }
    }
  }
}

template <bool BF16, int D, bool WEIGHTED>
hipError_t launch_merge_w(const Ctx &c, int nw_shift, size_t lds) {
  const Shape &sh = c.sh;
  hipError_t e = allow_full_lds<merge_csr_kernel>();
  if (e != hipSuccess) return e;
  {
    ProfScope ps(c.stream, KID_MERGE_CSR);
    // the member list is put together in LDS when that leaves the compute units as many workgroups as before:
    // two each, or one each when there are no more workgroups than compute units
    const size_t with_members = lds + (size_t)sh.maxE * 4;
    const long long wgs = (long long)sh.batch * sh.Hkv * sh.n_layers;
    // (short lists are not worth the extra pass over them: 19 against 23 us at 3700 members per list)
    const bool stage = sh.maxE >= 8192 &&
                       (with_members <= kLdsBytes / 2 - 1024 || (wgs <= 256 && with_members <= kLdsBytes - 8 * 1024));
    merge_csr_kernel<<<dim3(sh.batch, sh.Hkv, sh.n_layers), kCsrThreads, stage ? with_members : lds, c.stream>>>(
        c, nw_shift, stage ? (int)(lds / 4) : -1);
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
  const int shift = merge_csr_wave_shift(max_budget);
  return (((size_t)max_budget << shift) + csr_kept_words(max_budget, shift)) * 4;
}

hipError_t launch_merge(const Ctx &c) {
  const int shift = merge_csr_wave_shift(c.sh.maxB);
  const size_t lds = merge_csr_lds_bytes(c.sh.maxB);
  if (c.sh.bf16)
    return c.sh.d == 128 ? launch_merge_t<true, 128>(c, shift, lds) : launch_merge_t<true, 64>(c, shift, lds);
  return c.sh.d == 128 ? launch_merge_t<false, 128>(c, shift, lds) : launch_merge_t<false, 64>(c, shift, lds);
}

}  // namespace flowmm
