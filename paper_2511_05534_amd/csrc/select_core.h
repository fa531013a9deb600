// Top-B split of one unit, shared by the stand-alone select kernel and the unit-resident path.
// The B-th largest key is found by a 4-pass radix select over the float bit patterns (keys are
// non-negative floats, so unsigned order = value order); an ordered block scan compacts the
// pivots.  The last W tokens (the proxies) are pivots regardless of their key.
#pragma once
#include "device_common.h"

namespace flowmm {

template <int THREADS>
struct SelectScratch {
  int hist[256];
  int wave_sums[THREADS / 64 + 1];
  unsigned prefix;
  int remaining;
};

// exclusive prefix sum over the workgroup, in thread order; *total receives the block sum.
// T is int or long long (several small counters packed into one word scan together).
template <int THREADS, typename T>
__device__ __forceinline__ T block_exclusive_scan(T v, T *lds_wave /*[THREADS/64+1]*/, T *total) {
  constexpr int kWaves = THREADS / 64;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  T inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const T u = __shfl_up(inc, o, 64);
    if (lane >= o) inc += u;
  }
  __syncthreads();  // lds_wave may still be read from a previous call
  if (lane == 63) lds_wave[wave] = inc;
  __syncthreads();
  if (wave == 0) {
    const T w = lane < kWaves ? lds_wave[lane] : (T)0;
    T winc = w;
#pragma unroll
    for (int o = 1; o < kWaves; o <<= 1) {
      const T u = __shfl_up(winc, o, 64);
      if (lane >= o) winc += u;
    }
    if (lane < kWaves) lds_wave[lane] = winc - w;
    if (lane == kWaves - 1) lds_wave[kWaves] = winc;
  }
  __syncthreads();
  *total = lds_wave[kWaves];
  return lds_wave[wave] + inc - v;
}

// keys: L float bit patterns (LDS or global).  Writes kept[0..B) ascending and assign[0..L)
// (pivot: its slot; others: -2 = still to be matched).  All THREADS threads must call.
template <int THREADS>
__device__ __forceinline__ void compact_top_b(const unsigned *keys, int L, int W, unsigned thr, int need_eq,
                                              int *kept, int *assign, SelectScratch<THREADS> &sc);

template <int THREADS>
__device__ __forceinline__ void select_top_b(const unsigned *keys, int L, int W, int B, int *kept,
                                             int *assign, SelectScratch<THREADS> &sc) {
  static_assert(THREADS >= 256 && THREADS % 64 == 0, "the digit scan uses one thread per bin");
  const int lane = threadIdx.x & 63;
  const int nbody = L - W;
  const int need = B - W;      // pivots still to choose among the non-proxy tokens
  unsigned thr = 0xffffffffu;  // nothing in the body exceeds or equals this
  int need_eq = 0;
  if (need > 0) {
    unsigned prefix = 0, mask = 0;
    int remaining = need;
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      if (threadIdx.x < 256) sc.hist[threadIdx.x] = 0;
      __syncthreads();
      for (int i0 = 0; i0 < nbody; i0 += THREADS) {
        const int i = i0 + threadIdx.x;
        const unsigned k = i < nbody ? keys[i] : 0u;
        const bool act = i < nbody && (k & mask) == prefix;
        const int dg = (k >> shift) & 255;
        const unsigned long long am = __ballot(act);
        if (am) {
          // a whole wave on one digit is the common case for the exponent byte: one add instead of 64
          const int first = __ffsll((long long)am) - 1;
          const int d0 = __shfl(dg, first, 64);
          if (__ballot(act && dg == d0) == am) {
            if (lane == first) atomicAdd(&sc.hist[d0], __popcll(am));
          } else if (act) {
            atomicAdd(&sc.hist[dg], 1);
          }
        }
      }
      __syncthreads();
      // bins in descending order: thread t looks at bin 255 - t
      const int cnt = threadIdx.x < 256 ? sc.hist[255 - threadIdx.x] : 0;
      int total;
      const int before = block_exclusive_scan<THREADS, int>(cnt, sc.wave_sums, &total);
      if (threadIdx.x < 256 && before < remaining && remaining <= before + cnt) {
        sc.prefix = prefix | ((unsigned)(255 - threadIdx.x) << shift);
        sc.remaining = remaining - before;
      }
      __syncthreads();
      prefix = sc.prefix;
      remaining = sc.remaining;
      mask |= 255u << shift;
    }
    thr = prefix;
    need_eq = remaining;  // how many tokens equal to the threshold are still pivots
  }
  compact_top_b<THREADS>(keys, L, W, thr, need_eq, kept, assign, sc);
}

// Ordered compaction given the threshold: tokens above it and the first need_eq tokens equal to it
// are pivots, and so are the last W tokens.
template <int THREADS>
__device__ __forceinline__ void compact_top_b(const unsigned *keys, int L, int W, unsigned thr, int need_eq,
                                              int *kept, int *assign, SelectScratch<THREADS> &sc) {
  const int nbody = L - W;
  int gt_carry = 0, eq_carry = 0;
  for (int i0 = 0; i0 < L; i0 += THREADS) {
    const int i = i0 + threadIdx.x;
    int gt = 0, eq = 0;
    if (i < L) {
      if (i >= nbody) {
        gt = 1;
      } else {
        const unsigned k = keys[i];
        gt = k > thr;
        eq = k == thr;
      }
    }
    int total;
    const int before = block_exclusive_scan<THREADS, int>(gt | (eq << 16), sc.wave_sums, &total);
    const int gt_before = gt_carry + (before & 0xffff);
    const int eq_before = eq_carry + (before >> 16);
    if (i < L) {
      const bool is_kept = gt || (eq && eq_before < need_eq);
      const int slot = gt_before + min(eq_before, need_eq);
      if (is_kept) kept[slot] = i;
      assign[i] = is_kept ? slot : -2;
    }
    gt_carry += total & 0xffff;
    eq_carry += total >> 16;
  }
}

// ---- wave64 reductions on the data-parallel-primitive path (no LDS traffic) ---------------------
// dpp_ctrl: row_shr:n = 0x110 + n (shift right inside each row of 16 lanes), row_bcast:15 = 0x142
// (lane 15 of every row to the next row), row_bcast:31 = 0x143 (lane 31 to the upper half).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float old, float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_move(int old, int v) {
  return __builtin_amdgcn_update_dpp(old, v, CTRL, ROW_MASK, 0xf, false);
}

// maximum over each half-wave (lanes 0..31, 32..63); valid in lanes 31 and 63
__device__ __forceinline__ float half_wave_max_hi(float v) {
  v = fmaxf(v, dpp_move<0x111, 0xf>(v, v));
  v = fmaxf(v, dpp_move<0x112, 0xf>(v, v));
  v = fmaxf(v, dpp_move<0x114, 0xf>(v, v));
  v = fmaxf(v, dpp_move<0x118, 0xf>(v, v));
  v = fmaxf(v, dpp_move<0x142, 0xa>(v, v));
  return v;
}

// sum over each half-wave; valid in lanes 31 and 63
__device__ __forceinline__ float half_wave_sum_hi(float v) {
  v += dpp_move<0x111, 0xf>(0.f, v);
  v += dpp_move<0x112, 0xf>(0.f, v);
  v += dpp_move<0x114, 0xf>(0.f, v);
  v += dpp_move<0x118, 0xf>(0.f, v);
  v += dpp_move<0x142, 0xa>(0.f, v);
  return v;
}

// sum over the wave; valid in lane 63
__device__ __forceinline__ int wave_sum_hi(int v) {
  v += dpp_move<0x111, 0xf>(0, v);
  v += dpp_move<0x112, 0xf>(0, v);
  v += dpp_move<0x114, 0xf>(0, v);
  v += dpp_move<0x118, 0xf>(0, v);
  v += dpp_move<0x142, 0xa>(0, v);
  v += dpp_move<0x143, 0xc>(0, v);
  return v;
}

// inclusive prefix sum over the wave in lane order
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  v += dpp_move<0x111, 0xf>(0, v);
  v += dpp_move<0x112, 0xf>(0, v);
  v += dpp_move<0x114, 0xf>(0, v);
  v += dpp_move<0x118, 0xf>(0, v);
  v += dpp_move<0x142, 0xa>(0, v);
  v += dpp_move<0x143, 0xc>(0, v);
  return v;
}

template <int THREADS>
struct SmallSelectScratch {
  int hist[4][256];  // one histogram per radix pass, cleared once
  int wave_sums[THREADS / 64 + 1];
};

// Top-B split for L <= KPT * THREADS with few barriers: every thread keeps its KPT consecutive
// keys in registers, each radix pass costs one barrier (the 256-bin scan is repeated by every
// wave on its own instead of being shared), and the compaction is one block scan.
// keys: the thread's keys KPT t .. KPT t + KPT - 1 (anything where the index is >= L).  kept and
// assign may be LDS or global.  Same results as select_top_b.
// VEC_ASSIGN: assign + KPT t is 16-byte aligned for every thread t; a thread's assignments then go out
// as 16-byte chunks (consecutive words of LDS written one by one from 64 lanes KPT words apart meet
// in a few banks).
template <int THREADS, int KPT, bool VEC_ASSIGN = false>
__device__ __forceinline__ void select_top_b_regs(const unsigned (&keys)[KPT], int L, int W, int B, int *kept,
                                                  int *assign, SmallSelectScratch<THREADS> &sc) {
  static_assert(KPT * THREADS <= 65535, "the packed scan keeps two 16-bit counts");
  const int lane = threadIdx.x & 63;
  const int nbody = L - W;
  const int need = B - W;
  const int i0 = threadIdx.x * KPT;
  unsigned thr = 0xffffffffu;
  int need_eq = 0;
  for (int i = threadIdx.x; i < 4 * 256; i += THREADS) (&sc.hist[0][0])[i] = 0;
  __syncthreads();
  if (need > 0) {
    unsigned prefix = 0, mask = 0;
    int remaining = need;
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      int *hist = sc.hist[pass];
#pragma unroll
      for (int j = 0; j < KPT; ++j) {
        bool act = i0 + j < nbody && (keys[j] & mask) == prefix;
        const int dg = (keys[j] >> shift) & 255;
        unsigned long long am = __ballot(act);
        if (KPT > 4 && pass == 0) {
          // The exponent byte: a few digits per wave, and all waves add to the same few bins, where
          // additions take their turns.  Lanes with the same digit add once, through their first lane;
          // after four distinct digits the lanes that are left add by themselves.
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            if (!am) break;
            const int first = __ffsll((long long)am) - 1;
            const int d0 = __builtin_amdgcn_readlane(dg, first);
            const unsigned long long same = __ballot(act && dg == d0);
            if (lane == first) atomicAdd(&hist[d0], __popcll(same));
            act = act && dg != d0;
            am &= ~same;
          }
          if (act) atomicAdd(&hist[dg], 1);
        } else if (am) {  // a whole wave on one digit is the common case for the exponent byte
          const int first = __ffsll((long long)am) - 1;
          const int d0 = __builtin_amdgcn_readlane(dg, first);
          if (__ballot(act && dg == d0) == am) {
            if (lane == first) atomicAdd(&hist[d0], __popcll(am));
          } else if (act) {
            atomicAdd(&hist[dg], 1);
          }
        }
      }
      __syncthreads();
      // every wave scans the bins in descending order by itself: lane j owns bins 255-4j .. 252-4j
      int c4[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) c4[j] = hist[255 - 4 * lane - j];
      const int mine = c4[0] + c4[1] + c4[2] + c4[3];
      int before = wave_inclusive_scan(mine) - mine;  // keys in higher bins
      int digit = -1, rem_new = 0, in_bin = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (digit < 0 && before < remaining && remaining <= before + c4[j]) {
          digit = 255 - 4 * lane - j;
          rem_new = remaining - before;
          in_bin = c4[j];
        }
        before += c4[j];
      }
      const unsigned long long found = __ballot(digit >= 0);
      const int src = __ffsll((long long)found) - 1;
      digit = __builtin_amdgcn_readlane(digit, src);
      remaining = __builtin_amdgcn_readlane(rem_new, src);
      in_bin = __builtin_amdgcn_readlane(in_bin, src);
      prefix |= (unsigned)digit << shift;
      mask |= 255u << shift;
      // Every key of the bin is wanted: the digits below need not be looked at.  The prefix with zeros
      // under it then serves as the threshold (the keys of the bin are above it or equal to it, and as
      // many equal ones are wanted as the bin holds).  With float keys this ends most searches after
      // the second or third pass: the bin of the B-th largest key rarely holds another key by then.
      if (in_bin == remaining) break;
    }
    thr = prefix;
    need_eq = remaining;
  }
  // ordered compaction: one block scan over (above, equal) counts of the threads' keys
  int gtn = 0, eqn = 0;
  unsigned gtm = 0, eqm = 0;  // bit j: key j is above / equal to the threshold
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    const int i = i0 + j;
    const bool gt = i < L && (i >= nbody || keys[j] > thr);
    const bool eq = i < nbody && keys[j] == thr;
    gtm |= (unsigned)gt << j;
    eqm |= (unsigned)eq << j;
    gtn += gt;
    eqn += eq;
  }
  // block-wide exclusive scan of the packed counts: a wave scan on the DPP path, then the totals of
  // the earlier waves (one barrier)
  const int packed = gtn | (eqn << 16);
  const int inc = wave_inclusive_scan(packed);
  if (lane == 63) sc.wave_sums[threadIdx.x >> 6] = inc;
  __syncthreads();
  int before = inc - packed;
  for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) before += sc.wave_sums[w];
  int gt_before = before & 0xffff, eq_before = before >> 16;
  int mine[KPT];
#pragma unroll
  for (int j = 0; j < KPT; ++j) {
    const int i = i0 + j;
    const bool gt = (gtm >> j) & 1u, eq = (eqm >> j) & 1u;
    mine[j] = -2;
    if (i < L) {
      const bool is_kept = gt || (eq && eq_before < need_eq);
      const int slot = gt_before + min(eq_before, need_eq);
      if (is_kept) kept[slot] = i;
      mine[j] = is_kept ? slot : -2;
      if (!VEC_ASSIGN) assign[i] = mine[j];
    }
    gt_before += gt;
    eq_before += eq;
  }
  if constexpr (VEC_ASSIGN) {
    static_assert(KPT % 4 == 0, "whole 16-byte chunks");
#pragma unroll
    for (int q = 0; q < KPT / 4; ++q) {
      const int i = i0 + 4 * q;
      if (i + 3 < L) {
        *reinterpret_cast<int4 *>(assign + i) = make_int4(mine[4 * q], mine[4 * q + 1], mine[4 * q + 2], mine[4 * q + 3]);
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (i + j < L) assign[i + j] = mine[4 * q + j];
      }
    }
  }
}

template <int THREADS>
__device__ __forceinline__ void select_top_b_small(const unsigned (&keys4)[4], int L, int W, int B, int *kept,
                                                   int *assign, SmallSelectScratch<THREADS> &sc) {
  select_top_b_regs<THREADS, 4>(keys4, L, W, B, kept, assign, sc);
}

// The need-th largest of keys[0..nbody) (nbody <= 1024), found by ONE wave that holds 16 keys
// per lane and fixes the threshold bit by bit from the top; no barrier inside.  Returns the
// threshold and how many keys equal to it are still needed (wave-uniform).
__device__ __forceinline__ void wave_select_threshold(const unsigned *keys, int nbody, int need, unsigned *thr_out,
                                                      int *need_eq_out) {
  const int lane = threadIdx.x & 63;
  unsigned k[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int i = lane * 16 + j;
    k[j] = i < nbody ? keys[i] : 0u;  // padding keys are 0 and are masked by the index test below
  }
  const int mine = min(max(nbody - lane * 16, 0), 16);  // valid keys of this lane
  unsigned thr = 0;
  for (int bit = 30; bit >= 0; --bit) {  // keys are non-negative floats: bit 31 is clear
    const unsigned cand = thr | (1u << bit);
    int cnt = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) cnt += (j < mine && k[j] >= cand) ? 1 : 0;
    const int total = __builtin_amdgcn_readlane(wave_sum_hi(cnt), 63);
    if (total >= need) thr = cand;
  }
  int gt = 0;
#pragma unroll
  for (int j = 0; j < 16; ++j) gt += (j < mine && k[j] > thr) ? 1 : 0;
  *thr_out = thr;
  *need_eq_out = need - __builtin_amdgcn_readlane(wave_sum_hi(gt), 63);
}

}  // namespace flowmm
