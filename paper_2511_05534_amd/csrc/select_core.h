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

}  // namespace flowmm
