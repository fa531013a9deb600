// Pieces shared by the kernels that contract query rows staged in LDS with keys held in registers
// (score.hip: the proxy window; flow_exact.hip: every token of the prompt as a query).
#pragma once
#include "device_common.h"

namespace flowmm {

// lane i of the wave fetches 16 bytes from base + byte_off (base wave-uniform, in scalar registers;
// the lane's part is a 32-bit offset, so no lane keeps a 64-bit address); they land at
// lds_base + 16 i (lds_base wave-uniform).  Lanes that are switched off leave their 16 bytes alone.
// Inline assembly, so the compiler does not wait for it before unrelated LDS traffic (nothing else
// here uses M0); the caller waits with s_waitcnt vmcnt(0) and a barrier.
typedef __attribute__((address_space(3))) void lds_void;
__device__ __forceinline__ void load16_to_lds(const void *base, unsigned byte_off, void *lds_base) {
  const unsigned lds_addr = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_void *)lds_base);
  // the base goes through the first lane's copy of it: free when it already sits in scalar registers,
  // and it keeps the operand a scalar pair when the compiler has lost track of its uniformity
  const unsigned long long bits = (unsigned long long)(uintptr_t)base;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)bits), hi = __builtin_amdgcn_readfirstlane((unsigned)(bits >> 32));
  base = reinterpret_cast<const void *>((uintptr_t)(((unsigned long long)hi << 32) | lo));
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(byte_off), "s"(base), "s"(lds_addr) : "memory");
}

// The products of one block of 32 query rows with this wave's keys.  KEYS_AS_ROWS: accumulator
// rows are keys and lane n owns query row n (pass 1); otherwise rows are query rows and lane n owns
// key n of every group (pass 3).  Fragments are requested kAhead steps ahead, also across blocks.
template <bool BF16, int D, int KS, bool KEYS_AS_ROWS, int AHEAD>
__device__ __forceinline__ void block_products(f32x16_t (&acc)[KS], const uint4 (&kf)[KS][Cfg<BF16, D>::NF],
                                               uint4 (&pf)[AHEAD], const char *qrow, bool more) {
  constexpr int NF = Cfg<BF16, D>::NF, RS = Cfg<BF16, D>::NCH + 1;
#pragma unroll
  for (int sub = 0; sub < KS; ++sub)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[sub][i] = 0.f;
#pragma unroll
  for (int f = 0; f < NF; ++f) {
    const uint4 cur = pf[f % AHEAD];
    if (f + AHEAD < NF) pf[f % AHEAD] = *reinterpret_cast<const uint4 *>(qrow + 32 * (f + AHEAD));
#pragma unroll
    for (int sub = 0; sub < KS; ++sub) {
      if constexpr (KEYS_AS_ROWS) mma_chunk<BF16>(acc[sub], kf[sub][f], cur);
      else mma_chunk<BF16>(acc[sub], cur, kf[sub][f]);
    }
  }
  if (more) {
#pragma unroll
    for (int f = 0; f < AHEAD; ++f) pf[f] = *reinterpret_cast<const uint4 *>(qrow + 32 * RS * 16 + 32 * f);
  }
}

}  // namespace flowmm
