// Pieces shared by the kernels that contract query rows staged in LDS with keys held in registers
// (score.hip: the proxy window; flow_exact.hip: every token of the prompt as a query).
#pragma once
#include "device_common.h"

namespace flowmm {

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
