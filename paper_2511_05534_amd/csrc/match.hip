// Step "match": every non-pivot key goes to the pivot with the largest cosine similarity
// among the pivots that are not highly sensitive (importance <= tau) and, in an intra-modal
// layer, share its modality (FlowMM, Sensitivity-Adaptive Token Matching: cosine equation and
// thresholded argmax; the intra/cross rule of Information Flow Guided Merging).
//
// The select kernel leaves, per (sequence, kv head, layer) and token class (one class in a
// cross-modal layer, text / image in an intra-modal one), the list of pivots that may receive
// tokens, their K rows packed with the row stride used here, and their 1/norm.
// A workgroup owns a tile of tokens of one class (32*KS per wave, held as MFMA B operands in
// registers straight from HBM) and walks over the class's pivot list in LDS tiles that arrive by
// direct global->LDS loads, double buffered.  The similarity matrix is never stored: each 32x32
// block of dot products is scaled by the pivot's 1/norm, shifted by the token's norm (so every
// candidate is a non-negative float whose bit pattern orders like its value) and folded into a
// running maximum whose low four mantissa bits carry the row inside the lane's share of the block.
// The token's own norm is a positive factor common to all its candidates and is left out.
// Candidates therefore compare at 2^-19 relative resolution; below that the earlier list entry
// wins inside a lane's 16 rows of a block and the earlier block wins.
#include "device_common.h"
#include "kernels.h"
#include "profile.h"
#include "select_core.h"

namespace flowmm {

namespace {

constexpr int kThreads = kMatchWaves * 64;

// sum of squares of a chunk added to s; bf16 pairs go through the two-element dot product instruction
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
template <bool BF16>
__device__ __forceinline__ float chunk_sumsq_acc(const uint4 &c, float s) {
  if constexpr (BF16) {
    const unsigned w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bf16x2_t v;
      __builtin_memcpy(&v, &w[j], 4);
      s = __builtin_amdgcn_fdot2_f32_bf16(v, v, s, false);
    }
    return s;
  } else {
    return s + chunk_sumsq<false>(c);
  }
}

template <bool BF16, int D>
__global__ __launch_bounds__(kThreads, 4) void match_kernel(Ctx c) {
  using CF = Cfg<BF16, D>;
  constexpr int NCH = CF::NCH, NF = CF::NF;
  constexpr int KS = match_subs(BF16);
  constexpr int TILE = kMatchWaves * 32 * KS;
  constexpr int ROWS = match_tile_rows(NCH);  // list rows per LDS tile
  constexpr int kMfmaPerBlock = KS * NF * (BF16 ? 1 : 4);
  extern __shared__ uint4 lds[];
  constexpr int RS = NCH + 1;  // row stride in chunks: the odd stride keeps 16 rows' fragments on distinct banks
  uint4 *lds_rows = lds;                                             // [2][ROWS][RS]
  float *lds_w = reinterpret_cast<float *>(lds + 2 * ROWS * RS);     // [2][ROWS]
  int *lds_tok = reinterpret_cast<int *>(lds_w + 2 * ROWS);          // [TILE] tokens to assign, or -1

  const Shape &sh = c.sh;
  const int *meta = c.meta;
  // Workgroups are handed to the eight XCDs in turn.  All token tiles of a (layer, kv head) go to
  // one XCD, so its pivot pack is fetched into one L2 only.
  const int units = sh.n_layers * sh.Hkv;
  const int xcd = blockIdx.x & 7, k = blockIdx.x >> 3;
  const int ul = k / sh.tiles_match, x = k - ul * sh.tiles_match;
  const int unit_i = ul * 8 + xcd;
  if (unit_i >= units) return;
  const int l = unit_i / sh.Hkv, gkv = unit_i - l * sh.Hkv;
  const long long unit = unit_i;
  const int *cu = meta + meta[MW_OFF_CU_MATCH];
  const int b = find_seq(cu, meta[MW_BATCH], x);
  int tile = x - cu[b];
  const SeqInfo s = load_seq(meta, b);
  const bool cross = c.mode[l * sh.batch + b] != 0;
  // The tiles walk over the select kernel's list of the tokens to be matched (no pivot among them).
  // Token class of this tile: everything in a cross-modal layer, else text tiles then image tiles.
  const int *ev_n = c.ev_n + (unit * sh.batch + b) * 2;
  int cls = 0, cbeg = 0, cn = ev_n[0];
  if (!cross) {
    const int t0 = (cn + TILE - 1) / TILE;
    if (tile >= t0) {
      tile -= t0; cls = 1; cbeg = cn; cn = ev_n[1];
    }
  }
  const int v0 = tile * TILE;
  if (v0 >= cn) return;

  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, n = lane & 31, half = lane >> 5;
  const uint4 *K = reinterpret_cast<const uint4 *>(c.K) + (long long)l * sh.ks_layer +
                   (long long)gkv * sh.ks_head + (long long)s.tok_off * sh.ks_tok;
  const int *ev = c.ev_list + unit * sh.T + s.tok_off + cbeg;
  int *assign = c.assign + unit * sh.T + s.tok_off;
  const int Bp = (s.B + 31) & ~31;
  const long long lbase = unit * 2 * sh.SBP + 2 * (meta + meta[MW_OFF_CU_BP])[b] + cls * Bp;
  const uint4 *pack = c.pack + lbase * RS;
  const float *pl_w = c.pl_w + lbase;
  const int npc = c.pl_n[(unit * sh.batch + b) * 2 + cls];  // list length, a multiple of 32
  const int ntiles = (npc + ROWS - 1) / ROWS;

  auto stage = [&](int t, int buf) {
    const int r0 = t * ROWS;
    const int rows = min(ROWS, npc - r0);
    const uint4 *src = pack + (long long)r0 * RS;
    uint4 *dst = lds_rows + buf * ROWS * RS;
    const int nchunks = rows * RS;  // the tile is a plain copy of that part of the pack
    for (int q0 = wave * 64; q0 < nchunks; q0 += kThreads)
      if (q0 + lane < nchunks) load_to_lds<16>(src, (unsigned)(q0 + lane) * 16u, dst + q0);
    if (wave * 64 + lane < rows)
      load_to_lds<4>(pl_w + r0, (unsigned)(wave * 64 + lane) * 4u, lds_w + buf * ROWS + wave * 64);
  };
  // this wave's tokens as B operands, and their norms
  const int wv0 = v0 + wave * 32 * KS;
  const bool active = wv0 < cn;
  uint4 kf[KS][NF];
  float shift[KS];
  // position of this lane's token of every group (the class's last one past the end)
  int tok[KS];
#pragma unroll
  for (int sub = 0; sub < KS; ++sub) tok[sub] = ev[min(wv0 + sub * 32 + n, cn - 1)];
  // Their rows come in whole through the LDS that the pivot tiles use afterwards (every wave has its own
  // share of it), one token group at a time; rows that do not lie within 4 GiB, and rows too wide for that
  // share, are fetched fragment by fragment.
  constexpr bool kStaged = kMatchWaves * 32 * NCH <= 2 * ROWS * RS;
  if (kStaged && sh.rows32) {
#pragma unroll
    for (int sub = 0; sub < KS; ++sub)
      fetch_rows_staged<BF16, D>(K, (unsigned)sh.ks_tok, tok[sub], lds_rows + wave * 32 * NCH, kf[sub]);
    __syncthreads();  // the pivot tiles may overwrite the other waves' shares now
  } else {
#pragma unroll
    for (int sub = 0; sub < KS; ++sub) {
      const uint4 *row = K + (long long)tok[sub] * sh.ks_tok + half;
#pragma unroll
      for (int f = 0; f < NF; ++f) kf[sub][f] = row[2 * f];
    }
  }
  if (ntiles > 0) stage(0, 0);
#pragma unroll
  for (int sub = 0; sub < KS; ++sub)
    if (half == 0)
      lds_tok[wave * 32 * KS + sub * 32 + n] = wv0 + sub * 32 + n < cn ? tok[sub] : -1;
#pragma unroll
  for (int sub = 0; sub < KS; ++sub) {
    float ss = 0.f;
#pragma unroll
    for (int f = 0; f < NF; ++f) ss = chunk_sumsq_acc<BF16>(kf[sub][f], ss);
    ss += __shfl_xor(ss, 32, 64);
    shift[sub] = sqrtf(ss) * 1.001f;  // >= |<token, pivot>| / |pivot| for every pivot
  }
  unsigned best[KS];
  int bblk[KS];
#pragma unroll
  for (int sub = 0; sub < KS; ++sub) { best[sub] = 0u; bblk[sub] = 0; }

  // A block is 32 list rows against this wave's tokens: every fragment read from LDS feeds KS matrix
  // instructions (one per token group), the next fragment is requested before the current one is used,
  // then the KS x 16 dot products of each lane are folded into the running maxima.  The two waves
  // that share a SIMD overlap one's matrix phase with the other's folding.
  constexpr int NBLK = ROWS / 32;   // blocks per LDS tile
  constexpr int kBlockBytes = 32 * RS * 16;
  // one fragment ahead: with four waves per SIMD the others cover the LDS latency, and the registers
  // a deeper queue takes had to be found in scratch memory
  constexpr int kAhead = 1;
  const int fa = (n * RS + half) * 16;  // byte offset of this lane's first fragment inside a block
  const char *lds_bytes = reinterpret_cast<const char *>(lds);
  for (int t = 0; t < ntiles; ++t) {
    __builtin_amdgcn_s_waitcnt(0);  // this wave's part of tile t has landed
    __syncthreads();                // ... and everybody else's; tile t-1 is no longer read
    if (t + 1 < ntiles) stage(t + 1, (t + 1) & 1);
    if (!active) continue;
    const char *rows = lds_bytes + (t & 1) * (ROWS * RS * 16) + fa;
    const char *wt = reinterpret_cast<const char *>(lds_w + (t & 1) * ROWS) + 16 * half;
    const int nblk = min(ROWS, npc - t * ROWS) >> 5;
    uint4 pf[kAhead];  // the next fragments, requested ahead of their use (also across blocks of the tile)
#pragma unroll
    for (int f = 0; f < kAhead; ++f) pf[f] = *reinterpret_cast<const uint4 *>(rows + 32 * f);
#pragma unroll
    for (int pb = 0; pb < NBLK; ++pb) {
      if (pb < nblk) {
        const char *brow = rows + pb * kBlockBytes;
        f32x16_t acc[KS];
#pragma unroll
        for (int sub = 0; sub < KS; ++sub)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[sub][i] = 0.f;
#pragma unroll
        for (int f = 0; f < NF; ++f) {
          const uint4 cur = pf[f % kAhead];
          if (f + kAhead < NF) pf[f % kAhead] = *reinterpret_cast<const uint4 *>(brow + 32 * (f + kAhead));
#pragma unroll
          for (int sub = 0; sub < KS; ++sub) mma_chunk<BF16>(acc[sub], cur, kf[sub][f]);  // [pivot][token]
        }
        if (pb + 1 < nblk) {
#pragma unroll
          for (int f = 0; f < kAhead; ++f)
            pf[f] = *reinterpret_cast<const uint4 *>(brow + kBlockBytes + 32 * f);
        }
        const int blk = t * NBLK + pb;
        unsigned m[KS];
#pragma unroll
        for (int sub = 0; sub < KS; ++sub) m[sub] = 0u;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          // 1/norm of rows 8g + 4 half + j of the block, j = 0..3 (the fence keeps the compiler from
          // fetching all four groups up front: registers are short)
          const float4 w4 = *reinterpret_cast<const float4 *>(wt + pb * 128 + 32 * g);
          const float wv[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
          for (int sub = 0; sub < KS; ++sub) {
#pragma unroll
            for (int j = 0; j < 4; j += 2) {
              const int i = 4 * g + j;
              const unsigned p0 = (__float_as_uint(fmaf(acc[sub][i], wv[j], shift[sub])) & ~15u) | (unsigned)(15 - i);
              const unsigned p1 = (__float_as_uint(fmaf(acc[sub][i + 1], wv[j + 1], shift[sub])) & ~15u) | (unsigned)(14 - i);
              m[sub] = max(max(m[sub], p0), p1);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int sub = 0; sub < KS; ++sub) {
          if (m[sub] > best[sub]) { best[sub] = m[sub]; bblk[sub] = blk; }
        }
      }
    }
  }

  // the two half-waves saw disjoint rows of the same tokens
  const int *pl_slot = c.pl_slot + lbase;
  int dropped = 0;
#pragma unroll
  for (int sub = 0; sub < KS; ++sub) {
    int e = bblk[sub] * 32 + acc_row(15 - (int)(best[sub] & 15u), half);
    const unsigned mine = best[sub] >> 4;
    const unsigned other = __shfl_xor(best[sub], 32, 64) >> 4;
    const int oe = __shfl_xor(e, 32, 64);
    if (other > mine || (other == mine && oe < e)) e = oe;
    const int tk = half == 0 ? lds_tok[wave * 32 * KS + sub * 32 + n] : -1;  // written by this very lane
    if (tk >= 0) {
      const int slot = npc > 0 ? pl_slot[e] : -1;
      assign[tk] = slot;
      dropped += slot < 0;
    }
  }
  dropped = wave_sum_int(dropped);
  if (lane == 0 && dropped) atomicAdd(&c.n_dropped[unit * sh.batch + b], dropped);
}

template <bool BF16, int D>
hipError_t launch_match_t(const Ctx &c) {
  constexpr int NCH = Cfg<BF16, D>::NCH;
  constexpr int ROWS = match_tile_rows(NCH);
  const Shape &sh = c.sh;
  const size_t lds = 2 * (size_t)ROWS * (NCH + 1) * 16 + 2 * ROWS * sizeof(float) +
                     (size_t)match_tile_tokens(BF16) * sizeof(int);
  hipError_t e = allow_full_lds<match_kernel<BF16, D>>();
  if (e != hipSuccess) return e;
  const int units = sh.n_layers * sh.Hkv;
  const long long grid = (long long)((units + 7) / 8) * 8 * sh.tiles_match;
  if (grid > 0x7fffffffLL) return hipErrorInvalidConfiguration;
  ProfScope ps(c.stream, KID_MATCH);
  match_kernel<BF16, D><<<dim3((unsigned)grid), kThreads, lds, c.stream>>>(c);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_match(const Ctx &c) {
  if (c.sh.bf16) return c.sh.d == 128 ? launch_match_t<true, 128>(c) : launch_match_t<true, 64>(c);
  return c.sh.d == 128 ? launch_match_t<false, 128>(c) : launch_match_t<false, 64>(c);
}

}  // namespace flowmm
