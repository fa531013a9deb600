// Steps "flow" and "select", and the lists the match step works from.
//   flow  : rho = mean over query heads of the share of proxy attention that lands on tokens
//           of the other modality; the layer merges across modalities iff rho > theta
//           (FlowMM, Information Flow Guided Merging: rho equation and threshold rule).
//   select: the B most important tokens of each KV head form the pivot set, the rest are
//           merged into it (same section, top-B rule).  The proxy tokens themselves are always
//           pivots.  Ties go to the lower position, pivots are listed in ascending position.
//   lists : the pivots that may receive tokens (importance <= tau: Sensitivity-Adaptive Token
//           Matching), per token class (one class in a cross-modal layer, text / image in an
//           intra-modal one), in ascending slot order, padded to a multiple of 32 with copies of
//           the first entry; their K rows packed next to each other with the row stride of the
//           match kernel's LDS tiles (one 16-byte chunk of padding per row), and their 1/norm.
//           Ineligible pivots are in no list, so the match contraction never meets them.
// One workgroup per (sequence, kv head, layer).  The B-th largest importance is found by a
// 4-pass radix select on the float bit patterns (importances are non-negative, so the bits
// order like the values); a block-wide ordered scan then compacts the pivots.
#include <type_traits>

#include "device_common.h"
#include "kernels.h"
#include "profile.h"
#include "select_core.h"

namespace flowmm {

namespace {

constexpr int kThreads = 1024;
constexpr int kSelectRegisterKeys = 16 * kThreads;  // longest sequence whose keys stay in registers

template <bool BF16, int D>
// eight waves per SIMD (at most 64 vector and 96 scalar registers): two workgroups share a compute unit
__global__ __launch_bounds__(kThreads, 8) void select_kernel(Ctx c) {
  constexpr int NCH = Cfg<BF16, D>::NCH;
  __shared__ SelectScratch<kThreads> scratch;
  __shared__ SmallSelectScratch<kThreads> scratch_regs;
  extern __shared__ __align__(16) unsigned lds_keys[];  // [min(maxL, kSelectRegisterKeys)] keys, then assignments
  __shared__ float lds_head[kThreads];
  __shared__ float sh_rho;
  const Shape &sh = c.sh;
  const int *meta = c.meta;
  const int b = rotated_block_x(), gkv = blockIdx.y, l = blockIdx.z;
  const SeqInfo s = load_seq(meta, b);
  const long long unit = (long long)l * sh.Hkv + gkv;

  // ---- flow: every workgroup of the layer folds the same numbers in the same order -------------
  {
    const int *cu = meta + meta[MW_OFF_CU_SCORE];
    const int x0 = cu[b], x1 = cu[b + 1];
    float rho = 0.f;
    for (int h0 = 0; h0 < sh.Hq; h0 += kThreads) {
      const int h = h0 + threadIdx.x;
      if (h < sh.Hq) {
        const float *cp = c.cross_part + (long long)(l * sh.Hq + h) * sh.tiles_score;
        float v = 0.f;
        for (int x = x0; x < x1; ++x) v += cp[x];
        lds_head[threadIdx.x] = v / (float)sh.W;  // share of this head's proxy attention
      }
      __syncthreads();
      if (threadIdx.x == 0) {
        const int nh = min(kThreads, sh.Hq - h0);
        for (int i = 0; i < nh; ++i) rho += lds_head[i];
      }
      __syncthreads();
    }
    if (threadIdx.x == 0) {
      rho /= (float)sh.Hq;
      sh_rho = rho;
      if (gkv == 0) {
        c.rho[l * sh.batch + b] = rho;
        c.mode[l * sh.batch + b] = (rho > sh.theta) != (sh.invert_flow != 0) ? 1 : 0;
      }
      c.n_dropped[unit * sh.batch + b] = 0;
    }
  }
  // ---- top-B split -----------------------------------------------------------------------------
  const unsigned *imp = reinterpret_cast<const unsigned *>(c.importance) + unit * sh.T + s.tok_off;
  int *kept = c.kept_idx + unit * sh.SB + s.kept_off;
  int *assign = c.assign + unit * sh.T + s.tok_off;
  // Up to 16 keys per thread stay in registers for the four radix passes and the compaction (one
  // trip to memory instead of five); longer sequences read their keys again in every pass.  A
  // thread owns consecutive keys (the compaction is then one block scan), which is no shape to talk
  // to memory in: keys come in and assignments go out through LDS, in coalesced rows.
  auto from_registers = [&](auto kpt_tag) {
    constexpr int KPT = decltype(kpt_tag)::value;
    unsigned keys[KPT];
    const int i0 = threadIdx.x * KPT;
    if ((reinterpret_cast<uintptr_t>(imp) & 15) == 0) {
      // the thread's keys are KPT / 4 chunks of 16 bytes: all of them requested at once, no detour
#pragma unroll
      for (int q = 0; q < KPT / 4; ++q) {
        const int i = i0 + 4 * q;
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (i + 3 < s.L) {
          v = *reinterpret_cast<const uint4 *>(imp + i);
        } else {
          if (i < s.L) v.x = imp[i];
          if (i + 1 < s.L) v.y = imp[i + 1];
          if (i + 2 < s.L) v.z = imp[i + 2];
        }
        keys[4 * q] = v.x; keys[4 * q + 1] = v.y; keys[4 * q + 2] = v.z; keys[4 * q + 3] = v.w;
      }
    } else {
      // a sequence that does not start on a 16-byte boundary: coalesced rows through LDS, KPT requests in flight
      for (int base = 0; base < s.L; base += KPT * kThreads) {
        unsigned v[KPT];
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
          const int i = base + j * kThreads + threadIdx.x;
          v[j] = i < s.L ? imp[i] : 0u;
        }
#pragma unroll
        for (int j = 0; j < KPT; ++j) {
          const int i = base + j * kThreads + threadIdx.x;
          if (i < s.L) lds_keys[i] = v[j];
        }
      }
      __syncthreads();
#pragma unroll
      for (int j = 0; j < KPT; ++j) keys[j] = i0 + j < s.L ? lds_keys[i0 + j] : 0u;
    }
    // the same LDS words take the assignments (the call starts with a barrier of its own)
    int *lds_assign = reinterpret_cast<int *>(lds_keys);
    select_top_b_regs<kThreads, KPT, true>(keys, s.L, sh.W, s.B, kept, lds_assign, scratch_regs);
    __syncthreads();
    for (int i = threadIdx.x; i < s.L; i += kThreads) assign[i] = lds_assign[i];
  };
  // the launch reserves LDS for the longest sequence, or none when that one is too long
  const bool staged = sh.maxL <= kSelectRegisterKeys;
  if (staged && s.L <= 4 * kThreads) from_registers(std::integral_constant<int, 4>{});
  else if (staged && s.L <= 8 * kThreads) from_registers(std::integral_constant<int, 8>{});
  else if (staged) from_registers(std::integral_constant<int, 16>{});
  else select_top_b<kThreads>(imp, s.L, sh.W, s.B, kept, assign, scratch);
  __syncthreads();  // kept[] is read back below; sh_rho is set
  const bool cross = (sh_rho > sh.theta) != (sh.invert_flow != 0);

  // ---- the tokens to be matched, in class order --------------------------------------------------
  // (all of them ascending in a cross-modal layer; the text tokens, then the image tokens in an
  // intra-modal one).  The match kernel walks over this list, so pivots take no part in its contraction.
  // Consecutive threads look at consecutive list positions (the flags come out of LDS without bank
  // conflicts and the list goes to memory in nearly whole lines); the rank of a token is the count of
  // the (round, wave) cells before its own plus the flagged lanes below it.
  {
    constexpr int KPT = 16, kWaves = kThreads / 64;
    static_assert(KPT * kWaves <= 256, "one counter per (round, wave) in the histogram scratch");
    int *ev = c.ev_list + unit * sh.T + s.tok_off;
    const int *order = c.cls_order + s.tok_off;
    const int *asg = staged ? reinterpret_cast<const int *>(lds_keys) : assign;
    const int bound = cross ? s.L : s.n_text;  // class-order indices below it belong to the first class
    int *cell = scratch.hist;                  // [KPT][kWaves] counts, then exclusive offsets
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    auto flagged = [&](int v, int &tok) {
      tok = 0;
      if (v >= s.L) return false;
      tok = cross ? v : order[v];
      return asg[tok] == -2;
    };
    int carry = 0, carry0 = 0;
    for (int base = 0; base < s.L; base += KPT * kThreads) {
#pragma unroll
      for (int j = 0; j < KPT; ++j) {
        const int v = base + j * kThreads + threadIdx.x;
        int tok;
        const bool f = flagged(v, tok);
        const unsigned long long bal = __ballot(f), bal0 = __ballot(f && v < bound);
        if (lane == 0) cell[j * kWaves + wave] = __popcll(bal) | (__popcll(bal0) << 16);
      }
      __syncthreads();
      if (wave == 0) {  // exclusive scan of the KPT * kWaves cells in list order: four cells per lane
        int v4[4], sum = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) { v4[k] = 4 * lane + k < KPT * kWaves ? cell[4 * lane + k] : 0; sum += v4[k]; }
        int before = wave_inclusive_scan(sum) - sum;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          if (4 * lane + k < KPT * kWaves) cell[4 * lane + k] = before;
          before += v4[k];
        }
        if (lane == 63) scratch.remaining = before;  // the total of this round
      }
      __syncthreads();
#pragma unroll
      for (int j = 0; j < KPT; ++j) {
        const int v = base + j * kThreads + threadIdx.x;
        int tok;
        const bool f = flagged(v, tok);
        const unsigned long long bal = __ballot(f);
        if (f) ev[carry + (cell[j * kWaves + wave] & 0xffff) + __popcll(bal & ((1ull << lane) - 1))] = tok;
      }
      const int total = scratch.remaining;
      carry += total & 0xffff;
      carry0 += total >> 16;
      __syncthreads();  // the cells are counted into again
    }
    if (threadIdx.x == 0) {
      c.ev_n[(unit * sh.batch + b) * 2] = carry0;
      c.ev_n[(unit * sh.batch + b) * 2 + 1] = carry - carry0;
    }
  }

  // ---- lists of eligible pivots per token class --------------------------------------------------
  const int Bp = (s.B + 31) & ~31;
  const long long lbase = unit * 2 * sh.SBP + 2 * (meta + meta[MW_OFF_CU_BP])[b];
  const uint4 *K = reinterpret_cast<const uint4 *>(c.K) + (long long)l * sh.ks_layer +
                   (long long)gkv * sh.ks_head + (long long)s.tok_off * sh.ks_tok;
  const uint8_t *mod = c.mod + s.tok_off;
  const float *impf = c.importance + unit * sh.T + s.tok_off;
  int *pl_slot = c.pl_slot + lbase;
  int *pl_tok = c.pl_tok + lbase;
  float *pl_w = c.pl_w + lbase;
  uint4 *pack = c.pack + lbase * (NCH + 1);
  int n[2] = {0, 0};
  for (int s0 = 0; s0 < s.B; s0 += kThreads) {  // ordered placement of the eligible slots of each class
    const int slot = s0 + threadIdx.x;
    int f0 = 0, f1 = 0, tok = 0;
    if (slot < s.B) {
      tok = kept[slot];
      const bool ok = !(impf[tok] > s.tau);
      const int cls = cross ? 0 : mod[tok];
      f0 = ok && cls == 0;
      f1 = ok && cls == 1;
    }
    int tot;
    const int ex = block_exclusive_scan<kThreads, int>(f0 | (f1 << 16), scratch.wave_sums, &tot);
    if (f0 | f1) {
      const int pos = f0 ? n[0] + (ex & 0xffff) : Bp + n[1] + (ex >> 16);
      pl_slot[pos] = slot;
      pl_tok[pos] = tok;
    }
    n[0] += tot & 0xffff;
    n[1] += tot >> 16;
  }
  __syncthreads();
  const int np[2] = {(n[0] + 31) & ~31, (n[1] + 31) & ~31};
#pragma unroll
  for (int cls = 0; cls < 2; ++cls)
    for (int e = n[cls] + threadIdx.x; e < np[cls]; e += kThreads) {
      pl_slot[cls * Bp + e] = pl_slot[cls * Bp];
      pl_tok[cls * Bp + e] = pl_tok[cls * Bp];
    }
  if (threadIdx.x < 2) c.pl_n[(unit * sh.batch + b) * 2 + threadIdx.x] = np[threadIdx.x];
  __syncthreads();
  // rows and inverse norms: NCH lanes per row
  constexpr int RPP = kThreads / NCH;  // rows per pass; a multiple of 32, so a pass ends inside a padded list
  const int rl = threadIdx.x / NCH, ch = threadIdx.x % NCH;
  constexpr int U = 4;  // rows in flight per lane group: the dependent loads of a row overlap with the others'
#pragma unroll
  for (int cls = 0; cls < 2; ++cls) {
    for (int e0 = 0; e0 < np[cls]; e0 += U * RPP) {
      int e[U], tok[U];
      uint4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        e[u] = e0 + u * RPP + rl;  // e < np is uniform over the NCH lanes of a row
        tok[u] = e[u] < np[cls] ? pl_tok[cls * Bp + e[u]] : 0;
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        v[u] = make_uint4(0, 0, 0, 0);
        if (e[u] < np[cls]) v[u] = K[(long long)tok[u] * sh.ks_tok + ch];
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float ss = chunk_sumsq<BF16>(v[u]);
#pragma unroll
        for (int o = NCH / 2; o >= 1; o >>= 1) ss += __shfl_xor(ss, o, 64);
        if (e[u] < np[cls]) {
          pack[(long long)(cls * Bp + e[u]) * (NCH + 1) + ch] = v[u];
          if (ch == 0) pl_w[cls * Bp + e[u]] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;
        }
      }
    }
  }
}

}  // namespace

namespace {

template <bool BF16, int D>
hipError_t launch_select_t(const Ctx &c) {
  const size_t lds = c.sh.maxL <= kSelectRegisterKeys ? (size_t)c.sh.maxL * 4 : 0;
  hipError_t e = allow_full_lds<select_kernel<BF16, D>>();
  if (e != hipSuccess) return e;
  ProfScope ps(c.stream, KID_SELECT);
  select_kernel<BF16, D><<<dim3(c.sh.batch, c.sh.Hkv, c.sh.n_layers), kThreads, lds, c.stream>>>(c);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_select(const Ctx &c) {
  if (c.sh.bf16) return c.sh.d == 128 ? launch_select_t<true, 128>(c) : launch_select_t<true, 64>(c);
  return c.sh.d == 128 ? launch_select_t<false, 128>(c) : launch_select_t<false, 64>(c);
}

}  // namespace flowmm
