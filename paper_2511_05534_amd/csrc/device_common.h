// Device-side helpers shared by the gfx950 kernels: MFMA fragments read straight from global
// memory or LDS in 16-byte chunks, wave64 reductions, and metadata look-ups.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "layout.h"

namespace flowmm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

// A row of head_dim elements is NCH 16-byte chunks.  In every contraction lane (n, half) of a
// wave (n = lane & 31, half = lane >> 5) owns the chunks 2t+half, t = 0..NF-1, of row n of
// its operand tile, so both operands of an MFMA see the same channel in the same k slot.
template <bool BF16, int D>
struct Cfg {
  static constexpr int kElemBytes = BF16 ? 2 : 4;
  static constexpr int NCH = D * kElemBytes / 16;  // chunks per row
  static constexpr int NF = NCH / 2;               // fragments per lane per row
  static constexpr int kElemsPerChunk = 16 / kElemBytes;
};

// acc[m][n] += sum over the chunk's channels of a(row m) * b(row n); 32x32 tile, lane holds
// column n = lane & 31 and rows m = 8*(i/4) + 4*(lane>>5) + (i%4), i = 0..15.
template <bool BF16>
__device__ __forceinline__ void mma_chunk(f32x16_t &acc, const uint4 &a, const uint4 &b) {
  if constexpr (BF16) {
    bf16x8_t av, bv;
    __builtin_memcpy(&av, &a, 16);
    __builtin_memcpy(&bv, &b, 16);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc, 0, 0, 0);
  } else {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
  }
}

__device__ __forceinline__ int acc_row(int i, int half) { return 8 * (i >> 2) + 4 * half + (i & 3); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }

// round-to-nearest-even float -> bf16 bits (finite inputs; NaN stays NaN)
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

template <bool BF16>
__device__ __forceinline__ void chunk_to_floats(const uint4 &c, float *f) {
  if constexpr (BF16) {
    f[0] = bf16_bits_to_float(c.x & 0xffffu); f[1] = bf16_bits_to_float(c.x >> 16);
    f[2] = bf16_bits_to_float(c.y & 0xffffu); f[3] = bf16_bits_to_float(c.y >> 16);
    f[4] = bf16_bits_to_float(c.z & 0xffffu); f[5] = bf16_bits_to_float(c.z >> 16);
    f[6] = bf16_bits_to_float(c.w & 0xffffu); f[7] = bf16_bits_to_float(c.w >> 16);
  } else {
    f[0] = __uint_as_float(c.x); f[1] = __uint_as_float(c.y);
    f[2] = __uint_as_float(c.z); f[3] = __uint_as_float(c.w);
  }
}

template <bool BF16>
__device__ __forceinline__ uint4 floats_to_chunk(const float *f) {
  uint4 c;
  if constexpr (BF16) {
    c.x = float_to_bf16_bits(f[0]) | (float_to_bf16_bits(f[1]) << 16);
    c.y = float_to_bf16_bits(f[2]) | (float_to_bf16_bits(f[3]) << 16);
    c.z = float_to_bf16_bits(f[4]) | (float_to_bf16_bits(f[5]) << 16);
    c.w = float_to_bf16_bits(f[6]) | (float_to_bf16_bits(f[7]) << 16);
  } else {
    c.x = __float_as_uint(f[0]); c.y = __float_as_uint(f[1]);
    c.z = __float_as_uint(f[2]); c.w = __float_as_uint(f[3]);
  }
  return c;
}

template <bool BF16>
__device__ __forceinline__ float chunk_sumsq(const uint4 &c) {
  float f[8];
  chunk_to_floats<BF16>(c, f);
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < (BF16 ? 8 : 4); ++j) s = fmaf(f[j], f[j], s);
  return s;
}

// running (max, sum of exp2) pairs of a softmax row, in the log2 domain
__device__ __forceinline__ void stat_combine(float &m, float &z, float m2, float z2) {
  const float M = fmaxf(m, m2);
  if (M == -INFINITY) { m = M; z = 0.f; return; }
  z = z * fast_exp2(m - M) + z2 * fast_exp2(m2 - M);
  m = M;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__device__ __forceinline__ int wave_sum_int(int v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Direct global -> LDS load: lane i of the wave fetches BYTES (4 or 16) bytes from base + byte_off
// (base wave-uniform, in scalar registers; the lane's part is a 32-bit offset, so no lane keeps a
// 64-bit address) and they land at lds_base + i * BYTES (lds_base wave-uniform).  Lanes that are
// switched off leave their bytes alone.  Issued as inline assembly so that the compiler does not
// wait for it before unrelated LDS reads (it cannot tell two LDS buffers apart); the statement
// sets M0 and says so in its clobber list (the compiler keeps M0 out of register allocation and
// warns about any such entry; the entry is still what orders its own M0 writes around this one).
// The caller waits with s_waitcnt vmcnt(0) and a barrier before reading the data.
typedef __attribute__((address_space(3))) void lds_void;
template <int BYTES>
__device__ __forceinline__ void load_to_lds(const void *base, unsigned byte_off, void *lds_base) {
  static_assert(BYTES == 4 || BYTES == 16, "one dword or four per lane");
  const unsigned lds_addr = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(lds_void *)lds_base);
  // the base goes through the first lane's copy of it: free when it already sits in scalar registers,
  // and it keeps the operand a scalar pair when the compiler has lost track of its uniformity
  const unsigned long long bits = (unsigned long long)(uintptr_t)base;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)bits), hi = __builtin_amdgcn_readfirstlane((unsigned)(bits >> 32));
  base = reinterpret_cast<const void *>((uintptr_t)(((unsigned long long)hi << 32) | lo));
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
  if constexpr (BYTES == 16)
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(byte_off), "s"(base), "s"(lds_addr) : "memory", "m0");
  else
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(byte_off), "s"(base), "s"(lds_addr) : "memory", "m0");
#pragma clang diagnostic pop
}

// The rows of 32 tokens as MFMA operand fragments (this lane's chunks 2t+half of row n), fetched as
// whole rows.  Asked for straight from memory, those fragments make every load instruction touch 32
// cache lines for 32 bytes each, and a compute unit's L1 looks up one line per clock: 16 bytes per
// clock, and the waves wait at their load instructions meanwhile.  Here the wave fetches whole rows
// (64/NCH rows per instruction, every line touched once) into a staging area of its own in LDS with
// direct global->LDS loads; the chunk a lane asks for is chosen so that the chunks of row r land
// XOR-swizzled by r, and the fragments are then read from there without bank conflicts.
//   base  : wave-uniform; row t starts at base + t * row_stride chunks (32-bit byte offsets: the
//           caller has checked that the rows lie within 4 GiB of base)
//   tok   : the row this lane's fragments belong to (lanes n and n + 32 pass the same)
//   stage : 32 * NCH chunks of LDS that no other wave touches until the call has returned
template <bool BF16, int D>
__device__ __forceinline__ void request_rows_staged(const void *base, unsigned row_stride, int tok, uint4 *stage) {
  constexpr int NCH = Cfg<BF16, D>::NCH;
  static_assert(NCH <= 64 && (NCH & (NCH - 1)) == 0, "rows of a power-of-two number of chunks");
  constexpr int RPI = 64 / NCH;  // rows per load instruction
  const int lane = threadIdx.x & 63;
  const int rl = lane / NCH, slot = lane % NCH;
#pragma unroll
  for (int j = 0; j < 32 / RPI; ++j) {
    const int r = j * RPI + rl;
    const int t = __shfl(tok, r, 64);
    const int ch = slot ^ (r & (NCH - 1));
    load_to_lds<16>(base, ((unsigned)t * row_stride + (unsigned)ch) * 16u, stage + j * 64);
  }
}

// The fragments of the rows that request_rows_staged asked for (waits for this wave's outstanding loads
// first; only this wave reads the area, so no barrier), and a wait for the reads themselves: on return
// the area may be written again.
template <bool BF16, int D>
__device__ __forceinline__ void read_rows_staged(const uint4 *stage, uint4 (&frag)[Cfg<BF16, D>::NF]) {
  constexpr int NCH = Cfg<BF16, D>::NCH, NF = Cfg<BF16, D>::NF;
  const int lane = threadIdx.x & 63, n = lane & 31, half = lane >> 5;
  __builtin_amdgcn_s_waitcnt(0);
#pragma unroll
  for (int f = 0; f < NF; ++f) frag[f] = stage[n * NCH + ((2 * f + half) ^ (n & (NCH - 1)))];
  __builtin_amdgcn_s_waitcnt(0);
}

template <bool BF16, int D>
__device__ __forceinline__ void fetch_rows_staged(const void *base, unsigned row_stride, int tok, uint4 *stage,
                                                  uint4 (&frag)[Cfg<BF16, D>::NF]) {
  request_rows_staged<BF16, D>(base, row_stride, tok, stage);
  read_rows_staged<BF16, D>(stage, frag);
}

// For grids whose x extent counts sequences (or a fixed number of workgroups per sequence) and whose
// y, z are kv head and layer: workgroups go to the eight XCDs in turn by their linear index, so a
// batch of eight would pin each sequence, long ones included, to one XCD.  Rotating x by the other
// two coordinates spreads every sequence over all XCDs; for fixed (y, z) it is still a bijection.
__device__ __forceinline__ int rotated_block_x() { return (blockIdx.x + blockIdx.y + blockIdx.z) % gridDim.x; }

// sequence that owns flat index x given an increasing cumulative table cu[0..batch]
__device__ __forceinline__ int find_seq(const int *__restrict__ cu, int batch, int x) {
  int lo = 0, hi = batch;  // invariant: cu[lo] <= x < cu[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu[mid] <= x) lo = mid; else hi = mid;
  }
  return lo;
}

struct SeqInfo {
  int tok_off, L, B, kept_off, win_has_img, n_text;
  float tau;
};

__device__ __forceinline__ SeqInfo load_seq(const int *__restrict__ meta, int b) {
  const int *r = meta + meta[MW_OFF_SEQ] + b * SW_WORDS;
  SeqInfo s;
  s.tok_off = r[SW_TOK_OFF];
  s.L = r[SW_L];
  s.B = r[SW_B];
  s.kept_off = r[SW_KEPT_OFF];
  s.tau = __int_as_float(r[SW_TAU]);
  s.win_has_img = r[SW_WIN_HAS_IMG];
  s.n_text = r[SW_N_TEXT];
  return s;
}

__device__ __forceinline__ SeqInfo inline_seq(const InlineMeta &m, int b) {
  SeqInfo s;
  s.tok_off = m.tok_off[b];
  s.L = m.L[b];
  s.B = m.B[b];
  s.kept_off = m.kept_off[b];
  s.tau = m.tau[b];
  s.win_has_img = (m.win_has_img >> b) & 1u;
  s.n_text = 0;
  return s;
}

// modality (0 text, 1 image) of position i of sequence b: the first span that ends after i.
// The loop runs over the spans of the sequence with wave-uniform bounds, so the span table is read
// with scalar loads (a per-lane walk would turn it into vector loads from the argument block, which
// then queue behind every outstanding key load).
__device__ __forceinline__ int inline_mod(const InlineMeta &m, int b, int i) {
  const int first = m.span_off[b], last = m.span_off[b + 1] - 1;
  int mod = (m.span_is_image >> last) & 1u;
  for (int j = last - 1; j >= first; --j)
    if (i < m.span_end[j]) mod = (m.span_is_image >> j) & 1u;
  return mod;
}

}  // namespace flowmm
