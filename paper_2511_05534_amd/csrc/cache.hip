// Decode-time maintenance of the compacted cache: the cache-append equation of the paper's
// Preliminary section, K_t = [K_{t-1}, k_t], V_t = [V_{t-1}, v_t], on a cache that keeps head room
// for decoded tokens behind every sequence's merged prompt rows, and the copy that puts the rows of
// a re-merge back at the head of the sequence's range.  Pure data movement in 16-byte chunks.
#include "device_common.h"
#include "kernels.h"
#include "profile.h"

namespace flowmm {

namespace {

// grid (sequences of this launch, kv heads, layers); one thread per 16-byte chunk of the K row and of the V row
__global__ __launch_bounds__(64) void cache_append_kernel(AppendArgs a) {
  const int b = blockIdx.x, g = blockIdx.y, l = blockIdx.z;
  const int t = threadIdx.x;
  if (t >= 2 * a.nch) return;
  const int tensor = t / a.nch, ch = t - tensor * a.nch;
  const long long dst_row = (long long)l * a.ks_layer + (long long)g * a.ks_head + (long long)a.row[b] * a.ks_tok;
  const long long src_row = (((long long)l * gridDim.y + g) * a.batch + a.b0 + b) * a.nch;
  const uint4 *src = reinterpret_cast<const uint4 *>(tensor ? a.v_new : a.k_new);
  uint4 *dst = reinterpret_cast<uint4 *>(tensor ? a.V_c : a.K_c);
  dst[dst_row + ch] = src[src_row + ch];
}

// grid (row groups, kv heads, layers): rows [0, B) of the dense [Lyr][Hkv][B][d] source go to rows
// [row0, row0 + B) of the strided cache
__global__ __launch_bounds__(256) void cache_store_rows_kernel(StoreRowsArgs a) {
  const int g = blockIdx.y, l = blockIdx.z;
  const long long chunks = (long long)a.B * a.nch;
  const uint4 *srcK = reinterpret_cast<const uint4 *>(a.K_src) + ((long long)l * gridDim.y + g) * chunks;
  const uint4 *srcV = reinterpret_cast<const uint4 *>(a.V_src) + ((long long)l * gridDim.y + g) * chunks;
  uint4 *dstK = reinterpret_cast<uint4 *>(a.K_c) + (long long)l * a.ks_layer + (long long)g * a.ks_head + (long long)a.row0 * a.ks_tok;
  uint4 *dstV = reinterpret_cast<uint4 *>(a.V_c) + (long long)l * a.ks_layer + (long long)g * a.ks_head + (long long)a.row0 * a.ks_tok;
  for (long long q = (long long)blockIdx.x * 256 + threadIdx.x; q < chunks; q += (long long)gridDim.x * 256) {
    const long long s = q / a.nch;
    const int ch = (int)(q - s * a.nch);
    dstK[s * a.ks_tok + ch] = srcK[q];
    dstV[s * a.ks_tok + ch] = srcV[q];
  }
}

}  // namespace

hipError_t launch_cache_append(const AppendArgs &a, int n_seqs, int Hkv, int n_layers, hipStream_t stream) {
  ProfScope ps(stream, KID_CACHE_APPEND);
  cache_append_kernel<<<dim3(n_seqs, Hkv, n_layers), 64, 0, stream>>>(a);
  return hipGetLastError();
}

hipError_t launch_cache_store_rows(const StoreRowsArgs &a, int Hkv, int n_layers, hipStream_t stream) {
  const long long chunks = (long long)a.B * a.nch;
  const int gx = (int)((chunks + 255) / 256 < 64 ? (chunks + 255) / 256 : 64);
  ProfScope ps(stream, KID_CACHE_STORE_ROWS);
  cache_store_rows_kernel<<<dim3(gx > 0 ? gx : 1, Hkv, n_layers), 256, 0, stream>>>(a);
  return hipGetLastError();
}

}  // namespace flowmm
