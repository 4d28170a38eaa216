// KV-cache compaction (paper Sec. 3 and Sec. 4.3: the mask is applied to the target's cache and
// only the kept tokens remain): an ordered row gather, out[r, j, :] = in[r, idx[r, j], :], for K
// and V in one launch so the index read is shared.  Pure data movement in 16-byte pieces.
#include "common.hpp"
#include "kernels.hpp"

namespace pkv {
namespace {

constexpr int kUnroll = 4;

// grid (ceil(K / rows_per_block), rows); cpr = 16-byte chunks per token row.
__global__ __launch_bounds__(256) void compact_kernel(const u32x4* __restrict__ k_in, const u32x4* __restrict__ v_in,
                                                       const int32_t* __restrict__ idx, int64_t N, int K, int cpr,
                                                       u32x4* __restrict__ k_out, u32x4* __restrict__ v_out) {
  const int r = blockIdx.y;
  const int tokens_per_step = 256 / cpr;
  const int ch = threadIdx.x % cpr, tsub = threadIdx.x / cpr;
  const int j0 = blockIdx.x * tokens_per_step * kUnroll + tsub;
  const int32_t* ridx = idx + (size_t)r * K;
  const size_t in_base = (size_t)r * N * cpr, out_base = (size_t)r * K * cpr;
  u32x4 kv[kUnroll], vv[kUnroll];
  int jj[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    jj[u] = j0 + u * tokens_per_step;
    if (jj[u] < K && tsub < tokens_per_step) {
      const size_t src = in_base + (size_t)ridx[jj[u]] * cpr + ch;
      kv[u] = __builtin_nontemporal_load(k_in + src);
      vv[u] = __builtin_nontemporal_load(v_in + src);
    }
  }
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    if (jj[u] < K && tsub < tokens_per_step) {
      const size_t dst = out_base + (size_t)jj[u] * cpr + ch;
      __builtin_nontemporal_store(kv[u], k_out + dst);
      __builtin_nontemporal_store(vv[u], v_out + dst);
    }
  }
}

}  // namespace

hipError_t launch_compact(const void* k_in, const void* v_in, const int32_t* idx, int64_t rows, int64_t N, int64_t K,
                          int64_t row_bytes, void* k_out, void* v_out, hipStream_t stream) {
  if (rows <= 0 || K <= 0) return hipSuccess;
  const int cpr = (int)(row_bytes / 16);
  const int tokens_per_block = (256 / cpr) * kUnroll;
  dim3 grid((unsigned)((K + tokens_per_block - 1) / tokens_per_block), (unsigned)rows);
  compact_kernel<<<grid, 256, 0, stream>>>((const u32x4*)k_in, (const u32x4*)v_in, idx, N, (int)K, cpr,
                                           (u32x4*)k_out, (u32x4*)v_out);
  return hipGetLastError();
}

}  // namespace pkv
