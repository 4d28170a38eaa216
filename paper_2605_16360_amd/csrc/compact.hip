// KV-cache compaction (paper Sec. 3 and Sec. 4.3: the mask is applied to the target's cache and
// only the kept tokens remain): an ordered row gather, out[r, j, :] = in[r, idx[r, j], :], for K
// and V in one launch so the index read is shared.  Pure data movement in 16-byte pieces, two token rows in flight per thread (measured at
// N = 32 768, keep ratio 0.3: 0.436 ms with one or two, 0.45 ms with four, 0.96 ms with eight; plain instead of
// non-temporal loads 0.48 ms).
#include "common.hpp"
#include "kernels.hpp"

namespace pkv {
namespace {

constexpr int kUnroll = 2;

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

// ---------------------------------------------------------------------------------------------
// The same gather with the cache as its own destination (the paper's mask is applied to the target's
// cache where it lies): afterwards tokens 0 .. K-1 of every row r are the kept tokens in order; what
// lies behind them is not touched.  idx is ascending, so token j moves from idx[j] >= j: a destination
// never lies behind its source, and the only hazard is a later token's destination overwriting an
// earlier token's source before it was read.  One workgroup per row walks the kept tokens in chunks
// of 128 in order: the loads of chunk c+1 are issued, a barrier makes sure every thread holds chunk
// c, then chunk c is stored.  Chunk c+1 reads tokens at or behind (c+1)*128, which chunk c's stores
// (tokens below (c+1)*128) cannot touch, so the two overlap safely.
// grid (rows), 256 threads; cpr = 16-byte chunks per token (<= 32).
// ---------------------------------------------------------------------------------------------
constexpr int kInplaceTokens = 128;

// With counts != nullptr the rows are ragged (a budget shared by the `heads` rows of a layer): idx holds,
// per layer, heads * K flat indices h * N + n in ascending order, row r = (layer, h) keeps counts[r] of
// them, and its list starts behind those of the layer's earlier heads.
template <int PER>  // 16-byte pieces per thread and chunk, for each of K and V
__global__ __launch_bounds__(256) void compact_inplace_kernel(u32x4* __restrict__ k, u32x4* __restrict__ v,
                                                               const int32_t* __restrict__ idx, int64_t N, int K, int cpr,
                                                               const int32_t* __restrict__ counts, int heads) {
  const int r = blockIdx.x, tid = threadIdx.x;
  const int32_t* ridx = idx + (size_t)r * K;
  int32_t sub = 0;  // what a stored index is ahead of the row's token number
  if (counts != nullptr) {
    const int layer = r / heads, h = r % heads;
    int start = 0;
    for (int hh = 0; hh < h; ++hh) start += counts[layer * heads + hh];
    ridx = idx + (size_t)layer * heads * K + start;
    K = counts[r];
    sub = (int32_t)(h * N);
  }
  u32x4* kb = k + (size_t)r * N * cpr;
  u32x4* vb = v + (size_t)r * N * cpr;
  const int n_chunks = (K + kInplaceTokens - 1) / kInplaceTokens;
  u32x4 ka[PER], va[PER], kn[PER], vn[PER];
  auto load = [&](int c, u32x4 (&kr)[PER], u32x4 (&vr)[PER]) {
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int piece = tid + 256 * u, j = c * kInplaceTokens + piece / cpr, ch = piece % cpr;
      if (piece < kInplaceTokens * cpr && j < K) {
        const size_t src = (size_t)(ridx[j] - sub) * cpr + ch;
        kr[u] = __builtin_nontemporal_load(kb + src);
        vr[u] = __builtin_nontemporal_load(vb + src);
      }
    }
  };
  auto store = [&](int c, const u32x4 (&kr)[PER], const u32x4 (&vr)[PER]) {
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int piece = tid + 256 * u, j = c * kInplaceTokens + piece / cpr, ch = piece % cpr;
      if (piece < kInplaceTokens * cpr && j < K) {
        const size_t dst = (size_t)j * cpr + ch;
        kb[dst] = kr[u];
        vb[dst] = vr[u];
      }
    }
  };
  load(0, ka, va);
  for (int c = 0; c < n_chunks; ++c) {
    if (c + 1 < n_chunks) load(c + 1, kn, vn);
    // every thread holds its part of chunk c (and of every chunk before it) before any of chunk c is stored
    __syncthreads();
    store(c, ka, va);
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      ka[u] = kn[u];
      va[u] = vn[u];
    }
  }
}

// mask[r, n] = 1 for the kept tokens of row r, 0 elsewhere (uint8).  One workgroup per row clears the row,
// then sets the kept positions.
__global__ __launch_bounds__(256) void mask_kernel(const int32_t* __restrict__ idx, int64_t N, int K,
                                                    uint8_t* __restrict__ mask) {
  const int r = blockIdx.x, tid = threadIdx.x;
  uint8_t* row = mask + (size_t)r * N;
  // 16-byte stores over the aligned middle, bytes at the ragged ends
  const uintptr_t addr = reinterpret_cast<uintptr_t>(row);
  const int64_t head = (int64_t)((16 - (addr & 15)) & 15) < N ? (int64_t)((16 - (addr & 15)) & 15) : N;
  const int64_t n16 = (N - head) / 16;
  for (int64_t i = tid; i < head; i += 256) row[i] = 0;
  u32x4* mid = reinterpret_cast<u32x4*>(row + head);
  for (int64_t i = tid; i < n16; i += 256) mid[i] = u32x4{0, 0, 0, 0};
  for (int64_t i = head + n16 * 16 + tid; i < N; i += 256) row[i] = 0;
  __syncthreads();  // workgroup-scope release/acquire: the zeros are in place before the ones
  const int32_t* ridx = idx + (size_t)r * K;
  for (int j = tid; j < K; j += 256) row[ridx[j]] = 1;
}

// counts[layer, h] = number of a layer's kept flat indices (ascending, heads * K of them) that fall into
// [h * N, (h + 1) * N): the difference of two lower bounds.  One thread per (layer, head).
__global__ void head_counts_kernel(const int32_t* __restrict__ flat, int layers, int heads, int64_t N, int K,
                                   int32_t* __restrict__ counts) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= layers * heads) return;
  const int layer = t / heads, h = t % heads, n = heads * K;
  const int32_t* row = flat + (size_t)layer * n;
  auto lower_bound = [&](int64_t value) {  // first position whose index is >= value
    int lo = 0, hi = n;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if ((int64_t)row[mid] < value) lo = mid + 1;
      else hi = mid;
    }
    return lo;
  };
  counts[t] = lower_bound((int64_t)(h + 1) * N) - lower_bound((int64_t)h * N);
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

hipError_t launch_compact_inplace(void* k, void* v, const int32_t* idx, int64_t rows, int64_t N, int64_t K, int64_t row_bytes,
                                  const int32_t* counts, int heads, hipStream_t stream) {
  if (rows <= 0 || K <= 0) return hipSuccess;
  const int cpr = (int)(row_bytes / 16);
  const int per = (kInplaceTokens * cpr + 255) / 256;  // 16-byte pieces per thread and chunk
  u32x4 *kp = (u32x4*)k, *vp = (u32x4*)v;
  if (per <= 4) compact_inplace_kernel<4><<<(unsigned)rows, 256, 0, stream>>>(kp, vp, idx, N, (int)K, cpr, counts, heads);
  else if (per <= 8) compact_inplace_kernel<8><<<(unsigned)rows, 256, 0, stream>>>(kp, vp, idx, N, (int)K, cpr, counts, heads);
  else if (per <= 16) compact_inplace_kernel<16><<<(unsigned)rows, 256, 0, stream>>>(kp, vp, idx, N, (int)K, cpr, counts, heads);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_head_counts(const int32_t* flat, int64_t layers, int64_t heads, int64_t N, int64_t K, int32_t* counts,
                              hipStream_t stream) {
  const int64_t n = layers * heads;
  if (n <= 0) return hipSuccess;
  head_counts_kernel<<<(unsigned)((n + 255) / 256), 256, 0, stream>>>(flat, (int)layers, (int)heads, N, (int)K, counts);
  return hipGetLastError();
}

hipError_t launch_mask(const int32_t* idx, int64_t rows, int64_t N, int64_t K, uint8_t* mask, hipStream_t stream) {
  if (rows <= 0) return hipSuccess;
  mask_kernel<<<(unsigned)rows, 256, 0, stream>>>(idx, N, (int)K, mask);
  return hipGetLastError();
}

}  // namespace pkv
