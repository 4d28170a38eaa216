// Per-row Top-K selection (paper Sec. 3: the mask keeps the Top-K of the mapped scores per target
// layer and head; Sec. 4.3 names a Top-K kernel that materialises it).  Integer work only: scores
// are turned into order-preserving 32-bit keys, the K-th largest key is found by an 8-bit radix select
// (at most four passes) on the keys relative to the row's smallest key, and one more ordered pass emits the kept indices in ascending order, taking
// equal keys by lower index.  A row of up to 36 864 scores is read from global memory once and its keys stay in
// registers for all passes; longer rows are re-read (from L2) in every pass.
#include "common.hpp"
#include "kernels.hpp"

namespace pkv {
namespace {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / 64;

// Larger key <=> earlier in the selection order.  NaN maps to 0 (below -inf), -0.0 onto +0.0.
__device__ __forceinline__ uint32_t order_key(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// One workgroup per row; the row is re-read (from L2) in every pass.  For rows longer than kTopkRegMax.
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(const float* __restrict__ scores, int N, int K,
                                                            int32_t* __restrict__ idx_out) {
  const float* row = scores + (size_t)blockIdx.x * N;
  int32_t* out = idx_out + (size_t)blockIdx.x * K;
  __shared__ uint32_t hist[kTopkWaves][256];
  __shared__ uint32_t tot[256];
  __shared__ uint32_t s_prefix, s_krem;
  __shared__ uint32_t wave_gt[kTopkWaves], wave_eq[kTopkWaves];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  // f(key) for the keys tid, tid + 1024, ... of the row, sixteen loads in flight per thread (one workgroup per row:
  // the loop is bound by the bytes it keeps in flight)
  auto for_each_key = [&](auto&& f) {
    constexpr int kBatch = 16;
    for (int i0 = tid; i0 < N; i0 += kBatch * kTopkThreads) {
      float v[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int i = i0 + u * kTopkThreads;
        v[u] = row[i < N ? i : N - 1];
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u)
        if (i0 + u * kTopkThreads < N) f(order_key(v[u]));
    }
  };

  // Range of the row's keys: the radix digits are taken from key - kmin, top-aligned to the width of the
  // range.  Digits of the raw key are badly skewed (scores share sign and exponent), and lanes that add to
  // the same LDS counter are serialised; digits of the range-relative key are spread over all 256 bins.
  __syncthreads();
  uint32_t kmin = 0xffffffffu, kmax = 0u;
  for_each_key([&](uint32_t key) {
    kmin = key < kmin ? key : kmin;
    kmax = key > kmax ? key : kmax;
  });
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const uint32_t a = __shfl_xor(kmin, off, 64), c = __shfl_xor(kmax, off, 64);
    kmin = a < kmin ? a : kmin;
    kmax = c > kmax ? c : kmax;
  }
  if (lane == 0) {
    wave_gt[wave] = kmin;
    wave_eq[wave] = kmax;
  }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kTopkWaves; ++w) {
    kmin = wave_gt[w] < kmin ? wave_gt[w] : kmin;
    kmax = wave_eq[w] > kmax ? wave_eq[w] : kmax;
  }
  const uint32_t span = kmax - kmin;
  int prev_sh = span == 0 ? 0 : 32 - __builtin_clz(span);  // significant bits of key - kmin

  // radix select on rel = key - kmin: `prefix` = the bits of the K-th largest rel above bit prev_sh
  uint32_t prefix = 0, krem = (uint32_t)K;
  bool first = true;
  while (prev_sh > 0) {
    const int shift = prev_sh > 8 ? prev_sh - 8 : 0;
    const uint32_t dmask = (1u << (prev_sh - shift)) - 1u;
    for (int i = tid; i < kTopkWaves * 256; i += kTopkThreads) (&hist[0][0])[i] = 0;
    __syncthreads();
    for_each_key([&](uint32_t key) {
      const uint32_t rel = key - kmin;
      if (first || (rel >> prev_sh) == prefix) atomicAdd(&hist[wave][(rel >> shift) & dmask], 1u);
    });
    __syncthreads();
    if (tid < 256) {
      uint32_t s = 0;
#pragma unroll
      for (int w = 0; w < kTopkWaves; ++w) s += hist[w][tid];
      tot[tid] = s;
    }
    __syncthreads();
    if (wave == 0) {
      // lane owns bins 4*lane .. 4*lane+3; `above` = number of candidates in higher bins
      const uint32_t c0 = tot[4 * lane], c1 = tot[4 * lane + 1], c2 = tot[4 * lane + 2], c3 = tot[4 * lane + 3];
      const uint32_t mine = c0 + c1 + c2 + c3;
      uint32_t v = mine;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_down(v, off, 64);
        if (lane + off < 64) v += t;
      }
      const uint32_t a3 = v - mine, a2 = a3 + c3, a1 = a2 + c2, a0 = a1 + c1;
      const uint32_t above[4] = {a0, a1, a2, a3};
      const uint32_t cnt[4] = {c0, c1, c2, c3};
#pragma unroll
      for (int bsel = 0; bsel < 4; ++bsel) {
        if (above[bsel] < krem && krem <= above[bsel] + cnt[bsel]) {
          s_prefix = (prefix << (prev_sh - shift)) | (uint32_t)(4 * lane + bsel);
          s_krem = krem - above[bsel];
        }
      }
    }
    __syncthreads();
    prefix = s_prefix;
    krem = s_krem;
    prev_sh = shift;
    first = false;
  }
  prefix += kmin;  // back to a key; with all keys equal the loop did not run: T = kmin, K of them are taken
  __syncthreads();

  // `prefix` is now the K-th largest key T; `krem` of the keys equal to T are kept, lowest index first.
  // Ordered output without a barrier per tile: wave w owns the contiguous part [w * per_wave, (w + 1) * per_wave) of the
  // row.  A first sweep counts the keys above T and equal to T in every part, one prefix sum over the 16 parts gives each
  // wave its first output slot and the number of equal keys before it, and a second sweep writes the indices in order
  // with a running offset that lives in the wave.
  const uint32_t T = prefix, eq_take = krem;
  const int per_wave = ((N + kTopkWaves - 1) / kTopkWaves + 63) & ~63;
  const int w_lo = wave * per_wave < N ? wave * per_wave : N;
  const int w_hi = w_lo + per_wave < N ? w_lo + per_wave : N;
  uint32_t cnt_gt = 0, cnt_eq = 0;
  for (int i0 = w_lo + lane; i0 < w_hi; i0 += 16 * 64) {
    float v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = row[i0 + u * 64 < w_hi ? i0 + u * 64 : w_hi - 1];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const uint32_t key = order_key(v[u]);
      cnt_gt += (i0 + u * 64 < w_hi) && key > T;
      cnt_eq += (i0 + u * 64 < w_hi) && key == T;
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    cnt_gt += __shfl_xor(cnt_gt, off, 64);
    cnt_eq += __shfl_xor(cnt_eq, off, 64);
  }
  if (lane == 0) {
    wave_gt[wave] = cnt_gt;
    wave_eq[wave] = cnt_eq;
  }
  __syncthreads();
  uint32_t eq_before = 0, out_pos = 0;  // equal keys in earlier parts; first output slot of this part
#pragma unroll
  for (int w = 0; w < kTopkWaves; ++w) {
    if (w < wave) {
      const uint32_t e_after = eq_before + wave_eq[w];
      out_pos += wave_gt[w] + ((e_after < eq_take ? e_after : eq_take) - (eq_before < eq_take ? eq_before : eq_take));
      eq_before = e_after;
    }
  }
  const uint64_t lower = (1ull << lane) - 1ull;
  for (int base0 = w_lo; base0 < w_hi; base0 += 16 * 64) {
    float v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int i = base0 + u * 64 + lane;
      v[u] = row[i < w_hi ? i : w_hi - 1];
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int i = base0 + u * 64 + lane;
      const bool valid = i < w_hi;  // once false for a wave's tile it stays false: the counts below add nothing
      const uint32_t key = order_key(v[u]);
      const bool gt = valid && key > T, eq = valid && key == T;
      const uint64_t be = __builtin_amdgcn_ballot_w64(eq);
      const uint32_t eq_rank = eq_before + __popcll(be & lower);
      const bool take = gt || (eq && eq_rank < eq_take);
      const uint64_t bt = __builtin_amdgcn_ballot_w64(take);
      if (take) out[out_pos + __popcll(bt & lower)] = i;
      out_pos += __popcll(bt);
      eq_before += __popcll(be);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Rows of up to kTopkRegMax scores: thread t keeps the keys of the kTopkItems consecutive scores
// [t * kTopkItems, (t + 1) * kTopkItems) in registers, so the row is read from memory once, every radix
// pass runs on registers, and the ordered output needs one prefix sum over the threads' kept counts
// instead of one per tile.
// ---------------------------------------------------------------------------------------------
constexpr int kTopkItems = 36;
constexpr int kTopkRegMax = kTopkItems * kTopkThreads;

// exclusive prefix sum of one value per thread over the workgroup (16 waves); also returns the total
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wave_tot, int wave, int lane, uint32_t& total) {
  uint32_t inc = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t t = __shfl_up(inc, off, 64);
    if (lane >= off) inc += t;
  }
  if (lane == 63) wave_tot[wave] = inc;
  __syncthreads();
  uint32_t before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kTopkWaves; ++w) {
    const uint32_t t = wave_tot[w];
    if (w < wave) before += t;
    tot += t;
  }
  __syncthreads();
  total = tot;
  return before + inc - v;
}

__global__ __launch_bounds__(kTopkThreads) void topk_reg_kernel(const float* __restrict__ scores, int N, int K,
                                                                int32_t* __restrict__ idx_out) {
  const float* row = scores + (size_t)blockIdx.x * N;
  int32_t* out = idx_out + (size_t)blockIdx.x * K;
  __shared__ uint32_t hist[kTopkWaves][256];
  __shared__ uint32_t tot[256];
  __shared__ uint32_t s_prefix, s_krem;
  __shared__ uint32_t wave_a[kTopkWaves], wave_b[kTopkWaves];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int i0 = tid * kTopkItems;

  // keys of this thread's scores; positions at and past N hold the key 0 and are never counted
  uint32_t key[kTopkItems];
  if ((reinterpret_cast<uintptr_t>(row) & 15) == 0 && i0 + kTopkItems <= N) {
#pragma unroll
    for (int j = 0; j < kTopkItems; j += 4) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(row + i0 + j);
      key[j] = order_key(v[0]);
      key[j + 1] = order_key(v[1]);
      key[j + 2] = order_key(v[2]);
      key[j + 3] = order_key(v[3]);
    }
  } else {
#pragma unroll
    for (int j = 0; j < kTopkItems; ++j) key[j] = i0 + j < N ? order_key(row[i0 + j]) : 0u;
  }
  const int mine = N - i0 < 0 ? 0 : (N - i0 < kTopkItems ? N - i0 : kTopkItems);  // valid items of this thread

  uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
  for (int j = 0; j < kTopkItems; ++j) {
    if (j < mine) {
      kmin = key[j] < kmin ? key[j] : kmin;
      kmax = key[j] > kmax ? key[j] : kmax;
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const uint32_t a = __shfl_xor(kmin, off, 64), c = __shfl_xor(kmax, off, 64);
    kmin = a < kmin ? a : kmin;
    kmax = c > kmax ? c : kmax;
  }
  if (lane == 0) {
    wave_a[wave] = kmin;
    wave_b[wave] = kmax;
  }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kTopkWaves; ++w) {
    kmin = wave_a[w] < kmin ? wave_a[w] : kmin;
    kmax = wave_b[w] > kmax ? wave_b[w] : kmax;
  }
  const uint32_t span = kmax - kmin;
  int prev_sh = span == 0 ? 0 : 32 - __builtin_clz(span);

  uint32_t prefix = 0, krem = (uint32_t)K;
  bool first = true;
  while (prev_sh > 0) {
    const int shift = prev_sh > 8 ? prev_sh - 8 : 0;
    const uint32_t dmask = (1u << (prev_sh - shift)) - 1u;
    for (int i = tid; i < kTopkWaves * 256; i += kTopkThreads) (&hist[0][0])[i] = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kTopkItems; ++j) {
      const uint32_t rel = key[j] - kmin;
      if (j < mine && (first || (rel >> prev_sh) == prefix)) atomicAdd(&hist[wave][(rel >> shift) & dmask], 1u);
    }
    __syncthreads();
    if (tid < 256) {
      uint32_t sum = 0;
#pragma unroll
      for (int w = 0; w < kTopkWaves; ++w) sum += hist[w][tid];
      tot[tid] = sum;
    }
    __syncthreads();
    if (wave == 0) {
      const uint32_t c0 = tot[4 * lane], c1 = tot[4 * lane + 1], c2 = tot[4 * lane + 2], c3 = tot[4 * lane + 3];
      const uint32_t own = c0 + c1 + c2 + c3;
      uint32_t v = own;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_down(v, off, 64);
        if (lane + off < 64) v += t;
      }
      const uint32_t a3 = v - own, a2 = a3 + c3, a1 = a2 + c2, a0 = a1 + c1;
      const uint32_t above[4] = {a0, a1, a2, a3};
      const uint32_t cnt[4] = {c0, c1, c2, c3};
#pragma unroll
      for (int bsel = 0; bsel < 4; ++bsel) {
        if (above[bsel] < krem && krem <= above[bsel] + cnt[bsel]) {
          s_prefix = (prefix << (prev_sh - shift)) | (uint32_t)(4 * lane + bsel);
          s_krem = krem - above[bsel];
        }
      }
    }
    __syncthreads();
    prefix = s_prefix;
    krem = s_krem;
    prev_sh = shift;
    first = false;
  }
  const uint32_t T = prefix + kmin, eq_take = krem;

  // kept: keys above T, and the eq_take lowest-index keys equal to T
  uint32_t n_gt = 0, n_eq = 0;
#pragma unroll
  for (int j = 0; j < kTopkItems; ++j) {
    if (j < mine) {
      n_gt += key[j] > T;
      n_eq += key[j] == T;
    }
  }
  uint32_t tot_eq, tot_gt;
  const uint32_t eq_before = block_exclusive_scan(n_eq, wave_a, wave, lane, tot_eq);
  const uint32_t eq_mine = eq_before >= eq_take ? 0u : (eq_take - eq_before < n_eq ? eq_take - eq_before : n_eq);
  uint32_t pos = block_exclusive_scan(n_gt + eq_mine, wave_b, wave, lane, tot_gt);
  uint32_t eq_left = eq_mine;
#pragma unroll
  for (int j = 0; j < kTopkItems; ++j) {
    if (j < mine) {
      const bool take = key[j] > T || (key[j] == T && eq_left > 0);
      if (key[j] == T && eq_left > 0) --eq_left;
      if (take) out[pos++] = i0 + j;
    }
  }
}

}  // namespace

hipError_t launch_topk(const float* scores, int64_t rows, int64_t N, int64_t K, int32_t* idx_out,
                       hipStream_t stream) {
  if (rows <= 0) return hipSuccess;
  if (N <= kTopkRegMax) {
    topk_reg_kernel<<<dim3((unsigned)rows), kTopkThreads, 0, stream>>>(scores, (int)N, (int)K, idx_out);
  } else {
    topk_kernel<<<dim3((unsigned)rows), kTopkThreads, 0, stream>>>(scores, (int)N, (int)K, idx_out);
  }
  return hipGetLastError();
}

}  // namespace pkv
