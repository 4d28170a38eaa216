// Per-row Top-K selection (paper Sec. 3: the mask keeps the Top-K of the mapped scores per target
// layer and head; Sec. 4.3 names a Top-K kernel that materialises it).  Integer work only: scores
// are turned into order-preserving 32-bit keys, the K-th largest key is found by a four-pass
// 8-bit radix select, and one more ordered pass emits the kept indices in ascending order, taking
// equal keys by lower index.
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

// One workgroup per row.
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(const float* __restrict__ scores, int N, int K,
                                                            int32_t* __restrict__ idx_out) {
  const float* row = scores + (size_t)blockIdx.x * N;
  int32_t* out = idx_out + (size_t)blockIdx.x * K;
  __shared__ uint32_t hist[kTopkWaves][256];
  __shared__ uint32_t tot[256];
  __shared__ uint32_t s_prefix, s_krem;
  __shared__ uint32_t wave_gt[kTopkWaves], wave_eq[kTopkWaves];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

  uint32_t prefix = 0, krem = (uint32_t)K;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    for (int i = tid; i < kTopkWaves * 256; i += kTopkThreads) (&hist[0][0])[i] = 0;
    __syncthreads();
    for (int i = tid; i < N; i += kTopkThreads) {
      const uint32_t key = order_key(row[i]);
      if (pass == 0 || (key >> (shift + 8)) == prefix) atomicAdd(&hist[wave][(key >> shift) & 255u], 1u);
    }
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
          s_prefix = (prefix << 8) | (uint32_t)(4 * lane + bsel);
          s_krem = krem - above[bsel];
        }
      }
    }
    __syncthreads();
    prefix = s_prefix;
    krem = s_krem;
  }

  // `prefix` is now the K-th largest key T; `krem` of the keys equal to T are kept, lowest index first.
  const uint32_t T = prefix, eq_take = krem;
  uint32_t base_out = 0, base_eq = 0;
  for (int tile = 0; tile < N; tile += kTopkThreads) {
    const int i = tile + tid;
    const bool valid = i < N;
    const uint32_t key = valid ? order_key(row[i]) : 0u;
    const bool gt = valid && key > T, eq = valid && key == T;
    const uint64_t bg = __builtin_amdgcn_ballot_w64(gt), be = __builtin_amdgcn_ballot_w64(eq);
    const uint64_t lower = (1ull << lane) - 1ull;
    const uint32_t lane_gt = __popcll(bg & lower), lane_eq = __popcll(be & lower);
    if (lane == 0) {
      wave_gt[wave] = __popcll(bg);
      wave_eq[wave] = __popcll(be);
    }
    __syncthreads();
    uint32_t wg = 0, we = 0, tg = 0, te = 0;
#pragma unroll
    for (int w = 0; w < kTopkWaves; ++w) {
      const uint32_t g = wave_gt[w], e = wave_eq[w];
      if (w < wave) {
        wg += g;
        we += e;
      }
      tg += g;
      te += e;
    }
    const uint32_t eq_rank = base_eq + we + lane_eq;
    const uint32_t taken_before_tile = base_eq < eq_take ? base_eq : eq_take;
    const uint32_t taken_before_me = (eq_rank < eq_take ? eq_rank : eq_take) - taken_before_tile;
    if (gt || (eq && eq_rank < eq_take)) out[base_out + wg + lane_gt + taken_before_me] = i;
    const uint32_t eq_after = base_eq + te;
    base_out += tg + ((eq_after < eq_take ? eq_after : eq_take) - taken_before_tile);
    base_eq = eq_after;
    __syncthreads();
  }
}

}  // namespace

hipError_t launch_topk(const float* scores, int64_t rows, int64_t N, int64_t K, int32_t* idx_out,
                       hipStream_t stream) {
  if (rows <= 0) return hipSuccess;
  topk_kernel<<<dim3((unsigned)rows), kTopkThreads, 0, stream>>>(scores, (int)N, (int)K, idx_out);
  return hipGetLastError();
}

}  // namespace pkv
