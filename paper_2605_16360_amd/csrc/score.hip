// Proxy importance scoring (paper Sec. 3: per-query-row softmax of Q K^T / sqrt(d), reduced over
// the query axis to one score per context key), as two flash-style passes that never store the
// N_q x N logit matrix:
//   pass 1  score_lse_kernel     row log-sum-exp of every reconstruction query
//   pass 2  score_colmax_kernel  per context key, the maximum over queries and over the heads of
//                                the GQA group of exp(logit - lse)
// Both passes compute 32x32 tiles of K Q^T (pass 1) / Q K^T (pass 2) with
// v_mfma_f32_32x32x16_bf16.  One operand (the "columns": 32*NCOL per wave) stays in registers for
// the whole kernel, the other (the "rows") is streamed through a 16 KB LDS tile that is fetched
// from global memory one iteration ahead.  With rows on the MFMA M axis a lane owns ONE column and
// 16 rows of every tile, so both reductions (sum over keys in pass 1, max over queries in pass 2)
// run inside a lane and need a single cross-lane step at the very end.
//
// Exponentials are taken in base 2: with c = log2(e) / sqrt(d), softmax probability
// p = 2^(c*s - L2), L2 = log2(sum 2^(c*s)).  Pass 1 stores -L2 / c per query row; pass 2 feeds
// that value to the MFMA as the accumulator's initial value, so its tiles come out as s - L2/c
// and need nothing but a running maximum; one exp2 per context key is taken at the very end
// (max and exp commute).
#include "common.hpp"
#include "kernels.hpp"

namespace pkv {
namespace {

template <int D>
struct ScoreCfg {
  static constexpr int CPR = D / 8;             // 16-byte chunks per row
  static constexpr int ROWS = 8192 / D;         // rows of one streamed tile (16 KB)
  static constexpr int SUB = ROWS / 32;         // 32-row sub-tiles per tile
  static constexpr int KK = D / 16;             // MFMA k-steps per 32x32 tile
  static constexpr int LOADS = ROWS * CPR / 256;  // 16-byte chunks staged per thread and tile
};

// XOR swizzle of the 16-byte chunk index inside a row; keeps both the 16-byte tile stores and the
// MFMA fragment reads (32 consecutive rows, same chunk) spread over all LDS banks.
template <int D>
__device__ __forceinline__ int swz(int row) {
  if constexpr (D == 64) return (row & 7) ^ ((row >> 3) & 1);
  else return row & 15;
}

template <int D>
struct TileRegs {
  u32x4 v[ScoreCfg<D>::LOADS];
};

// Fetches rows [row0, row0 + ROWS) of a [*, D] bf16 matrix; rows >= row_limit re-read the last
// valid row so that every access stays inside the matrix (the caller masks them).
template <int D>
__device__ __forceinline__ void tile_fetch(TileRegs<D>& r, const uint16_t* base, int row0, int row_limit, int tid) {
  using C = ScoreCfg<D>;
#pragma unroll
  for (int i = 0; i < C::LOADS; ++i) {
    const int id = tid + 256 * i;
    const int row = id / C::CPR, ch = id % C::CPR;
    int grow = row0 + row;
    grow = grow < row_limit ? grow : row_limit - 1;
    r.v[i] = *reinterpret_cast<const u32x4*>(base + (size_t)grow * D + ch * 8);
  }
}

template <int D>
__device__ __forceinline__ void tile_store(const TileRegs<D>& r, u32x4* lds, int tid) {
  using C = ScoreCfg<D>;
#pragma unroll
  for (int i = 0; i < C::LOADS; ++i) {
    const int id = tid + 256 * i;
    const int row = id / C::CPR, ch = id % C::CPR;
    lds[row * C::CPR + (ch ^ swz<D>(row))] = r.v[i];
  }
}

template <int D>
__device__ __forceinline__ bf16x8 frag_read(const u32x4* lds, int row, int ch) {
  return as_bf16x8(lds[row * ScoreCfg<D>::CPR + (ch ^ swz<D>(row))]);
}

__device__ __forceinline__ float max16(const f32x16& a, float seed) {
  float m = max3f(seed, a[0], a[1]);
  m = max3f(m, a[2], a[3]);
  m = max3f(m, a[4], a[5]);
  m = max3f(m, a[6], a[7]);
  m = max3f(m, a[8], a[9]);
  m = max3f(m, a[10], a[11]);
  m = max3f(m, a[12], a[13]);
  m = max3f(m, a[14], a[15]);
  return m;
}

constexpr float kNegInf = -__builtin_huge_valf();
constexpr float kRescaleGap = 64.0f;  // a lane re-bases its partial sum once a logit exceeds its reference by 2^64

// ---------------------------------------------------------------------------------------------
// pass 1: neg_lse[l, h, i] = -L2(i) / c
// grid (ceil(N_q / (128*NCOL)), H_q, L_s), 256 threads; wave w owns queries
// [i0 + 32*NCOL*w, +32*NCOL) as the resident B operand.
// ---------------------------------------------------------------------------------------------
template <int D, int NCOL>
__global__ __launch_bounds__(256, 2) void score_lse_kernel(const uint16_t* __restrict__ q,
                                                            const uint16_t* __restrict__ k_ctx,
                                                            const uint16_t* __restrict__ k_rec,
                                                            float* __restrict__ neg_lse, int H_q, int G, int N,
                                                            int N_q, int chunk, float c, float inv_c) {
  using C = ScoreCfg<D>;
  __shared__ u32x4 lds[C::ROWS * C::CPR];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int h = blockIdx.y, l = blockIdx.z, H_kv = H_q / G, hs = h / G;
  constexpr int QB = 128 * NCOL;
  const int i0 = blockIdx.x * QB;
  const uint16_t* qh = q + (size_t)(l * H_q + h) * N_q * D;
  const uint16_t* kc = k_ctx + (size_t)(l * H_kv + hs) * N * D;
  const uint16_t* kr = k_rec + (size_t)(l * H_kv + hs) * N_q * D;

  bf16x8 b[NCOL][C::KK];
  int qi[NCOL], qlo[NCOL];
#pragma unroll
  for (int cs = 0; cs < NCOL; ++cs) {
    qi[cs] = i0 + (wave * NCOL + cs) * 32 + l32;
    qlo[cs] = (qi[cs] / chunk) * chunk;
    const int row = qi[cs] < N_q ? qi[cs] : N_q - 1;
#pragma unroll
    for (int kk = 0; kk < C::KK; ++kk)
      b[cs][kk] = as_bf16x8(*reinterpret_cast<const u32x4*>(qh + (size_t)row * D + kk * 16 + half * 8));
  }
  float m_ref[NCOL], lsum[NCOL];
#pragma unroll
  for (int cs = 0; cs < NCOL; ++cs) {
    m_ref[cs] = -1.0e30f;
    lsum[cs] = 0.0f;
  }

  const int n_ctx = (N + C::ROWS - 1) / C::ROWS;
  const int i_end = (i0 + QB < N_q ? i0 + QB : N_q);  // one past the block's last query
  const int rec_lo = (i0 / chunk) * chunk;            // first reconstruction key any query of the block sees
  const int n_rec = (i_end - rec_lo + C::ROWS - 1) / C::ROWS;
  const int total = n_ctx + n_rec;
  const int wave_i_lo = i0 + wave * NCOL * 32;  // first query of this wave

  TileRegs<D> regs;
  tile_fetch<D>(regs, kc, 0, N, tid);
  for (int t = 0; t < total; ++t) {
    __syncthreads();
    tile_store<D>(regs, lds, tid);
    __syncthreads();
    if (t + 1 < total) {
      if (t + 1 < n_ctx) tile_fetch<D>(regs, kc, (t + 1) * C::ROWS, N, tid);
      else tile_fetch<D>(regs, kr, rec_lo + (t + 1 - n_ctx) * C::ROWS, i_end, tid);
    }
    const bool is_rec = t >= n_ctx;
    const int row0 = is_rec ? rec_lo + (t - n_ctx) * C::ROWS : t * C::ROWS;
    const int limit = is_rec ? i_end : N;
#pragma unroll
    for (int s = 0; s < C::SUB; ++s) {
      const int jbase = row0 + s * 32;
      if (jbase >= limit) break;
      if (is_rec && jbase > wave_i_lo + NCOL * 32 - 1) break;  // keys after the wave's last query
      bf16x8 a[C::KK];
#pragma unroll
      for (int kk = 0; kk < C::KK; ++kk) a[kk] = frag_read<D>(lds, s * 32 + l32, kk * 2 + half);
#pragma unroll
      for (int cs = 0; cs < NCOL; ++cs) {
        const int cs_i_lo = wave_i_lo + cs * 32;
        if (is_rec && jbase > cs_i_lo + 31) continue;  // wave-uniform
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
        for (int kk = 0; kk < C::KK; ++kk) acc = mfma_32x32x16(a[kk], b[cs][kk], acc);
        // a mask is needed on a ragged context tail and wherever causality or a chunk boundary cuts
        // the tile: not when every key of the sub-tile is <= the first query and >= every query's chunk start
        const bool cut = is_rec ? !(jbase + 31 <= cs_i_lo && jbase >= ((cs_i_lo + 31) / chunk) * chunk)
                                : (jbase + 32 > limit);
        if (cut) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = jbase + (r >> 2) * 8 + half * 4 + (r & 3);
            const bool vis = is_rec ? (j <= qi[cs] && j >= qlo[cs]) : (j < N);
            acc[r] = vis ? acc[r] : kNegInf;
          }
        }
        const float tm = max16(acc, kNegInf) * c;
        const bool up = tm - m_ref[cs] > kRescaleGap;
        if (__builtin_amdgcn_ballot_w64(up)) {
          const float nm = up ? tm : m_ref[cs];
          lsum[cs] *= __builtin_amdgcn_exp2f(m_ref[cs] - nm);
          m_ref[cs] = nm;
        }
        const float nref = -m_ref[cs];
        float s0 = 0.0f, s1 = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          s0 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r], c, nref));
          s1 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r + 1], c, nref));
        }
        lsum[cs] += s0 + s1;
      }
    }
  }
#pragma unroll
  for (int cs = 0; cs < NCOL; ++cs) {
    const float m2 = swap_halves(m_ref[cs]), l2 = swap_halves(lsum[cs]);
    const float m = __builtin_fmaxf(m_ref[cs], m2);
    const float tot = lsum[cs] * __builtin_amdgcn_exp2f(m_ref[cs] - m) + l2 * __builtin_amdgcn_exp2f(m2 - m);
    const float L2 = m + __builtin_amdgcn_logf(tot);
    if (half == 0 && qi[cs] < N_q) neg_lse[(size_t)(l * H_q + h) * N_q + qi[cs]] = -L2 * inv_c;
  }
}

// ---------------------------------------------------------------------------------------------
// pass 2: x[l, hs, n] = 2^(c * max_{g, i} (<q^{(hs*G+g)}_i, k_n> + neg_lse[l, hs*G+g, i]))
// grid (ceil(N / (128*NCOL)), H_kv, L_s), 256 threads; wave w owns context keys
// [n0 + 32*NCOL*w, +32*NCOL) as the resident B operand and streams all G*N_q queries.
// ---------------------------------------------------------------------------------------------
template <int D, int NCOL>
__global__ __launch_bounds__(256, 2) void score_colmax_kernel(const uint16_t* __restrict__ q,
                                                               const uint16_t* __restrict__ k_ctx,
                                                               const float* __restrict__ neg_lse,
                                                               float* __restrict__ x, int H_q, int G, int N, int N_q,
                                                               float c) {
  using C = ScoreCfg<D>;
  __shared__ u32x4 lds[C::ROWS * C::CPR];
  __shared__ __attribute__((aligned(16))) float lds_nl[C::ROWS];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int hs = blockIdx.y, l = blockIdx.z, H_kv = H_q / G;
  constexpr int KB = 128 * NCOL;
  const int n0 = blockIdx.x * KB;
  const uint16_t* kc = k_ctx + (size_t)(l * H_kv + hs) * N * D;

  bf16x8 b[NCOL][C::KK];
  int kn[NCOL];
#pragma unroll
  for (int cs = 0; cs < NCOL; ++cs) {
    kn[cs] = n0 + (wave * NCOL + cs) * 32 + l32;
    const int row = kn[cs] < N ? kn[cs] : N - 1;
#pragma unroll
    for (int kk = 0; kk < C::KK; ++kk)
      b[cs][kk] = as_bf16x8(*reinterpret_cast<const u32x4*>(kc + (size_t)row * D + kk * 16 + half * 8));
  }
  float runmax[NCOL];
#pragma unroll
  for (int cs = 0; cs < NCOL; ++cs) runmax[cs] = kNegInf;

  const int nqt = (N_q + C::ROWS - 1) / C::ROWS;
  const int total = G * nqt;
  TileRegs<D> regs;
  float nl_reg = kNegInf;
  auto fetch = [&](int t) {
    const int g = t / nqt, qt = t - g * nqt;
    const size_t head = (size_t)(l * H_q + hs * G + g);
    tile_fetch<D>(regs, q + head * N_q * D, qt * C::ROWS, N_q, tid);
    if (tid < C::ROWS) {
      const int i = qt * C::ROWS + tid;
      nl_reg = i < N_q ? neg_lse[head * N_q + i] : kNegInf;
    }
  };
  fetch(0);
  for (int t = 0; t < total; ++t) {
    __syncthreads();
    tile_store<D>(regs, lds, tid);
    if (tid < C::ROWS) lds_nl[tid] = nl_reg;
    __syncthreads();
    if (t + 1 < total) fetch(t + 1);
    const int row0 = (t % nqt) * C::ROWS;
#pragma unroll
    for (int s = 0; s < C::SUB; ++s) {
      if (row0 + s * 32 >= N_q) break;
      bf16x8 a[C::KK];
#pragma unroll
      for (int kk = 0; kk < C::KK; ++kk) a[kk] = frag_read<D>(lds, s * 32 + l32, kk * 2 + half);
      // accumulator rows of this lane: (r/4)*8 + half*4 + r%4
      f32x16 init;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(&lds_nl[s * 32 + j * 8 + half * 4]);
        init[4 * j + 0] = v[0];
        init[4 * j + 1] = v[1];
        init[4 * j + 2] = v[2];
        init[4 * j + 3] = v[3];
      }
#pragma unroll
      for (int cs = 0; cs < NCOL; ++cs) {
        f32x16 acc = mfma_32x32x16(a[0], b[cs][0], init);
#pragma unroll
        for (int kk = 1; kk < C::KK; ++kk) acc = mfma_32x32x16(a[kk], b[cs][kk], acc);
        runmax[cs] = max16(acc, runmax[cs]);
      }
    }
  }
#pragma unroll
  for (int cs = 0; cs < NCOL; ++cs) {
    const float m = __builtin_fmaxf(runmax[cs], swap_halves(runmax[cs]));
    if (half == 0 && kn[cs] < N) x[(size_t)(l * H_kv + hs) * N + kn[cs]] = __builtin_amdgcn_exp2f(c * m);
  }
}

__global__ void f32_to_bf16_kernel(const float* __restrict__ in, uint16_t* __restrict__ out, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) out[i] = f32_to_bf16_bits(in[i]);
}

}  // namespace

hipError_t launch_f32_to_bf16(const float* in, uint16_t* out, int64_t n, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  const int blocks = (int)((n + 255) / 256 < 65536 ? (n + 255) / 256 : 65536);
  f32_to_bf16_kernel<<<blocks, 256, 0, stream>>>(in, out, n);
  return hipGetLastError();
}

hipError_t launch_score_lse(const uint16_t* q, const uint16_t* k_ctx, const uint16_t* k_rec, float* neg_lse,
                            int L_s, int H_q, int H_kv, int d, int64_t N, int64_t N_q, int chunk,
                            hipStream_t stream) {
  const int G = H_q / H_kv;
  const float c = 1.4426950408889634f / sqrtf((float)d), inv_c = 1.0f / c;
  constexpr int NCOL = 2;
  dim3 grid((unsigned)((N_q + 128 * NCOL - 1) / (128 * NCOL)), (unsigned)H_q, (unsigned)L_s);
  if (d == 64)
    score_lse_kernel<64, NCOL><<<grid, 256, 0, stream>>>(q, k_ctx, k_rec, neg_lse, H_q, G, (int)N, (int)N_q, chunk, c, inv_c);
  else
    score_lse_kernel<128, NCOL><<<grid, 256, 0, stream>>>(q, k_ctx, k_rec, neg_lse, H_q, G, (int)N, (int)N_q, chunk, c, inv_c);
  return hipGetLastError();
}

hipError_t launch_score_colmax(const uint16_t* q, const uint16_t* k_ctx, const float* neg_lse, float* x, int L_s,
                               int H_q, int H_kv, int d, int64_t N, int64_t N_q, hipStream_t stream) {
  const int G = H_q / H_kv;
  const float c = 1.4426950408889634f / sqrtf((float)d);
  if (d == 64) {
    constexpr int NCOL = 4;
    dim3 grid((unsigned)((N + 128 * NCOL - 1) / (128 * NCOL)), (unsigned)H_kv, (unsigned)L_s);
    score_colmax_kernel<64, NCOL><<<grid, 256, 0, stream>>>(q, k_ctx, neg_lse, x, H_q, G, (int)N, (int)N_q, c);
  } else {
    constexpr int NCOL = 2;
    dim3 grid((unsigned)((N + 128 * NCOL - 1) / (128 * NCOL)), (unsigned)H_kv, (unsigned)L_s);
    score_colmax_kernel<128, NCOL><<<grid, 256, 0, stream>>>(q, k_ctx, neg_lse, x, H_q, G, (int)N, (int)N_q, c);
  }
  return hipGetLastError();
}

}  // namespace pkv
