// Proxy importance scoring, pass 2 (paper Sec. 3: the softmax probabilities of Q K^T / sqrt(d),
// reduced over the query axis to one score per context key): per context key, the maximum over all
// reconstruction queries and over the query heads of the GQA group of exp(logit - lse).
//
// The logit matrix is never stored: Q K^T tiles are recomputed with v_mfma_f32_32x32x16_bf16.  The
// context keys of a workgroup (the "columns", 32*NCOL per wave) stay in registers as the MFMA B
// operand for the whole kernel; the queries (the "rows") stream through 16 KB LDS tiles.  With
// rows on the MFMA M axis a lane owns ONE key column and 16 query rows of every tile, so the
// maximum over queries runs inside a lane and needs one cross-lane step (lane ^ 32) at the end.
//
// With c = log2(e) / sqrt(d) the probability is p = 2^(c*s - L2), L2 the row's log2-sum-exp2.
// Pass 1 stores -L2 / c per query row; it is fed to the MFMA as the accumulator's initial value,
// so tiles come out as s - L2/c and need nothing but a running maximum (v_max3); one exp2 per
// context key is taken at the very end (max and exp commute).  The result is a probability: rounding in
// s - L2/c can carry it a few ulp past one, so it is clamped to one.
//
// Streaming: three LDS buffers and one barrier per tile.  While tile t is computed, tile t+2 goes
// from registers to LDS and tile t+3 is fetched from global memory into registers, all issued
// behind the first MFMAs of the tile.  The issue order inside a tile is written out by hand and
// pinned with scheduling barriers: the MFMAs of one pair of column sub-tiles alternate with the
// v_max3 that reduce the previous pair.
#include "kernels.hpp"
#include "score_common.hpp"

namespace pkv {
namespace {

// ---------------------------------------------------------------------------------------------
// pass 2: x[l, hs, n] = 2^(c * max_{g, i} (<q^{(hs*G+g)}_i, k_n> + neg_lse[l, hs*G+g, i]))
// one-dimensional grid over (KV group, key block of 128*NCOL keys), 256 threads; wave w owns context keys
// [n0 + 32*NCOL*w, +32*NCOL) as the resident B operand and streams all G*N_q queries.
// Rows past N_q carry -inf as their initial value, so every sub-tile is processed without a branch.
// Chains are handled in pairs (two column sub-tiles): the MFMAs of pair i are issued while the
// VALU reduces the accumulators of pair i-1 (also across tile boundaries).
// ---------------------------------------------------------------------------------------------
template <int D, int NCOL>
__global__ __launch_bounds__(256, D == 128 ? 1 : 2) void score_colmax_kernel(const uint16_t* __restrict__ q,
                                                               const uint16_t* __restrict__ k_ctx,
                                                               const float* __restrict__ neg_lse,
                                                               float* __restrict__ x, int L_s, int H_q, int G, int N, int N_q,
                                                               float c) {
  using C = ScoreCfg<D>;
  static_assert(NCOL % 2 == 0, "column sub-tiles are processed in pairs");
  __shared__ u32x4 lds[kNBuf * C::TILE_U4];
  __shared__ __attribute__((aligned(16))) float lds_nl[kNBuf * C::ROWS];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  constexpr int KB = 128 * NCOL;
  const int H_kv = H_q / G;
  const GroupBlock gb = group_block((N + KB - 1) / KB);  // a group's blocks: its key blocks (they stream the same queries)
  if (gb.group >= L_s * H_kv) return;
  const int l = gb.group / H_kv, hs = gb.group % H_kv;
  const int n0 = gb.item * KB;
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

  // tiles are fetched in order: head g = 0..G-1 of the group, query tile qt = 0..nqt-1
  const int nqt = (N_q + C::ROWS - 1) / C::ROWS;
  const int total = G * nqt;
  TileRegs<D> regs;
  float nl_reg = kNegInf;
  int fg = 0, fqt = 0;
  auto fetch_next = [&]() {
    const size_t head = (size_t)(l * H_q + hs * G + fg);
    tile_fetch<D>(regs, q + head * N_q * D, fqt * C::ROWS, N_q, tid);
    if (tid < C::ROWS) {
      const int i = fqt * C::ROWS + tid;
      nl_reg = i < N_q ? neg_lse[head * N_q + i] : kNegInf;
    }
    if (++fqt == nqt) {
      fqt = 0;
      ++fg;
    }
  };
  auto store = [&](int t) {
    tile_store<D>(regs, lds + (t % kNBuf) * C::TILE_U4, tid);
    if (tid < C::ROWS) lds_nl[(t % kNBuf) * C::ROWS + tid] = nl_reg;
  };
  fetch_next();
  store(0);
  if (total > 1) {
    fetch_next();
    store(1);
  }
  if (total > 2) fetch_next();
  __syncthreads();

  // Fragments and initial values of the current 32-row sub-tile, refilled in place: a[kk] right behind
  // the last MFMA that consumes it, init behind the pair's second MFMA (the last one that reads it).
  bf16x8 a[C::KK];
  f32x16 init;
  auto load_a = [&](int t, int s, int kk) {
    a[kk] = frag_read<D>(lds + (t % kNBuf) * C::TILE_U4, s * 32 + l32, kk * 2 + half);
  };
  auto load_init = [&](int t, int s) {
    const float* nl = lds_nl + (t % kNBuf) * C::ROWS;
    // accumulator rows of this lane: (r/4)*8 + half*4 + r%4
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(&nl[s * 32 + j * 8 + half * 4]);
      init[4 * j + 0] = v[0];
      init[4 * j + 1] = v[1];
      init[4 * j + 2] = v[2];
      init[4 * j + 3] = v[3];
    }
  };
#pragma unroll
  for (int kk = 0; kk < C::KK; ++kk) load_a(0, 0, kk);
  load_init(0, 0);
  f32x16 pend0 = splat16(kNegInf), pend1 = splat16(kNegInf);
  constexpr int NP = NCOL / 2;  // pairs per sub-tile
  for (int t = 0; t < total; ++t) {
    static_for<C::SUB * NP>([&](auto ic) {
      constexpr int i = decltype(ic)::value, s = i / NP, pr = i % NP;
      constexpr int pp = (pr + NP - 1) % NP;  // pair whose accumulators are pending
      constexpr int NM = 2 * C::KK;
      f32x16 c0, c1;
      MaxTree w0, w1;
      static_for<NM>([&](auto jc) {
        constexpr int j = decltype(jc)::value, kk = j / 2;
        if constexpr (j == 0) c0 = mfma_32x32x16(a[0], b[2 * pr][0], init);
        else if constexpr (j == 1) c1 = mfma_32x32x16(a[0], b[2 * pr + 1][0], init);
        else if constexpr (j % 2 == 0) c0 = mfma_32x32x16(a[kk], b[2 * pr][kk], c0);
        else c1 = mfma_32x32x16(a[kk], b[2 * pr + 1][kk], c1);
        if constexpr (i == 0 && j == 1) {
          // every wave has finished tile t-1: its buffer takes tile t+2, the registers take tile t+3
          __syncthreads();
          if (t + 2 < total) store(t + 2);
          if (t + 3 < total) fetch_next();
        }
        if constexpr (pr == NP - 1 && (j & 1)) {
          // last pair of the sub-tile: refill from the next sub-tile (sub-tile 0 of the next tile after the last)
          if constexpr (s + 1 < C::SUB) {
            load_a(t, s + 1, kk);
            if constexpr (j == 1) load_init(t, s + 1);
          } else {  // past the last tile this reads a stale buffer, harmlessly
            load_a(t + 1, 0, kk);
            if constexpr (j == 1) load_init(t + 1, 0);
          }
        }
        // the 16 v_max3 of the pending pair behind MFMAs 2, 3, ... (its last MFMA has retired by then)
        if constexpr (j >= 2) {
          constexpr int g = j - 2, lo = (16 * g) / (NM - 2), hi = (16 * (g + 1)) / (NM - 2);
          static_for<hi - lo>([&](auto vc) {
            constexpr int v = lo + decltype(vc)::value;
            if constexpr (v < 8) max_step<v>(pend0, w0, runmax[2 * pp]);
            else max_step<v - 8>(pend1, w1, runmax[2 * pp + 1]);
          });
        }
        __builtin_amdgcn_sched_barrier(0);
      });
      pend0 = c0;
      pend1 = c1;
    });
  }
  runmax[NCOL - 2] = max16_tree(pend0, runmax[NCOL - 2]);
  runmax[NCOL - 1] = max16_tree(pend1, runmax[NCOL - 1]);
#pragma unroll
  for (int cs = 0; cs < NCOL; ++cs) {
    const float m = __builtin_fmaxf(runmax[cs], swap_halves(runmax[cs]));
    if (half == 0 && kn[cs] < N) x[(size_t)(l * H_kv + hs) * N + kn[cs]] = __builtin_fminf(__builtin_amdgcn_exp2f(c * m), 1.0f);
  }
}

// ---------------------------------------------------------------------------------------------
// pass 2, sum form (the accumulation over the query axis that Sec. 3 prints for the proxy feature):
//   x[l, hs, n] = sum over the heads g of the group and all queries i of 2^(c * (<q_i, k_n> + neg_lse[l, h, i]))
// Same geometry as the max form (a workgroup owns 128*NCOL context keys as the resident B operand and
// streams all G*N_q queries, -L2/c as the accumulator's initial value), but every element is exponentiated
// and added: mul, exp2, add per element, so this kernel is bound by the vector ALU like pass 1.  A probability
// never exceeds one, so there is no reference to track.  Rows past N_q carry -inf and add zero.
// ---------------------------------------------------------------------------------------------
//
// CAUSAL: the proxy's own prefill attention (N_q == N, the keys are the sequence's own): query i sees keys n <= i, so a
// workgroup starts at the query tile that holds its first key and masks the tiles that the diagonal cuts.
template <int D, int NCOL, bool CAUSAL>
__global__ __launch_bounds__(256, 2) void score_colsum_kernel(const uint16_t* __restrict__ q,
                                                               const uint16_t* __restrict__ k_ctx,
                                                               const float* __restrict__ neg_lse,
                                                               float* __restrict__ x, int L_s, int H_q, int G, int N, int N_q,
                                                               float c) {
  using C = ScoreCfg<D>;
  __shared__ u32x4 lds[kNBuf * C::TILE_U4];
  __shared__ __attribute__((aligned(16))) float lds_nl[kNBuf * C::ROWS];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  constexpr int KB = 128 * NCOL;
  const int H_kv = H_q / G;
  const GroupBlock gb = group_block((N + KB - 1) / KB);  // a group's blocks: its key blocks (they stream the same queries)
  if (gb.group >= L_s * H_kv) return;
  const int l = gb.group / H_kv, hs = gb.group % H_kv;
  const int n0 = gb.item * KB;
  const uint16_t* kc = k_ctx + (size_t)(l * H_kv + hs) * N * D;

  bf16x8 b[NCOL][C::KK];
  int kn[NCOL];
  float colsum[NCOL];
#pragma unroll
  for (int cs = 0; cs < NCOL; ++cs) {
    kn[cs] = n0 + (wave * NCOL + cs) * 32 + l32;
    const int row = kn[cs] < N ? kn[cs] : N - 1;
#pragma unroll
    for (int kk = 0; kk < C::KK; ++kk)
      b[cs][kk] = as_bf16x8(*reinterpret_cast<const u32x4*>(kc + (size_t)row * D + kk * 16 + half * 8));
    colsum[cs] = 0.0f;
  }

  // tiles are fetched in order: head g = 0..G-1 of the group, query tile qt = 0..nqt-1
  const int nqt = (N_q + C::ROWS - 1) / C::ROWS;
  const int qt_first = CAUSAL ? n0 / C::ROWS : 0;  // KB is a multiple of ROWS
  const int total = G * (nqt - qt_first);
  TileRegs<D> regs;
  float nl_reg = kNegInf;
  int fg = 0, fqt = qt_first;
  auto fetch_next = [&]() {
    const size_t head = (size_t)(l * H_q + hs * G + fg);
    tile_fetch<D>(regs, q + head * N_q * D, fqt * C::ROWS, N_q, tid);
    if (tid < C::ROWS) {
      const int i = fqt * C::ROWS + tid;
      nl_reg = i < N_q ? neg_lse[head * N_q + i] : kNegInf;
    }
    if (++fqt == nqt) {
      fqt = qt_first;
      ++fg;
    }
  };
  auto store = [&](int t) {
    tile_store<D>(regs, lds + (t % kNBuf) * C::TILE_U4, tid);
    if (tid < C::ROWS) lds_nl[(t % kNBuf) * C::ROWS + tid] = nl_reg;
  };
  fetch_next();
  store(0);
  if (total > 1) {
    fetch_next();
    store(1);
  }
  if (total > 2) fetch_next();

  int cqt = qt_first;  // query tile of step t
  for (int t = 0; t < total; ++t) {
    // every wave has finished tile t-1: its buffer takes tile t+2, the registers take tile t+3
    __syncthreads();
    if (t + 2 < total) store(t + 2);
    if (t + 3 < total) fetch_next();
    const u32x4* buf = lds + (t % kNBuf) * C::TILE_U4;
    const float* nl = lds_nl + (t % kNBuf) * C::ROWS;
    const int row0 = cqt * C::ROWS;
    const bool diag = CAUSAL && row0 < n0 + KB - 1;  // some query of the tile lies before some key of the block
    if (++cqt == nqt) cqt = qt_first;
#pragma unroll
    for (int s = 0; s < C::SUB; ++s) {
      bf16x8 a[C::KK];
#pragma unroll
      for (int kk = 0; kk < C::KK; ++kk) a[kk] = frag_read<D>(buf, s * 32 + l32, kk * 2 + half);
      // accumulator rows of this lane: (r/4)*8 + half*4 + r%4
      f32x16 init;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(&nl[s * 32 + j * 8 + half * 4]);
        init[4 * j + 0] = v[0];
        init[4 * j + 1] = v[1];
        init[4 * j + 2] = v[2];
        init[4 * j + 3] = v[3];
      }
#pragma unroll
      for (int cp = 0; cp < NCOL; cp += 2) {
        f32x16 acc[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          acc[e] = init;
#pragma unroll
          for (int kk = 0; kk < C::KK; ++kk) acc[e] = mfma_32x32x16(a[kk], b[cp + e][kk], acc[e]);
        }
        if (diag) {
#pragma unroll
          for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int i = row0 + s * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
              acc[e][r] = i >= kn[cp + e] ? acc[e][r] : kNegInf;
            }
        }
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          float s0 = __builtin_amdgcn_exp2f(acc[e][0] * c), s1 = __builtin_amdgcn_exp2f(acc[e][1] * c);
          float s2 = __builtin_amdgcn_exp2f(acc[e][2] * c), s3 = __builtin_amdgcn_exp2f(acc[e][3] * c);
#pragma unroll
          for (int r = 4; r < 16; r += 4) {
            s0 += __builtin_amdgcn_exp2f(acc[e][r + 0] * c);
            s1 += __builtin_amdgcn_exp2f(acc[e][r + 1] * c);
            s2 += __builtin_amdgcn_exp2f(acc[e][r + 2] * c);
            s3 += __builtin_amdgcn_exp2f(acc[e][r + 3] * c);
          }
          colsum[cp + e] += (s0 + s1) + (s2 + s3);
        }
      }
    }
  }
#pragma unroll
  for (int cs = 0; cs < NCOL; ++cs) {
    const float tot = colsum[cs] + swap_halves(colsum[cs]);
    if (half == 0 && kn[cs] < N) x[(size_t)(l * H_kv + hs) * N + kn[cs]] = tot;
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

hipError_t launch_score_colsum(const uint16_t* q, const uint16_t* k_ctx, const float* neg_lse, float* x, int L_s,
                               int H_q, int H_kv, int d, int64_t N, int64_t N_q, bool causal, hipStream_t stream) {
  const int G = H_q / H_kv;
  const float c = 1.4426950408889634f / sqrtf((float)d);
  constexpr int NCOL = 2;
  if (causal && N != N_q) return hipErrorInvalidValue;
  const unsigned grid = group_grid((int64_t)L_s * H_kv, (N + 128 * NCOL - 1) / (128 * NCOL));
  if (grid == 0) return hipErrorInvalidValue;
  const int n = (int)N, nq = (int)N_q;
  if (d == 64) {
    if (causal) score_colsum_kernel<64, NCOL, true><<<grid, 256, 0, stream>>>(q, k_ctx, neg_lse, x, L_s, H_q, G, n, nq, c);
    else score_colsum_kernel<64, NCOL, false><<<grid, 256, 0, stream>>>(q, k_ctx, neg_lse, x, L_s, H_q, G, n, nq, c);
  } else {
    if (causal) score_colsum_kernel<128, NCOL, true><<<grid, 256, 0, stream>>>(q, k_ctx, neg_lse, x, L_s, H_q, G, n, nq, c);
    else score_colsum_kernel<128, NCOL, false><<<grid, 256, 0, stream>>>(q, k_ctx, neg_lse, x, L_s, H_q, G, n, nq, c);
  }
  return hipGetLastError();
}

hipError_t launch_score_colmax(const uint16_t* q, const uint16_t* k_ctx, const float* neg_lse, float* x, int L_s,
                               int H_q, int H_kv, int d, int64_t N, int64_t N_q, hipStream_t stream) {
  const int G = H_q / H_kv;
  const float c = 1.4426950408889634f / sqrtf((float)d);
  if (d == 64) {
    constexpr int NCOL = 4;
    const unsigned grid = group_grid((int64_t)L_s * H_kv, (N + 128 * NCOL - 1) / (128 * NCOL));
    if (grid == 0) return hipErrorInvalidValue;
    score_colmax_kernel<64, NCOL><<<grid, 256, 0, stream>>>(q, k_ctx, neg_lse, x, L_s, H_q, G, (int)N, (int)N_q, c);
  } else {
    // one workgroup per CU (the resident keys of 4 column sub-tiles alone take 128 registers): a wave has the SIMD's
    // whole register file, and the pinned issue order keeps the matrix pipe fed without a second wave
    constexpr int NCOL = 4;
    const unsigned grid = group_grid((int64_t)L_s * H_kv, (N + 128 * NCOL - 1) / (128 * NCOL));
    if (grid == 0) return hipErrorInvalidValue;
    score_colmax_kernel<128, NCOL><<<grid, 256, 0, stream>>>(q, k_ctx, neg_lse, x, L_s, H_q, G, (int)N, (int)N_q, c);
  }
  return hipGetLastError();
}

}  // namespace pkv
