// Proxy importance scoring, pass 1 (paper Sec. 3: softmax of Q K^T / sqrt(d) per query row): the
// row log-sum-exp of every reconstruction query over the N context keys plus the reconstruction
// keys of its own chunk up to and including itself.
//
// The logit matrix is never stored: K Q^T tiles are computed with v_mfma_f32_32x32x16_bf16.  The
// queries of a workgroup (the "columns", 32*NCOL per wave) stay in registers as the MFMA B operand
// for the whole kernel; the keys (the "rows") stream through 16 KB LDS tiles.  With rows on the
// MFMA M axis a lane owns ONE query column and 16 key rows of every tile, so the sum over keys runs
// inside a lane and needs one cross-lane step (lane ^ 32) at the end.
//
// With c = log2(e) / sqrt(d) the kernel accumulates lsum = sum 2^(c*s - m_ref) per lane and column.
// The vector ALU, not the matrix pipe, bounds this pass (one v_exp_f32 costs two ALU slots), so the
// work per element is cut to the three instructions that cannot be avoided (fma, exp2, add): no
// running maximum is tracked.  The reference m_ref is an attained logit of the column; it is only
// replaced when the sum of one 16-element chain leaves [0, 2^64), which the first chain of every
// column does by construction (m_ref starts at -1e30) and later chains practically never do.  A term
// can exceed the reference by up to 2^64 and every term far below it is negligible against the
// attained one, so neither overflow nor underflow loses anything.  The kernel writes -L2 / c per
// row, L2 = m_ref + log2(lsum), which pass 2 uses as the accumulator's initial value.
//
// Streaming: three LDS buffers and one barrier per tile.  While tile t is computed, tile t+2 goes
// from registers to LDS and tile t+3 is fetched from global memory into registers.
#include "kernels.hpp"
#include "score_common.hpp"

namespace pkv {
namespace {

// A chain's sum outside [0, kRebase) makes its lanes take a new reference.
constexpr float kRebase = 1.8446744e19f;  // 2^64
// Interior tiles are summed without any check; a column's running sum outside [0, kTileRedo) afterwards
// undoes the tile and sums it again chain by chain with the check.
constexpr float kTileRedo = 1.2676506e30f;  // 2^100

template <int D, int NCOL, int MINB>
__global__ __launch_bounds__(256, MINB) void score_lse_kernel(const uint16_t* __restrict__ q,
                                                               const uint16_t* __restrict__ k_ctx,
                                                               const uint16_t* __restrict__ k_rec,
                                                               float* __restrict__ neg_lse, int H_q, int G, int N,
                                                               int N_q, int chunk, float c, float inv_c) {
  using C = ScoreCfg<D>;
  __shared__ u32x4 lds[kNBuf * C::TILE_U4];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int h = blockIdx.y, l = blockIdx.z, H_kv = H_q / G, hs = h / G;
  constexpr int QB = 128 * NCOL;
  const int i0 = blockIdx.x * QB;
  const uint16_t* qh = q + (size_t)(l * H_q + h) * N_q * D;
  const uint16_t* kc = k_ctx + (size_t)(l * H_kv + hs) * N * D;
  const uint16_t* kr = k_rec + (size_t)(l * H_kv + hs) * N_q * D;

  // resident B operand: the wave's queries
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
  float nref[NCOL], lsum[NCOL];  // nref = -m_ref
#pragma unroll
  for (int cs = 0; cs < NCOL; ++cs) {
    nref[cs] = 1.0e30f;
    lsum[cs] = 0.0f;
  }

  // tile list: the context tiles, then the reconstruction tiles from the start of the block's chunk to
  // its last query
  const int n_ctx = (N + C::ROWS - 1) / C::ROWS;
  const int i_end = (i0 + QB < N_q ? i0 + QB : N_q);  // one past the block's last query
  const int rec_lo = (i0 / chunk) * chunk;            // first reconstruction key any query of the block sees
  const int n_rec = (i_end - rec_lo + C::ROWS - 1) / C::ROWS;
  const int total = n_ctx + n_rec;
  const int wave_i_lo = i0 + wave * NCOL * 32;  // first query of this wave
  TileRegs<D> regs;
  auto fetch = [&](int t) {
    if (t < n_ctx) tile_fetch<D>(regs, kc, t * C::ROWS, N, tid);
    else tile_fetch<D>(regs, kr, rec_lo + (t - n_ctx) * C::ROWS, i_end, tid);
  };

  // sum of one chain: 16 x (fma, exp2, add); re-based when it leaves [0, 2^64)
  auto accumulate = [&](const f32x16& acc, int cs) {
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
#pragma unroll
    for (int r = 0; r < 16; r += 4) {
      s0 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r + 0], c, nref[cs]));
      s1 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r + 1], c, nref[cs]));
      s2 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r + 2], c, nref[cs]));
      s3 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r + 3], c, nref[cs]));
    }
    float sum = (s0 + s1) + (s2 + s3);
    const bool bad = !(sum < kRebase);  // too large, infinite or NaN
    if (__builtin_amdgcn_ballot_w64(bad)) {
      if (bad) {
        const float tm = max16_tree(acc, kNegInf) * c;
        // all 16 rows masked: keep the reference (their terms are zero under any finite reference)
        const float nm = tm > -1.0e30f ? tm : -nref[cs];
        lsum[cs] *= __builtin_amdgcn_exp2f(-nref[cs] - nm);
        nref[cs] = -nm;
        sum = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r], c, nref[cs]));
      }
    }
    lsum[cs] += sum;
  };

  // sum of one chain, no check: 16 x (fma, exp2, add)
  auto fast_sum = [&](const f32x16& acc, int cs) {
    float s0 = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[0], c, nref[cs]));
    float s1 = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[1], c, nref[cs]));
    float s2 = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[2], c, nref[cs]));
    float s3 = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[3], c, nref[cs]));
#pragma unroll
    for (int r = 4; r < 16; r += 4) {
      s0 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r + 0], c, nref[cs]));
      s1 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r + 1], c, nref[cs]));
      s2 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r + 2], c, nref[cs]));
      s3 += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[r + 3], c, nref[cs]));
    }
    return (s0 + s1) + (s2 + s3);
  };
  // the keys of an interior tile, visible to every query of the block, summed without checks
  auto interior_tile = [&](const u32x4* buf) {
#pragma unroll
    for (int s = 0; s < C::SUB; ++s) {
      bf16x8 a[C::KK];
#pragma unroll
      for (int kk = 0; kk < C::KK; ++kk) a[kk] = frag_read<D>(buf, s * 32 + l32, kk * 2 + half);
      f32x16 acc[NCOL];
#pragma unroll
      for (int cs = 0; cs < NCOL; ++cs) {
        acc[cs] = splat16(0.0f);
#pragma unroll
        for (int kk = 0; kk < C::KK; ++kk) acc[cs] = mfma_32x32x16(a[kk], b[cs][kk], acc[cs]);
      }
#pragma unroll
      for (int cs = 0; cs < NCOL; ++cs) lsum[cs] += fast_sum(acc[cs], cs);
    }
  };

  fetch(0);
  tile_store<D>(regs, lds, tid);
  if (total > 1) {
    fetch(1);
    tile_store<D>(regs, lds + C::TILE_U4, tid);
  }
  if (total > 2) fetch(2);

  for (int t = 0; t < total; ++t) {
    // every wave has finished tile t-1: its buffer takes tile t+2, the registers take tile t+3
    __syncthreads();
    if (t + 2 < total) tile_store<D>(regs, lds + ((t + 2) % kNBuf) * C::TILE_U4, tid);
    if (t + 3 < total) fetch(t + 3);
    const u32x4* buf = lds + (t % kNBuf) * C::TILE_U4;
    const bool is_rec = t >= n_ctx;
    const int row0 = is_rec ? rec_lo + (t - n_ctx) * C::ROWS : t * C::ROWS;
    // interior tile: summed without checks, and again chain by chain with them if a sum went out of
    // range (the very first tile does: the reference starts at -1e30)
    // a reconstruction tile is interior too when all its keys lie at or before the block's first query and inside the
    // chunk of its last one (then inside every query's chunk)
    bool careful = is_rec ? !(row0 + C::ROWS - 1 <= i0 && row0 >= ((i_end - 1) / chunk) * chunk) : (row0 + C::ROWS > N);
    if (!careful) {
      float before[NCOL];
#pragma unroll
      for (int cs = 0; cs < NCOL; ++cs) before[cs] = lsum[cs];
      interior_tile(buf);
      bool bad = false;
#pragma unroll
      for (int cs = 0; cs < NCOL; ++cs) bad |= !(lsum[cs] < kTileRedo);
      if (__builtin_amdgcn_ballot_w64(bad)) {
#pragma unroll
        for (int cs = 0; cs < NCOL; ++cs) lsum[cs] = before[cs];
        careful = true;
      }
    }
    if (careful) {
      // ragged context tail, a reconstruction tile where causality and chunk boundaries cut, or a redo
      const int limit = is_rec ? i_end : N;
#pragma unroll
      for (int s = 0; s < C::SUB; ++s) {
        const int jbase = row0 + s * 32;
        if (jbase >= limit) break;
        if (is_rec && jbase > wave_i_lo + NCOL * 32 - 1) break;  // keys after the wave's last query
        bf16x8 a[C::KK];
#pragma unroll
        for (int kk = 0; kk < C::KK; ++kk) a[kk] = frag_read<D>(buf, s * 32 + l32, kk * 2 + half);
#pragma unroll
        for (int cs = 0; cs < NCOL; ++cs) {
          const int cs_i_lo = wave_i_lo + cs * 32;
          if (is_rec && jbase > cs_i_lo + 31) continue;  // wave-uniform: keys after the sub-tile's last query
          f32x16 acc = splat16(0.0f);
#pragma unroll
          for (int kk = 0; kk < C::KK; ++kk) acc = mfma_32x32x16(a[kk], b[cs][kk], acc);
          // no mask needed when every key of the sub-tile is <= the first query and >= every query's chunk start
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
          accumulate(acc, cs);
        }
      }
    }
  }
#pragma unroll
  for (int cs = 0; cs < NCOL; ++cs) {
    const float m1 = -nref[cs];
    const float m2 = swap_halves(m1), l2 = swap_halves(lsum[cs]);
    const float m = __builtin_fmaxf(m1, m2);
    const float tot = lsum[cs] * __builtin_amdgcn_exp2f(m1 - m) + l2 * __builtin_amdgcn_exp2f(m2 - m);
    const float L2 = m + __builtin_amdgcn_logf(tot);
    if (half == 0 && qi[cs] < N_q) neg_lse[(size_t)(l * H_q + h) * N_q + qi[cs]] = -L2 * inv_c;
  }
}

}  // namespace

hipError_t launch_score_lse(const uint16_t* q, const uint16_t* k_ctx, const uint16_t* k_rec, float* neg_lse,
                            int L_s, int H_q, int H_kv, int d, int64_t N, int64_t N_q, int chunk,
                            hipStream_t stream) {
  const int G = H_q / H_kv;
  const float c = 1.4426950408889634f / sqrtf((float)d), inv_c = 1.0f / c;
  // two column sub-tiles per wave; three workgroups per CU at d = 64 (at most 168 registers), two at d = 128
  constexpr int NCOL = 2;
  // the query blocks of a head are dealt over all XCDs (measured: fewer L2 misses than one KV group per XCD, whose
  // blocks drift apart along a key stream slightly larger than the L2)
  dim3 grid((unsigned)((N_q + 128 * NCOL - 1) / (128 * NCOL)), (unsigned)H_q, (unsigned)L_s);
  if (d == 64)
    score_lse_kernel<64, NCOL, 3><<<grid, 256, 0, stream>>>(q, k_ctx, k_rec, neg_lse, H_q, G, (int)N, (int)N_q, chunk, c, inv_c);
  else
    score_lse_kernel<128, NCOL, 2><<<grid, 256, 0, stream>>>(q, k_ctx, k_rec, neg_lse, H_q, G, (int)N, (int)N_q, chunk, c, inv_c);
  return hipGetLastError();
}

}  // namespace pkv
