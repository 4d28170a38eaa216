// HybridAxialMapper forward (paper Sec. 4.1) for one proxy layer at a time:
//   stage 1  conv stem            stem_conv1_kernel (fp32 ALU) + conv 2 as an fp16 MFMA GEMM whose A rows
//                                 are overlapping 3-token spans of the padded conv-1 output
//   stage 2  time-axis encoder    gather_pe_kernel, then per layer: QKV GEMM (writes q, k row-major and v transposed
//                                 for the attention's second product) -> window attention -> out-proj GEMM whose
//                                 epilogue adds the residual and normalises the row -> FFN-1 GEMM -> FFN-2 GEMM
//                                 with the same epilogue; all sliding windows of the layer are batched along the
//                                 GEMM M axis
//            overlap averaging    overlap_avg_kernel
//   stage 3  head-axis attention  K/V projection GEMM (inner products with queries / output weights in its epilogue)
//                                  + stage3_kernel (softmax over the slots per token and head, fp32 ALU)
// Matrix products take IEEE half (fp16) operands and accumulate in fp32 on v_mfma_f32_32x32x16_f16; the
// residual stream, normalisation, softmax and GELU are fp32.
#include "common.hpp"
#include "context.hpp"
#include "kernels.hpp"

namespace pkv {
namespace {

typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

constexpr float kNegInf = -__builtin_huge_valf();
constexpr int kDT = 512;    // d_time
constexpr int kWin = 2048;  // window length
constexpr int kStride = 1024;
constexpr int kHeads = 8;   // encoder heads, 64 wide

__device__ __forceinline__ float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

__device__ __forceinline__ uint16_t to_h(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }

// 8 chunks of 16 bytes per 128-byte LDS row, XOR-swizzled so that 16-byte tile stores and MFMA fragment reads
// (32 consecutive rows, same chunk) both spread over all LDS banks
__device__ __forceinline__ int swz8(int row) { return (row & 7) ^ ((row >> 3) & 1); }

// ------------------------------------------------------------------------------------------
// Range of the first convolution's output.  The scores of Sec. 3 in their sum form are not bounded by one (an
// attention sink collects up to G * N_q), so GELU(BN(conv1(x))) can exceed what IEEE half holds.  The operand of the
// second convolution is therefore stored as half(h1 * 2^-s) with one exponent s per proxy layer, taken from the
// largest score of the layer, and the second convolution's per-channel scale is multiplied by 2^s: exact, since only
// the exponent moves.  s = 0 (nothing changes) whenever the bound below stays under 2^15.
//   slot[0]: bits of max |x| (atomicMax, cleared again by stem_scale_kernel), slot[1] = 2^-s, slot[2] = 2^s (floats)
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void absmax_kernel(const float* __restrict__ x, int64_t n, uint32_t* __restrict__ slot) {
  uint32_t m = 0;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const uint32_t a = __float_as_uint(x[i]) & 0x7fffffffu;
    m = a > m ? a : m;
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const uint32_t o = __shfl_xor(m, off, 64);
    m = o > m ? o : m;
  }
  if ((threadIdx.x & 63) == 0) atomicMax(slot, m);
}

// |h1| <= |scale_c| * sum |w_c| * max|x| + |shift_c| <= cw * max|x| + cs  (|GELU(y)| <= |y|)
__global__ void stem_scale_kernel(uint32_t* __restrict__ slot, float cw, float cs) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  const float bound = __builtin_fmaf(cw, __uint_as_float(slot[0]), cs);
  const int e = (int)((__float_as_uint(bound) >> 23) & 255u) - 127;  // floor(log2(bound)); 128 for inf or NaN
  const int sh = e >= 15 ? e - 14 : 0;                                 // bound * 2^-sh < 2^15
  slot[1] = (uint32_t)(127 - sh) << 23;
  slot[2] = (uint32_t)(127 + sh) << 23;
  slot[0] = 0u;
}

// ------------------------------------------------------------------------------------------
// stage 1, first convolution: h1[t+1, c] = half(2^-s * GELU(scale[c] * sum_{h,tap} w[c,h,tap] * x[h, t+tap-1] + shift[c]))
// rows 0 and N+1 of h1 are zero (the padding of the second convolution).
// grid ceil(N / 64), 256 threads; thread owns channels tid, tid+256, ...
// ------------------------------------------------------------------------------------------
constexpr int kStemTok = 64;
constexpr int kMaxHs = 16;

__global__ __launch_bounds__(256) void stem_conv1_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                          const float* __restrict__ scale,
                                                          const float* __restrict__ shift,
                                                          const float* __restrict__ range_slot,
                                                          uint16_t* __restrict__ h1, int H_s, int N, int c_mid) {
  __shared__ float xs[kMaxHs][kStemTok + 2];
  const float down = range_slot[1];  // 2^-s
  const int t0 = blockIdx.x * kStemTok;
  for (int i = threadIdx.x; i < H_s * (kStemTok + 2); i += 256) {
    const int h = i / (kStemTok + 2), tt = i % (kStemTok + 2);
    const int t = t0 + tt - 1;
    xs[h][tt] = (t >= 0 && t < N) ? x[(size_t)h * N + t] : 0.0f;
  }
  __syncthreads();
  for (int c = threadIdx.x; c < c_mid; c += 256) {
    float wr[kMaxHs * 3];
#pragma unroll
    for (int i = 0; i < kMaxHs * 3; ++i) wr[i] = (i < H_s * 3) ? w[(size_t)c * H_s * 3 + i] : 0.0f;
    const float sc = scale[c], sh = shift[c];
    for (int tt = 0; tt < kStemTok && t0 + tt < N; ++tt) {
      float acc = 0.0f;
#pragma unroll
      for (int h = 0; h < kMaxHs; ++h) {
        if (h < H_s) {
          acc = __builtin_fmaf(wr[h * 3 + 0], xs[h][tt + 0], acc);
          acc = __builtin_fmaf(wr[h * 3 + 1], xs[h][tt + 1], acc);
          acc = __builtin_fmaf(wr[h * 3 + 2], xs[h][tt + 2], acc);
        }
      }
      h1[(size_t)(t0 + tt + 1) * c_mid + c] = to_h(gelu_erf(__builtin_fmaf(acc, sc, sh)) * down);
    }
    if (blockIdx.x == 0) h1[c] = 0;
    if (blockIdx.x == gridDim.x - 1) h1[(size_t)(N + 1) * c_mid + c] = 0;
  }
}

// ------------------------------------------------------------------------------------------
// fp16 GEMM  C[M, Nn] = A[M, K] * W[Nn, K]^T  (+ epilogue), fp32 accumulation.
// A rows start lda elements apart (lda < K gives the overlapping rows of the second convolution).
//
// Persistent kernel, one 512-thread workgroup per CU.  Block tile BM (rows of A) x BN (rows of W), 256 x 256 or
// 128 x 512, K step 64 (full 128-byte lines per row), 8 waves, each 64 x 128 = 2 x 4 MFMA tiles.  A tile
// of this size needs 1 byte from L2 per 100 to 128 flop; smaller tiles are bound by the L2 -> CU path, not by
// the matrix pipe.  The 128 x 512 shape spans a whole row of the encoder's width, so its epilogue can normalise
// the row (residual add + LayerNorm) before anything goes to memory.
//
// The A rows go on the MFMA M axis and the W rows on the N axis, so a lane owns output COLUMNS.  The
// W rows of a wave's 128-column block are staged in the order n = 4*l + jn (l = lane & 31, jn = MFMA
// tile), so a lane holds four adjacent columns in its four tiles and every store instruction writes
// whole 256-byte (fp16) or 512-byte (fp32) row segments, 8 or 16 bytes per lane.  Output (and residual)
// buffers have their row count padded to a multiple of 256, so the epilogue has no row predicate; rows
// at and past M are written with values that nobody reads (the stem's epilogue, which writes a token's row into
// the windows that hold it, skips them instead).
//
// The K steps of all tiles of a workgroup form one stream: two LDS stages (64 or 80 KB each) and ONE barrier
// per step.  A step is four phases of 8 MFMAs; the fragments of phase kk+1 are read from LDS between
// the MFMAs of phase kk (phase 3 reads phase 0 of the next step, behind the barrier), step s+1 goes
// from registers to LDS during phase 2 and each register is refilled with its part of step s+2 right
// behind that -- across tile boundaries, so the next tile's loads are in flight during an epilogue.
// The issue order is written out and pinned with scheduling barriers.
//
// Tile order: blocks are dealt round-robin to the 8 XCDs by the hardware, so XCD x = block % 8 takes the
// row tiles x, x+8, ... and its workgroups take that list's (row tile, column tile) pairs round-robin:
// the Nn / BN column tiles of one row tile run at the same time on one XCD and share its L2 copy of
// the A rows.
// K % 64 == 0, Nn % BN == 0.
// ------------------------------------------------------------------------------------------
enum Epilogue {
  kEpiGeluPeWin,      // z = GELU(acc * (p0[n] * *p2) + p1[n]) of token m goes, plus the positional row of its place, into the
                      // row of every window that holds the token: out_f32 and out_h (second stem convolution -> stage-2 input)
  kEpiQkvH,           // columns below 2 * d_time: out_h[m, n] = half(acc + p0[n]), rows ldc apart (q and k);
                      // the others (v): out_v in the transposed, key-permuted layout of the attention kernel
  kEpiBiasReluH,      // out_h = relu(acc + p0[n])
  kEpiStage3,         // columns = stage-3 key and value slots of 64: per token and slot the inner products of
                      // acc + p0 with the learned queries (p1, n_head of them, times 1/8) or with the output weights (g)
  kEpiResLn           // BN = 512: y = LayerNorm(res[m, :] + acc + p0) * g + b -> out_f32 (may be res) and out_h
};

struct EpiArgs {
  const float* p0;
  const float* p1;
  const float* p2;
  const float* g;
  const float* b;
  const float* res;
  float* out_f32;
  uint16_t* out_h;
  uint16_t* out_v;
  int ldc;  // elements between output rows
  const float* pe;  // kEpiGeluPeWin: positional table [kWin, d_time]
  int n_win;        // kEpiGeluPeWin: number of windows
  int n_slot, n_head;  // kEpiStage3: slots H_s (keys in columns [0, 64 H_s), values in [64 H_s, 128 H_s)) and queries H_l
};

// epilogue stores bypass L2 allocation: the output is not read again by this kernel and would evict W and A rows
#define PKV_ST(ptr, val) __builtin_nontemporal_store((val), (ptr))

constexpr int kGemmBK = 64;
constexpr int kXcds = 8;

// Sum of v[0..15] over the 32 lanes that share bit 5 of the lane number, sixteen sums at once: in every step a lane
// keeps the half of its values that its own lane bit selects, hands the other half to the partner and adds what it
// receives; after four steps it holds one value, the row (lane & 31) >> 1 of the sixteen, summed over sixteen lanes,
// and the last step adds the neighbour's.  31 exchanges instead of 80.
__device__ __forceinline__ float reduce16_over_lanes(float (&v)[16], int l32) {
  static_for<4>([&](auto sc) {
    constexpr int step = decltype(sc)::value, n = 8 >> step, mask = 16 >> step;
    const bool up = (l32 & mask) != 0;
#pragma unroll
    for (int j = 0; j < n; ++j) {
      const float send = up ? v[j] : v[j + n];
      const float keep = up ? v[j + n] : v[j];
      v[j] = keep + __shfl_xor(send, mask, 64);
    }
  });
  return v[0] + __shfl_xor(v[0], 1, 64);
}

// Sum of v[0..15] over the 16 lanes that share the upper bits of the lane number, sixteen sums at once, by the same
// halving exchange: afterwards lane j (lane & 15) holds the sum of v[j].  15 exchanges.
__device__ __forceinline__ float reduce16_over_16_lanes(float (&v)[16], int lane) {
  static_for<4>([&](auto sc) {
    constexpr int step = decltype(sc)::value, n = 8 >> step, mask = 8 >> step;
    const bool up = (lane & mask) != 0;
#pragma unroll
    for (int j = 0; j < n; ++j) {
      const float send = up ? v[j] : v[j + n];
      const float keep = up ? v[j + n] : v[j];
      v[j] = keep + __shfl_xor(send, mask, 64);
    }
  });
  return v[0];
}

template <int EPI, int BM, int BN>
__global__ __launch_bounds__(512, 1) void gemm_f16_kernel(const uint16_t* __restrict__ A, int lda,
                                                            const uint16_t* __restrict__ W, int M, int Nn, int K,
                                                            EpiArgs ep) {
  constexpr int WM = BM / 64, WN = 8 / WM;       // waves along M and N
  constexpr int NA = BM / 64, NS = (BM + BN) / 64;  // 64-row parts of a stage: A parts, then W parts
  constexpr int kStageU4 = (BM + BN) * (kGemmBK / 8);  // 16-byte units per stage
  static_assert(WM * WN == 8 && BN / WN == 128, "a wave computes 64 x 128");
  static_assert(EPI != kEpiResLn || BN == kDT, "the normalising epilogue needs the whole row in one tile");
  extern __shared__ u32x4 lds[];  // 2 stages
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int wm = wave / WN, wn = wave % WN;
  const int n_tiles = Nn / BN;
  const int nk = K / kGemmBK;
  const int xcd = blockIdx.x % kXcds, wg = blockIdx.x / kXcds, wg_per_xcd = gridDim.x / kXcds;
  // tile `it` of this workgroup: entry it * wg_per_xcd + wg of the XCD's list
  auto tile_of = [&](int it, int& m0, int& n0) {
    const int u = it * wg_per_xcd + wg;
    m0 = ((u / n_tiles) * kXcds + xcd) * BM;
    n0 = (u % n_tiles) * BN;
    return m0 < M;
  };
  int my_tiles = 0;
  {
    int a, b;
    while (tile_of(my_tiles, a, b)) ++my_tiles;
  }
  const int total = my_tiles * nk;
  if (total == 0) return;

  // staging: thread t moves chunk t % 8 of LDS rows t / 8 + 64 * i (i < NA: A rows, i >= NA: W rows).
  // LDS row wl = 64 (i - NA) + t / 8 of the W part holds W row n0 + 128 (wl / 128) + 4 (wl % 32) + (wl % 128) / 32.
  const int srow = tid >> 3, sch = tid & 7;
  const int sslot = srow * 8 + (sch ^ swz8(srow));  // swz8(srow + 64 * i) == swz8(srow)
  u32x4 rg[NS];
  int f_m0 = 0, f_n0 = 0, f_k = 0, f_it = 0;  // position of the next step to fetch
  tile_of(0, f_m0, f_n0);
  auto fetch_one = [&](int i) {
    const int k0 = f_k * kGemmBK + sch * 8;
    if (i < NA) {
      int m = f_m0 + srow + 64 * i;
      m = m < M ? m : M - 1;
      rg[i] = *reinterpret_cast<const u32x4*>(A + (size_t)m * lda + k0);
    } else {
      const int wl = srow + 64 * (i - NA);
      const int n = f_n0 + (wl & ~127) + 4 * (wl & 31) + ((wl & 127) >> 5);
      rg[i] = *reinterpret_cast<const u32x4*>(W + (size_t)n * K + k0);
    }
  };
  // moves on to the following step; past the end it stays on the last step (re-reads valid memory)
  auto fetch_advance = [&]() {
    if (++f_k == nk) {
      if (f_it + 1 < my_tiles) {
        f_k = 0;
        ++f_it;
        tile_of(f_it, f_m0, f_n0);
      } else {
        f_k = nk - 1;
      }
    }
  };

  f32x16 acc[2][4];
  auto zero_acc = [&]() {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int jn = 0; jn < 4; ++jn) acc[i][jn] = f32x16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  };
  zero_acc();
  // bias (and scale) of the current tile's columns n .. n+3, loaded when the tile starts: a load inside
  // the epilogue would have to wait for the prefetch of the next step as well
  f32x4 p0, p1 = {0.0f, 0.0f, 0.0f, 0.0f};
  auto load_bias = [&](int it) {
    int m0, n0;
    tile_of(it < my_tiles ? it : my_tiles - 1, m0, n0);
    const int n = n0 + wn * 128 + 4 * l32;
    p0 = *reinterpret_cast<const f32x4*>(ep.p0 + n);
    if constexpr (EPI == kEpiGeluPeWin) {
      p0 *= *ep.p2;
      p1 = *reinterpret_cast<const f32x4*>(ep.p1 + n);
    }
  };
  load_bias(0);

  // prologue: step 0 to LDS, step 1 in registers, fragments of (step 0, phase 0) in registers
#pragma unroll
  for (int i = 0; i < NS; ++i) fetch_one(i);
  fetch_advance();
#pragma unroll
  for (int i = 0; i < NS; ++i) lds[sslot + 64 * 8 * i] = rg[i];
#pragma unroll
  for (int i = 0; i < NS; ++i) fetch_one(i);
  fetch_advance();
  __syncthreads();
  const int fsw = swz8(l32);  // all fragment rows of this lane are l32 plus a multiple of 32
  const int xrow = (wm * 64 + l32) * 8, wrow = (BM + wn * 128 + l32) * 8;
  f16x8 fx[2][2], fw[2][4];
  auto read_frag = [&](const u32x4* st, int kk, int set, int which) {
    const int slot = (kk * 2 + half) ^ fsw;
    if (which < 2) fx[set][which] = as_f16x8(st[xrow + which * 32 * 8 + slot]);
    else fw[set][which - 2] = as_f16x8(st[wrow + (which - 2) * 32 * 8 + slot]);
  };
#pragma unroll
  for (int wh = 0; wh < 6; ++wh) read_frag(lds, 0, 0, wh);

  for (int s = 0; s < total; ++s) {
    u32x4* st = lds + (s & 1) * kStageU4;
    u32x4* st_next = lds + ((s + 1) & 1) * kStageU4;
    static_for<4>([&](auto kc) {
      constexpr int kk = decltype(kc)::value, cur = kk & 1, nxt = cur ^ 1;
      if constexpr (kk == 3) {
        // every wave has read the last fragments of this step and written its part of step s+1
        __syncthreads();
      }
      static_for<8>([&](auto jc) {
        constexpr int j = decltype(jc)::value, i = j >> 2, jn = j & 3;
        acc[i][jn] = mfma_f16_32x32x16(fx[cur][i], fw[cur][jn], acc[i][jn]);
        if constexpr (j < 6) {
          if constexpr (kk < 3) read_frag(st, kk + 1, nxt, j);
          else read_frag(st_next, 0, nxt, j);
        }
        if constexpr (kk == 2) {
          // the register is refilled as soon as it is free: a whole step lies between a load and its use
          st_next[sslot + 64 * 8 * j] = rg[j];
          fetch_one(j);
          if constexpr (j + 8 < NS) {
            st_next[sslot + 64 * 8 * (j + 8)] = rg[j + 8];
            fetch_one(j + 8);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      });
    });
    fetch_advance();
    if (s % nk != nk - 1) continue;

    // epilogue: lane holds columns n .. n+3; register r of tile (i, jn) holds row mb + (r/4)*8 + r%4
    int m0, n0;
    tile_of(s / nk, m0, n0);
    const int n = n0 + wn * 128 + 4 * l32;
    if constexpr (EPI == kEpiResLn) {
      // (1) pre-norm sum in place, acc += bias + residual row, and (2) row sums and sums of squares: four columns in
      // the lane, 32 lanes by exchange, 4 waves through LDS (the stage that this step has used up is free until
      // phase 2 of the next step)
      struct Pair {
        float s1, s2;
      };
      Pair* red = reinterpret_cast<Pair*>(st);  // [128 rows][4 waves along N]
      int own_row[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const float* rb = ep.res + (size_t)(m0 + wm * 64 + i * 32 + half * 4) * kDT + n;
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          f32x4 rv[4];
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) rv[e4] = *reinterpret_cast<const f32x4*>(rb + (size_t)(qd * 8 + e4) * kDT);
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4)
#pragma unroll
            for (int jn = 0; jn < 4; ++jn) acc[i][jn][qd * 4 + e4] += rv[e4][jn] + p0[jn];
        }
        float t[2];
#pragma unroll
        for (int which = 0; which < 2; ++which) {
          float sv[16];
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float a0 = acc[i][0][r], a1 = acc[i][1][r], a2 = acc[i][2][r], a3 = acc[i][3][r];
            sv[r] = which == 0 ? (a0 + a1) + (a2 + a3) : (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
          }
          t[which] = reduce16_over_lanes(sv, l32);
        }
        own_row[i] = ((wm * 2 + i) * 2 + half) * 16 + (l32 >> 1);
        if ((l32 & 1) == 0) red[own_row[i] * 4 + wn] = Pair{t[0], t[1]};
      }
      __syncthreads();
      float mean_o[2], rstd_o[2];  // of the row this lane reduced
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const f32x4 lo = *reinterpret_cast<const f32x4*>(&red[own_row[i] * 4]);
        const f32x4 hi = *reinterpret_cast<const f32x4*>(&red[own_row[i] * 4 + 2]);
        const float sum = (lo[0] + lo[2]) + (hi[0] + hi[2]), sq = (lo[1] + lo[3]) + (hi[1] + hi[3]);
        const float mu = sum * (1.0f / kDT);
        const float var = __builtin_fmaxf(__builtin_fmaf(-mu, mu, sq * (1.0f / kDT)), 0.0f);
        mean_o[i] = mu;
        rstd_o[i] = 1.0f / sqrtf(var + 1e-5f);
      }
      // (3) normalise and store: the statistics of row r sit in lanes 2r and 2r+1 of the lane's own half
      const f32x4 g4 = *reinterpret_cast<const f32x4*>(ep.g + n), b4 = *reinterpret_cast<const f32x4*>(ep.b + n);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const size_t ob = (size_t)(m0 + wm * 64 + i * 32 + half * 4) * kDT + n;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float mu = __shfl(mean_o[i], (half << 5) | (2 * r), 64), rs = __shfl(rstd_o[i], (half << 5) | (2 * r), 64);
          f32x4 v = {acc[i][0][r], acc[i][1][r], acc[i][2][r], acc[i][3][r]};
          v = (v - mu) * rs * g4 + b4;
          const size_t o = ob + (size_t)((r >> 2) * 8 + (r & 3)) * kDT;
          PKV_ST(reinterpret_cast<f32x4*>(ep.out_f32 + o), v);
          PKV_ST(reinterpret_cast<f16x4*>(ep.out_h + o), __builtin_convertvector(v, f16x4));
        }
      }
      __syncthreads();  // the stage may be overwritten again
    } else if constexpr (EPI == kEpiStage3) {
      // The 64 columns of a slot sit in 16 lanes (four columns each).  Per 32-row block: the lane's share of every row's
      // inner product with one coefficient vector, sixteen rows reduced over the 16 lanes at once, lane j keeps row j of
      // the sixteen that its half-wave holds.  Key slots take the n_head queries in turn, value slots the output weights.
      const int col = n0 + wn * 128 + (l32 >> 4) * 64;  // first column of the lane group's slot
      const int slot = col >> 6, e0 = (l32 & 15) * 4;
      const bool is_k = slot < ep.n_slot, is_v = !is_k && slot < 2 * ep.n_slot;
      const int sv = is_k ? slot : slot - ep.n_slot;
      const int j16 = l32 & 15;
      const int n_pass = ep.n_head;  // uniform; value slots use pass 0 only
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int row = m0 + wm * 64 + i * 32 + (j16 >> 2) * 8 + half * 4 + (j16 & 3);  // the row this lane ends up with
        float* orow = ep.out_f32 + (size_t)row * ep.ldc;
        for (int h = 0; h < n_pass; ++h) {
          const float* cf = is_k ? ep.p1 + (size_t)h * 64 + e0 : ep.g + e0;
          const f32x4 c4 = *reinterpret_cast<const f32x4*>(cf);
          float part[16];
#pragma unroll
          for (int r = 0; r < 16; ++r)
            part[r] = (acc[i][0][r] + p0[0]) * c4[0] + (acc[i][1][r] + p0[1]) * c4[1] + (acc[i][2][r] + p0[2]) * c4[2] +
                      (acc[i][3][r] + p0[3]) * c4[3];
          const float tot = reduce16_over_16_lanes(part, l32);
          if (row < M) {
            if (is_k) orow[h * ep.n_slot + sv] = tot * 0.125f;
            else if (is_v && h == 0) orow[ep.n_head * ep.n_slot + sv] = tot;
          }
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        if constexpr (EPI == kEpiQkvH) {
          if (n0 >= 2 * kDT) {
            // v: element (token m, column vc) goes to vt[(window * heads + head) * 64 + dd][pos]; the lane's eight tokens
            // of a 16-token group (rows r = 8u .. 8u+7 of the tile pair qd = 2u, 2u+1) land in positions half*8 .. +7
            const int vc = n - 2 * kDT;  // columns vc .. vc+3: one head, dd .. dd+3
            const int mg = m0 + wm * 64 + i * 32;
            uint16_t* vb = ep.out_v + ((size_t)((mg / kWin) * kHeads + (vc >> 6)) * 64 + (vc & 63)) * kWin + (mg % kWin) + half * 8;
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
              for (int jn = 0; jn < 4; ++jn) {
                f32x8 t;
#pragma unroll
                for (int e = 0; e < 8; ++e) t[e] = acc[i][jn][u * 8 + e] + p0[jn];
                PKV_ST(reinterpret_cast<f16x8*>(vb + (size_t)jn * kWin + u * 16), __builtin_convertvector(t, f16x8));
              }
            continue;
          }
        }
        const size_t ob = (size_t)(m0 + wm * 64 + i * 32 + half * 4) * ep.ldc + n;
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
#pragma unroll
          for (int e4 = 0; e4 < 4; ++e4) {
            const int r = qd * 4 + e4;
            f32x4 v = {acc[i][0][r], acc[i][1][r], acc[i][2][r], acc[i][3][r]};
            const size_t o = ob + (size_t)(qd * 8 + e4) * ep.ldc;
            if constexpr (EPI == kEpiGeluPeWin) {
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] = gelu_erf(__builtin_fmaf(v[e], p0[e], p1[e]));
              // token t sits at place t - 1024 k of window k = min(t / 1024, n_win - 1) and, if that window is not the
              // first and the token lies in its first half, at place + 1024 of the window before
              const int t = m0 + wm * 64 + i * 32 + half * 4 + qd * 8 + e4;
              if (t < M) {
                const int kq = t / kStride, k1 = kq < ep.n_win ? kq : ep.n_win - 1, p1w = t - k1 * kStride;
                const size_t o1 = ((size_t)k1 * kWin + p1w) * kDT + n;
                const f32x4 y1 = v + *reinterpret_cast<const f32x4*>(ep.pe + (size_t)p1w * kDT + n);
                PKV_ST(reinterpret_cast<f32x4*>(ep.out_f32 + o1), y1);
                PKV_ST(reinterpret_cast<f16x4*>(ep.out_h + o1), __builtin_convertvector(y1, f16x4));
                if (k1 >= 1 && kq == k1) {
                  const size_t o0 = o1 - (size_t)(kWin - kStride) * kDT;  // window k1 - 1, place p1w + 1024
                  const f32x4 y0 = v + *reinterpret_cast<const f32x4*>(ep.pe + (size_t)(p1w + kStride) * kDT + n);
                  PKV_ST(reinterpret_cast<f32x4*>(ep.out_f32 + o0), y0);
                  PKV_ST(reinterpret_cast<f16x4*>(ep.out_h + o0), __builtin_convertvector(y0, f16x4));
                }
              }
            } else if constexpr (EPI == kEpiQkvH) {
              PKV_ST(reinterpret_cast<f16x4*>(ep.out_h + o), __builtin_convertvector(v + p0, f16x4));
            } else if constexpr (EPI == kEpiBiasReluH) {
              v += p0;
#pragma unroll
              for (int e = 0; e < 4; ++e) v[e] = __builtin_fmaxf(v[e], 0.0f);
              PKV_ST(reinterpret_cast<f16x4*>(ep.out_h + o), __builtin_convertvector(v, f16x4));
            }
          }
        }
      }
    }
    zero_acc();
    load_bias(s / nk + 1);
  }
}

// ------------------------------------------------------------------------------------------
// Window attention (8 heads x 64, full bidirectional attention inside each window).
// qk [T, 2 * d_time] holds q then k of every window row; vt [window][head][64][win] holds v transposed, the keys of
// every 16-group in the order the second product consumes them (both written by the QKV GEMM's epilogue).
// Computes S^T = K Q^T so that a lane owns one query column; P^T then feeds the second MFMA as its
// B operand straight from the accumulator registers, with V^T tiles as the A operand.
// 256 threads; a workgroup owns 256 queries of one (window, head), a wave 64 of them (two 32-column
// sub-tiles); keys stream in tiles of 64 through three LDS stages (K tile + V^T tile, 16 KB each) with one
// barrier per tile: while tile t is computed, tile t+2 goes from registers to LDS and tile t+3 is
// fetched from global memory.
// Online softmax with a lazily raised reference: a column's reference only moves when a logit exceeds it
// by more than 2^8, so the rescaling of the output accumulators is rare; probabilities stay below 2^8,
// which half holds with its full relative precision.
// Block -> work mapping: blocks are dealt round-robin to the 8 XCDs, so block b takes q-block (b / 8) % 8
// of item (b / 64) * 8 + b % 8: the 8 q-blocks of one (window, head) run on one XCD and share its L2 copy of
// that head's K and V.
// ------------------------------------------------------------------------------------------
constexpr float kAttnLazy = 8.0f;

// max over the 32 elements of two accumulator tiles (v_max3 tree)
__device__ __forceinline__ float max16_8(const f32x16& a, const f32x16& b) {
  float m = max3f(a[0], a[1], a[2]);
#pragma unroll
  for (int r = 3; r < 15; r += 2) m = max3f(m, a[r], a[r + 1]);
  m = max3f(m, a[15], b[0]);
#pragma unroll
  for (int r = 1; r < 15; r += 2) m = max3f(m, b[r], b[r + 1]);
  return __builtin_fmaxf(m, b[15]);
}

// max / sum over the two half-waves without an LDS round trip: the swap leaves the lower half's value in both
// halves of the first register and the upper half's in both halves of the second
__device__ __forceinline__ float halves_max(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __builtin_fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float halves_sum(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__global__ __launch_bounds__(256, 2) void window_attention_kernel(const uint16_t* __restrict__ qk,
                                                                   const uint16_t* __restrict__ vt,
                                                                   uint16_t* __restrict__ ao, int64_t T, int n_win) {
  __shared__ u32x4 lds[3 * 1024];  // stage = K tile (64 keys x 8 chunks) then V^T tile (64 d rows x 8 chunks)
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int bj = blockIdx.x >> 3, item = (bj >> 3) * kXcds + (blockIdx.x & 7);
  const int wk = item / kHeads, hd = item % kHeads;
  const int64_t base = (int64_t)wk * kWin;
  const int len = (wk < n_win - 1) ? kWin : (int)(T - base);
  const int i0 = (bj & 7) * 256;
  if (i0 >= len) return;
  constexpr float c = 1.4426950408889634f * 0.125f;  // log2(e) / sqrt(64)

  f16x8 bq[2][4];
  int qi[2];
#pragma unroll
  for (int cs = 0; cs < 2; ++cs) {
    qi[cs] = i0 + wave * 64 + cs * 32 + l32;
    const int row = qi[cs] < len ? qi[cs] : len - 1;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk)
      bq[cs][kk] = as_f16x8(*reinterpret_cast<const u32x4*>(qk + (size_t)(base + row) * (2 * kDT) + hd * 64 + kk * 16 + half * 8));
  }
  f32x16 o[2][2];  // [d half][query sub-tile]
#pragma unroll
  for (int ds = 0; ds < 2; ++ds)
#pragma unroll
    for (int cs = 0; cs < 2; ++cs) o[ds][cs] = f32x16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  float m_run[2] = {-1.0e30f, -1.0e30f}, l_run[2] = {0.0f, 0.0f};

  const uint16_t* kbase = qk + (size_t)base * (2 * kDT) + kDT + hd * 64;
  const uint16_t* vbase = vt + (size_t)(wk * kHeads + hd) * 64 * kWin;
  const int n_tiles = (len + 63) / 64;
  // staging: thread moves chunk tid % 8 of rows tid / 8 and tid / 8 + 32 of both tiles
  const int srow = tid >> 3, sch = tid & 7;
  const int sslot = srow * 8 + (sch ^ swz8(srow));  // swz8(srow + 32) == swz8(srow)
  u32x4 rk[2], rv[2];
  auto fetch = [&](int t) {
    const int j0 = t * 64;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int row = srow + 32 * i;
      int j = j0 + row;
      j = j < len ? j : len - 1;
      rk[i] = *reinterpret_cast<const u32x4*>(kbase + (size_t)j * (2 * kDT) + sch * 8);
      rv[i] = *reinterpret_cast<const u32x4*>(vbase + (size_t)row * kWin + j0 + sch * 8);
    }
  };
  auto store = [&](int t) {
    u32x4* st = lds + (t % 3) * 1024;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      st[sslot + 32 * 8 * i] = rk[i];
      st[512 + sslot + 32 * 8 * i] = rv[i];
    }
  };
  fetch(0);
  store(0);
  if (n_tiles > 1) {
    fetch(1);
    store(1);
  }
  if (n_tiles > 2) fetch(2);
  const int fsw = swz8(l32);
  // Every load so far (the wave's query fragments among them) has landed before the loop starts.  Without this the
  // compiler, which cannot tell at the loop head that the query fragments arrived long ago, waits for ALL outstanding
  // loads in front of the first MFMAs of every tile (the counter is in order), i.e. for the prefetch it has just issued.
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)

  typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
  const f16x2 ones = {(_Float16)1.0f, (_Float16)1.0f};
  // LDS reads run ahead of their use: the first four K fragments of tile t+1 are read in the tail of tile t (its stage
  // has been complete since the barrier of tile t), the other four behind the first MFMAs; the V^T fragments of a
  // 16-key step are read one step ahead and serve both query sub-tiles.
  auto read_k = [&](const u32x4* st, int ks, f16x8 (&fk)[4]) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) fk[kk] = as_f16x8(st[(ks * 32 + l32) * 8 + ((kk * 2 + half) ^ fsw)]);
  };
  auto read_v = [&](const u32x4* st, int u, f16x8 (&fv)[2]) {
#pragma unroll
    for (int ds = 0; ds < 2; ++ds) fv[ds] = as_f16x8(st[512 + (ds * 32 + l32) * 8 + ((u * 2 + half) ^ fsw)]);  // d row, step u
  };
  f16x8 fk0[4];
  for (int t = 0; t < n_tiles; ++t) {
    // every wave has finished tile t-1: its stage takes tile t+2, the registers take tile t+3
    __syncthreads();
    if (t + 2 < n_tiles) store(t + 2);
    if (t + 3 < n_tiles) fetch(t + 3);
    const u32x4* st = lds + (t % 3) * 1024;
    const int j0 = t * 64;
    const bool ragged = j0 + 64 > len;
    if (t == 0) read_k(st, 0, fk0);

    // S^T tiles of both query sub-tiles: s[cs][ks] = K[ks] Q[cs]^T
    f32x16 s[2][2];
    f16x8 fk1[4], fv[2][2];
    read_k(st, 1, fk1);
    read_v(st, 0, fv[0]);
#pragma unroll
    for (int cs = 0; cs < 2; ++cs) {
      f32x16 acc = f32x16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) acc = mfma_f16_32x32x16(fk0[kk], bq[cs][kk], acc);
      s[cs][0] = acc;
    }
#pragma unroll
    for (int cs = 0; cs < 2; ++cs) {
      f32x16 acc = f32x16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) acc = mfma_f16_32x32x16(fk1[kk], bq[cs][kk], acc);
      s[cs][1] = acc;
    }
    if (ragged) {
      const int lim = len - j0 - half * 4;  // element r of tile ks is key j0 + ks*32 + (r>>2)*8 + half*4 + (r&3)
#pragma unroll
      for (int cs = 0; cs < 2; ++cs)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[cs][ks][r] = (ks * 32 + (r >> 2) * 8 + (r & 3)) < lim ? s[cs][ks][r] : kNegInf;
    }
    float tmax[2];
#pragma unroll
    for (int cs = 0; cs < 2; ++cs) tmax[cs] = halves_max(max16_8(s[cs][0], s[cs][1])) * c;
    if (__builtin_amdgcn_ballot_w64(tmax[0] > m_run[0] + kAttnLazy || tmax[1] > m_run[1] + kAttnLazy)) {
#pragma unroll
      for (int cs = 0; cs < 2; ++cs) {
        const float nm = tmax[cs] > m_run[cs] + kAttnLazy ? tmax[cs] : m_run[cs];
        const float alpha = __builtin_amdgcn_exp2f(m_run[cs] - nm);
        l_run[cs] *= alpha;
#pragma unroll
        for (int ds = 0; ds < 2; ++ds)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[ds][cs][r] *= alpha;
        m_run[cs] = nm;
      }
    }
    // Four steps of 16 keys.  A wave issues in order, so an MFMA that finds the matrix pipe busy holds back the vector
    // instructions behind it: the four MFMAs of step u-1 are therefore spread between the vector instructions of
    // step u (one MFMA, then a quarter of the step's exponentials, conversions and sums), each finding the pipe free.
    float lsum[2] = {0.0f, 0.0f};
    f16x8 pb[2][2];  // [step parity][query sub-tile]
    static_for<5>([&](auto uc) {
      constexpr int u = decltype(uc)::value;
      if constexpr (u > 0) {
#pragma unroll
        for (int ds = 0; ds < 2; ++ds)
#pragma unroll
          for (int cs = 0; cs < 2; ++cs) o[ds][cs] = mfma_f16_32x32x16(fv[(u - 1) & 1][ds], pb[(u - 1) & 1][cs], o[ds][cs]);
      }
      if constexpr (u < 4) {
        constexpr int ks = u >> 1, u2 = u & 1;
#pragma unroll
        for (int cs = 0; cs < 2; ++cs) {
          const float nref = -m_run[cs];
          f32x8 p;
#pragma unroll
          for (int e = 0; e < 8; ++e) p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[cs][ks][u2 * 8 + e], c, nref));
          pb[u & 1][cs] = __builtin_convertvector(p, f16x8);
          // the row sum takes the probabilities as the second product sees them (rounded to half), two per instruction
#pragma unroll
          for (int e = 0; e < 8; e += 2)
            lsum[cs] = __builtin_amdgcn_fdot2(f16x2{pb[u & 1][cs][e], pb[u & 1][cs][e + 1]}, ones, lsum[cs], false);
        }
        // pins the row sums to this step: left alone, the compiler moves all of them behind the last step
        asm volatile("" : "+v"(lsum[0]), "+v"(lsum[1]));
        if constexpr (u > 0) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x002, 12, 0);  // twelve vector instructions
          }
        }
        // V^T fragments of step u+1 into the buffer that the MFMAs of step u-1 have just released
        if constexpr (u < 3) read_v(st, u + 1, fv[(u + 1) & 1]);
      } else {
        if (t + 1 < n_tiles) read_k(lds + ((t + 1) % 3) * 1024, 0, fk0);
      }
      __builtin_amdgcn_sched_barrier(0);
    });
#pragma unroll
    for (int cs = 0; cs < 2; ++cs) l_run[cs] += lsum[cs];
  }

  // output: O^T / row sum, through LDS so that every query row is written as 128 contiguous bytes
  __syncthreads();
  uint16_t* ot = reinterpret_cast<uint16_t*>(lds) + wave * (64 * 72);  // [64 queries][64 d + 8 pad] per wave
#pragma unroll
  for (int cs = 0; cs < 2; ++cs) {
    const float inv = 1.0f / halves_sum(l_run[cs]);
#pragma unroll
    for (int ds = 0; ds < 2; ++ds)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        f16x4 pk;
#pragma unroll
        for (int e = 0; e < 4; ++e) pk[e] = (_Float16)(o[ds][cs][rg * 4 + e] * inv);
        *reinterpret_cast<f16x4*>(ot + (cs * 32 + l32) * 72 + ds * 32 + rg * 8 + half * 4) = pk;
      }
  }
  // the wave reads back its own rows only: no barrier needed beyond the wave's own LDS ordering
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int id = lane + 64 * i, row = id >> 3, ch = id & 7;  // 64 rows x 8 chunks of 16 bytes
    const int q = i0 + wave * 64 + row;
    if (q < len)
      *reinterpret_cast<u32x4*>(ao + (size_t)(base + q) * kDT + hd * 64 + ch * 8) =
          *reinterpret_cast<const u32x4*>(ot + row * 72 + ch * 8);
  }
}

// ------------------------------------------------------------------------------------------
// overlap averaging: zg[t] = half(mean over the windows covering token t of x[row of t in that window])
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void overlap_avg_kernel(const float* __restrict__ x, uint16_t* __restrict__ zg,
                                                           int64_t N, int n_win) {
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (gid >= N * (kDT / 4)) return;
  const int64_t t = gid / (kDT / 4);
  const int c4 = (int)(gid % (kDT / 4));
  f32x4 sum = {0.0f, 0.0f, 0.0f, 0.0f};
  float cnt = 0.0f;
  const int64_t khi = t / kStride;
#pragma unroll
  for (int dk = 0; dk < 2; ++dk) {
    const int64_t k = khi - dk;
    if (k < 0 || k >= n_win) continue;
    const int64_t p = t - k * kStride;
    if (p >= kWin) continue;
    sum += *reinterpret_cast<const f32x4*>(x + (size_t)(k * kWin + p) * kDT + c4 * 4);
    cnt += 1.0f;
  }
  const f32x4 mean = sum / cnt;
  *reinterpret_cast<f16x4*>(zg + (size_t)t * kDT + c4 * 4) = __builtin_convertvector(mean, f16x4);
}

// ------------------------------------------------------------------------------------------
// stage 3 per token (Eq. 3), after the K/V projection GEMM whose epilogue has already taken the inner products:
// s3[t] = [ <Q_l[h], K[s]> / 8 for h < H_l, s < H_s | <w_o, V[s]> for s < H_s ];
// yhat[ll, h, t] = sum_s softmax_s(logit[h][s]) * u[s] + b_o for every paired target layer ll.
// Block = 256 threads = (256 / H_l) tokens x H_l target heads, token index fastest.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void stage3_kernel(const float* __restrict__ s3, float b_o, float* __restrict__ yhat,
                                                      int64_t N, int H_s, int H_l, int ll_lo, int ll_hi) {
  const int tok_per_block = 256 / H_l;
  const int tt = threadIdx.x % tok_per_block, h = threadIdx.x / tok_per_block;
  const int64_t t = (int64_t)blockIdx.x * tok_per_block + tt;
  if (h >= H_l || t >= N) return;
  const float* row = s3 + (size_t)t * ((H_l + 1) * H_s);
  const float* lg = row + h * H_s;
  const float* u = row + H_l * H_s;
  float mx = kNegInf;
  for (int s = 0; s < H_s; ++s) mx = __builtin_fmaxf(mx, lg[s]);
  float den = 0.0f, num = 0.0f;
  for (int s = 0; s < H_s; ++s) {
    const float e = __expf(lg[s] - mx);
    den += e;
    num += e * u[s];
  }
  const float y = num / den + b_o;
  for (int ll = ll_lo; ll < ll_hi; ++ll) yhat[((size_t)ll * H_l + h) * N + t] = y;
}

template <int EPI, int BM, int BN>
hipError_t launch_gemm(const uint16_t* A, int lda, const uint16_t* W, int64_t M, int Nn, int K, const EpiArgs& ep,
                       int n_cu, hipStream_t stream) {
  constexpr int kLdsBytes = 2 * (BM + BN) * (kGemmBK / 8) * 16;
  static bool attr_set = false;  // per instantiation; setting it again is harmless
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_f16_kernel<EPI, BM, BN>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  if (Nn % BN != 0 || K % kGemmBK != 0 || M <= 0) return hipErrorInvalidValue;
  const int m_tiles = (int)((M + BM - 1) / BM), n_tiles = Nn / BN;
  // one workgroup per CU, a multiple of the XCD count, no more than there are tiles per XCD list
  const int per_xcd_tiles = ((m_tiles + kXcds - 1) / kXcds) * n_tiles;
  int wg_per_xcd = n_cu / kXcds;
  if (wg_per_xcd < 1) wg_per_xcd = 1;
  if (wg_per_xcd > per_xcd_tiles) wg_per_xcd = per_xcd_tiles;
  gemm_f16_kernel<EPI, BM, BN><<<kXcds * wg_per_xcd, 512, kLdsBytes, stream>>>(A, lda, W, (int)M, Nn, K, ep);
  return hipGetLastError();
}

#define PKV_TRY(call)                  \
  do {                                 \
    hipError_t e_ = (call);            \
    if (e_ != hipSuccess) return e_;   \
  } while (0)

}  // namespace

namespace {

// The network for one proxy layer (input rows xl [H_kv, N]); writes yhat rows of the target layers ll .. ll_hi - 1.
hipError_t mapper_layer(proxykv_ctx* ctx, MapperWorkspace& m, const float* xl, int64_t N, float* yhat, int ll, int ll_hi,
                        int n_cu, hipStream_t stream) {
  const proxykv_config& c = ctx->cfg;
  const MapperWeights& w = ctx->w;
  int64_t n_win, T;
  window_plan(N, c.win, c.stride, &n_win, &T);
  uint16_t* h1 = (uint16_t*)m.h1.ptr;
  float* x = (float*)m.x.ptr;
  uint16_t* xb = (uint16_t*)m.xb.ptr;
  uint16_t* qk = (uint16_t*)m.qk.ptr;
  uint16_t* vt = (uint16_t*)m.vt.ptr;
  uint16_t* ao = (uint16_t*)m.ao.ptr;
  uint16_t* hid = (uint16_t*)m.hid.ptr;
  uint16_t* zg = (uint16_t*)m.zg.ptr;
  float* s3 = (float*)m.s3.ptr;
  uint32_t* range = (uint32_t*)m.range.ptr;
  const unsigned ew_blocks_N = (unsigned)((N * (kDT / 4) + 255) / 256);

  // stage 1
  {
    const int64_t n_x = (int64_t)c.H_kv * N;
    const unsigned blocks = (unsigned)((n_x + 256 * 16 - 1) / (256 * 16) < 1024 ? (n_x + 256 * 16 - 1) / (256 * 16) : 1024);
    absmax_kernel<<<blocks, 256, 0, stream>>>(xl, n_x, range);
    PKV_TRY(hipGetLastError());
    stem_scale_kernel<<<1, 64, 0, stream>>>(range, w.stem_cw, w.stem_cs);
    PKV_TRY(hipGetLastError());
  }
  stem_conv1_kernel<<<(unsigned)((N + kStemTok - 1) / kStemTok), 256, 0, stream>>>(
      xl, w.conv1_w, w.bn1_scale, w.bn1_shift, reinterpret_cast<const float*>(range), h1, c.H_kv, (int)N, c.c_mid);
  PKV_TRY(hipGetLastError());
  EpiArgs e2 = {};
  e2.p0 = w.bn2_scale;
  e2.p1 = w.bn2_shift;
  e2.p2 = reinterpret_cast<const float*>(range) + 2;
  e2.out_f32 = x;
  e2.out_h = xb;
  e2.ldc = kDT;
  e2.pe = w.pe;
  e2.n_win = (int)n_win;
  PKV_TRY((launch_gemm<kEpiGeluPeWin, 256, 256>(h1, c.c_mid, w.conv2_w, N, kDT, 3 * c.c_mid, e2, n_cu, stream)));

  // stage 2 (the stem's epilogue has written its input rows)
  for (int li = 0; li < c.n_enc_layers; ++li) {
    const EncoderLayerWeights& e = w.enc[li];
    EpiArgs eq = {};
    eq.p0 = e.in_b;
    eq.out_h = qk;
    eq.out_v = vt;
    eq.ldc = 2 * kDT;
    PKV_TRY((launch_gemm<kEpiQkvH, 256, 256>(xb, kDT, e.in_w, T, 3 * kDT, kDT, eq, n_cu, stream)));
    window_attention_kernel<<<(unsigned)(n_win * kHeads * (kWin / 256)), 256, 0, stream>>>(qk, vt, ao, T, (int)n_win);
    PKV_TRY(hipGetLastError());
    EpiArgs eo = {};
    eo.p0 = e.out_b;
    eo.g = e.ln1_g;
    eo.b = e.ln1_b;
    eo.res = x;
    eo.out_f32 = x;
    eo.out_h = xb;
    eo.ldc = kDT;
    PKV_TRY((launch_gemm<kEpiResLn, 128, 512>(ao, kDT, e.out_w, T, kDT, kDT, eo, n_cu, stream)));
    EpiArgs e1 = {};
    e1.p0 = e.ffn1_b;
    e1.out_h = hid;
    e1.ldc = c.d_ffn;
    PKV_TRY((launch_gemm<kEpiBiasReluH, 256, 256>(xb, kDT, e.ffn1_w, T, c.d_ffn, kDT, e1, n_cu, stream)));
    EpiArgs ef = eo;
    ef.p0 = e.ffn2_b;
    ef.g = e.ln2_g;
    ef.b = e.ln2_b;
    PKV_TRY((launch_gemm<kEpiResLn, 128, 512>(hid, c.d_ffn, e.ffn2_w, T, kDT, c.d_ffn, ef, n_cu, stream)));
  }
  overlap_avg_kernel<<<ew_blocks_N, 256, 0, stream>>>(x, zg, N, (int)n_win);
  PKV_TRY(hipGetLastError());

  // stage 3
  const int nkv = kv3_stride(c);
  EpiArgs e3 = {};
  e3.p0 = w.kv_b;
  e3.p1 = w.queries;
  e3.g = w.out_w;
  e3.out_f32 = s3;
  e3.ldc = (c.H_l + 1) * c.H_kv;
  e3.n_slot = c.H_kv;
  e3.n_head = c.H_l;
  PKV_TRY((launch_gemm<kEpiStage3, 256, 256>(zg, kDT, w.kv_w, N, nkv, kDT, e3, n_cu, stream)));
  const int tok_per_block = 256 / c.H_l;
  stage3_kernel<<<(unsigned)((N + tok_per_block - 1) / tok_per_block), 256, 0, stream>>>(s3, w.out_b, yhat, N, c.H_kv, c.H_l, ll,
                                                                                        ll_hi);
  return hipGetLastError();
}

}  // namespace

hipError_t mapper_forward(proxykv_ctx* ctx, const float* x_in, int64_t N, float* yhat, hipStream_t stream) {
  const proxykv_config& c = ctx->cfg;
  int n_cu = 0, dev = 0;
  PKV_TRY(hipGetDevice(&dev));
  PKV_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  int64_t n_win, T;
  window_plan(N, c.win, c.stride, &n_win, &T);
  // distinct proxy layers are dealt round-robin to the lanes; lane 0 is the caller's stream, the others start behind
  // the work already queued there and are joined into it at the end
  const int lanes = map_lanes(T, ctx->distinct_layers);
  if (lanes > 1) {
    PKV_TRY(hipEventRecord(ctx->lane_fork, stream));
    for (int lane = 1; lane < lanes; ++lane) PKV_TRY(hipStreamWaitEvent(ctx->lane_stream[lane], ctx->lane_fork, 0));
  }
  int ll = 0, item = 0;
  while (ll < c.L_l) {
    const int ls = ctx->pairing[ll];
    int ll_hi = ll + 1;
    while (ll_hi < c.L_l && ctx->pairing[ll_hi] == ls) ++ll_hi;
    const int lane = item % lanes;
    PKV_TRY(mapper_layer(ctx, ctx->m[lane], x_in + (size_t)ls * c.H_kv * N, N, yhat, ll, ll_hi, n_cu,
                         lane == 0 ? stream : ctx->lane_stream[lane]));
    ll = ll_hi;
    ++item;
  }
  for (int lane = 1; lane < lanes; ++lane) {
    PKV_TRY(hipEventRecord(ctx->lane_join[lane], ctx->lane_stream[lane]));
    PKV_TRY(hipStreamWaitEvent(stream, ctx->lane_join[lane], 0));
  }
  return hipSuccess;
}

}  // namespace pkv
