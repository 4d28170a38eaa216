// HybridAxialMapper forward (paper Sec. 4.1) for one proxy layer at a time:
//   stage 1  conv stem            stem_conv1_kernel (fp32 ALU) + conv 2 as an fp16 MFMA GEMM whose A rows
//                                 are overlapping 3-token spans of the padded conv-1 output
//   stage 2  time-axis encoder    gather_pe_kernel, then per layer: QKV GEMM -> window attention ->
//                                 out-proj GEMM (+residual) -> LayerNorm -> FFN GEMMs -> LayerNorm;
//                                 all sliding windows of the layer are batched along the GEMM M axis
//            overlap averaging    overlap_avg_kernel
//   stage 3  head-axis attention  K/V projection GEMM + stage3_kernel (per token, fp32 ALU)
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

// 8 chunks of 16 bytes per 128-byte LDS row, XOR-swizzled (see score.hip)
__device__ __forceinline__ int swz8(int row) { return (row & 7) ^ ((row >> 3) & 1); }

// ------------------------------------------------------------------------------------------
// stage 1, first convolution: h1[t+1, c] = half(GELU(scale[c] * sum_{h,tap} w[c,h,tap] * x[h, t+tap-1] + shift[c]))
// rows 0 and N+1 of h1 are zero (the padding of the second convolution).
// grid ceil(N / 64), 256 threads; thread owns channels tid, tid+256, ...
// ------------------------------------------------------------------------------------------
constexpr int kStemTok = 64;
constexpr int kMaxHs = 16;

__global__ __launch_bounds__(256) void stem_conv1_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                          const float* __restrict__ scale,
                                                          const float* __restrict__ shift, uint16_t* __restrict__ h1,
                                                          int H_s, int N, int c_mid) {
  __shared__ float xs[kMaxHs][kStemTok + 2];
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
      h1[(size_t)(t0 + tt + 1) * c_mid + c] = to_h(gelu_erf(__builtin_fmaf(acc, sc, sh)));
    }
    if (blockIdx.x == 0) h1[c] = 0;
    if (blockIdx.x == gridDim.x - 1) h1[(size_t)(N + 1) * c_mid + c] = 0;
  }
}

// ------------------------------------------------------------------------------------------
// fp16 GEMM  C[M, Nn] = A[M, K] * W[Nn, K]^T  (+ epilogue), fp32 accumulation.
// A rows start lda elements apart (lda < K gives the overlapping rows of the second convolution).
// 128 x 128 block tile, K step 64, 4 waves in 2 x 2, each 64 x 64 = 2 x 2 MFMA tiles.
// grid (Nn / 128, ceil(M / 128)); K % 64 == 0, Nn % 128 == 0.
// ------------------------------------------------------------------------------------------
enum Epilogue {
  kEpiAffineGeluF32,  // out_f32 = GELU(acc * p0[n] + p1[n])                       (second stem convolution)
  kEpiQkv,            // acc + p0[n]: columns < 2*d_time -> out_h [M, 2*d_time]; the rest -> vt (transposed)
  kEpiBiasResidF32,   // out_f32 = acc + p0[n] + resid[m, n]
  kEpiBiasReluH,   // out_h = relu(acc + p0[n])
  kEpiBiasF32         // out_f32 = acc + p0[n]
};

struct EpiArgs {
  const float* p0;
  const float* p1;
  const float* resid;
  float* out_f32;
  uint16_t* out_h;
  uint16_t* vt;
};

template <int EPI>
__global__ __launch_bounds__(256, 2) void gemm_f16_kernel(const uint16_t* __restrict__ A, int lda,
                                                            const uint16_t* __restrict__ W, int M, int Nn, int K,
                                                            EpiArgs ep) {
  __shared__ u32x4 lds_a[128 * 8];
  __shared__ u32x4 lds_b[128 * 8];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int wm = wave >> 1, wn = wave & 1;
  const int n0 = blockIdx.x * 128, m0 = blockIdx.y * 128;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  u32x4 ra[4], rb[4];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + 256 * i, row = id >> 3, ch = id & 7;
      int m = m0 + row;
      m = m < M ? m : M - 1;
      ra[i] = *reinterpret_cast<const u32x4*>(A + (size_t)m * lda + k0 + ch * 8);
      rb[i] = *reinterpret_cast<const u32x4*>(W + (size_t)(n0 + row) * K + k0 + ch * 8);
    }
  };
  fetch(0);
  for (int k0 = 0; k0 < K; k0 += 64) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int id = tid + 256 * i, row = id >> 3, ch = id & 7;
      lds_a[row * 8 + (ch ^ swz8(row))] = ra[i];
      lds_b[row * 8 + (ch ^ swz8(row))] = rb[i];
    }
    __syncthreads();
    if (k0 + 64 < K) fetch(k0 + 64);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      f16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int ra_row = wm * 64 + i * 32 + l32, rb_row = wn * 64 + i * 32 + l32;
        fa[i] = as_f16x8(lds_a[ra_row * 8 + ((kk * 2 + half) ^ swz8(ra_row))]);
        fb[i] = as_f16x8(lds_b[rb_row * 8 + ((kk * 2 + half) ^ swz8(rb_row))]);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = mfma_f16_32x32x16(fa[i], fb[j], acc[i][j]);
    }
  }

  // epilogue: lane holds column n, rows m_base + (r/4)*8 + half*4 + r%4
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int n = n0 + wn * 64 + j * 32 + l32;
    const float p0 = ep.p0[n];
    const float p1 = (EPI == kEpiAffineGeluF32) ? ep.p1[n] : 0.0f;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int mb = m0 + wm * 64 + i * 32 + rg * 8 + half * 4;  // 4 consecutive rows mb .. mb+3
        if (mb >= M) continue;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[i][j][rg * 4 + e];
        if constexpr (EPI == kEpiQkv) {
          if (n < 2 * kDT) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (mb + e < M) ep.out_h[(size_t)(mb + e) * (2 * kDT) + n] = to_h(v[e] + p0);
          } else {
            // v transposed: vt[window][head][dd][pos], pos = 16-token groups with bits 2 and 3 of the
            // in-group offset swapped, which is the order the P*V MFMA consumes keys in
            const int f = n - 2 * kDT, hd = f >> 6, dd = f & 63;
            const int wk = mb / kWin, p = mb % kWin;
            const int w16 = p & 15;
            const int pos = (p & ~15) | (w16 & 3) | ((w16 & 4) << 1) | ((w16 & 8) >> 1);
            uint16_t* dst = ep.vt + ((size_t)(wk * kHeads + hd) * 64 + dd) * kWin + pos;
            if (mb + 3 < M) {
              f16x4 pk;
#pragma unroll
              for (int e = 0; e < 4; ++e) pk[e] = (_Float16)(v[e] + p0);
              *reinterpret_cast<f16x4*>(dst) = pk;
            } else {
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (mb + e < M) dst[e] = to_h(v[e] + p0);
            }
          }
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int m = mb + e;
            if (m >= M) continue;
            const size_t o = (size_t)m * Nn + n;
            if constexpr (EPI == kEpiAffineGeluF32) ep.out_f32[o] = gelu_erf(__builtin_fmaf(v[e], p0, p1));
            else if constexpr (EPI == kEpiBiasResidF32) ep.out_f32[o] = v[e] + p0 + ep.resid[o];
            else if constexpr (EPI == kEpiBiasReluH) ep.out_h[o] = to_h(__builtin_fmaxf(v[e] + p0, 0.0f));
            else ep.out_f32[o] = v[e] + p0;
          }
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// stage 2 input: window row r = 2048*k + p holds token 1024*k + p;  x = z_local[token] + pe[p]
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void gather_pe_kernel(const float* __restrict__ z_local, const float* __restrict__ pe,
                                                         float* __restrict__ x, uint16_t* __restrict__ xb, int64_t T) {
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;  // one float4 each
  if (gid >= T * (kDT / 4)) return;
  const int64_t r = gid / (kDT / 4);
  const int c4 = (int)(gid % (kDT / 4));
  const int64_t k = r / kWin;
  const int p = (int)(r % kWin);
  const f32x4 a = *reinterpret_cast<const f32x4*>(z_local + (size_t)(k * kStride + p) * kDT + c4 * 4);
  const f32x4 b = *reinterpret_cast<const f32x4*>(pe + (size_t)p * kDT + c4 * 4);
  const f32x4 s = a + b;
  *reinterpret_cast<f32x4*>(x + (size_t)r * kDT + c4 * 4) = s;
  *reinterpret_cast<f16x4*>(xb + (size_t)r * kDT + c4 * 4) = __builtin_convertvector(s, f16x4);
}

// ------------------------------------------------------------------------------------------
// LayerNorm over rows of 512 (eps 1e-5): x = LN(in) * g + b, plus an fp16 copy.  One wave per row.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void layernorm_kernel(const float* __restrict__ in, const float* __restrict__ g,
                                                         const float* __restrict__ b, float* __restrict__ x,
                                                         uint16_t* __restrict__ xb, int64_t T) {
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= T) return;
  const int lane = threadIdx.x & 63;
  const float* src = in + (size_t)row * kDT;
  f32x4 v0 = *reinterpret_cast<const f32x4*>(src + lane * 4);
  f32x4 v1 = *reinterpret_cast<const f32x4*>(src + 256 + lane * 4);
  float s = (v0[0] + v0[1]) + (v0[2] + v0[3]) + (v1[0] + v1[1]) + (v1[2] + v1[3]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
  const float mu = s * (1.0f / kDT);
  v0 -= mu;
  v1 -= mu;
  float q = (v0[0] * v0[0] + v0[1] * v0[1]) + (v0[2] * v0[2] + v0[3] * v0[3]) + (v1[0] * v1[0] + v1[1] * v1[1]) +
            (v1[2] * v1[2] + v1[3] * v1[3]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) q += __shfl_xor(q, off, 64);
  const float rstd = 1.0f / sqrtf(q * (1.0f / kDT) + 1e-5f);
  const f32x4 g0 = *reinterpret_cast<const f32x4*>(g + lane * 4), g1 = *reinterpret_cast<const f32x4*>(g + 256 + lane * 4);
  const f32x4 b0 = *reinterpret_cast<const f32x4*>(b + lane * 4), b1 = *reinterpret_cast<const f32x4*>(b + 256 + lane * 4);
  const f32x4 y0 = v0 * rstd * g0 + b0, y1 = v1 * rstd * g1 + b1;
  *reinterpret_cast<f32x4*>(x + (size_t)row * kDT + lane * 4) = y0;
  *reinterpret_cast<f32x4*>(x + (size_t)row * kDT + 256 + lane * 4) = y1;
  *reinterpret_cast<f16x4*>(xb + (size_t)row * kDT + lane * 4) = __builtin_convertvector(y0, f16x4);
  *reinterpret_cast<f16x4*>(xb + (size_t)row * kDT + 256 + lane * 4) = __builtin_convertvector(y1, f16x4);
}

// ------------------------------------------------------------------------------------------
// Window attention (8 heads x 64, full bidirectional attention inside each window).
// Computes S^T = K Q^T so that a lane owns one query column; P^T then feeds the second MFMA as its
// B operand straight from the accumulator registers, with V^T tiles as the A operand.
// grid (2048 / 256, 8 heads, n_win), 256 threads; wave owns 64 queries.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 2) void window_attention_kernel(const uint16_t* __restrict__ qk,
                                                                   const uint16_t* __restrict__ vt,
                                                                   uint16_t* __restrict__ ao, int64_t T, int n_win) {
  __shared__ u32x4 lds_k[64 * 8];
  __shared__ u32x4 lds_v[64 * 8];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, half = lane >> 5, l32 = lane & 31;
  const int hd = blockIdx.y, wk = blockIdx.z;
  const int64_t base = (int64_t)wk * kWin;
  const int len = (wk < n_win - 1) ? kWin : (int)(T - base);
  const int i0 = blockIdx.x * 256;
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
    for (int cs = 0; cs < 2; ++cs)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[ds][cs][r] = 0.0f;
  float m_run[2] = {-1.0e30f, -1.0e30f}, l_run[2] = {0.0f, 0.0f};

  const uint16_t* kbase = qk + (size_t)base * (2 * kDT) + kDT + hd * 64;
  const uint16_t* vbase = vt + (size_t)(wk * kHeads + hd) * 64 * kWin;
  u32x4 rk[2], rv[2];
  auto fetch = [&](int j0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int id = tid + 256 * i, row = id >> 3, ch = id & 7;
      int j = j0 + row;
      j = j < len ? j : len - 1;
      rk[i] = *reinterpret_cast<const u32x4*>(kbase + (size_t)j * (2 * kDT) + ch * 8);
      rv[i] = *reinterpret_cast<const u32x4*>(vbase + (size_t)row * kWin + j0 + ch * 8);
    }
  };
  fetch(0);
  for (int j0 = 0; j0 < len; j0 += 64) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int id = tid + 256 * i, row = id >> 3, ch = id & 7;
      lds_k[row * 8 + (ch ^ swz8(row))] = rk[i];
      lds_v[row * 8 + (ch ^ swz8(row))] = rv[i];
    }
    __syncthreads();
    if (j0 + 64 < len) fetch(j0 + 64);
    const bool ragged = j0 + 64 > len;
#pragma unroll
    for (int cs = 0; cs < 2; ++cs) {
      f32x16 s[2];
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[ks][r] = 0.0f;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const int row = ks * 32 + l32;
          const f16x8 fk = as_f16x8(lds_k[row * 8 + ((kk * 2 + half) ^ swz8(row))]);
          s[ks] = mfma_f16_32x32x16(fk, bq[cs][kk], s[ks]);
        }
        if (ragged) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = j0 + ks * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
            s[ks][r] = j < len ? s[ks][r] : kNegInf;
          }
        }
      }
      float tmax = kNegInf;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int r = 0; r < 16; r += 2) tmax = max3f(tmax, s[ks][r], s[ks][r + 1]);
      tmax = __builtin_fmaxf(tmax, swap_halves(tmax)) * c;
      if (__builtin_amdgcn_ballot_w64(tmax > m_run[cs])) {
        const float nm = __builtin_fmaxf(m_run[cs], tmax);
        const float alpha = __builtin_amdgcn_exp2f(m_run[cs] - nm);
        l_run[cs] *= alpha;
#pragma unroll
        for (int ds = 0; ds < 2; ++ds)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[ds][cs][r] *= alpha;
        m_run[cs] = nm;
      }
      const float nref = -m_run[cs];
      float lsum = 0.0f;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
        for (int u2 = 0; u2 < 2; ++u2) {
          f32x8 p;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[ks][u2 * 8 + e], c, nref));
            lsum += p[e];
          }
          const f16x8 pb = __builtin_convertvector(p, f16x8);
          const int u = ks * 2 + u2;
#pragma unroll
          for (int ds = 0; ds < 2; ++ds) {
            const int row = ds * 32 + l32;  // V^T fragment: d row, 16-key step u
            const f16x8 fv = as_f16x8(lds_v[row * 8 + ((u * 2 + half) ^ swz8(row))]);
            o[ds][cs] = mfma_f16_32x32x16(fv, pb, o[ds][cs]);
          }
        }
      }
      l_run[cs] += lsum;
    }
  }
#pragma unroll
  for (int cs = 0; cs < 2; ++cs) {
    const float inv = 1.0f / (l_run[cs] + swap_halves(l_run[cs]));
    if (qi[cs] < len) {
      uint16_t* dst = ao + (size_t)(base + qi[cs]) * kDT + hd * 64;
#pragma unroll
      for (int ds = 0; ds < 2; ++ds)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          f16x4 pk;
#pragma unroll
          for (int e = 0; e < 4; ++e) pk[e] = (_Float16)(o[ds][cs][rg * 4 + e] * inv);
          *reinterpret_cast<f16x4*>(dst + ds * 32 + rg * 8 + half * 4) = pk;
        }
    }
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
// stage 3 per token (Eq. 3): kv3[t] = [K slots | V slots] (H_s x 64 each, biases included);
// yhat[ll, h, t] = sum_s softmax_s(<Q_l[h], K[s]> / 8) * <w_o, V[s]> + b_o for every paired target layer ll.
// Block = 256 threads = (256 / H_l) tokens x H_l target heads, token index fastest.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void stage3_kernel(const float* __restrict__ kv3, const float* __restrict__ queries,
                                                      const float* __restrict__ w_o, float b_o, float* __restrict__ yhat,
                                                      int64_t N, int H_s, int H_l, int ll_lo, int ll_hi) {
  __shared__ float u_lds[256 * kMaxHs / 1];  // [token][slot], at most 256 tokens... sized for H_l = 1
  const int tok_per_block = 256 / H_l;
  const int64_t t0 = (int64_t)blockIdx.x * tok_per_block;
  const int row_f = 2 * H_s * 64;
  // phase 1: u[token][s] = <w_o, V[s]>
  for (int i = threadIdx.x; i < tok_per_block * H_s; i += 256) {
    const int tt = i % tok_per_block, s = i / tok_per_block;
    const int64_t t = t0 + tt;
    float acc = 0.0f;
    if (t < N) {
      const float* v = kv3 + (size_t)t * row_f + (H_s + s) * 64;
#pragma unroll
      for (int e = 0; e < 64; e += 4) {
        const f32x4 vv = *reinterpret_cast<const f32x4*>(v + e);
        const f32x4 ww = *reinterpret_cast<const f32x4*>(w_o + e);
        acc += vv[0] * ww[0] + vv[1] * ww[1] + vv[2] * ww[2] + vv[3] * ww[3];
      }
    }
    u_lds[tt * kMaxHs + s] = acc;
  }
  __syncthreads();
  const int tt = threadIdx.x % tok_per_block, h = threadIdx.x / tok_per_block;
  const int64_t t = t0 + tt;
  if (h >= H_l || t >= N) return;
  float logit[kMaxHs];
#pragma unroll
  for (int s = 0; s < kMaxHs; ++s) logit[s] = kNegInf;
  const float* qh = queries + (size_t)h * 64;
#pragma unroll
  for (int s = 0; s < kMaxHs; ++s) {
    if (s < H_s) {
      const float* k = kv3 + (size_t)t * row_f + s * 64;
      float acc = 0.0f;
#pragma unroll
      for (int e = 0; e < 64; e += 4) {
        const f32x4 kk = *reinterpret_cast<const f32x4*>(k + e);
        const f32x4 qq = *reinterpret_cast<const f32x4*>(qh + e);
        acc += kk[0] * qq[0] + kk[1] * qq[1] + kk[2] * qq[2] + kk[3] * qq[3];
      }
      logit[s] = acc * 0.125f;
    }
  }
  float mx = kNegInf;
#pragma unroll
  for (int s = 0; s < kMaxHs; ++s) mx = __builtin_fmaxf(mx, logit[s]);
  float den = 0.0f, num = 0.0f;
#pragma unroll
  for (int s = 0; s < kMaxHs; ++s) {
    if (s < H_s) {
      const float e = __expf(logit[s] - mx);
      den += e;
      num += e * u_lds[tt * kMaxHs + s];
    }
  }
  const float y = num / den + b_o;
  for (int ll = ll_lo; ll < ll_hi; ++ll) yhat[((size_t)ll * H_l + h) * N + t] = y;
}

template <int EPI>
hipError_t launch_gemm(const uint16_t* A, int lda, const uint16_t* W, int64_t M, int Nn, int K, const EpiArgs& ep,
                       hipStream_t stream) {
  dim3 grid((unsigned)(Nn / 128), (unsigned)((M + 127) / 128));
  gemm_f16_kernel<EPI><<<grid, 256, 0, stream>>>(A, lda, W, (int)M, Nn, K, ep);
  return hipGetLastError();
}

#define PKV_TRY(call)                  \
  do {                                 \
    hipError_t e_ = (call);            \
    if (e_ != hipSuccess) return e_;   \
  } while (0)

}  // namespace

hipError_t mapper_forward(proxykv_ctx* ctx, const float* x_in, int64_t N, float* yhat, hipStream_t stream) {
  const proxykv_config& c = ctx->cfg;
  const MapperWeights& w = ctx->w;
  MapperWorkspace& m = ctx->m;
  int64_t n_win, T;
  window_plan(N, c.win, c.stride, &n_win, &T);
  uint16_t* h1 = (uint16_t*)m.h1.ptr;
  float* z_local = (float*)m.z_local.ptr;
  float* x = (float*)m.x.ptr;
  uint16_t* xb = (uint16_t*)m.xb.ptr;
  uint16_t* qk = (uint16_t*)m.qk.ptr;
  uint16_t* vt = (uint16_t*)m.vt.ptr;
  uint16_t* ao = (uint16_t*)m.ao.ptr;
  float* tmp = (float*)m.tmp.ptr;
  uint16_t* hid = (uint16_t*)m.hid.ptr;
  uint16_t* zg = (uint16_t*)m.zg.ptr;
  float* kv3 = (float*)m.kv3.ptr;
  const unsigned ew_blocks_T = (unsigned)((T * (kDT / 4) + 255) / 256);
  const unsigned ew_blocks_N = (unsigned)((N * (kDT / 4) + 255) / 256);

  int ll = 0;
  while (ll < c.L_l) {
    const int ls = ctx->pairing[ll];
    int ll_hi = ll + 1;
    while (ll_hi < c.L_l && ctx->pairing[ll_hi] == ls) ++ll_hi;
    const float* xl = x_in + (size_t)ls * c.H_kv * N;

    // stage 1
    stem_conv1_kernel<<<(unsigned)((N + kStemTok - 1) / kStemTok), 256, 0, stream>>>(xl, w.conv1_w, w.bn1_scale, w.bn1_shift,
                                                                                    h1, c.H_kv, (int)N, c.c_mid);
    PKV_TRY(hipGetLastError());
    EpiArgs e2 = {w.bn2_scale, w.bn2_shift, nullptr, z_local, nullptr, nullptr};
    PKV_TRY(launch_gemm<kEpiAffineGeluF32>(h1, c.c_mid, w.conv2_w, N, kDT, 3 * c.c_mid, e2, stream));

    // stage 2
    gather_pe_kernel<<<ew_blocks_T, 256, 0, stream>>>(z_local, w.pe, x, xb, T);
    PKV_TRY(hipGetLastError());
    for (int li = 0; li < c.n_enc_layers; ++li) {
      const EncoderLayerWeights& e = w.enc[li];
      EpiArgs eq = {e.in_b, nullptr, nullptr, nullptr, qk, vt};
      PKV_TRY(launch_gemm<kEpiQkv>(xb, kDT, e.in_w, T, 3 * kDT, kDT, eq, stream));
      window_attention_kernel<<<dim3(kWin / 256, kHeads, (unsigned)n_win), 256, 0, stream>>>(qk, vt, ao, T, (int)n_win);
      PKV_TRY(hipGetLastError());
      EpiArgs eo = {e.out_b, nullptr, x, tmp, nullptr, nullptr};
      PKV_TRY(launch_gemm<kEpiBiasResidF32>(ao, kDT, e.out_w, T, kDT, kDT, eo, stream));
      layernorm_kernel<<<(unsigned)((T + 3) / 4), 256, 0, stream>>>(tmp, e.ln1_g, e.ln1_b, x, xb, T);
      PKV_TRY(hipGetLastError());
      EpiArgs e1 = {e.ffn1_b, nullptr, nullptr, nullptr, hid, nullptr};
      PKV_TRY(launch_gemm<kEpiBiasReluH>(xb, kDT, e.ffn1_w, T, c.d_ffn, kDT, e1, stream));
      EpiArgs ef = {e.ffn2_b, nullptr, x, tmp, nullptr, nullptr};
      PKV_TRY(launch_gemm<kEpiBiasResidF32>(hid, c.d_ffn, e.ffn2_w, T, kDT, c.d_ffn, ef, stream));
      layernorm_kernel<<<(unsigned)((T + 3) / 4), 256, 0, stream>>>(tmp, e.ln2_g, e.ln2_b, x, xb, T);
      PKV_TRY(hipGetLastError());
    }
    overlap_avg_kernel<<<ew_blocks_N, 256, 0, stream>>>(x, zg, N, (int)n_win);
    PKV_TRY(hipGetLastError());

    // stage 3
    const int nkv = 2 * c.H_kv * c.d_head_x;
    EpiArgs e3 = {w.kv_b, nullptr, nullptr, kv3, nullptr, nullptr};
    PKV_TRY(launch_gemm<kEpiBiasF32>(zg, kDT, w.kv_w, N, nkv, kDT, e3, stream));
    const int tok_per_block = 256 / c.H_l;
    stage3_kernel<<<(unsigned)((N + tok_per_block - 1) / tok_per_block), 256, 0, stream>>>(
        kv3, w.queries, w.out_w, w.out_b, yhat, N, c.H_kv, c.H_l, ll, ll_hi);
    PKV_TRY(hipGetLastError());
    ll = ll_hi;
  }
  return hipSuccess;
}

}  // namespace pkv
