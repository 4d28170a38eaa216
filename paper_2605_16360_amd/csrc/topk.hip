// Per-row Top-K selection (paper Sec. 3: the mask keeps the Top-K of the mapped scores per target
// layer and head; Sec. 4.3 names a Top-K kernel that materialises it).  Integer work only: scores
// are turned into order-preserving 32-bit keys, the K-th largest key is found by an 8-bit radix select
// (at most four passes) on the keys relative to the row's smallest key, and one more ordered pass emits the kept indices in ascending order, taking
// equal keys by lower index.  A row of up to 36 864 scores is read from global memory once and its keys stay in
// registers for all passes.  A longer row is split into parts of at most 36 864 scores, one workgroup each, so that
// few long rows still fill the chip: four launches of an 8-bit radix pass on the raw keys whose per-part histograms
// meet in a per-row histogram in device scratch memory (the last workgroup of a row to arrive picks the digit), then
// one launch that writes every part's kept indices behind those of the parts before it.
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

// ---------------------------------------------------------------------------------------------
// Rows of up to kTopkRegMax scores: thread t keeps the keys of the kTopkItems consecutive scores
// [t * kTopkItems, (t + 1) * kTopkItems) in registers, so the row is read from memory once, every radix
// pass runs on registers, and the ordered output needs one prefix sum over the threads' kept counts
// instead of one per tile.  The K-th largest key is found on the keys relative to the row's smallest key, top-aligned
// to the width of the range: digits of the raw key are badly skewed (scores share sign and exponent) and lanes that
// add to the same LDS counter are serialised; digits of the range-relative key are spread over all 256 bins.
// ---------------------------------------------------------------------------------------------
constexpr int kTopkItems = 36;
constexpr int kTopkRegMax = kTopkItems * kTopkThreads;
static_assert(kTopkRegMax == kTopkSingleMax, "kernels.hpp states the longest single-workgroup row");

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

// Ordered gather of the token rows a workgroup has just selected (the mask applied to the target's cache, Sec. 4.3):
// dst[j, :] = src[list[j], :] for j in [j_lo, j_hi), K and V together.  `list` was written by this workgroup before
// the barrier that precedes the call.  cpr = 16-byte chunks per token row.
struct GatherArgs {
  const u32x4* k_in;
  const u32x4* v_in;
  u32x4* k_out;
  u32x4* v_out;
  int cpr;
};
__device__ __forceinline__ void gather_rows(const GatherArgs& ga, size_t in_base, size_t out_base, const int32_t* list,
                                            int j_lo, int j_hi, int tid) {
  const int cpr = ga.cpr, tokens_per_step = kTopkThreads / cpr;
  const int ch = tid % cpr, tsub = tid / cpr;
  if (tsub >= tokens_per_step) return;
  constexpr int kU = 2;
  for (int j0 = j_lo + tsub; j0 < j_hi; j0 += kU * tokens_per_step) {
    u32x4 kv[kU], vv[kU];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const int j = j0 + u * tokens_per_step;
      if (j < j_hi) {
        const size_t src = in_base + (size_t)list[j] * cpr + ch;
        kv[u] = __builtin_nontemporal_load(ga.k_in + src);
        vv[u] = __builtin_nontemporal_load(ga.v_in + src);
      }
    }
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const int j = j0 + u * tokens_per_step;
      if (j < j_hi) {
        const size_t dst = out_base + (size_t)j * cpr + ch;
        __builtin_nontemporal_store(kv[u], ga.k_out + dst);
        __builtin_nontemporal_store(vv[u], ga.v_out + dst);
      }
    }
  }
}

template <bool GATHER>
__global__ __launch_bounds__(kTopkThreads) void topk_reg_kernel(const float* __restrict__ scores, int N, int K,
                                                                int32_t* __restrict__ idx_out, GatherArgs ga) {
  const float* row = scores + (size_t)blockIdx.x * N;
  int32_t* out = idx_out + (size_t)blockIdx.x * K;
  __shared__ uint32_t hist[kTopkWaves][256];
  __shared__ uint32_t tot[2][256];
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

  // the first pass's histograms (one per wave) are cleared under the barrier of the range reduction
  for (int i = tid; i < kTopkWaves * 256; i += kTopkThreads) (&hist[0][0])[i] = 0;
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

  // Pass p counts into tot[p & 1].  First pass: every key counts, one histogram per wave keeps lanes of different waves
  // off the same counter, and their sum goes to tot[0].  Later passes: only the keys under the prefix (a 256th of the
  // row per pass) count, straight into tot[p & 1], which was cleared while the pass before picked its digit.
  uint32_t prefix = 0, krem = (uint32_t)K;
  int pass = 0;
  while (prev_sh > 0) {
    const int shift = prev_sh > 8 ? prev_sh - 8 : 0;
    const uint32_t dmask = (1u << (prev_sh - shift)) - 1u;
    uint32_t* cur = tot[pass & 1];
    if (pass == 0) {
#pragma unroll
      for (int j = 0; j < kTopkItems; ++j)
        if (j < mine) atomicAdd(&hist[wave][((key[j] - kmin) >> shift) & dmask], 1u);
      __syncthreads();
      if (tid < 256) {
        uint32_t sum = 0;
#pragma unroll
        for (int w = 0; w < kTopkWaves; ++w) sum += hist[w][tid];
        cur[tid] = sum;
      }
    } else {
#pragma unroll
      for (int j = 0; j < kTopkItems; ++j) {
        const uint32_t rel = key[j] - kmin;
        if (j < mine && (rel >> prev_sh) == prefix) atomicAdd(&cur[(rel >> shift) & dmask], 1u);
      }
    }
    __syncthreads();
    if (tid < 256) tot[(pass + 1) & 1][tid] = 0;
    if (wave == 0) {
      const uint32_t c0 = cur[4 * lane], c1 = cur[4 * lane + 1], c2 = cur[4 * lane + 2], c3 = cur[4 * lane + 3];
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
    ++pass;
  }
  const uint32_t T = prefix + kmin, eq_take = krem;

  // kept: keys above T, and the eq_take lowest-index keys equal to T.  One prefix sum over the threads carries both
  // counts (each at most 36 864, so 16 bits apiece): the kept equal keys before a thread are min(equal before, eq_take).
  uint32_t n_gt = 0, n_eq = 0;
#pragma unroll
  for (int j = 0; j < kTopkItems; ++j) {
    if (j < mine) {
      n_gt += key[j] > T;
      n_eq += key[j] == T;
    }
  }
  static_assert(kTopkRegMax < 65536, "two 16-bit counts share one prefix sum");
  uint32_t both_total;
  const uint32_t both = block_exclusive_scan((n_gt << 16) | n_eq, wave_a, wave, lane, both_total);
  const uint32_t eq_before = both & 0xffffu, gt_before = both >> 16;
  uint32_t pos = gt_before + (eq_before < eq_take ? eq_before : eq_take);
  uint32_t eq_left = eq_before >= eq_take ? 0u : (eq_take - eq_before < n_eq ? eq_take - eq_before : n_eq);
#pragma unroll
  for (int j = 0; j < kTopkItems; ++j) {
    if (j < mine) {
      const bool take = key[j] > T || (key[j] == T && eq_left > 0);
      if (key[j] == T && eq_left > 0) --eq_left;
      if (take) out[pos++] = i0 + j;
    }
  }
  if constexpr (GATHER) {
    __syncthreads();  // the row's list is complete and visible to the whole workgroup
    gather_rows(ga, (size_t)blockIdx.x * N * ga.cpr, (size_t)blockIdx.x * K * ga.cpr, out, 0, K, tid);
  }
}

// ---------------------------------------------------------------------------------------------
// Rows longer than kTopkRegMax are cut into parts of at most kMwPartMax = 45 056 scores (170 000 scores: four parts,
// so that 112 rows are 448 workgroups, one round on 256 CUs); part p of a row (thread t keeps the keys of the
// consecutive scores [p * part_len + t * kMwItems, + kMwItems) in registers) is one workgroup.  Scratch memory per row (32-bit words):
//   [0, 16)                      state: prefix, krem, then one arrival counter per pass at [4 + pass]
//   [16, 16 + 4 * 256)           the row's histogram of every pass
//   [1040, 1040 + parts * 257)   per part: its histogram of the last pass (256), then its number of keys above the
//                                24-bit prefix that the last pass starts from
// mw_init_kernel clears the first 1040 words of every row; the per-part words are all written by pass 3.
// Pass `pass` takes the digit (key >> (24 - 8 * pass)) & 255 of the keys whose higher bits equal the prefix found so
// far; the workgroup that arrives last at the row's counter has every part's contribution in the row's histogram
// (each part adds its bins, fences, then takes its ticket) and picks the bin that holds the krem-th largest key.
// ---------------------------------------------------------------------------------------------
constexpr int kMwItems = 44, kMwPartMax = kMwItems * kTopkThreads;  // scores per thread and per part
constexpr int kMwStateWords = 16, kMwRowFixedWords = kMwStateWords + 4 * 256, kMwPartWords = 257;

__global__ void mw_init_kernel(uint32_t* __restrict__ scratch, int rows, int row_words, int K) {
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (int64_t)rows * kMwRowFixedWords) return;
  const int r = (int)(gid / kMwRowFixedWords), w = (int)(gid % kMwRowFixedWords);
  scratch[(size_t)r * row_words + w] = (w == 1) ? (uint32_t)K : 0u;  // word 0: prefix, word 1: krem
}

// keys of part `part` of the row in registers; positions at and past the part's end hold key 0 and are never counted
__device__ __forceinline__ int mw_load_keys(const float* row, int N, int part_len, int part, int tid, uint32_t (&key)[kMwItems],
                                            int& i0) {
  const int lo = part * part_len, hi = lo + part_len < N ? lo + part_len : N;
  i0 = lo + tid * kMwItems;
  if ((reinterpret_cast<uintptr_t>(row + i0) & 15) == 0 && i0 + kMwItems <= hi) {
#pragma unroll
    for (int j = 0; j < kMwItems; j += 4) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(row + i0 + j);
      key[j] = order_key(v[0]);
      key[j + 1] = order_key(v[1]);
      key[j + 2] = order_key(v[2]);
      key[j + 3] = order_key(v[3]);
    }
  } else {
#pragma unroll
    for (int j = 0; j < kMwItems; ++j) key[j] = i0 + j < hi ? order_key(row[i0 + j]) : 0u;
  }
  return hi - i0 < 0 ? 0 : (hi - i0 < kMwItems ? hi - i0 : kMwItems);
}

// grid (parts, rows)
__global__ __launch_bounds__(kTopkThreads) void mw_pass_kernel(const float* __restrict__ scores, int N, int part_len,
                                                               int pass, uint32_t* __restrict__ scratch, int row_words) {
  const int part = blockIdx.x, parts = gridDim.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float* row = scores + (size_t)blockIdx.y * N;
  uint32_t* rs = scratch + (size_t)blockIdx.y * row_words;
  __shared__ uint32_t hist[kTopkWaves][256];
  __shared__ uint32_t tot[256];
  __shared__ uint32_t s_last, wave_hi[kTopkWaves];
  uint32_t key[kMwItems];
  int i0;
  const int mine = mw_load_keys(row, N, part_len, part, tid, key, i0);
  const uint32_t prefix = rs[0];  // the bits above `shift + 8` of the K-th largest key (written by the previous launch)
  const int shift = 24 - 8 * pass;
  for (int i = tid; i < kTopkWaves * 256; i += kTopkThreads) (&hist[0][0])[i] = 0;
  __syncthreads();
  uint32_t n_hi = 0;  // last pass: keys above the prefix
#pragma unroll
  for (int j = 0; j < kMwItems; ++j) {
    const bool valid = j < mine;
    const bool match = valid && (pass == 0 || (key[j] >> (shift + 8)) == prefix);
    const uint32_t digit = (key[j] >> shift) & 255u;
    // scores of one row share sign and exponent, so in the first passes most lanes of a wave hit one counter: a wave
    // whose matching lanes all carry the same digit adds their number once
    const uint64_t bm = __builtin_amdgcn_ballot_w64(match);
    if (bm != 0) {
      const uint32_t d0 = __builtin_amdgcn_readlane(digit, __builtin_ctzll(bm));
      const uint64_t same = __builtin_amdgcn_ballot_w64(match && digit == d0);
      if (same == bm) {
        if (lane == (int)__builtin_ctzll(bm)) atomicAdd(&hist[wave][d0], (uint32_t)__popcll(bm));
      } else if (match) {
        atomicAdd(&hist[wave][digit], 1u);
      }
    }
    if (pass == 3) n_hi += valid && (key[j] >> 8) > prefix;
  }
  __syncthreads();
  if (tid < 256) {
    uint32_t sum = 0;
#pragma unroll
    for (int w = 0; w < kTopkWaves; ++w) sum += hist[w][tid];
    if (sum) atomicAdd(&rs[kMwStateWords + pass * 256 + tid], sum);
    if (pass == 3) rs[kMwRowFixedWords + part * kMwPartWords + tid] = sum;
  }
  if (pass == 3) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) n_hi += __shfl_xor(n_hi, off, 64);
    if (lane == 0) wave_hi[wave] = n_hi;
    __syncthreads();
    if (tid == 0) {
      uint32_t t = 0;
#pragma unroll
      for (int w = 0; w < kTopkWaves; ++w) t += wave_hi[w];
      rs[kMwRowFixedWords + part * kMwPartWords + 256] = t;
    }
  }
  // This part's bins are in the row's histogram before its ticket is taken: the adds are device-scope atomics, carried
  // out where all workgroups meet, and the barrier lets no wave pass before its own adds have been acknowledged.  (A
  // device-wide fence here instead costs a write-back of the whole L2 per workgroup: 200 us per launch at 560 groups.)
  __syncthreads();
  if (tid == 0) s_last = (atomicAdd(&rs[4 + pass], 1u) == (uint32_t)(parts - 1));
  __syncthreads();
  if (!s_last) return;
  if (tid < 256) tot[tid] = atomicAdd(&rs[kMwStateWords + pass * 256 + tid], 0u);  // read where the adds met
  __syncthreads();
  if (wave == 0) {
    const uint32_t krem = rs[1];
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
        rs[0] = (prefix << 8) | (uint32_t)(4 * lane + bsel);
        rs[1] = krem - above[bsel];
      }
    }
  }
}

// grid (parts, rows): rs[0] is the K-th largest key T, rs[1] the number of keys equal to T that are kept (lowest
// index first).  A part's first output slot follows from the last-pass histograms of the parts before it.
template <bool GATHER>
__global__ __launch_bounds__(kTopkThreads) void mw_write_kernel(const float* __restrict__ scores, int N, int K, int part_len,
                                                                const uint32_t* __restrict__ scratch, int row_words,
                                                                int32_t* __restrict__ idx_out, GatherArgs ga) {
  const int part = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float* row = scores + (size_t)blockIdx.y * N;
  const uint32_t* rs = scratch + (size_t)blockIdx.y * row_words;
  int32_t* out = idx_out + (size_t)blockIdx.y * K;
  __shared__ uint32_t wave_a[kTopkWaves], wave_b[kTopkWaves];
  uint32_t key[kMwItems];
  int i0;
  const int mine = mw_load_keys(row, N, part_len, part, tid, key, i0);
  const uint32_t T = rs[0], eq_take = rs[1], t8 = T & 255u;
  // keys above T and keys equal to T in the parts before this one
  uint32_t g = 0, e = 0;
  if (tid < 256) {
    for (int q = 0; q < part; ++q) {
      const uint32_t* ph = rs + kMwRowFixedWords + q * kMwPartWords;
      const uint32_t h = ph[tid];
      g += (uint32_t)tid > t8 ? h : 0u;
      e += (uint32_t)tid == t8 ? h : 0u;
      if (tid == 0) g += ph[256];
    }
  }
  uint32_t gt_before, eq_before_parts;
  (void)block_exclusive_scan(g, wave_a, wave, lane, gt_before);
  (void)block_exclusive_scan(e, wave_b, wave, lane, eq_before_parts);

  uint32_t n_gt = 0, n_eq = 0;
#pragma unroll
  for (int j = 0; j < kMwItems; ++j) {
    if (j < mine) {
      n_gt += key[j] > T;
      n_eq += key[j] == T;
    }
  }
  uint32_t tot_eq, tot_kept;
  const uint32_t eq_before = eq_before_parts + block_exclusive_scan(n_eq, wave_a, wave, lane, tot_eq);
  const uint32_t eq_mine = eq_before >= eq_take ? 0u : (eq_take - eq_before < n_eq ? eq_take - eq_before : n_eq);
  const uint32_t part_pos = gt_before + (eq_before_parts < eq_take ? eq_before_parts : eq_take);
  uint32_t pos = part_pos + block_exclusive_scan(n_gt + eq_mine, wave_b, wave, lane, tot_kept);
  uint32_t eq_left = eq_mine;
#pragma unroll
  for (int j = 0; j < kMwItems; ++j) {
    if (j < mine) {
      const bool take = key[j] > T || (key[j] == T && eq_left > 0);
      if (key[j] == T && eq_left > 0) --eq_left;
      if (take) out[pos++] = i0 + j;
    }
  }
  if constexpr (GATHER) {
    __syncthreads();  // this part's stretch of the list is complete and visible to the whole workgroup
    gather_rows(ga, (size_t)blockIdx.y * N * ga.cpr, (size_t)blockIdx.y * K * ga.cpr, out, (int)part_pos,
                (int)(part_pos + tot_kept), tid);
  }
}

}  // namespace

// parts of a row that is too long for one register-resident workgroup (may be one)
static int topk_parts(int64_t N) { return (int)((N + kMwPartMax - 1) / kMwPartMax); }

size_t topk_scratch_bytes(int64_t rows, int64_t N) {
  if (N <= kTopkRegMax || rows <= 0) return 0;
  const int parts = topk_parts(N);
  return (size_t)rows * (size_t)(kMwRowFixedWords + parts * kMwPartWords) * 4;
}

// gather != nullptr: every workgroup also gathers the token rows it selected (k/v in [rows, N, row_bytes], out [rows, K, row_bytes])
static hipError_t launch_topk_impl(const float* scores, int64_t rows, int64_t N, int64_t K, int32_t* idx_out, void* scratch,
                                   const GatherArgs* gather, hipStream_t stream) {
  if (rows <= 0) return hipSuccess;
  const GatherArgs none = {nullptr, nullptr, nullptr, nullptr, 0};
  const int parts = topk_parts(N);
  if (N <= kTopkRegMax) {
    if (gather) topk_reg_kernel<true><<<dim3((unsigned)rows), kTopkThreads, 0, stream>>>(scores, (int)N, (int)K, idx_out, *gather);
    else topk_reg_kernel<false><<<dim3((unsigned)rows), kTopkThreads, 0, stream>>>(scores, (int)N, (int)K, idx_out, none);
    return hipGetLastError();
  }
  if (scratch == nullptr || rows > 65535) return hipErrorInvalidValue;
  // parts of equal length, a multiple of four scores (16-byte loads when the row itself is aligned)
  const int part_len = (int)((((N + parts - 1) / parts) + 3) & ~(int64_t)3);
  const int row_words = kMwRowFixedWords + parts * kMwPartWords;
  uint32_t* sc = (uint32_t*)scratch;
  const int64_t init_words = rows * kMwRowFixedWords;
  mw_init_kernel<<<(unsigned)((init_words + 255) / 256), 256, 0, stream>>>(sc, (int)rows, row_words, (int)K);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const dim3 grid((unsigned)parts, (unsigned)rows);
  for (int pass = 0; pass < 4; ++pass) {
    mw_pass_kernel<<<grid, kTopkThreads, 0, stream>>>(scores, (int)N, part_len, pass, sc, row_words);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (gather) mw_write_kernel<true><<<grid, kTopkThreads, 0, stream>>>(scores, (int)N, (int)K, part_len, sc, row_words, idx_out, *gather);
  else mw_write_kernel<false><<<grid, kTopkThreads, 0, stream>>>(scores, (int)N, (int)K, part_len, sc, row_words, idx_out, none);
  return hipGetLastError();
}

hipError_t launch_topk(const float* scores, int64_t rows, int64_t N, int64_t K, int32_t* idx_out, void* scratch,
                       hipStream_t stream) {
  return launch_topk_impl(scores, rows, N, K, idx_out, scratch, nullptr, stream);
}

hipError_t launch_topk_gather(const float* scores, int64_t rows, int64_t N, int64_t K, int32_t* idx_out, void* scratch,
                              const void* k_in, const void* v_in, int64_t row_bytes, void* k_out, void* v_out,
                              hipStream_t stream) {
  const GatherArgs ga = {(const u32x4*)k_in, (const u32x4*)v_in, (u32x4*)k_out, (u32x4*)v_out, (int)(row_bytes / 16)};
  if (ga.cpr < 1 || ga.cpr > kTopkThreads || kTopkThreads % ga.cpr != 0) return hipErrorInvalidValue;
  return launch_topk_impl(scores, rows, N, K, idx_out, scratch, &ga, stream);
}

}  // namespace pkv
