// Helpers shared by the two scoring passes: tile geometry, the XOR-swizzled LDS tile layout, the
// global -> register -> LDS staging of a tile, MFMA fragment reads and the v_max3 reduction tree.
#pragma once
#include "common.hpp"

namespace pkv {
namespace {

template <int D>
struct ScoreCfg {
  static constexpr int CPR = D / 8;             // 16-byte chunks per row
  static constexpr int ROWS = 8192 / D;         // rows of one streamed tile (16 KB)
  static constexpr int SUB = ROWS / 32;         // 32-row sub-tiles per tile
  static constexpr int KK = D / 16;             // MFMA k-steps per 32x32 tile
  static constexpr int LOADS = ROWS * CPR / 256;  // 16-byte chunks staged per thread and tile
  static constexpr int TILE_U4 = ROWS * CPR;    // 16-byte units per tile
};
constexpr int kNBuf = 3;

// Block -> (group, item) on a one-dimensional grid.  The hardware deals blocks round-robin to the 8 XCDs, so XCD x
// = block % 8 takes the (layer, KV head) groups x, x + 8, ... one after the other: the `per_group` blocks of a group run
// on one XCD at about the same time and share its L2 copy of the queries they all stream in pass 2 (measured: 4.9 GB
// leave the L2s per launch at N = 32k instead of 18.5 GB with the key blocks of a group dealt over all XCDs).
constexpr int kScoreXcds = 8;
struct GroupBlock {
  int group, item;
};
__device__ __forceinline__ GroupBlock group_block(int per_group) {
  const int xcd = blockIdx.x % kScoreXcds, j = blockIdx.x / kScoreXcds;
  return {(j / per_group) * kScoreXcds + xcd, j % per_group};
}
// number of blocks of such a grid; 0 if it does not fit a one-dimensional launch
inline unsigned group_grid(int64_t n_groups, int64_t per_group) {
  const int64_t blocks = kScoreXcds * ((n_groups + kScoreXcds - 1) / kScoreXcds) * per_group;
  return blocks < (1ll << 31) ? (unsigned)blocks : 0u;
}

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
  const char* tb = reinterpret_cast<const char*>(base) + (size_t)row0 * (D * 2);
  if (row0 + C::ROWS <= row_limit) {  // interior tile: uniform base plus a per-thread 32-bit offset
    const uint32_t off = (uint32_t)(tid / C::CPR) * (D * 2) + (uint32_t)(tid % C::CPR) * 16;
#pragma unroll
    for (int i = 0; i < C::LOADS; ++i)
      r.v[i] = *reinterpret_cast<const u32x4*>(tb + off + (uint32_t)i * (256 / C::CPR) * (D * 2));
  } else {
#pragma unroll
    for (int i = 0; i < C::LOADS; ++i) {
      const int id = tid + 256 * i;
      const int row = id / C::CPR, ch = id % C::CPR;
      int grow = row0 + row;
      grow = grow < row_limit ? grow : row_limit - 1;
      r.v[i] = *reinterpret_cast<const u32x4*>(base + (size_t)grow * D + ch * 8);
    }
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

// max(seed, a[0..15]) as a tree of v_max3 (depth three); the steps can be placed one by one.
struct MaxTree {
  float m0, m1, m2, m3, m4, t0, t1;
};
template <int I>
__device__ __forceinline__ void max_step(const f32x16& a, MaxTree& w, float& run) {
  if constexpr (I == 0) w.m0 = max3f(a[0], a[1], a[2]);
  else if constexpr (I == 1) w.m1 = max3f(a[3], a[4], a[5]);
  else if constexpr (I == 2) w.m2 = max3f(a[6], a[7], a[8]);
  else if constexpr (I == 3) w.m3 = max3f(a[9], a[10], a[11]);
  else if constexpr (I == 4) w.m4 = max3f(a[12], a[13], a[14]);
  else if constexpr (I == 5) w.t0 = max3f(w.m0, w.m1, w.m2);
  else if constexpr (I == 6) w.t1 = max3f(w.m3, w.m4, a[15]);
  else run = max3f(run, w.t0, w.t1);
}
__device__ __forceinline__ float max16_tree(const f32x16& a, float seed) {
  MaxTree w;
  float run = seed;
  static_for<8>([&](auto ic) { max_step<decltype(ic)::value>(a, w, run); });
  return run;
}

constexpr float kNegInf = -__builtin_huge_valf();
// A lane re-bases its partial sum when a logit exceeds its reference by more than 2^kRescaleGap.
constexpr float kRescaleGap = 60.0f;

__device__ __forceinline__ f32x16 splat16(float v) {
  f32x16 r;
#pragma unroll
  for (int i = 0; i < 16; ++i) r[i] = v;
  return r;
}

}  // namespace
}  // namespace pkv
