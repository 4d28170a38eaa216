// Host-side state behind the opaque proxykv_ctx: configuration, device workspace and the device
// copy of the mapper weights.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

#include <vector>

#include "../../include/proxykv.h"

namespace pkv {

struct DeviceBuffer {
  void* ptr = nullptr;
  size_t bytes = 0;
};

// Device pointers into one allocation that holds the prepared mapper weights.
struct EncoderLayerWeights {
  const uint16_t* in_w;   // fp16 [3*d_time, d_time]
  const float* in_b;      // [3*d_time]
  const uint16_t* out_w;  // fp16 [d_time, d_time]
  const float* out_b;
  const float *ln1_g, *ln1_b;
  const uint16_t* ffn1_w;  // fp16 [d_ffn, d_time]
  const float* ffn1_b;
  const uint16_t* ffn2_w;  // fp16 [d_time, d_ffn]
  const float* ffn2_b;
  const float *ln2_g, *ln2_b;
};

struct MapperWeights {
  const float* conv1_w;                  // fp32 [c_mid, H_kv*3]
  const float *bn1_scale, *bn1_shift;    // batch norm and conv bias folded: y = conv * scale + shift
  float stem_cw = 0.0f, stem_cs = 0.0f;  // |first conv block's output| <= stem_cw * max|x| + stem_cs (host values)
  const uint16_t* conv2_w;               // fp16 [d_time, 3*c_mid], k index = tap * c_mid + channel
  const float *bn2_scale, *bn2_shift;
  std::vector<EncoderLayerWeights> enc;
  const uint16_t* kv_w;                  // fp16 [2*H_kv*d_head_x, d_time]: key rows, then value rows
  const float* kv_b;                     // [2*H_kv*d_head_x]
  const float* queries;                  // [H_l, d_head_x]
  const float* out_w;                    // [d_head_x]
  float out_b;
  const float* pe;                       // fp32 [win, d_time] sinusoidal table
};

// Mapper activations for ONE proxy layer (the network runs once per distinct proxy layer).
// Row length of the stage-3 K/V projection's output: 2*H_kv*d_head_x rounded up to the GEMM's column tile.
inline int kv3_stride(const proxykv_config& c) { return (2 * c.H_kv * c.d_head_x + 255) / 256 * 256; }

// Distinct proxy layers are independent, so kMapLanes of them run side by side, each on a stream ("lane") and in a
// workspace of its own; lane 0 is the caller's stream.  Short contexts leave most of the chip idle inside one layer's
// kernels (at N = 8192 a layer is 14 336 window rows: 112 output tiles for 256 CUs; 26.7 ms with one lane, 20.3 ms
// with four); at long ones a layer's kernels fill the chip and the lanes only close the gaps at kernel boundaries
// (N = 32 768: 88.6, 86.7, 85.8, 85.2 ms with one to four lanes).
// The environment variable PROXYKV_MAP_LANES (1 .. kMapLanes) overrides the choice, for measurements.
constexpr int kMapLanes = 4;
inline int map_lanes(int64_t window_rows, int distinct_layers) {
  (void)window_rows;
  int lanes = kMapLanes;
  if (const char* env = getenv("PROXYKV_MAP_LANES")) {
    const int v = atoi(env);
    if (v >= 1 && v <= kMapLanes) lanes = v;
  }
  return lanes < distinct_layers ? lanes : (distinct_layers > 0 ? distinct_layers : 1);
}

struct MapperWorkspace {
  DeviceBuffer h1;       // fp16 [(N+2), c_mid]  stem conv1 output with one zero row at each end
  DeviceBuffer x;        // fp32 [T, d_time]     residual stream over all window rows
  DeviceBuffer xb;       // fp16 [T, d_time]     fp16 copy feeding the GEMMs
  DeviceBuffer qk;       // fp16 [T, 2*d_time]   q and k of the current layer
  DeviceBuffer vt;       // fp16 [n_win, heads, 64, win]  v transposed per window and head
  DeviceBuffer ao;       // fp16 [T, d_time]     attention output
  DeviceBuffer hid;      // fp16 [T, d_ffn]
  DeviceBuffer zg;       // fp16 [N, d_time]     overlap-averaged encoder output
  DeviceBuffer s3;       // fp32 [N, (H_l + 1) * H_s]  stage 3: per token the H_l x H_s logits, then <w_o, V[s]> of every slot
  DeviceBuffer range;    // 3 words: largest |score| of the layer (bits), 2^-s and 2^s of the stem's range exponent
};

}  // namespace pkv

struct proxykv_ctx {
  proxykv_config cfg;
  int last_hip_error = 0;
  bool weights_set = false;
  // stage timing: events at the boundaries of the PROXYKV_N_STAGES stages of proxykv_prune
  bool profile = false, ev_created = false;
  hipEvent_t ev[PROXYKV_N_STAGES + 1] = {};
  bool ev_recorded[PROXYKV_N_STAGES + 1] = {};
  pkv::DeviceBuffer weight_blob;
  pkv::MapperWeights w;
  std::vector<int32_t> pairing;  // [L_l] 0-based proxy layer per target layer
  // workspace
  pkv::DeviceBuffer q_bf16, kctx_bf16, krec_bf16;  // bf16 copies of fp32 inputs
  pkv::DeviceBuffer neg_lse;                       // fp32 [L_s, H_q, N_q]
  pkv::DeviceBuffer x_ws;                          // fp32 [L_s, H_kv, N]
  pkv::DeviceBuffer yhat_ws;                       // fp32 [L_l, H_l, N]
  pkv::DeviceBuffer topk_ws;                       // per-row histograms and counters of the Top-K of rows split over workgroups
  bool fused_select = false;                       // proxykv_prune: selection and gather in one launch (measured slower)
  pkv::MapperWorkspace m[pkv::kMapLanes];          // one per lane; only the lanes a length needs are allocated
  // lanes 1 .. kMapLanes-1: streams (default priority, non-blocking) and the events that fork them from and join
  // them into the caller's stream
  bool lanes_created = false;
  hipStream_t lane_stream[pkv::kMapLanes] = {};
  hipEvent_t lane_fork = nullptr, lane_join[pkv::kMapLanes] = {};
  int distinct_layers = 1;                         // distinct proxy layers in `pairing`
};

namespace pkv {

// Number of windows and total window rows for context length N.
inline void window_plan(int64_t N, int win, int stride, int64_t* n_win, int64_t* total_rows) {
  if (N <= win) {
    *n_win = 1;
    *total_rows = N;
    return;
  }
  const int64_t k = (N - win + stride - 1) / stride + 1;
  *n_win = k;
  *total_rows = (k - 1) * (int64_t)win + (N - (k - 1) * (int64_t)stride);
}

// Runs the mapper for every distinct proxy layer; implemented in mapper.hip.
// Returns a hipError_t; the workspace must already be large enough.
hipError_t mapper_forward(proxykv_ctx* ctx, const float* x, int64_t N, float* yhat, hipStream_t stream);

}  // namespace pkv
