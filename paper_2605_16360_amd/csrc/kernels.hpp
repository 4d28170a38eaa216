// Launchers of the HIP kernels; each enqueues on `stream` and returns the launch's hipError_t.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace pkv {

// fp32 -> bf16 (round to nearest even), n elements.
hipError_t launch_f32_to_bf16(const float* in, uint16_t* out, int64_t n, hipStream_t stream);

// Scoring, pass 1: neg_lse[l, h, i] = -log2(sum_k 2^(c * <q_i, k>)) / c with c = log2(e) / sqrt(d),
// the sum running over the N context keys and the visible reconstruction keys of query i.
hipError_t launch_score_lse(const uint16_t* q, const uint16_t* k_ctx, const uint16_t* k_rec, float* neg_lse,
                            int L_s, int H_q, int H_kv, int d, int64_t N, int64_t N_q, int chunk,
                            hipStream_t stream);
// Scoring, pass 2: x[l, g, n] = 2^(c * max over (head of group g, query i) of (<q_i, k_n> + neg_lse[l, h, i])).
hipError_t launch_score_colmax(const uint16_t* q, const uint16_t* k_ctx, const float* neg_lse, float* x,
                               int L_s, int H_q, int H_kv, int d, int64_t N, int64_t N_q,
                               hipStream_t stream);

// Scoring, pass 2 in the sum form: x[l, g, n] = sum over (head of group g, query i) of 2^(c * (<q_i, k_n> + neg_lse[l, h, i])).
// causal: the keys are the queries' own sequence (N == N_q) and query i adds to keys n <= i only.
hipError_t launch_score_colsum(const uint16_t* q, const uint16_t* k_ctx, const float* neg_lse, float* x,
                               int L_s, int H_q, int H_kv, int d, int64_t N, int64_t N_q, bool causal,
                               hipStream_t stream);
// Per-row Top-K.  Rows longer than 36 864 scores are split over several workgroups and need `scratch`
// (topk_scratch_bytes(rows, N) bytes of device memory, any contents, 256-byte aligned; rows <= 65535 then).
constexpr int64_t kTopkSingleMax = 36864;  // longest row one workgroup selects from
size_t topk_scratch_bytes(int64_t rows, int64_t N);
hipError_t launch_topk(const float* scores, int64_t rows, int64_t N, int64_t K, int32_t* idx_out, void* scratch,
                       hipStream_t stream);
// The same selection with every workgroup gathering the token rows it kept: k_out[r, j, :] = k_in[r, idx[r, j], :] and
// likewise v (row_bytes per token, 1024 / (row_bytes / 16) a whole number).
hipError_t launch_topk_gather(const float* scores, int64_t rows, int64_t N, int64_t K, int32_t* idx_out, void* scratch,
                              const void* k_in, const void* v_in, int64_t row_bytes, void* k_out, void* v_out,
                              hipStream_t stream);

hipError_t launch_compact(const void* k_in, const void* v_in, const int32_t* idx, int64_t rows, int64_t N,
                          int64_t K, int64_t row_bytes, void* k_out, void* v_out, hipStream_t stream);

// In-place variant: tokens 0 .. K-1 of every row of k and v become the kept tokens in order.
hipError_t launch_compact_inplace(void* k, void* v, const int32_t* idx, int64_t rows, int64_t N, int64_t K, int64_t row_bytes,
                                  const int32_t* counts, int heads, hipStream_t stream);
// counts [layers, heads] from a layer's ascending flat indices h * N + n (heads * K per layer)
hipError_t launch_head_counts(const int32_t* flat, int64_t layers, int64_t heads, int64_t N, int64_t K, int32_t* counts,
                              hipStream_t stream);
// mask[r, n] = 1 if n is one of idx[r, :], else 0.
hipError_t launch_mask(const int32_t* idx, int64_t rows, int64_t N, int64_t K, uint8_t* mask, hipStream_t stream);
}  // namespace pkv
