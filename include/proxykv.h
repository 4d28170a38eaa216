/*
 * proxykv.h -- C ABI of the MI355X (gfx950) implementation of the ProxyKV hot path:
 *
 *     score  ->  map  ->  top-k  ->  compact        (and the fused  prune)
 *
 * ProxyKV ("Cross-Model Proxy Pruning for Efficient Long-Context LLM Inference") lets a small
 * proxy model score the importance of every context token, maps those scores onto the layers and
 * heads of the large target model with the HybridAxialMapper, keeps the Top-K tokens per target
 * head and evicts the rest of the target's KV cache.  This library is that data path; the two
 * language models themselves are not part of it.
 *
 * Notation (paper, Sec. 3): proxy with L_s layers, H_q query heads, H_kv (= the paper's H_s) KV
 * heads, head width d; context length N; N_q reconstruction queries handled in chunks of `chunk`
 * queries; target with L_l layers, H_l KV heads, head width D; retention ratio rho; B = 1.
 *
 * Conventions for every entry point
 *   - Tensor arguments are DEVICE pointers owned by the caller, dense row-major in the stated
 *     layout and 16-byte aligned, unless the comment says "host".  The library never frees or
 *     reallocates them and keeps no reference after the call's work has run.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream) and the
 *     call returns without synchronising.  Outputs are valid once the stream has been synchronised.
 *   - A context owns device workspace (row log-sum-exps, mapper activations, histograms) and a
 *     device copy of the mapper weights.  Workspace grows on demand inside a call; call
 *     proxykv_reserve beforehand to keep allocation out of a timed or captured region.
 *     One context serves one stream at a time; concurrent calls on one context race.
 *   - Return value: PROXYKV_OK (0) or a negative proxykv_status.  All argument checks run before
 *     the first HIP call, so PROXYKV_EINVAL / PROXYKV_EUNSUPPORTED are returned on any machine.
 *     PROXYKV_EHIP means a HIP runtime call failed; proxykv_last_hip_error gives its code.
 */
#ifndef PROXYKV_H
#define PROXYKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct proxykv_ctx proxykv_ctx;

typedef enum {
  PROXYKV_OK = 0,
  PROXYKV_EINVAL = -1,       /* null pointer, non-positive size, ratio outside (0,1], K outside [1,N], ... */
  PROXYKV_EUNSUPPORTED = -2, /* a shape or switch this build has no kernel for */
  PROXYKV_ENOMEM = -3,       /* device allocation failed */
  PROXYKV_ESTATE = -4,       /* mapper weights not set, context destroyed, ... */
  PROXYKV_EHIP = -5,         /* a HIP runtime call failed */
  PROXYKV_ELIMIT = -6        /* a size beyond the fixed limit that the entry point documents */
} proxykv_status;

typedef enum { PROXYKV_BF16 = 0, PROXYKV_FP32 = 1 } proxykv_dtype;

/* Reduction over the query axis that turns attention probabilities into a per-key score.
 * MAX: maximum over reconstruction queries and over the query heads of a GQA group (the
 * reconstruction-style score the proxy runs in place of the target's second prefill, Sec. 1/3).
 * SUM: the accumulation over the query axis printed in Sec. 3, summed over the heads of the group as
 * well; the same reconstruction queries, chunks and visibility as MAX. */
typedef enum { PROXYKV_REDUCE_MAX = 0, PROXYKV_REDUCE_SUM = 1 } proxykv_reduce;

typedef struct {
  /* proxy and target shapes */
  int32_t L_s, H_q, H_kv, d; /* d in {64, 128}; H_q a multiple of H_kv */
  int32_t L_l, H_l, D;       /* D*2 bytes must be a multiple of 16 */
  /* HybridAxialMapper (Sec. 4.1).  The paper fixes d_time = 512, 6 encoder layers, 8 heads,
   * FFN 4*d_time, window 2048, stride 1024; c_mid (width between the two stem convolutions) and
   * d_head_x (width of the stage-3 head slots) are not given there: 256 and 64 are this build's
   * reading.  This build has kernels for d_time = 512, n_enc_heads = 8 (head width 64),
   * d_head_x = 64, c_mid and d_ffn multiples of 256, win = 2048, stride = 1024, H_kv <= 16,
   * H_l <= 64 (PROXYKV_EUNSUPPORTED otherwise). */
  int32_t d_time, c_mid, n_enc_layers, n_enc_heads, d_ffn, d_head_x, win, stride;
  int32_t reduce; /* proxykv_reduce */
  int32_t device; /* HIP device ordinal */
} proxykv_config;

/* Fills the mapper fields of *cfg with the values above (512, 256, 6, 8, 2048, 64, 2048, 1024),
 * reduce = MAX, device = 0.  Shapes are left untouched. */
void proxykv_default_mapper(proxykv_config* cfg);

/* Creates a context.  Validates cfg; touches no device. */
int proxykv_create(proxykv_ctx** out, const proxykv_config* cfg);
/* Frees the context's device memory and the context.  NULL is allowed. */
int proxykv_destroy(proxykv_ctx* ctx);

/* Number of floats in the mapper weight blob for cfg; 0 if cfg is invalid.  Blob layout (all
 * fp32, concatenated in this order, each tensor dense row-major):
 *   stem: conv1.weight [c_mid, H_kv, 3], conv1.bias [c_mid], bn1.gamma, bn1.beta, bn1.mean,
 *         bn1.var [c_mid each]; conv2.weight [d_time, c_mid, 3], conv2.bias [d_time], bn2.gamma,
 *         bn2.beta, bn2.mean, bn2.var [d_time each]                        (Sec. 4.1, Eq. 2)
 *   for each encoder layer: in_proj.weight [3*d_time, d_time] (rows: q, k, v), in_proj.bias,
 *         out_proj.weight [d_time, d_time], out_proj.bias, ln1.gamma, ln1.beta,
 *         ffn1.weight [d_ffn, d_time], ffn1.bias, ffn2.weight [d_time, d_ffn], ffn2.bias,
 *         ln2.gamma, ln2.beta                                              (Sec. 4.1, stage 2)
 *   head: k_proj.weight [H_kv*d_head_x, d_time], k_proj.bias, v_proj.weight, v_proj.bias,
 *         queries [H_l, d_head_x], out.weight [d_head_x], out.bias [1]    (Sec. 4.1, Eq. 3) */
size_t proxykv_mapper_weight_count(const proxykv_config* cfg);
/* Copies the blob (HOST pointer, n_floats as above) to the device, pre-rounding matrix operands to
 * fp16 and folding the inference-mode batch-norm statistics into per-channel scale/shift.
 * Synchronous. */
int proxykv_set_mapper_weights(proxykv_ctx* ctx, const float* blob_host, size_t n_floats);

/* Device workspace, in bytes, that score + map + top-k + compact need for this context length. */
int proxykv_workspace_bytes(const proxykv_config* cfg, int64_t N, int64_t N_q, size_t* out_bytes);
/* Allocates that workspace now (synchronous) so that later calls do not allocate. */
int proxykv_reserve(proxykv_ctx* ctx, int64_t N, int64_t N_q);

/* K = clamp(floor(keep_ratio * N), 1, N), evaluated in IEEE double (Sec. 3: Top-K at retention
 * ratio rho in (0,1]; the rounding is this build's reading).  *K_out is a host integer. */
int proxykv_keep_count(int64_t N, double keep_ratio, int64_t* K_out);
/* Depth-proportional layer pairing (Sec. 4.1): pairing_host[l_l] = ceil((l_l+1)*L_s/L_l) - 1 for
 * l_l = 0..L_l-1 (0-based proxy layer for each 0-based target layer).  HOST array of L_l ints. */
int proxykv_layer_pairing(const proxykv_config* cfg, int32_t* pairing_host);

/* Proxy importance score (Sec. 3, system overview and problem formulation).
 *   q_rec [L_s, H_q, N_q, d]  reconstruction queries (post-RoPE)
 *   k_ctx [L_s, H_kv, N, d]   context keys
 *   k_rec [L_s, H_kv, N_q, d] keys of the reconstruction tokens
 *   dtype: element type of the three inputs; fp32 inputs are rounded to bf16 (nearest even) first
 *   x_out [L_s, H_kv, N] fp32
 * Query i of query head h (KV head h / (H_q/H_kv)) sees the N context keys and the reconstruction
 * keys j of its own chunk (i / chunk == j / chunk) with j <= i; probabilities are the softmax of
 * <q, k> / sqrt(d) over that set; x_out[l, g, n] is the maximum probability that context key n
 * receives from any query of any head of group g (reduce = MAX), or the sum of those probabilities
 * over all of them (reduce = SUM).  QK^T runs on bf16 MFMA with fp32 accumulation. */
int proxykv_score(proxykv_ctx* ctx, const void* q_rec, const void* k_ctx, const void* k_rec,
                  int32_t dtype, int64_t N, int64_t N_q, int32_t chunk, float* x_out, void* stream);

/* The proxy feature in the form Sec. 3 (system overview) prints: the post-softmax attention of the
 * proxy's own prefill accumulated over the query axis,
 *   x_out[l, g, n] = sum over the heads h of group g and the queries i >= n of
 *                    softmax_{j <= i}(<q_i, k_j> / sqrt(d))[n]
 * (causal, as in a decoder's prefill; the G query heads of a KV head are summed).
 *   q [L_s, H_q, N, d], k [L_s, H_kv, N, d] (DEVICE, dtype as in proxykv_score); x_out [L_s, H_kv, N] fp32.
 * The scores of one (layer, KV head) add up to G * N.  The reduce field of the config is not used. */
int proxykv_score_self(proxykv_ctx* ctx, const void* q, const void* k, int32_t dtype, int64_t N,
                       float* x_out, void* stream);

/* HybridAxialMapper forward (Sec. 4.1): x [L_s, H_kv, N] fp32 -> yhat [L_l, H_l, N] fp32 raw logits.
 * Target layer l_l reads proxy layer pairing[l_l]; weights are shared, so target layers paired with
 * the same proxy layer receive identical rows and the network runs once per distinct proxy layer.
 * Stage 1: two Conv1D(k=3, pad 1) + batch norm (inference) + GELU(erf); stage 2: sinusoidal
 * positions restarting in every window, post-norm encoder layers (ReLU FFN) on windows
 * [stride*k, min(stride*k + win, N)), outputs averaged where windows overlap; stage 3: per-token
 * attention of the H_l learned queries over H_kv projected slots, then a linear map to one logit.
 * Matrix products take IEEE half (fp16) operands and accumulate in fp32; the rest is fp32.
 * Needs proxykv_set_mapper_weights (ESTATE otherwise).
 * Distinct proxy layers run side by side on up to four streams that the context owns (default priority); they start
 * behind the work already queued on `stream` and are joined into it by events before the call returns, so for the
 * caller everything is ordered on `stream` as for the other entry points. */
int proxykv_map(proxykv_ctx* ctx, const float* x, int64_t N, float* yhat, void* stream);

/* Per-row Top-K (Sec. 3: mask M by Top-K thresholding of the mapped scores; Sec. 4.3).
 *   scores [rows, N] fp32, idx_out [rows, K] int32.
 * Keeps the K entries that come first under the total order (higher score first, equal scores by
 * lower index; -0.0 == +0.0; NaN below every number) and writes their indices in ascending order.
 * A row of up to 36 864 scores is selected by one workgroup; a longer row is split over several, which meet in
 * per-row histograms in the context's workspace (then rows <= 65535, PROXYKV_EUNSUPPORTED otherwise). */
int proxykv_topk(proxykv_ctx* ctx, const float* scores, int64_t rows, int64_t N, int64_t K,
                 int32_t* idx_out, void* stream);

/* proxykv_topk for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same result, but the call allocates nothing (no hipMalloc, no hipFree, no
 * workspace growth): the per-row histograms and counters that rows longer than 36 864 scores need live in a fixed
 * array of 8 MiB inside the library's device image (every GPU the library runs on holds it until the process ends).
 * Rows of up to 36 864 scores need none of it.  For longer rows the call needs
 *     rows * (1040 + 257 * ceil(N / 45056)) * 4 bytes <= proxykv_topk_static_limit() = 8 MiB
 * (1014 rows of 170 000 scores, 812 of 262 144) and returns PROXYKV_ELIMIT beyond that, before any device work.
 * All calls on one GPU share the array: calls that overlap in time on one GPU (different streams or contexts) race;
 * calls on one stream are ordered and each clears what it needs with a kernel of its own (no memset node, so the
 * call can be captured).  The first call on a device looks up the array's address (the runtime loads the device
 * image then): make one call of any size before capturing. */
int proxykv_topk_static(proxykv_ctx* ctx, const float* scores, int64_t rows, int64_t N, int64_t K,
                        int32_t* idx_out, void* stream);
size_t proxykv_topk_static_limit(void);

/* Applies the mask to the target cache (Sec. 3, Sec. 4.3): for r < rows, j < K
 *   k_out[r, j, :] = k_in[r, idx[r, j], :]   and the same for v.
 *   k_in, v_in [rows, N, D] 16-bit elements; idx [rows, K] int32 in [0, N); k_out, v_out
 *   [rows, K, D].  rows = L_l * H_l.  Outputs must not overlap inputs.  Indices are not checked
 *   on the device: out-of-range indices are the caller's error (proxykv_topk never produces one).
 *   Limits: rows <= 65535 (PROXYKV_EINVAL); D*2 bytes a multiple of 16, at most 4096, and D*2/16 a divisor of
 *   256 (PROXYKV_EUNSUPPORTED). */
int proxykv_compact(proxykv_ctx* ctx, const void* k_in, const void* v_in, const int32_t* idx,
                    int64_t rows, int64_t N, int64_t K, int64_t D, void* k_out, void* v_out,
                    void* stream);

/* The same gather applied to the cache where it lies (Sec. 4.3: the mask is applied to the target's
 * cache; App. B: the target's memory drops once it is): k, v [rows, N, D] 16-bit elements are both
 * source and destination.  Afterwards tokens 0 .. K-1 of every row are the kept tokens in order
 * (k[r, j, :] = old k[r, idx[r, j], :]); tokens K .. N-1 are left as they were.  idx [rows, K] must be
 * strictly ascending within a row (as proxykv_topk writes it): the kernel relies on idx[r, j] >= j.
 * D*2 bytes a multiple of 16 and at most 512. */
int proxykv_compact_inplace(proxykv_ctx* ctx, void* k, void* v, const int32_t* idx, int64_t rows,
                            int64_t N, int64_t K, int64_t D, void* stream);

/* The binary mask M of Sec. 3 from the kept indices: mask_out [rows, N] uint8 (DEVICE),
 * mask_out[r, n] = 1 if n is one of idx[r, 0 .. K-1], else 0.  Every byte of mask_out is written. */
int proxykv_mask(proxykv_ctx* ctx, const int32_t* idx, int64_t rows, int64_t N, int64_t K,
                 uint8_t* mask_out, void* stream);

/* Top-K with one budget per target layer instead of one per head (Sec. 3 thresholds the mapped scores
 * at a retention ratio and does not say whether heads share it; KVZip, whose scores the mapper
 * imitates, lets them): scores [layers, heads, N] fp32; of a layer's heads*N (head, token) pairs the
 * heads*K that come first under proxykv_topk's order (ties to the lower flat index h*N + n) are kept.
 *   flat_out [layers, heads*K] int32: the kept flat indices h*N + n, ascending, so the tokens of
 *     head h are the entries in [h*N, (h+1)*N) minus h*N, ascending, and follow those of head h-1;
 *   counts_out [layers, heads] int32: how many of them belong to each head (sum = heads*K).
 * heads*N must stay below 2^31 - 4096. */
int proxykv_topk_pooled(proxykv_ctx* ctx, const float* scores, int64_t layers, int64_t heads,
                        int64_t N, int64_t K, int32_t* flat_out, int32_t* counts_out, void* stream);

/* proxykv_compact_inplace for the lists proxykv_topk_pooled writes: k, v [layers, heads, N, D] 16-bit
 * elements; afterwards tokens 0 .. counts[l, h]-1 of row (l, h) are that head's kept tokens in order,
 * the rest of the row is left as it was.  flat and counts must be a pair written by
 * proxykv_topk_pooled with the same layers, heads, N, K (not checked on the device). */
int proxykv_compact_pooled(proxykv_ctx* ctx, void* k, void* v, const int32_t* flat,
                           const int32_t* counts, int64_t layers, int64_t heads, int64_t N, int64_t K,
                           int64_t D, void* stream);

/* The whole path on one stream: score -> map -> top-k -> compact, with
 * K = proxykv_keep_count(N, keep_ratio) written to *K_host (HOST, may be NULL).
 *   k_in, v_in [L_l, H_l, N, D]; k_out, v_out [L_l, H_l, K, D]; idx_out [L_l, H_l, K] int32;
 *   x_out [L_s, H_kv, N] and yhat_out [L_l, H_l, N] are optional (NULL = kept in workspace). */
int proxykv_prune(proxykv_ctx* ctx, const void* q_rec, const void* k_ctx, const void* k_rec,
                  int32_t dtype, int64_t N, int64_t N_q, int32_t chunk, double keep_ratio,
                  const void* k_in, const void* v_in, void* k_out, void* v_out, int32_t* idx_out,
                  float* x_out, float* yhat_out, int64_t* K_host, void* stream);

/* Sec. 4.3 names a Top-K kernel that materialises the mask in place.  With this switch on proxykv_prune runs
 * selection and gather as ONE launch: the workgroup that has written a stretch of a row's kept indices moves those
 * tokens' K and V rows itself (stage timing then books the whole launch as the compaction stage).  Off (the default:
 * measured faster, a row's gather is then spread over many small workgroups): the kernels of proxykv_topk and
 * proxykv_compact one after the other.  Same bits either way. */
int proxykv_set_fused_select(proxykv_ctx* ctx, int on);

/* Stage timing of proxykv_prune, for benchmarks.  With timing switched on, proxykv_prune records a
 * HIP event on its stream at each stage boundary (no synchronisation, no allocation in the call).
 * proxykv_profile_read waits for the last event of the most recent proxykv_prune and writes the
 * PROXYKV_N_STAGES durations in milliseconds to ms_host (HOST array): score pass 1 (row
 * log-sum-exp), score pass 2 (column max), mapper, top-k, compaction.  ESTATE if timing is off or
 * the context's most recent scoring call was not a complete proxykv_prune. */
#define PROXYKV_N_STAGES 5
int proxykv_profile_enable(proxykv_ctx* ctx, int on);
int proxykv_profile_read(proxykv_ctx* ctx, float* ms_host);

/* Static description of a status code. */
const char* proxykv_strerror(int status);
/* hipError_t of the last failed HIP call on this context (0 if none). */
int proxykv_last_hip_error(const proxykv_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* PROXYKV_H */
