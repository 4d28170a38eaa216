// C ABI of the ProxyKV hot path: argument validation, context and workspace management, and the
// sequencing of the kernels.  Every check runs before the first HIP call of an entry point.
#include <math.h>
#include <string.h>

#include <new>
#include <vector>

#include "context.hpp"
#include "kernels.hpp"

using pkv::DeviceBuffer;

namespace {

inline bool hip_ok(proxykv_ctx* ctx, hipError_t e) {
  if (e == hipSuccess) return true;
  if (ctx) ctx->last_hip_error = (int)e;
  (void)hipGetLastError();
  return false;
}

#define PKV_HIP(ctx, call)                                \
  do {                                                    \
    if (!hip_ok((ctx), (call))) return PROXYKV_EHIP;      \
  } while (0)

int validate_config(const proxykv_config* c) {
  if (!c) return PROXYKV_EINVAL;
  if (c->L_s <= 0 || c->H_q <= 0 || c->H_kv <= 0 || c->d <= 0 || c->L_l <= 0 || c->H_l <= 0 || c->D <= 0)
    return PROXYKV_EINVAL;
  if (c->H_q % c->H_kv != 0) return PROXYKV_EINVAL;
  if (c->d_time <= 0 || c->c_mid <= 0 || c->n_enc_layers < 0 || c->n_enc_heads <= 0 || c->d_ffn <= 0 ||
      c->d_head_x <= 0 || c->win <= 0 || c->stride <= 0 || c->stride > c->win || c->device < 0)
    return PROXYKV_EINVAL;
  if (c->reduce != PROXYKV_REDUCE_MAX && c->reduce != PROXYKV_REDUCE_SUM) return PROXYKV_EINVAL;
  if (c->d != 64 && c->d != 128) return PROXYKV_EUNSUPPORTED;
  if ((c->D * 2) % 16 != 0) return PROXYKV_EUNSUPPORTED;
  if (c->d_time != 512 || c->n_enc_heads != 8 || c->d_head_x != 64 || c->win != 2048 || c->stride != 1024 ||
      c->c_mid % 256 != 0 || c->d_ffn % 256 != 0 || c->H_kv > 16 || c->H_l > 64)
    return PROXYKV_EUNSUPPORTED;
  return PROXYKV_OK;
}

int validate_lengths(int64_t N, int64_t N_q, int64_t chunk) {
  if (N <= 0 || N_q <= 0 || chunk <= 0) return PROXYKV_EINVAL;
  if (N >= (1ll << 31) - 4096 || N_q >= (1ll << 31) - 4096 || chunk >= (1ll << 31)) return PROXYKV_EINVAL;
  return PROXYKV_OK;
}

int ensure(proxykv_ctx* ctx, DeviceBuffer& b, size_t bytes, hipStream_t stream) {
  if (bytes <= b.bytes) return PROXYKV_OK;
  if (b.ptr) {
    // earlier work on the stream may still read the old buffer
    PKV_HIP(ctx, hipStreamSynchronize(stream));
    PKV_HIP(ctx, hipFree(b.ptr));
    b.ptr = nullptr;
    b.bytes = 0;
  }
  void* p = nullptr;
  hipError_t e = hipMalloc(&p, bytes);
  if (e != hipSuccess) {
    hip_ok(ctx, e);
    return e == hipErrorOutOfMemory ? PROXYKV_ENOMEM : PROXYKV_EHIP;
  }
  // start from zeros: padded regions that no kernel writes (the tail of a short last window in the
  // transposed-V buffer) must hold finite values
  e = hipMemset(p, 0, bytes);
  if (e != hipSuccess) {
    hip_ok(ctx, e);
    (void)hipFree(p);
    return PROXYKV_EHIP;
  }
  b.ptr = p;
  b.bytes = bytes;
  return PROXYKV_OK;
}

struct Sizes {
  size_t neg_lse, x_ws, yhat_ws, h1, x, xb, qk, vt, ao, hid, zg, s3, range;
  size_t mapper() const { return h1 + x + xb + qk + vt + ao + hid + zg + s3 + range; }  // one lane's activations
  size_t total() const { return neg_lse + x_ws + yhat_ws + mapper(); }
};

Sizes workspace_sizes(const proxykv_config& c, int64_t N, int64_t N_q) {
  Sizes s;
  int64_t n_win, T;
  pkv::window_plan(N, c.win, c.stride, &n_win, &T);
  // rows of GEMM outputs (and of the residuals they read) are padded to the GEMM's 256-row tile
  const size_t Tp = ((size_t)T + 255) / 256 * 256, Np = (size_t)N, Npad = (Np + 255) / 256 * 256, dt = (size_t)c.d_time;
  s.neg_lse = (size_t)c.L_s * c.H_q * (size_t)N_q * 4;
  s.x_ws = (size_t)c.L_s * c.H_kv * Np * 4;
  s.yhat_ws = (size_t)c.L_l * c.H_l * Np * 4;
  s.h1 = (Np + 2) * (size_t)c.c_mid * 2;
  s.x = Tp * dt * 4;
  s.xb = Tp * dt * 2;
  s.qk = Tp * 2 * dt * 2;
  s.vt = (size_t)n_win * dt * (size_t)c.win * 2;
  s.ao = Tp * dt * 2;
  s.hid = Tp * (size_t)c.d_ffn * 2;
  s.zg = Np * dt * 2;
  s.s3 = Npad * (size_t)(c.H_l + 1) * (size_t)c.H_kv * 4;
  s.range = 256;
  return s;
}

int reserve_all(proxykv_ctx* ctx, int64_t N, int64_t N_q, bool score_part, bool map_part, bool prune_part,
                hipStream_t stream) {
  const Sizes s = workspace_sizes(ctx->cfg, N, N_q);
  int rc = PROXYKV_OK;
  if (score_part && (rc = ensure(ctx, ctx->neg_lse, s.neg_lse, stream))) return rc;
  if (prune_part) {
    if ((rc = ensure(ctx, ctx->x_ws, s.x_ws, stream))) return rc;
    if ((rc = ensure(ctx, ctx->yhat_ws, s.yhat_ws, stream))) return rc;
    if ((rc = ensure(ctx, ctx->topk_ws, pkv::topk_scratch_bytes((int64_t)ctx->cfg.L_l * ctx->cfg.H_l, N), stream))) return rc;
  }
  if (map_part) {
    int64_t n_win, T;
    pkv::window_plan(N, ctx->cfg.win, ctx->cfg.stride, &n_win, &T);
    const int lanes = pkv::map_lanes(T, ctx->distinct_layers);
    if (lanes > 1 && !ctx->lanes_created) {
      for (int i = 1; i < pkv::kMapLanes; ++i) {
        PKV_HIP(ctx, hipStreamCreateWithFlags(&ctx->lane_stream[i], hipStreamNonBlocking));
        PKV_HIP(ctx, hipEventCreateWithFlags(&ctx->lane_join[i], hipEventDisableTiming));
      }
      PKV_HIP(ctx, hipEventCreateWithFlags(&ctx->lane_fork, hipEventDisableTiming));
      ctx->lanes_created = true;
    }
   for (int lane = 0; lane < lanes; ++lane) {
    pkv::MapperWorkspace& m = ctx->m[lane];
    if ((rc = ensure(ctx, m.h1, s.h1, stream))) return rc;
    if ((rc = ensure(ctx, m.x, s.x, stream))) return rc;
    if ((rc = ensure(ctx, m.xb, s.xb, stream))) return rc;
    if ((rc = ensure(ctx, m.qk, s.qk, stream))) return rc;
    if ((rc = ensure(ctx, m.vt, s.vt, stream))) return rc;
    if ((rc = ensure(ctx, m.ao, s.ao, stream))) return rc;
    if ((rc = ensure(ctx, m.hid, s.hid, stream))) return rc;
    if ((rc = ensure(ctx, m.zg, s.zg, stream))) return rc;
    if ((rc = ensure(ctx, m.s3, s.s3, stream))) return rc;
    if ((rc = ensure(ctx, m.range, s.range, stream))) return rc;
   }
  }
  return rc;
}

// fp32 -> IEEE half bits, round to nearest even (subnormals and overflow to infinity included)
uint16_t host_f16(float f) {
  uint32_t x;
  memcpy(&x, &f, 4);
  const uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
  const uint32_t ax = x & 0x7fffffffu;
  if (ax > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);
  if (ax >= 0x477ff000u) return (uint16_t)(sign | 0x7c00u);  // >= 65520 rounds to infinity
  if (ax < 0x38800000u) {                                      // below 2^-14: half subnormal, unit 2^-24
    float a;
    memcpy(&a, &ax, 4);
    return (uint16_t)(sign | (uint32_t)nearbyint((double)a * 16777216.0));
  }
  const uint32_t mant = ax & 0x7fffffu, exp = (ax >> 23) - 127 + 15;
  uint32_t h = (exp << 10) | (mant >> 13);
  const uint32_t rem = mant & 0x1fffu;
  if (rem > 0x1000u || (rem == 0x1000u && (h & 1u))) ++h;
  return (uint16_t)(sign | h);
}

// Builds the prepared weight image on the host: a byte vector plus offsets of every section.
struct Stager {
  std::vector<uint8_t> bytes;
  size_t put_f32(const float* src, size_t n) {
    const size_t off = (bytes.size() + 255) & ~(size_t)255;
    bytes.resize(off + n * 4);
    memcpy(bytes.data() + off, src, n * 4);
    return off;
  }
  size_t put_f16(const float* src, size_t n) {
    const size_t off = (bytes.size() + 255) & ~(size_t)255;
    bytes.resize(off + n * 2);
    uint16_t* d = reinterpret_cast<uint16_t*>(bytes.data() + off);
    for (size_t i = 0; i < n; ++i) d[i] = host_f16(src[i]);
    return off;
  }
};

void free_buffer(DeviceBuffer& b) {
  if (b.ptr) (void)hipFree(b.ptr);
  b.ptr = nullptr;
  b.bytes = 0;
}

// Records stage boundary `i` on the stream when stage timing is switched on.
int mark(proxykv_ctx* ctx, int i, hipStream_t stream) {
  if (!ctx->profile) return PROXYKV_OK;
  PKV_HIP(ctx, hipEventRecord(ctx->ev[i], stream));
  ctx->ev_recorded[i] = true;
  return PROXYKV_OK;
}

int score_impl(proxykv_ctx* ctx, const void* q_rec, const void* k_ctx, const void* k_rec, int32_t dtype, int64_t N,
               int64_t N_q, int32_t chunk, float* x_out, hipStream_t stream) {
  const proxykv_config& c = ctx->cfg;
  const uint16_t *q = (const uint16_t*)q_rec, *kc = (const uint16_t*)k_ctx, *kr = (const uint16_t*)k_rec;
  int rc;
  if (dtype == PROXYKV_FP32) {
    const size_t nq = (size_t)c.L_s * c.H_q * (size_t)N_q * c.d, nkc = (size_t)c.L_s * c.H_kv * (size_t)N * c.d,
                 nkr = (size_t)c.L_s * c.H_kv * (size_t)N_q * c.d;
    if ((rc = ensure(ctx, ctx->q_bf16, nq * 2, stream))) return rc;
    if ((rc = ensure(ctx, ctx->kctx_bf16, nkc * 2, stream))) return rc;
    if ((rc = ensure(ctx, ctx->krec_bf16, nkr * 2, stream))) return rc;
    PKV_HIP(ctx, pkv::launch_f32_to_bf16((const float*)q_rec, (uint16_t*)ctx->q_bf16.ptr, (int64_t)nq, stream));
    PKV_HIP(ctx, pkv::launch_f32_to_bf16((const float*)k_ctx, (uint16_t*)ctx->kctx_bf16.ptr, (int64_t)nkc, stream));
    PKV_HIP(ctx, pkv::launch_f32_to_bf16((const float*)k_rec, (uint16_t*)ctx->krec_bf16.ptr, (int64_t)nkr, stream));
    q = (const uint16_t*)ctx->q_bf16.ptr;
    kc = (const uint16_t*)ctx->kctx_bf16.ptr;
    kr = (const uint16_t*)ctx->krec_bf16.ptr;
  }
  if ((rc = reserve_all(ctx, N, N_q, true, false, false, stream))) return rc;
  float* nl = (float*)ctx->neg_lse.ptr;
  int rcm;
  if ((rcm = mark(ctx, 0, stream))) return rcm;
  PKV_HIP(ctx, pkv::launch_score_lse(q, kc, kr, nl, c.L_s, c.H_q, c.H_kv, c.d, N, N_q, chunk, stream));
  if ((rcm = mark(ctx, 1, stream))) return rcm;
  if (c.reduce == PROXYKV_REDUCE_SUM)
    PKV_HIP(ctx, pkv::launch_score_colsum(q, kc, nl, x_out, c.L_s, c.H_q, c.H_kv, c.d, N, N_q, false, stream));
  else
    PKV_HIP(ctx, pkv::launch_score_colmax(q, kc, nl, x_out, c.L_s, c.H_q, c.H_kv, c.d, N, N_q, stream));
  if ((rcm = mark(ctx, 2, stream))) return rcm;
  return PROXYKV_OK;
}

// causal self-attention, summed over the query axis: pass 1 with no context keys and one chunk that spans the
// sequence (query i sees its own keys j <= i), then the causal column sum
int score_self_impl(proxykv_ctx* ctx, const void* q_in, const void* k_in, int32_t dtype, int64_t N, float* x_out,
                    hipStream_t stream) {
  const proxykv_config& c = ctx->cfg;
  const uint16_t *q = (const uint16_t*)q_in, *k = (const uint16_t*)k_in;
  int rc;
  if (dtype == PROXYKV_FP32) {
    const size_t nq = (size_t)c.L_s * c.H_q * (size_t)N * c.d, nk = (size_t)c.L_s * c.H_kv * (size_t)N * c.d;
    if ((rc = ensure(ctx, ctx->q_bf16, nq * 2, stream))) return rc;
    if ((rc = ensure(ctx, ctx->krec_bf16, nk * 2, stream))) return rc;
    PKV_HIP(ctx, pkv::launch_f32_to_bf16((const float*)q_in, (uint16_t*)ctx->q_bf16.ptr, (int64_t)nq, stream));
    PKV_HIP(ctx, pkv::launch_f32_to_bf16((const float*)k_in, (uint16_t*)ctx->krec_bf16.ptr, (int64_t)nk, stream));
    q = (const uint16_t*)ctx->q_bf16.ptr;
    k = (const uint16_t*)ctx->krec_bf16.ptr;
  }
  if ((rc = reserve_all(ctx, N, N, true, false, false, stream))) return rc;
  float* nl = (float*)ctx->neg_lse.ptr;
  int rcm;
  if ((rcm = mark(ctx, 0, stream))) return rcm;
  PKV_HIP(ctx, pkv::launch_score_lse(q, k, k, nl, c.L_s, c.H_q, c.H_kv, c.d, 0, N, (int)N, stream));
  if ((rcm = mark(ctx, 1, stream))) return rcm;
  PKV_HIP(ctx, pkv::launch_score_colsum(q, k, nl, x_out, c.L_s, c.H_q, c.H_kv, c.d, N, N, true, stream));
  if ((rcm = mark(ctx, 2, stream))) return rcm;
  return PROXYKV_OK;
}

int map_impl(proxykv_ctx* ctx, const float* x, int64_t N, float* yhat, hipStream_t stream) {
  int rc;
  if ((rc = reserve_all(ctx, N, 1, false, true, false, stream))) return rc;
  PKV_HIP(ctx, pkv::mapper_forward(ctx, x, N, yhat, stream));
  return PROXYKV_OK;
}

}  // namespace

extern "C" {

void proxykv_default_mapper(proxykv_config* cfg) {
  if (!cfg) return;
  cfg->d_time = 512;
  cfg->c_mid = 256;
  cfg->n_enc_layers = 6;
  cfg->n_enc_heads = 8;
  cfg->d_ffn = 2048;
  cfg->d_head_x = 64;
  cfg->win = 2048;
  cfg->stride = 1024;
  cfg->reduce = PROXYKV_REDUCE_MAX;
  cfg->device = 0;
}

int proxykv_create(proxykv_ctx** out, const proxykv_config* cfg) {
  if (!out) return PROXYKV_EINVAL;
  *out = nullptr;
  const int rc = validate_config(cfg);
  if (rc) return rc;
  proxykv_ctx* ctx = new (std::nothrow) proxykv_ctx();
  if (!ctx) return PROXYKV_ENOMEM;
  ctx->cfg = *cfg;
  ctx->pairing.resize(cfg->L_l);
  for (int ll = 0; ll < cfg->L_l; ++ll)
    ctx->pairing[ll] = (int32_t)(((int64_t)(ll + 1) * cfg->L_s + cfg->L_l - 1) / cfg->L_l - 1);
  ctx->distinct_layers = 0;
  for (int ll = 0; ll < cfg->L_l; ++ll) ctx->distinct_layers += (ll == 0 || ctx->pairing[ll] != ctx->pairing[ll - 1]);
  *out = ctx;
  return PROXYKV_OK;
}

int proxykv_destroy(proxykv_ctx* ctx) {
  if (!ctx) return PROXYKV_OK;
  std::vector<DeviceBuffer*> all = {&ctx->weight_blob, &ctx->q_bf16, &ctx->kctx_bf16, &ctx->krec_bf16,
                                    &ctx->neg_lse,     &ctx->x_ws,   &ctx->yhat_ws, &ctx->topk_ws};
  for (pkv::MapperWorkspace& m : ctx->m)
    for (DeviceBuffer* b : {&m.h1, &m.x, &m.xb, &m.qk, &m.vt, &m.ao, &m.hid, &m.zg, &m.s3, &m.range}) all.push_back(b);
  bool any = ctx->ev_created || ctx->lanes_created;
  for (DeviceBuffer* b : all) any = any || b->ptr;
  if (any) {
    (void)hipSetDevice(ctx->cfg.device);
    (void)hipDeviceSynchronize();
    for (DeviceBuffer* b : all) free_buffer(*b);
    if (ctx->ev_created)
      for (int i = 0; i < PROXYKV_N_STAGES + 1; ++i) (void)hipEventDestroy(ctx->ev[i]);
    if (ctx->lanes_created) {
      for (int i = 1; i < pkv::kMapLanes; ++i) {
        if (ctx->lane_stream[i]) (void)hipStreamDestroy(ctx->lane_stream[i]);
        if (ctx->lane_join[i]) (void)hipEventDestroy(ctx->lane_join[i]);
      }
      if (ctx->lane_fork) (void)hipEventDestroy(ctx->lane_fork);
    }
  }
  delete ctx;
  return PROXYKV_OK;
}

size_t proxykv_mapper_weight_count(const proxykv_config* c) {
  if (validate_config(c)) return 0;
  const size_t D = c->d_time, C1 = c->c_mid, F = c->d_ffn, dh = c->d_head_x, Hs = c->H_kv, Hl = c->H_l;
  size_t n = C1 * Hs * 3 + C1 + 4 * C1 + D * C1 * 3 + D + 4 * D;
  n += (size_t)c->n_enc_layers * (3 * D * D + 3 * D + D * D + D + 2 * D + F * D + F + D * F + D + 2 * D);
  n += 2 * (Hs * dh * D + Hs * dh) + Hl * dh + dh + 1;
  return n;
}

int proxykv_set_mapper_weights(proxykv_ctx* ctx, const float* blob, size_t n_floats) {
  if (!ctx || !blob) return PROXYKV_EINVAL;
  const proxykv_config& c = ctx->cfg;
  if (n_floats != proxykv_mapper_weight_count(&c)) return PROXYKV_EINVAL;
  const size_t D = c.d_time, C1 = c.c_mid, F = c.d_ffn, dh = c.d_head_x, Hs = c.H_kv, Hl = c.H_l;
  const double eps = 1e-5;
  const float* p = blob;
  auto take = [&](size_t n) {
    const float* r = p;
    p += n;
    return r;
  };
  Stager st;
  // stem: fold conv bias and inference batch norm into scale/shift (host double arithmetic)
  auto fold = [&](const float* bias, const float* g, const float* b, const float* mu, const float* var, size_t n,
                  size_t* off_scale, size_t* off_shift) {
    std::vector<float> sc(n), sh(n);
    for (size_t i = 0; i < n; ++i) {
      const double s = (double)g[i] / sqrt((double)var[i] + eps);
      sc[i] = (float)s;
      sh[i] = (float)(((double)bias[i] - (double)mu[i]) * s + (double)b[i]);
    }
    *off_scale = st.put_f32(sc.data(), n);
    *off_shift = st.put_f32(sh.data(), n);
  };
  const float* c1w = take(C1 * Hs * 3);
  const float* c1b = take(C1);
  const float *g1 = take(C1), *b1 = take(C1), *m1 = take(C1), *v1 = take(C1);
  const size_t o_c1w = st.put_f32(c1w, C1 * Hs * 3);
  size_t o_s1, o_h1;
  fold(c1b, g1, b1, m1, v1, C1, &o_s1, &o_h1);
  // bound of the first block's output, |GELU(y)| <= |y| <= |scale_c| * sum |w_c| * max|x| + |shift_c|
  double cw = 0.0, cs = 0.0;
  for (size_t ch = 0; ch < C1; ++ch) {
    const double sgn = (double)g1[ch] / sqrt((double)v1[ch] + eps), sc = fabs(sgn);
    double wsum = 0.0;
    for (size_t i = 0; i < Hs * 3; ++i) wsum += fabs((double)c1w[ch * Hs * 3 + i]);
    const double sh = fabs(((double)c1b[ch] - (double)m1[ch]) * sgn + (double)b1[ch]);
    if (sc * wsum > cw) cw = sc * wsum;
    if (sh > cs) cs = sh;
  }
  ctx->w.stem_cw = (float)(cw * 1.0001);
  ctx->w.stem_cs = (float)(cs * 1.0001 + 1e-6);
  const float* c2w = take(D * C1 * 3);
  const float* c2b = take(D);
  const float *g2 = take(D), *b2 = take(D), *m2 = take(D), *v2 = take(D);
  std::vector<float> c2r(D * C1 * 3);  // [c][c1][tap] -> [c][tap][c1]
  for (size_t co = 0; co < D; ++co)
    for (size_t ci = 0; ci < C1; ++ci)
      for (size_t tap = 0; tap < 3; ++tap) c2r[(co * 3 + tap) * C1 + ci] = c2w[(co * C1 + ci) * 3 + tap];
  const size_t o_c2w = st.put_f16(c2r.data(), c2r.size());
  size_t o_s2, o_h2;
  fold(c2b, g2, b2, m2, v2, D, &o_s2, &o_h2);
  struct EncOff {
    size_t in_w, in_b, out_w, out_b, ln1_g, ln1_b, f1_w, f1_b, f2_w, f2_b, ln2_g, ln2_b;
  };
  std::vector<EncOff> eo(c.n_enc_layers);
  for (int i = 0; i < c.n_enc_layers; ++i) {
    EncOff& e = eo[i];
    e.in_w = st.put_f16(take(3 * D * D), 3 * D * D);
    e.in_b = st.put_f32(take(3 * D), 3 * D);
    e.out_w = st.put_f16(take(D * D), D * D);
    e.out_b = st.put_f32(take(D), D);
    e.ln1_g = st.put_f32(take(D), D);
    e.ln1_b = st.put_f32(take(D), D);
    e.f1_w = st.put_f16(take(F * D), F * D);
    e.f1_b = st.put_f32(take(F), F);
    e.f2_w = st.put_f16(take(D * F), D * F);
    e.f2_b = st.put_f32(take(D), D);
    e.ln2_g = st.put_f32(take(D), D);
    e.ln2_b = st.put_f32(take(D), D);
  }
  // head: key and value projections stacked into one [2*Hs*dh, D] matrix
  const float* kw = take(Hs * dh * D);
  const float* kb = take(Hs * dh);
  const float* vw = take(Hs * dh * D);
  const float* vb = take(Hs * dh);
  // rows padded with zeros to the GEMM's 256-column tile (pkv::kv3_stride)
  const size_t kv_rows = (size_t)pkv::kv3_stride(c);
  std::vector<float> kvw(kv_rows * D, 0.0f), kvb(kv_rows, 0.0f);
  memcpy(kvw.data(), kw, Hs * dh * D * 4);
  memcpy(kvw.data() + Hs * dh * D, vw, Hs * dh * D * 4);
  memcpy(kvb.data(), kb, Hs * dh * 4);
  memcpy(kvb.data() + Hs * dh, vb, Hs * dh * 4);
  const size_t o_kvw = st.put_f16(kvw.data(), kvw.size());
  const size_t o_kvb = st.put_f32(kvb.data(), kvb.size());
  const size_t o_q = st.put_f32(take(Hl * dh), Hl * dh);
  const size_t o_ow = st.put_f32(take(dh), dh);
  const float out_b = *take(1);
  // sinusoidal positions 0 .. win-1 (Sec. 4.1, stage 2), evaluated in double
  std::vector<float> pe((size_t)c.win * D);
  for (int pos = 0; pos < c.win; ++pos)
    for (size_t i = 0; i < D; i += 2) {
      const double ang = (double)pos / pow(10000.0, (double)i / (double)D);
      pe[(size_t)pos * D + i] = (float)sin(ang);
      pe[(size_t)pos * D + i + 1] = (float)cos(ang);
    }
  const size_t o_pe = st.put_f32(pe.data(), pe.size());

  PKV_HIP(ctx, hipSetDevice(c.device));
  int rc = ensure(ctx, ctx->weight_blob, st.bytes.size(), nullptr);
  if (rc) return rc;
  PKV_HIP(ctx, hipMemcpy(ctx->weight_blob.ptr, st.bytes.data(), st.bytes.size(), hipMemcpyHostToDevice));
  const uint8_t* base = (const uint8_t*)ctx->weight_blob.ptr;
  auto F32 = [&](size_t off) { return (const float*)(base + off); };
  auto B16 = [&](size_t off) { return (const uint16_t*)(base + off); };
  pkv::MapperWeights& w = ctx->w;
  w.conv1_w = F32(o_c1w);
  w.bn1_scale = F32(o_s1);
  w.bn1_shift = F32(o_h1);
  w.conv2_w = B16(o_c2w);
  w.bn2_scale = F32(o_s2);
  w.bn2_shift = F32(o_h2);
  w.enc.resize(c.n_enc_layers);
  for (int i = 0; i < c.n_enc_layers; ++i) {
    const EncOff& e = eo[i];
    w.enc[i] = {B16(e.in_w), F32(e.in_b), B16(e.out_w), F32(e.out_b), F32(e.ln1_g), F32(e.ln1_b),
                B16(e.f1_w), F32(e.f1_b), B16(e.f2_w),  F32(e.f2_b),  F32(e.ln2_g), F32(e.ln2_b)};
  }
  w.kv_w = B16(o_kvw);
  w.kv_b = F32(o_kvb);
  w.queries = F32(o_q);
  w.out_w = F32(o_ow);
  w.out_b = out_b;
  w.pe = F32(o_pe);
  ctx->weights_set = true;
  return PROXYKV_OK;
}

int proxykv_workspace_bytes(const proxykv_config* cfg, int64_t N, int64_t N_q, size_t* out_bytes) {
  if (!out_bytes) return PROXYKV_EINVAL;
  int rc = validate_config(cfg);
  if (rc) return rc;
  if ((rc = validate_lengths(N, N_q, 1))) return rc;
  const Sizes s = workspace_sizes(*cfg, N, N_q);
  int64_t n_win, T;
  pkv::window_plan(N, cfg->win, cfg->stride, &n_win, &T);
  int distinct = 0, prev = -1;
  for (int ll = 0; ll < cfg->L_l; ++ll) {
    const int ls = (int)(((int64_t)(ll + 1) * cfg->L_s + cfg->L_l - 1) / cfg->L_l - 1);
    distinct += ls != prev;
    prev = ls;
  }
  *out_bytes = s.total() + (size_t)(pkv::map_lanes(T, distinct) - 1) * s.mapper();
  return PROXYKV_OK;
}

int proxykv_reserve(proxykv_ctx* ctx, int64_t N, int64_t N_q) {
  if (!ctx) return PROXYKV_EINVAL;
  const int rc = validate_lengths(N, N_q, 1);
  if (rc) return rc;
  PKV_HIP(ctx, hipSetDevice(ctx->cfg.device));
  return reserve_all(ctx, N, N_q, true, true, true, nullptr);
}

int proxykv_keep_count(int64_t N, double keep_ratio, int64_t* K_out) {
  if (!K_out || N <= 0 || !(keep_ratio > 0.0) || !(keep_ratio <= 1.0)) return PROXYKV_EINVAL;
  int64_t K = (int64_t)floor(keep_ratio * (double)N);
  if (K < 1) K = 1;
  if (K > N) K = N;
  *K_out = K;
  return PROXYKV_OK;
}

int proxykv_layer_pairing(const proxykv_config* cfg, int32_t* pairing_host) {
  if (!cfg || !pairing_host || cfg->L_s <= 0 || cfg->L_l <= 0) return PROXYKV_EINVAL;
  for (int ll = 0; ll < cfg->L_l; ++ll)
    pairing_host[ll] = (int32_t)(((int64_t)(ll + 1) * cfg->L_s + cfg->L_l - 1) / cfg->L_l - 1);
  return PROXYKV_OK;
}

int proxykv_score(proxykv_ctx* ctx, const void* q_rec, const void* k_ctx, const void* k_rec, int32_t dtype, int64_t N,
                  int64_t N_q, int32_t chunk, float* x_out, void* stream) {
  if (!ctx || !q_rec || !k_ctx || !k_rec || !x_out) return PROXYKV_EINVAL;
  if (dtype != PROXYKV_BF16 && dtype != PROXYKV_FP32) return PROXYKV_EINVAL;
  const int rc = validate_lengths(N, N_q, chunk);
  if (rc) return rc;
  PKV_HIP(ctx, hipSetDevice(ctx->cfg.device));
  // stage timing describes a whole proxykv_prune: a score call on its own leaves no complete record behind
  const int rcs = score_impl(ctx, q_rec, k_ctx, k_rec, dtype, N, N_q, chunk, x_out, (hipStream_t)stream);
  for (int i = 0; i < PROXYKV_N_STAGES + 1; ++i) ctx->ev_recorded[i] = false;
  return rcs;
}

int proxykv_score_self(proxykv_ctx* ctx, const void* q, const void* k, int32_t dtype, int64_t N, float* x_out, void* stream) {
  if (!ctx || !q || !k || !x_out) return PROXYKV_EINVAL;
  if (dtype != PROXYKV_BF16 && dtype != PROXYKV_FP32) return PROXYKV_EINVAL;
  const int rc = validate_lengths(N, N, N);
  if (rc) return rc;
  PKV_HIP(ctx, hipSetDevice(ctx->cfg.device));
  const int rcs = score_self_impl(ctx, q, k, dtype, N, x_out, (hipStream_t)stream);
  for (int i = 0; i < PROXYKV_N_STAGES + 1; ++i) ctx->ev_recorded[i] = false;
  return rcs;
}

int proxykv_map(proxykv_ctx* ctx, const float* x, int64_t N, float* yhat, void* stream) {
  if (!ctx || !x || !yhat) return PROXYKV_EINVAL;
  const int rc = validate_lengths(N, 1, 1);
  if (rc) return rc;
  if (!ctx->weights_set) return PROXYKV_ESTATE;
  PKV_HIP(ctx, hipSetDevice(ctx->cfg.device));
  return map_impl(ctx, x, N, yhat, (hipStream_t)stream);
}

int proxykv_topk(proxykv_ctx* ctx, const float* scores, int64_t rows, int64_t N, int64_t K, int32_t* idx_out,
                 void* stream) {
  if (!ctx || !scores || !idx_out) return PROXYKV_EINVAL;
  if (rows <= 0 || rows >= (1ll << 31) || N <= 0 || N >= (1ll << 31) - 4096 || K < 1 || K > N) return PROXYKV_EINVAL;
  if (N > pkv::kTopkSingleMax && rows > 65535) return PROXYKV_EUNSUPPORTED;
  PKV_HIP(ctx, hipSetDevice(ctx->cfg.device));
  const int rc = ensure(ctx, ctx->topk_ws, pkv::topk_scratch_bytes(rows, N), (hipStream_t)stream);
  if (rc) return rc;
  PKV_HIP(ctx, pkv::launch_topk(scores, rows, N, K, idx_out, ctx->topk_ws.ptr, (hipStream_t)stream));
  return PROXYKV_OK;
}

int proxykv_compact(proxykv_ctx* ctx, const void* k_in, const void* v_in, const int32_t* idx, int64_t rows, int64_t N,
                    int64_t K, int64_t D, void* k_out, void* v_out, void* stream) {
  if (!ctx || !k_in || !v_in || !idx || !k_out || !v_out) return PROXYKV_EINVAL;
  if (rows <= 0 || rows > 65535 || N <= 0 || N >= (1ll << 31) || K < 1 || K > N || D <= 0) return PROXYKV_EINVAL;
  if ((D * 2) % 16 != 0 || D * 2 > 4096 || 256 % ((D * 2) / 16) != 0) return PROXYKV_EUNSUPPORTED;
  PKV_HIP(ctx, hipSetDevice(ctx->cfg.device));
  PKV_HIP(ctx, pkv::launch_compact(k_in, v_in, idx, rows, N, K, D * 2, k_out, v_out, (hipStream_t)stream));
  return PROXYKV_OK;
}

int proxykv_compact_inplace(proxykv_ctx* ctx, void* k, void* v, const int32_t* idx, int64_t rows, int64_t N, int64_t K,
                            int64_t D, void* stream) {
  if (!ctx || !k || !v || !idx) return PROXYKV_EINVAL;
  if (rows <= 0 || N <= 0 || N >= (1ll << 31) || K < 1 || K > N || D <= 0) return PROXYKV_EINVAL;
  if ((D * 2) % 16 != 0 || D * 2 > 512) return PROXYKV_EUNSUPPORTED;
  PKV_HIP(ctx, hipSetDevice(ctx->cfg.device));
  PKV_HIP(ctx, pkv::launch_compact_inplace(k, v, idx, rows, N, K, D * 2, nullptr, 1, (hipStream_t)stream));
  return PROXYKV_OK;
}

int proxykv_topk_pooled(proxykv_ctx* ctx, const float* scores, int64_t layers, int64_t heads, int64_t N, int64_t K,
                        int32_t* flat_out, int32_t* counts_out, void* stream) {
  if (!ctx || !scores || !flat_out || !counts_out) return PROXYKV_EINVAL;
  if (layers <= 0 || heads <= 0 || N <= 0 || K < 1 || K > N) return PROXYKV_EINVAL;
  if (layers * heads >= (1ll << 31) || heads * N >= (1ll << 31) - 4096) return PROXYKV_EINVAL;
  if (heads * N > pkv::kTopkSingleMax && layers > 65535) return PROXYKV_EUNSUPPORTED;
  PKV_HIP(ctx, hipSetDevice(ctx->cfg.device));
  const int rc = ensure(ctx, ctx->topk_ws, pkv::topk_scratch_bytes(layers, heads * N), (hipStream_t)stream);
  if (rc) return rc;
  PKV_HIP(ctx, pkv::launch_topk(scores, layers, heads * N, heads * K, flat_out, ctx->topk_ws.ptr, (hipStream_t)stream));
  PKV_HIP(ctx, pkv::launch_head_counts(flat_out, layers, heads, N, K, counts_out, (hipStream_t)stream));
  return PROXYKV_OK;
}

int proxykv_compact_pooled(proxykv_ctx* ctx, void* k, void* v, const int32_t* flat, const int32_t* counts, int64_t layers,
                           int64_t heads, int64_t N, int64_t K, int64_t D, void* stream) {
  if (!ctx || !k || !v || !flat || !counts) return PROXYKV_EINVAL;
  if (layers <= 0 || heads <= 0 || N <= 0 || K < 1 || K > N || D <= 0) return PROXYKV_EINVAL;
  if (layers * heads >= (1ll << 31) || heads * N >= (1ll << 31) - 4096) return PROXYKV_EINVAL;
  if ((D * 2) % 16 != 0 || D * 2 > 512) return PROXYKV_EUNSUPPORTED;
  PKV_HIP(ctx, hipSetDevice(ctx->cfg.device));
  PKV_HIP(ctx, pkv::launch_compact_inplace(k, v, flat, layers * heads, N, K, D * 2, counts, (int)heads, (hipStream_t)stream));
  return PROXYKV_OK;
}

int proxykv_mask(proxykv_ctx* ctx, const int32_t* idx, int64_t rows, int64_t N, int64_t K, uint8_t* mask_out, void* stream) {
  if (!ctx || !idx || !mask_out) return PROXYKV_EINVAL;
  if (rows <= 0 || N <= 0 || N >= (1ll << 31) || K < 1 || K > N) return PROXYKV_EINVAL;
  PKV_HIP(ctx, hipSetDevice(ctx->cfg.device));
  PKV_HIP(ctx, pkv::launch_mask(idx, rows, N, K, mask_out, (hipStream_t)stream));
  return PROXYKV_OK;
}

int proxykv_prune(proxykv_ctx* ctx, const void* q_rec, const void* k_ctx, const void* k_rec, int32_t dtype, int64_t N,
                  int64_t N_q, int32_t chunk, double keep_ratio, const void* k_in, const void* v_in, void* k_out,
                  void* v_out, int32_t* idx_out, float* x_out, float* yhat_out, int64_t* K_host, void* stream) {
  if (!ctx || !q_rec || !k_ctx || !k_rec || !k_in || !v_in || !k_out || !v_out || !idx_out) return PROXYKV_EINVAL;
  if (dtype != PROXYKV_BF16 && dtype != PROXYKV_FP32) return PROXYKV_EINVAL;
  int rc = validate_lengths(N, N_q, chunk);
  if (rc) return rc;
  int64_t K = 0;
  if ((rc = proxykv_keep_count(N, keep_ratio, &K))) return rc;
  if (!ctx->weights_set) return PROXYKV_ESTATE;
  const proxykv_config& c = ctx->cfg;
  const int64_t rows = (int64_t)c.L_l * c.H_l;
  if (rows > 65535 || 256 % ((c.D * 2) / 16) != 0) return PROXYKV_EUNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  PKV_HIP(ctx, hipSetDevice(c.device));
  if ((rc = reserve_all(ctx, N, N_q, true, true, true, s))) return rc;
  float* x = x_out ? x_out : (float*)ctx->x_ws.ptr;
  float* y = yhat_out ? yhat_out : (float*)ctx->yhat_ws.ptr;
  if ((rc = score_impl(ctx, q_rec, k_ctx, k_rec, dtype, N, N_q, chunk, x, s))) return rc;
  if ((rc = map_impl(ctx, x, N, y, s))) return rc;
  if ((rc = mark(ctx, 3, s))) return rc;
  const int cpr = c.D * 2 / 16;
  if (ctx->fused_select && 1024 % cpr == 0) {
    // selection and gather in one launch: the workgroup that has written a stretch of a row's kept indices moves those
    // tokens' K and V rows; the whole launch is booked as the compaction stage
    if ((rc = mark(ctx, 4, s))) return rc;
    PKV_HIP(ctx, pkv::launch_topk_gather(y, rows, N, K, idx_out, ctx->topk_ws.ptr, k_in, v_in, (int64_t)c.D * 2, k_out, v_out, s));
  } else {
    PKV_HIP(ctx, pkv::launch_topk(y, rows, N, K, idx_out, ctx->topk_ws.ptr, s));
    if ((rc = mark(ctx, 4, s))) return rc;
    PKV_HIP(ctx, pkv::launch_compact(k_in, v_in, idx_out, rows, N, K, (int64_t)c.D * 2, k_out, v_out, s));
  }
  if ((rc = mark(ctx, 5, s))) return rc;
  if (K_host) *K_host = K;
  return PROXYKV_OK;
}

int proxykv_set_fused_select(proxykv_ctx* ctx, int on) {
  if (!ctx) return PROXYKV_EINVAL;
  ctx->fused_select = on != 0;
  return PROXYKV_OK;
}

int proxykv_profile_enable(proxykv_ctx* ctx, int on) {
  if (!ctx) return PROXYKV_EINVAL;
  if (on && !ctx->ev_created) {
    PKV_HIP(ctx, hipSetDevice(ctx->cfg.device));
    for (int i = 0; i < PROXYKV_N_STAGES + 1; ++i) PKV_HIP(ctx, hipEventCreate(&ctx->ev[i]));
    ctx->ev_created = true;
  }
  ctx->profile = on != 0;
  for (int i = 0; i < PROXYKV_N_STAGES + 1; ++i) ctx->ev_recorded[i] = false;
  return PROXYKV_OK;
}

int proxykv_profile_read(proxykv_ctx* ctx, float* ms_host) {
  if (!ctx || !ms_host) return PROXYKV_EINVAL;
  if (!ctx->profile || !ctx->ev_created) return PROXYKV_ESTATE;
  for (int i = 0; i < PROXYKV_N_STAGES + 1; ++i)
    if (!ctx->ev_recorded[i]) return PROXYKV_ESTATE;
  PKV_HIP(ctx, hipEventSynchronize(ctx->ev[PROXYKV_N_STAGES]));
  for (int i = 0; i < PROXYKV_N_STAGES; ++i) PKV_HIP(ctx, hipEventElapsedTime(&ms_host[i], ctx->ev[i], ctx->ev[i + 1]));
  return PROXYKV_OK;
}

const char* proxykv_strerror(int status) {
  switch (status) {
    case PROXYKV_OK: return "ok";
    case PROXYKV_EINVAL: return "invalid argument";
    case PROXYKV_EUNSUPPORTED: return "shape or option not supported by this build";
    case PROXYKV_ENOMEM: return "out of device memory";
    case PROXYKV_ESTATE: return "context not ready (mapper weights not set)";
    case PROXYKV_EHIP: return "HIP runtime error";
    case PROXYKV_ELIMIT: return "size beyond a fixed limit of this entry point";
    default: return "unknown status";
  }
}

int proxykv_last_hip_error(const proxykv_ctx* ctx) { return ctx ? ctx->last_hip_error : 0; }

}  // extern "C"
