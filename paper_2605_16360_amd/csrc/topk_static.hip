// proxykv_topk for callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses that
// forbid hipMalloc): the per-row histograms and counters that the Top-K of long rows needs live in a fixed array in
// the library's device image instead of the context's workspace, and the call allocates nothing.
#include "context.hpp"
#include "kernels.hpp"

namespace {

// Every GPU the library runs on holds its own copy of this array, at its own address, until the process ends.
constexpr size_t kScratchBytes = 8u << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each device, looked up on first use

}  // namespace

extern "C" int proxykv_topk_static(proxykv_ctx* ctx, const float* scores, int64_t rows, int64_t N, int64_t K,
                                   int32_t* idx_out, void* stream) {
  if (!ctx || !scores || !idx_out) return PROXYKV_EINVAL;
  if (rows <= 0 || rows >= (1ll << 31) || N <= 0 || N >= (1ll << 31) - 4096 || K < 1 || K > N) return PROXYKV_EINVAL;
  if (N > pkv::kTopkSingleMax && rows > 65535) return PROXYKV_EUNSUPPORTED;
  const size_t need = pkv::topk_scratch_bytes(rows, N);
  if (need > kScratchBytes) return PROXYKV_ELIMIT;
  const int dev = ctx->cfg.device;
  if (dev < 0 || dev >= kMaxDevices) return PROXYKV_EUNSUPPORTED;
  hipError_t e = hipSetDevice(dev);
  if (e == hipSuccess && g_scratch_ptr[dev] == nullptr) {
    // in host code the array's name is only a handle: its address on the current device comes from the runtime
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e == hipSuccess) g_scratch_ptr[dev] = p;
  }
  if (e == hipSuccess) e = pkv::launch_topk(scores, rows, N, K, idx_out, g_scratch_ptr[dev], (hipStream_t)stream);
  if (e != hipSuccess) {
    ctx->last_hip_error = (int)e;
    (void)hipGetLastError();
    return PROXYKV_EHIP;
  }
  return PROXYKV_OK;
}

extern "C" size_t proxykv_topk_static_limit(void) { return kScratchBytes; }
