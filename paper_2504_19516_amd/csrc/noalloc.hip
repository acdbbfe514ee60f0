// A GEMM entry point that allocates nothing, for callers that cannot call hipMalloc: code that
// runs under HIP graph capture, tight serving loops, harnesses that forbid allocation. It is
// sts_op_gemm's fp32-store form on the caller's DEVICE buffers; the split-K partial sums and the
// partial tiles of a cut last wave, which sts_op_gemm keeps in temporary allocations, live in a
// fixed file-scope device array instead.
#include <hip/hip_runtime.h>

#include <mutex>

#include "kernels.h"
#include "sts.h"

using namespace sts;

namespace {

constexpr size_t SCRATCH_FLOATS = STS_NOALLOC_SCRATCH_BYTES / sizeof(float);
// One copy per GPU the library's code object is loaded on, held until the process ends. In host
// code this name is only a handle for hipGetSymbolAddress: the device address is looked up once
// per device and every launch below takes that pointer.
static __device__ __align__(256) float scratch[SCRATCH_FLOATS];

constexpr int MAX_DEVICES = 16;
std::mutex g_mu;
float* g_scratch_ptr[MAX_DEVICES] = {nullptr};

// Device address of `scratch` on the current device (looked up on the first call there).
int scratch_on_current_device(float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return STS_EHIP;
  std::lock_guard<std::mutex> g(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return STS_EHIP;
    g_scratch_ptr[dev] = reinterpret_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return STS_OK;
}

}  // namespace

extern "C" int sts_op_gemm_noalloc(const void* a_dev, const void* w_dev, float* c_dev, int32_t m, int32_t n, int32_t k,
                                   int32_t tile_cfg, int32_t split_k, int32_t tail_slots, void* stream) {
  if (!a_dev || !w_dev || !c_dev || m < 1 || n < 1 || k < 1 || tile_cfg < 0 || tile_cfg >= GEMM_NCFG) return STS_EINVAL;
  if (split_k < 1 || split_k > 8 || tail_slots < 0 || (tail_slots > 0 && split_k != 1)) return STS_EINVAL;
  if (k % 64 != 0 || n % gemm_tile_n(tile_cfg) != 0) return STS_EINVAL;
  // what the call would put into the scratch array must fit it
  if (split_k > 1 && (size_t)split_k * (size_t)m * (size_t)n > SCRATCH_FLOATS) return STS_EINVAL;
  const size_t tile_floats = (size_t)gemm_tile_m(tile_cfg) * gemm_tile_n(tile_cfg);
  if (tail_slots > 0 && (size_t)tail_slots * tile_floats > SCRATCH_FLOATS) return STS_EINVAL;
  float* ws = nullptr;
  const int rc = scratch_on_current_device(&ws);
  if (rc != STS_OK) return rc;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const bf16* A = reinterpret_cast<const bf16*>(a_dev);
  const bf16* W = reinterpret_cast<const bf16*>(w_dev);
  hipError_t e;
  if (split_k > 1) {
    e = gemm_bf16(st, tile_cfg, EPI_F32, A, k, W, k, ws, n, m, n, k, split_k, (long long)m * n, nullptr, false);
    if (e != hipSuccess) return e == hipErrorInvalidValue ? STS_EINVAL : STS_EHIP;
    // the tiled kernel launches only as many splits as the K extent can feed: sum exactly those
    const int ksteps = k / 64, per = (ksteps + split_k - 1) / split_k;
    const int used = (ksteps + per - 1) / per;
    e = reduce_f32(st, c_dev, ws, used, (long long)m * n, (size_t)m * n);
  } else {
    // one partial tile per slot, as sts_op_gemm sizes its temporary buffer
    const GemmTail tail{tail_slots, ws, (size_t)tail_slots * tile_floats * sizeof(float)};
    e = gemm_bf16(st, tile_cfg, EPI_F32, A, k, W, k, c_dev, n, m, n, k, 1, 0, tail_slots > 0 ? &tail : nullptr, false);
  }
  if (e != hipSuccess) return e == hipErrorInvalidValue ? STS_EINVAL : STS_EHIP;
  return STS_OK;
}
