// Single-operation entry points on host data: each uploads fp32 inputs (rounded to bf16 on
// the device), runs exactly one of the engine's kernels, and returns fp32. They exist so that
// every kernel can be compared with the CPU oracle on identical bf16-rounded inputs.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <vector>

#include "kernels.h"
#include "sts.h"

using namespace sts;

namespace {

struct DevBufs {
  std::vector<void*> ptrs;
  ~DevBufs() { for (void* p : ptrs) (void)hipFree(p); }
  template <typename T> T* get(size_t n) {
    void* p = nullptr;
    if (hipMalloc(&p, std::max<size_t>(n, 1) * sizeof(T)) != hipSuccess) return nullptr;
    ptrs.push_back(p);
    return reinterpret_cast<T*>(p);
  }
};

__global__ void f32_to_bf16_kernel(bf16* dst, const float* src, size_t n) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < n) dst[i] = f2bf(src[i]);
}
__global__ void bf16_to_f32_kernel(float* dst, const bf16* src, size_t n) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < n) dst[i] = bf2f(src[i]);
}

// host fp32 -> device bf16
bf16* upload_bf16(DevBufs& b, const float* host, size_t n) {
  float* tmp = b.get<float>(n);
  bf16* out = b.get<bf16>(n);
  if (!tmp || !out) return nullptr;
  if (hipMemcpy(tmp, host, n * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) return nullptr;
  hipLaunchKernelGGL(f32_to_bf16_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, nullptr, out, tmp, n);
  return out;
}
int download_bf16(DevBufs& b, float* host, const bf16* dev, size_t n) {
  float* tmp = b.get<float>(n);
  if (!tmp) return STS_EHIP;
  hipLaunchKernelGGL(bf16_to_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, nullptr, tmp, dev, n);
  return hipMemcpy(host, tmp, n * sizeof(float), hipMemcpyDeviceToHost) == hipSuccess ? STS_OK : STS_EHIP;
}

}  // namespace

extern "C" int64_t sts_weight_packed_index(int32_t row, int32_t col, int32_t ld) {
  if (row < 0 || col < 0 || ld < 64 || ld % 64 != 0 || col >= ld) return -1;
  return (int64_t)weight_packed_index(row, col, ld);
}

extern "C" int sts_op_gemm(const float* a, const float* w, float* c_inout, int32_t m, int32_t n, int32_t k,
                           int32_t tile_cfg, int32_t epilogue, int32_t split_k, int32_t tail_slots) {
  if (!a || !w || !c_inout || m < 1 || n < 1 || k < 1 || tile_cfg < 0 || tile_cfg >= GEMM_NCFG) return STS_EINVAL;
  if (k % 64 != 0 || (epilogue == EPI_SWIGLU_BF16 ? 2 * n : n) % gemm_tile_n(tile_cfg) != 0) return STS_EINVAL;    // checked before the weights are packed into 32 x 64 blocks
  if (epilogue < 0 || epilogue > 3 || split_k < 1 || split_k > 8 || tail_slots < 0 || (tail_slots > 0 && split_k != 1)) return STS_EINVAL;
  DevBufs b;
  GemmTail tail{tail_slots, nullptr, 0};
  if (tail_slots > 0) {                                            // room for one partial tile per slot
    tail.ws_bytes = (size_t)tail_slots * gemm_tile_m(tile_cfg) * gemm_tile_n(tile_cfg) * sizeof(float);
    tail.ws = b.get<float>(tail.ws_bytes / sizeof(float));
    if (!tail.ws) return STS_EHIP;
  }
  const GemmTail* tp = tail_slots > 0 ? &tail : nullptr;
  const int wn = epilogue == EPI_SWIGLU_BF16 ? 2 * n : n;          // physical rows of W
  bf16* dA = upload_bf16(b, a, (size_t)m * k);
  bf16* dW = b.get<bf16>((size_t)wn * k);
  if (!dA || !dW) return STS_EHIP;
  {
    float* tmp = b.get<float>((size_t)wn * k);
    if (!tmp || hipMemcpy(tmp, w, (size_t)wn * k * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) return STS_EHIP;
    hipError_t e;
    if (epilogue == EPI_SWIGLU_BF16) {
      if (n % 32) return STS_EINVAL;
      e = convert_weight(nullptr, dW, k, tmp, n, k, 0, 32, 0, 1);
      if (e == hipSuccess) e = convert_weight(nullptr, dW, k, tmp + (size_t)n * k, n, k, 0, 32, 1, 1);
    } else {
      e = convert_weight(nullptr, dW, k, tmp, n, k, 0, 0, 0, 1);
    }
    if (e != hipSuccess) return STS_EHIP;
  }
  hipError_t e;
  int rc = STS_OK;
  if (epilogue == EPI_BF16 || epilogue == EPI_SWIGLU_BF16) {
    bf16* dC = b.get<bf16>((size_t)m * n);
    if (!dC) return STS_EHIP;
    e = gemm_bf16(nullptr, tile_cfg, epilogue, dA, k, dW, k, dC, n, m, wn, k, 1, 0, tp);
    if (e != hipSuccess) return e == hipErrorInvalidValue ? STS_EINVAL : STS_EHIP;
    rc = download_bf16(b, c_inout, dC, (size_t)m * n);
  } else if (epilogue == EPI_F32) {
    float* part = b.get<float>((size_t)split_k * m * n);
    float* dC = b.get<float>((size_t)m * n);
    if (!part || !dC) return STS_EHIP;
    e = gemm_bf16(nullptr, tile_cfg, EPI_F32, dA, k, dW, k, part, n, m, n, k, split_k, (long long)m * n, tp);
    if (e != hipSuccess) return e == hipErrorInvalidValue ? STS_EINVAL : STS_EHIP;
    // the tiled kernel launches only as many splits as the K extent can feed: sum exactly those
    const int ksteps = k / 64, per = (ksteps + split_k - 1) / split_k;
    const int used = (ksteps + per - 1) / per;
    if (reduce_f32(nullptr, dC, part, used, (long long)m * n, (size_t)m * n) != hipSuccess) return STS_EHIP;
    if (hipMemcpy(c_inout, dC, (size_t)m * n * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess) return STS_EHIP;
  } else {
    float* dC = b.get<float>((size_t)m * n);
    if (!dC || hipMemcpy(dC, c_inout, (size_t)m * n * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) return STS_EHIP;
    e = gemm_bf16(nullptr, tile_cfg, EPI_RESID_F32, dA, k, dW, k, dC, n, m, n, k, 1, 0, tp);
    if (e != hipSuccess) return e == hipErrorInvalidValue ? STS_EINVAL : STS_EHIP;
    if (hipMemcpy(c_inout, dC, (size_t)m * n * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess) return STS_EHIP;
  }
  if (hipDeviceSynchronize() != hipSuccess) return STS_EHIP;
  return rc;
}

extern "C" int sts_op_attn_prefill(const float* q, const float* k, const float* v, float* out, int32_t t, int32_t prior,
                                   int32_t n_q, int32_t n_kv, int32_t d, const int32_t* pages, int32_t n_pool_pages) {
  if (!q || !k || !v || !out || !pages || t < 1 || prior < 0 || n_q < 1 || n_kv < 1 || n_q % n_kv || (d != 64 && d != 128)) return STS_EINVAL;
  const int total = prior + t, np = (total + 15) / 16;
  for (int i = 0; i < np; i++) {
    if (pages[i] < 0 || pages[i] >= n_pool_pages) return STS_EINVAL;
    for (int j = 0; j < i; j++) if (pages[j] == pages[i]) return STS_EINVAL;
  }
  DevBufs b;
  KvGeom geo{n_kv, d, 16};
  bf16* pool = b.get<bf16>((size_t)n_pool_pages * geo.page_elems());
  int* d_bt = b.get<int>(np);
  float* dk = b.get<float>((size_t)total * n_kv * d);
  float* dv = b.get<float>((size_t)total * n_kv * d);
  bf16* dq = upload_bf16(b, q, (size_t)t * n_q * d);
  bf16* dout = b.get<bf16>((size_t)t * n_q * d);
  PrefillSeq* d_seq = b.get<PrefillSeq>(1);
  const int bq = attn_prefill_tile_q(), n_items = (t + bq - 1) / bq;
  AttnItem* d_items = b.get<AttnItem>(n_items);
  if (!pool || !d_bt || !dk || !dv || !dq || !dout || !d_seq || !d_items) return STS_EHIP;
  std::vector<AttnItem> items;
  for (int q0 = 0; q0 < t; q0 += bq) items.push_back(AttnItem{0, q0});
  PrefillSeq sq{0, t, prior, 0, np};
  if (hipMemset(pool, 0, (size_t)n_pool_pages * geo.page_elems() * sizeof(bf16)) != hipSuccess ||
      hipMemcpy(d_bt, pages, np * sizeof(int), hipMemcpyHostToDevice) != hipSuccess ||
      hipMemcpy(dk, k, (size_t)total * n_kv * d * sizeof(float), hipMemcpyHostToDevice) != hipSuccess ||
      hipMemcpy(dv, v, (size_t)total * n_kv * d * sizeof(float), hipMemcpyHostToDevice) != hipSuccess ||
      hipMemcpy(d_seq, &sq, sizeof(sq), hipMemcpyHostToDevice) != hipSuccess ||
      hipMemcpy(d_items, items.data(), n_items * sizeof(AttnItem), hipMemcpyHostToDevice) != hipSuccess) return STS_EHIP;
  if (kv_write_tokens(nullptr, pool, geo, d_bt, 0, total, dk, dv) != hipSuccess) return STS_EHIP;
  hipError_t e = attn_prefill(nullptr, dq, n_q * d, dout, n_q * d, d_seq, d_items, n_items, d_bt, pool, geo, n_q);
  if (e != hipSuccess) return e == hipErrorInvalidValue ? STS_EINVAL : STS_EHIP;
  int rc = download_bf16(b, out, dout, (size_t)t * n_q * d);
  if (hipDeviceSynchronize() != hipSuccess) return STS_EHIP;
  return rc;
}

extern "C" int sts_op_attn_decode(const float* q, const float* k, const float* v, float* out, int32_t n, const int32_t* ctx,
                                  int32_t n_q, int32_t n_kv, int32_t d, int32_t chunk_pages) {
  if (!q || !k || !v || !out || !ctx || n < 1 || n_q < 1 || n_kv < 1 || n_q % n_kv || (d != 64 && d != 128) || chunk_pages < 1) return STS_EINVAL;
  size_t total = 0; int max_pages = 0, tot_pages = 0;
  for (int i = 0; i < n; i++) {
    if (ctx[i] < 1) return STS_EINVAL;
    total += ctx[i];
    const int np = (ctx[i] + 15) / 16;
    max_pages = std::max(max_pages, np); tot_pages += np;
  }
  if (chunk_pages * 16 > attn_decode_max_chunk_tokens()) return STS_EINVAL;
  const int max_chunks = (max_pages + chunk_pages - 1) / chunk_pages;
  DevBufs b;
  KvGeom geo{n_kv, d, 16};
  bf16* pool = b.get<bf16>((size_t)tot_pages * geo.page_elems());
  int* d_bt = b.get<int>((size_t)n * max_pages);
  DecodeSeq* d_seq = b.get<DecodeSeq>(n);
  float* dk = b.get<float>(total * n_kv * d);
  float* dv = b.get<float>(total * n_kv * d);
  bf16* dq = upload_bf16(b, q, (size_t)n * n_q * d);
  bf16* dout = b.get<bf16>((size_t)n * n_q * d);
  float* ws = b.get<float>(attn_decode_ws_floats(n, n_q, d, max_chunks));
  if (!pool || !d_bt || !d_seq || !dk || !dv || !dq || !dout || !ws) return STS_EHIP;
  std::vector<int> bt((size_t)n * max_pages, 0);
  std::vector<DecodeSeq> seqs(n);
  // pages are handed out in reverse so that logical and physical order differ
  int next_page = tot_pages - 1;
  for (int i = 0; i < n; i++) {
    const int np = (ctx[i] + 15) / 16;
    for (int j = 0; j < np; j++) bt[(size_t)i * max_pages + j] = next_page--;
    seqs[i] = DecodeSeq{ctx[i] - 1, i * max_pages, np};      // the kernel attends to cl + 1 = ctx tokens
  }
  if (hipMemset(pool, 0, (size_t)tot_pages * geo.page_elems() * sizeof(bf16)) != hipSuccess ||
      hipMemcpy(d_bt, bt.data(), bt.size() * sizeof(int), hipMemcpyHostToDevice) != hipSuccess ||
      hipMemcpy(d_seq, seqs.data(), n * sizeof(DecodeSeq), hipMemcpyHostToDevice) != hipSuccess ||
      hipMemcpy(dk, k, total * n_kv * d * sizeof(float), hipMemcpyHostToDevice) != hipSuccess ||
      hipMemcpy(dv, v, total * n_kv * d * sizeof(float), hipMemcpyHostToDevice) != hipSuccess) return STS_EHIP;
  size_t off = 0;
  for (int i = 0; i < n; i++) {
    if (kv_write_tokens(nullptr, pool, geo, d_bt + (size_t)i * max_pages, 0, ctx[i], dk + off * n_kv * d, dv + off * n_kv * d) != hipSuccess) return STS_EHIP;
    off += ctx[i];
  }
  std::vector<DecodeItem> items;
  for (int i = 0; i < n; i++)
    for (int ch = 0; ch < (seqs[i].n_pages + chunk_pages - 1) / chunk_pages; ch++) items.push_back(DecodeItem{i, ch, seqs[i].cl, seqs[i].bt_off});
  DecodeItem* d_items = b.get<DecodeItem>(items.size());
  if (!d_items || hipMemcpy(d_items, items.data(), items.size() * sizeof(DecodeItem), hipMemcpyHostToDevice) != hipSuccess) return STS_EHIP;
  std::vector<int> multi;
  for (int i = 0; i < n; i++) if (seqs[i].n_pages > chunk_pages) multi.push_back(i);
  int* d_multi = b.get<int>(std::max<size_t>(1, multi.size()));
  if (!d_multi || (!multi.empty() && hipMemcpy(d_multi, multi.data(), multi.size() * sizeof(int), hipMemcpyHostToDevice) != hipSuccess)) return STS_EHIP;
  hipError_t e = attn_decode(nullptr, dq, dout, d_seq, d_items, (int)items.size(), d_multi, (int)multi.size(), d_bt, pool, geo, n, n_q, chunk_pages, max_chunks, ws);
  if (e != hipSuccess) return e == hipErrorInvalidValue ? STS_EINVAL : STS_EHIP;
  int rc = download_bf16(b, out, dout, (size_t)n * n_q * d);
  if (hipDeviceSynchronize() != hipSuccess) return STS_EHIP;
  return rc;
}
