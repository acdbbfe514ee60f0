// Memory-bound kernels between the contractions: weight generation, embedding, RMSNorm,
// rotary embedding + KV page writes, split-K reductions fused with residual/norm/SwiGLU,
// greedy argmax, and the copy kernel used as the bandwidth probe.
#include "kernels.h"

namespace sts {

// ------------------------------------------------------------------ counter-based generator
// Twelve-term Irwin-Hall approximation of a normal deviate from three 64-bit hashes of
// (seed, tensor id, element index): integer arithmetic plus one fp32 multiply, so a host
// implementation of the same recipe reproduces every value exactly.
__host__ __device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
__device__ __forceinline__ int irwin_hall12(uint64_t base, uint64_t i) {
  int s = 0;
#pragma unroll
  for (int j = 0; j < 3; j++) {
    uint64_t r = mix64(base ^ (4 * i + j));
    s += (int)(r & 0xFFFF) + (int)((r >> 16) & 0xFFFF) + (int)((r >> 32) & 0xFFFF) + (int)(r >> 48);
  }
  return s - 393210;
}

__device__ __forceinline__ int phys_row(int r, int row_offset, int ib, int phase) {
  return ib > 0 ? (r / ib) * 2 * ib + phase * ib + r % ib : row_offset + r;
}

// Where element (physical row r, column c) of a weight matrix with ld columns lives. Row-major, or the
// packed layout of the GEMM weights (weight_packed_index in kernels.h).
__device__ __forceinline__ size_t weight_elem(int r, int c, int ld, int packed) {
  return packed ? weight_packed_index(r, c, ld) : (size_t)r * ld + c;
}

__global__ void init_weight_kernel(bf16* dst, int ld, uint64_t base, int rows, int cols, int row_offset, int ib, int phase, int packed) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i >= (size_t)rows * cols) return;
  int r = (int)(i / cols), c = (int)(i % cols);
  float w = (float)irwin_hall12(base, i) * 0.02f * 1.52587890625e-05f;   // * 2^-16, exact
  dst[weight_elem(phys_row(r, row_offset, ib, phase), c, ld, packed)] = f2bf(w);
}
hipError_t init_weight(hipStream_t s, bf16* dst, int ld, uint64_t seed, uint64_t tensor_id, int rows, int cols,
                       int row_offset, int ib, int phase, int packed) {
  size_t n = (size_t)rows * cols;
  uint64_t base = mix64(seed ^ mix64(tensor_id));
  hipLaunchKernelGGL(init_weight_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, dst, ld, base, rows, cols, row_offset, ib, phase, packed);
  return hipGetLastError();
}

__global__ void convert_weight_kernel(bf16* dst, int ld, const float* src, int rows, int cols, int row_offset, int ib, int phase, int packed) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i >= (size_t)rows * cols) return;
  int r = (int)(i / cols), c = (int)(i % cols);
  dst[weight_elem(phys_row(r, row_offset, ib, phase), c, ld, packed)] = f2bf(src[i]);
}
hipError_t convert_weight(hipStream_t s, bf16* dst, int ld, const float* src, int rows, int cols, int row_offset, int ib, int phase, int packed) {
  size_t n = (size_t)rows * cols;
  hipLaunchKernelGGL(convert_weight_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, dst, ld, src, rows, cols, row_offset, ib, phase, packed);
  return hipGetLastError();
}
__global__ void export_weight_kernel(float* dst, const bf16* src, int ld, int rows, int cols, int row_offset, int ib, int phase, int packed) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i >= (size_t)rows * cols) return;
  int r = (int)(i / cols), c = (int)(i % cols);
  dst[i] = bf2f(src[weight_elem(phys_row(r, row_offset, ib, phase), c, ld, packed)]);
}
hipError_t export_weight(hipStream_t s, float* dst, const bf16* src, int ld, int rows, int cols, int row_offset, int ib, int phase, int packed) {
  size_t n = (size_t)rows * cols;
  hipLaunchKernelGGL(export_weight_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, dst, src, ld, rows, cols, row_offset, ib, phase, packed);
  return hipGetLastError();
}

__global__ void fill_f32_kernel(float* dst, float v, size_t n) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < n) dst[i] = v;
}
hipError_t fill_f32(hipStream_t s, float* dst, float v, size_t n) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, dst, v, n);
  return hipGetLastError();
}

// ------------------------------------------------------------------ embedding, gather
__global__ void embed_kernel(float* X, const bf16* emb, const int* tokens, int h) {
  const int row = blockIdx.x;
  const bf16* e = emb + (size_t)tokens[row] * h;
  for (int c = threadIdx.x * 8; c < h; c += blockDim.x * 8) {
    bf16x8 v = *reinterpret_cast<const bf16x8*>(e + c);
    float* o = X + (size_t)row * h + c;
#pragma unroll
    for (int j = 0; j < 8; j++) o[j] = bf2f(v[j]);
  }
}
hipError_t embed_rows(hipStream_t s, float* X, const bf16* emb, const int* tokens, int n, int h) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(embed_kernel, dim3(n), dim3(256), 0, s, X, emb, tokens, h);
  return hipGetLastError();
}
__global__ void gather_rows_kernel(float* dst, const float* src, const int* rows, int h) {
  const float* a = src + (size_t)rows[blockIdx.x] * h;
  for (int c = threadIdx.x; c < h; c += blockDim.x) dst[(size_t)blockIdx.x * h + c] = a[c];
}
hipError_t gather_rows_f32(hipStream_t s, float* dst, const float* src, const int* rows, int n, int h) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(gather_rows_kernel, dim3(n), dim3(256), 0, s, dst, src, rows, h);
  return hipGetLastError();
}

// ------------------------------------------------------------------ RMSNorm
__device__ __forceinline__ float block_sum(float v, float* red) {   // red: one float per wave (<= 16)
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
  for (int w = 0; w < (int)(blockDim.x >> 6); w++) t += red[w];
  __syncthreads();
  return t;
}

// A workgroup normalises R rows at once: all their loads are issued before the first reduction, so
// the launch is one round of latency-bound workgroups instead of two. Rows of up to 4096 * PER / 4
// elements stay in registers between the sum of squares and the scaling (PER 16-byte loads per
// thread and row); longer rows are read a second time.
template <int R, int PER>
__global__ void __launch_bounds__(256) rmsnorm_kernel(bf16* out, const float* X, const float* gain, float eps, int h, int n) {
  __shared__ float red[R][16];
  const int row0 = blockIdx.x * R;
  const bool in_regs = h <= 1024 * PER;
  f32x4 v[R][PER];
  float ss[R];
#pragma unroll
  for (int r = 0; r < R; r++) {
    ss[r] = 0.f;
    const float* x = X + (size_t)min(row0 + r, n - 1) * h;
    if (in_regs) {
#pragma unroll
      for (int i = 0; i < PER; i++) {
        const int c = threadIdx.x * 4 + i * 1024;
        v[r][i] = c < h ? *reinterpret_cast<const f32x4*>(x + c) : f32x4{0.f, 0.f, 0.f, 0.f};
      }
    }
  }
#pragma unroll
  for (int r = 0; r < R; r++) {
    if (in_regs) {
#pragma unroll
      for (int i = 0; i < PER; i++) ss[r] += v[r][i][0] * v[r][i][0] + v[r][i][1] * v[r][i][1] + v[r][i][2] * v[r][i][2] + v[r][i][3] * v[r][i][3];
    } else {
      const float* x = X + (size_t)min(row0 + r, n - 1) * h;
      for (int c = threadIdx.x * 4; c < h; c += 1024) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(x + c);
        ss[r] += t[0] * t[0] + t[1] * t[1] + t[2] * t[2] + t[3] * t[3];
      }
    }
  }
  // block sums of the R rows with one pair of barriers
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int r = 0; r < R; r++) {
    const float w = wave_sum(ss[r]);
    if (lane == 0) red[r][wave] = w;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < R; r++) {
    if (row0 + r >= n) break;
    const float tot = red[r][0] + red[r][1] + red[r][2] + red[r][3];
    const float inv = rsqrtf(tot / (float)h + eps);
    const float* x = X + (size_t)(row0 + r) * h;
    bf16* o_row = out + (size_t)(row0 + r) * h;
    if (in_regs) {
#pragma unroll
      for (int i = 0; i < PER; i++) {
        const int c = threadIdx.x * 4 + i * 1024;
        if (c < h) {
          const f32x4 g = *reinterpret_cast<const f32x4*>(gain + c);
          bf16x4 o;
#pragma unroll
          for (int j = 0; j < 4; j++) o[j] = f2bf(v[r][i][j] * inv * g[j]);
          *reinterpret_cast<bf16x4*>(o_row + c) = o;
        }
      }
    } else {
      for (int c = threadIdx.x * 4; c < h; c += 1024) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(x + c);
        const f32x4 g = *reinterpret_cast<const f32x4*>(gain + c);
        bf16x4 o;
#pragma unroll
        for (int j = 0; j < 4; j++) o[j] = f2bf(t[j] * inv * g[j]);
        *reinterpret_cast<bf16x4*>(o_row + c) = o;
      }
    }
  }
}
// Embedding rows and the first layer's RMSNorm in one pass: the row is in registers anyway, so the residual stream
// (fp32) and its normalised bf16 copy are written together and the stream is not read back. One workgroup per row,
// 8 elements per thread and 2048-column slab, rows of up to 8192 elements.
__global__ void __launch_bounds__(256) embed_norm_kernel(float* X, bf16* out, const bf16* emb, const int* tokens, const float* gain, float eps, int h) {
  constexpr int PER = 4;
  __shared__ float red[4];
  const int row = blockIdx.x;
  const bf16* e = emb + (size_t)tokens[row] * h;
  bf16x8 v[PER];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < PER; i++) {
    const int c = threadIdx.x * 8 + i * 2048;
    if (c < h) {
      v[i] = *reinterpret_cast<const bf16x8*>(e + c);
#pragma unroll
      for (int j = 0; j < 8; j++) { const float f = bf2f(v[i][j]); ss += f * f; }
    }
  }
  const float w = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = w;
  __syncthreads();
  const float inv = rsqrtf((red[0] + red[1] + red[2] + red[3]) / (float)h + eps);
#pragma unroll
  for (int i = 0; i < PER; i++) {
    const int c = threadIdx.x * 8 + i * 2048;
    if (c < h) {
      float* x = X + (size_t)row * h + c;
      const f32x4 g0 = *reinterpret_cast<const f32x4*>(gain + c), g1 = *reinterpret_cast<const f32x4*>(gain + c + 4);
      f32x4 x0, x1;
      bf16x8 o;
#pragma unroll
      for (int j = 0; j < 4; j++) {
        x0[j] = bf2f(v[i][j]); x1[j] = bf2f(v[i][j + 4]);
        o[j] = f2bf(x0[j] * inv * g0[j]); o[j + 4] = f2bf(x1[j] * inv * g1[j]);
      }
      *reinterpret_cast<f32x4*>(x) = x0;
      *reinterpret_cast<f32x4*>(x + 4) = x1;
      *reinterpret_cast<bf16x8*>(out + (size_t)row * h + c) = o;
    }
  }
}
hipError_t embed_norm_rows(hipStream_t s, float* X, bf16* out, const bf16* emb, const int* tokens, const float* gain, float eps, int n, int h) {
  if (n == 0) return hipSuccess;
  if (h > 8192 || h % 8 != 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(embed_norm_kernel, dim3(n), dim3(256), 0, s, X, out, emb, tokens, gain, eps, h);
  return hipGetLastError();
}

hipError_t rmsnorm_rows(hipStream_t s, bf16* out, const float* X, const float* gain, float eps, int n, int h) {
  if (n == 0) return hipSuccess;
  if (n >= 1024) hipLaunchKernelGGL((rmsnorm_kernel<2, 4>), dim3((n + 1) / 2), dim3(256), 0, s, out, X, gain, eps, h, n);
  else hipLaunchKernelGGL((rmsnorm_kernel<1, 8>), dim3(n), dim3(256), 0, s, out, X, gain, eps, h, n);
  return hipGetLastError();
}

// ------------------------------------------------------------------ rotary + KV page write (prefill)
// One workgroup per token row. cos/sin of the row's position are computed once (in double:
// positions reach tens of thousands of radians) and applied to every head. Q is rotated in
// place; K is rotated and scattered to its page; V is scattered transposed (page_tokens = 16).
__global__ void __launch_bounds__(256) rope_kv_prefill_kernel(bf16* qkv, int ld, const PrefillSeq* seqs, int n_seqs,
                                                              const int* block_tables, const double* inv_freq,
                                                              bf16* pool, KvGeom geo, int n_q) {
  __shared__ float cs[128], sn[128];
  const int row = blockIdx.x, d = geo.d, half = d >> 1;
  int si = 0;
  while (si + 1 < n_seqs && row >= seqs[si + 1].row0) si++;
  const PrefillSeq sq = seqs[si];
  const int pos = sq.p + (row - sq.row0);
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    double sv, cv;
    sincos((double)pos * inv_freq[i], &sv, &cv);
    cs[i] = (float)cv; sn[i] = (float)sv;
  }
  __syncthreads();
  const int page = block_tables[sq.bt_off + pos / geo.page_tokens], slot = pos % geo.page_tokens;
  bf16* r = qkv + (size_t)row * ld;
  // eight rotation pairs (two 16-byte loads, two 16-byte stores) per work item
  const int per_head = half >> 3, n_rot = (n_q + geo.n_kv) * per_head;
  for (int t = threadIdx.x; t < n_rot; t += blockDim.x) {
    const int hd = t / per_head, i0 = (t % per_head) * 8;
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(r + hd * d + i0);
    const bf16x8 b = *reinterpret_cast<const bf16x8*>(r + hd * d + i0 + half);
    bf16x8 ya, yb;
#pragma unroll
    for (int e = 0; e < 8; e++) {
      const float fa = bf2f(a[e]), fb = bf2f(b[e]);
      ya[e] = f2bf(fa * cs[i0 + e] - fb * sn[i0 + e]);
      yb[e] = f2bf(fa * sn[i0 + e] + fb * cs[i0 + e]);
    }
    bf16* dst = hd < n_q ? r + hd * d : pool + ((size_t)page * geo.n_kv + (hd - n_q)) * geo.head_elems() + (size_t)slot * d;
    *reinterpret_cast<bf16x8*>(dst + i0) = ya;
    *reinterpret_cast<bf16x8*>(dst + i0 + half) = yb;
  }
  // V^T: a page row holds 16 tokens of one (head, dd). Where the chunk covers a whole group of 8
  // tokens, the workgroup of the group's first row writes all 8 at once (one 16-byte store per
  // (head, dd), the 8 values gathered from the 8 rows with lane-contiguous loads) and the other
  // seven rows write nothing; a group the chunk covers only partly is written element by element.
  const bf16* vsrc = r + (n_q + geo.n_kv) * d;
  const int g0 = pos & ~7;                                  // first position of this row's group of 8
  const bool whole_group = g0 >= sq.p && g0 + 8 <= sq.p + sq.sl;
  if (whole_group) {
    if (pos != g0) return;
    for (int t = threadIdx.x; t < geo.n_kv * d; t += blockDim.x) {
      const int hd = t / d, dd = t % d;
      bf16x8 pack;
#pragma unroll
      for (int e = 0; e < 8; e++) pack[e] = vsrc[(size_t)e * ld + t];
      bf16* v = pool + ((size_t)page * geo.n_kv + hd) * geo.head_elems() + (size_t)geo.page_tokens * d;
      *reinterpret_cast<bf16x8*>(v + (size_t)dd * geo.page_tokens + slot) = pack;
    }
    return;
  }
  for (int t = threadIdx.x; t < geo.n_kv * d; t += blockDim.x) {
    const int hd = t / d, dd = t % d;
    bf16* v = pool + ((size_t)page * geo.n_kv + hd) * geo.head_elems() + (size_t)geo.page_tokens * d;
    v[(size_t)dd * geo.page_tokens + slot] = vsrc[t];
  }
}
hipError_t rope_kv_write_prefill(hipStream_t s, bf16* qkv, int ld, const PrefillSeq* seqs, int n_seqs,
                                 const int* block_tables, const double* inv_freq, bf16* pool, KvGeom geo,
                                 int n_rows, int n_q) {
  if (n_rows == 0) return hipSuccess;
  hipLaunchKernelGGL(rope_kv_prefill_kernel, dim3(n_rows), dim3(256), 0, s, qkv, ld, seqs, n_seqs, block_tables,
                     inv_freq, pool, geo, n_q);
  return hipGetLastError();
}

// ------------------------------------------------------------------ decode: QKV finish
// Sums the split-K partials of the QKV projection, rotates q and k for position cl, stores q
// (bf16) for the attention kernel and appends k and v to the request's last page.
__global__ void __launch_bounds__(256) decode_qkv_finish_kernel(const float* partials, int splits, long long split_stride, int ld,
                                                                const DecodeSeq* seqs, const int* block_tables,
                                                                const double* inv_freq, bf16* q_out, bf16* pool,
                                                                KvGeom geo, int n_q) {
  // blockIdx.x = request, blockIdx.y = group of 8 head slots out of n_q (Q) + n_kv (K) + n_kv (V)
  __shared__ float cs[128], sn[128];
  const int row = blockIdx.x, d = geo.d, half = d >> 1;
  const int slot0 = blockIdx.y * 8, n_slots = n_q + 2 * geo.n_kv, slot1 = min(n_slots, slot0 + 8);
  const DecodeSeq sq = seqs[row];
  const int pos = sq.cl;
  if (slot0 < n_q + geo.n_kv) {               // this group holds rotated heads
    for (int i = threadIdx.x; i < half; i += blockDim.x) {
      double sv, cv;
      sincos((double)pos * inv_freq[i], &sv, &cv);
      cs[i] = (float)cv; sn[i] = (float)sv;
    }
  }
  __syncthreads();
  const int page = block_tables[sq.bt_off + pos / geo.page_tokens], slot = pos % geo.page_tokens;
  const float* pr = partials + (size_t)row * ld;
  // a work item is four consecutive rotation pairs of a Q or K head, or four consecutive elements of a V head
  const int per_rot = half >> 2, per_v = d >> 2;
  const int n_rot_slots = max(0, min(slot1, n_q + geo.n_kv) - slot0), n_v_slots = (slot1 - slot0) - n_rot_slots;
  const int n_items = n_rot_slots * per_rot + n_v_slots * per_v;
  for (int t = threadIdx.x; t < n_items; t += blockDim.x) {
    if (t < n_rot_slots * per_rot) {
      const int hd = slot0 + t / per_rot, i0 = (t % per_rot) * 4;
      f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
      for (int z = 0; z < splits; z++) {
        a += *reinterpret_cast<const f32x4*>(pr + z * split_stride + hd * d + i0);
        b += *reinterpret_cast<const f32x4*>(pr + z * split_stride + hd * d + i0 + half);
      }
      bf16x4 ya, yb;
#pragma unroll
      for (int e = 0; e < 4; e++) {
        // the projection's result is rounded to bf16 before the rotation, as in the prefill path
        const float fa = bf2f(f2bf(a[e])), fb = bf2f(f2bf(b[e]));
        ya[e] = f2bf(fa * cs[i0 + e] - fb * sn[i0 + e]);
        yb[e] = f2bf(fa * sn[i0 + e] + fb * cs[i0 + e]);
      }
      bf16* dst = hd < n_q ? q_out + (size_t)row * n_q * d + hd * d
                           : pool + ((size_t)page * geo.n_kv + (hd - n_q)) * geo.head_elems() + (size_t)slot * d;
      *reinterpret_cast<bf16x4*>(dst + i0) = ya;
      *reinterpret_cast<bf16x4*>(dst + i0 + half) = yb;
    } else {
      const int tv = t - n_rot_slots * per_rot;
      const int hd = slot0 + n_rot_slots + tv / per_v, dd0 = (tv % per_v) * 4;
      const int vh = hd - n_q - geo.n_kv;
      f32x4 a = {0.f, 0.f, 0.f, 0.f};
      for (int z = 0; z < splits; z++) a += *reinterpret_cast<const f32x4*>(pr + z * split_stride + hd * d + dd0);
      bf16* v = pool + ((size_t)page * geo.n_kv + vh) * geo.head_elems() + (size_t)geo.page_tokens * d;
#pragma unroll
      for (int e = 0; e < 4; e++) v[(size_t)(dd0 + e) * geo.page_tokens + slot] = f2bf(a[e]);
    }
  }
}
hipError_t decode_qkv_finish(hipStream_t s, const float* partials, int splits, long long split_stride, int ld,
                             const DecodeSeq* seqs, const int* block_tables, const double* inv_freq,
                             bf16* q_out, bf16* pool, KvGeom geo, int n, int n_q) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(decode_qkv_finish_kernel, dim3(n, (n_q + 2 * geo.n_kv + 7) / 8), dim3(256), 0, s, partials, splits, split_stride, ld, seqs,
                     block_tables, inv_freq, q_out, pool, geo, n_q);
  return hipGetLastError();
}

// ------------------------------------------------------------------ split-K reductions
// X[row] += sum of partials; optionally out = rmsnorm(X[row]) * gain (bf16).
__global__ void __launch_bounds__(1024) reduce_resid_norm_kernel(float* X, const float* partials, int splits, long long split_stride,
                                                                 bf16* out, const float* gain, float eps, int h) {
  __shared__ float red[16];
  float* x = X + (size_t)blockIdx.x * h;
  const float* p = partials + (size_t)blockIdx.x * h;
  const int step = blockDim.x * 4;
  float ss = 0.f;
  for (int c = threadIdx.x * 4; c < h; c += step) {
    f32x4 v = *reinterpret_cast<const f32x4*>(x + c);
    for (int z = 0; z < splits; z++) {
      f32x4 q = *reinterpret_cast<const f32x4*>(p + z * split_stride + c);
      v += q;
    }
    *reinterpret_cast<f32x4*>(x + c) = v;
    ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
  }
  if (out == nullptr) return;
  const float inv = rsqrtf(block_sum(ss, red) / (float)h + eps);
  for (int c = threadIdx.x * 4; c < h; c += step) {
    f32x4 v = *reinterpret_cast<const f32x4*>(x + c);     // this thread wrote these itself
    f32x4 g = *reinterpret_cast<const f32x4*>(gain + c);
    bf16x4 o;
#pragma unroll
    for (int j = 0; j < 4; j++) o[j] = f2bf(v[j] * inv * g[j]);
    *reinterpret_cast<bf16x4*>(out + (size_t)blockIdx.x * h + c) = o;
  }
}
hipError_t reduce_resid_norm(hipStream_t s, float* X, const float* partials, int splits, long long split_stride,
                             bf16* out_norm, const float* gain, float eps, int n, int h) {
  if (n == 0) return hipSuccess;
  const int threads = h >= 4096 ? 1024 : (h >= 2048 ? 512 : 256);      // one float4 per thread where the row allows
  hipLaunchKernelGGL(reduce_resid_norm_kernel, dim3(n), dim3(threads), 0, s, X, partials, splits, split_stride, out_norm, gain, eps, h);
  return hipGetLastError();
}

// H[row][j] = silu(sum gate_j) * sum up_j; gate/up columns are interleaved in blocks of 32.
__global__ void __launch_bounds__(256) reduce_swiglu_kernel(bf16* H, const float* partials, int splits, long long split_stride, int mlp) {
  const int row = blockIdx.y;
  const int j = (blockIdx.x * blockDim.x + threadIdx.x) * 4;         // four consecutive outputs, inside one block of 32
  if (j >= mlp) return;
  const float* p = partials + (size_t)row * 2 * mlp + (j >> 5) * 64 + (j & 31);
  f32x4 g = {0.f, 0.f, 0.f, 0.f}, u = {0.f, 0.f, 0.f, 0.f};
  for (int z = 0; z < splits; z++) {
    g += *reinterpret_cast<const f32x4*>(p + z * split_stride);
    u += *reinterpret_cast<const f32x4*>(p + z * split_stride + 32);
  }
  bf16x4 o;
#pragma unroll
  for (int e = 0; e < 4; e++) o[e] = f2bf(g[e] / (1.f + __expf(-g[e])) * u[e]);
  *reinterpret_cast<bf16x4*>(H + (size_t)row * mlp + j) = o;
}
hipError_t reduce_swiglu(hipStream_t s, bf16* H, const float* partials, int splits, long long split_stride, int n, int mlp) {
  if (n == 0) return hipSuccess;
  if (mlp % 32 != 0 || split_stride % 4 != 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(reduce_swiglu_kernel, dim3((mlp / 4 + 255) / 256, n), dim3(256), 0, s, H, partials, splits, split_stride, mlp);
  return hipGetLastError();
}

__global__ void reduce_f32_kernel(float* out, const float* partials, int splits, long long split_stride, size_t n) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i >= n) return;
  float a = 0.f;
  for (int z = 0; z < splits; z++) a += partials[z * split_stride + i];
  out[i] = a;
}
hipError_t reduce_f32(hipStream_t s, float* out, const float* partials, int splits, long long split_stride, size_t n) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(reduce_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, out, partials, splits, split_stride, n);
  return hipGetLastError();
}

// ------------------------------------------------------------------ greedy sampling
// One workgroup of 1024 threads per row; 16-byte loads, four in flight per thread. The first
// maximum wins: a thread scans its indices in ascending order and the tree keeps the lower index
// on equal values.
__global__ void __launch_bounds__(1024) argmax_kernel(int* out, const float* logits, int vocab) {
  __shared__ float bv[1024];
  __shared__ int bi[1024];
  const float* l = logits + (size_t)blockIdx.x * vocab;
  float best = -INFINITY; int idx = 0x7FFFFFFF;
  auto take = [&](float v, int c) { if (v > best) { best = v; idx = c; } };
  if ((vocab & 3) == 0) {
    const float4* l4 = reinterpret_cast<const float4*>(l);
    const int n4 = vocab >> 2;
    int q = threadIdx.x;
    for (; q + 3 * 1024 < n4; q += 4 * 1024) {
      const float4 a = l4[q], b = l4[q + 1024], c = l4[q + 2048], d = l4[q + 3072];
      take(a.x, 4 * q); take(a.y, 4 * q + 1); take(a.z, 4 * q + 2); take(a.w, 4 * q + 3);
      take(b.x, 4 * q + 4096); take(b.y, 4 * q + 4097); take(b.z, 4 * q + 4098); take(b.w, 4 * q + 4099);
      take(c.x, 4 * q + 8192); take(c.y, 4 * q + 8193); take(c.z, 4 * q + 8194); take(c.w, 4 * q + 8195);
      take(d.x, 4 * q + 12288); take(d.y, 4 * q + 12289); take(d.z, 4 * q + 12290); take(d.w, 4 * q + 12291);
    }
    for (; q < n4; q += 1024) {
      const float4 a = l4[q];
      take(a.x, 4 * q); take(a.y, 4 * q + 1); take(a.z, 4 * q + 2); take(a.w, 4 * q + 3);
    }
  } else {
    for (int c = threadIdx.x; c < vocab; c += 1024) take(l[c], c);
  }
  bv[threadIdx.x] = best; bi[threadIdx.x] = idx;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if (threadIdx.x < o) {
      const float v = bv[threadIdx.x + o]; const int i = bi[threadIdx.x + o];
      if (v > bv[threadIdx.x] || (v == bv[threadIdx.x] && i < bi[threadIdx.x])) { bv[threadIdx.x] = v; bi[threadIdx.x] = i; }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) out[blockIdx.x] = bi[0] == 0x7FFFFFFF ? 0 : bi[0];     // a row without any value above -inf
}
hipError_t argmax_rows(hipStream_t s, int* out, const float* logits, int n, int vocab) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(argmax_kernel, dim3(n), dim3(1024), 0, s, out, logits, vocab);
  return hipGetLastError();
}

// ------------------------------------------------------------------ bandwidth probe
__global__ void __launch_bounds__(256) copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n) {
  size_t i = blockIdx.x * (size_t)256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i + 3 * stride < n; i += 4 * stride) {
    uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
  }
  for (; i < n; i += stride) dst[i] = src[i];
}
// The read half of the copy alone: what a partition pulls from memory when nothing is written back. The loads carry the
// non-temporal hint (every byte is used once); `sink` receives a word only if the data's XOR hits one particular value,
// which keeps the loads alive.
__global__ void __launch_bounds__(256) read_kernel(const u32x4* __restrict__ src, size_t n, unsigned* __restrict__ sink) {
  size_t i = blockIdx.x * (size_t)256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (; i + 7 * stride < n; i += 8 * stride) {
    u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; u++) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < 8; u++) acc ^= v[u];
  }
  for (; i < n; i += stride) acc ^= src[i];
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x5a17c0deu) *sink = 1u;
}
hipError_t read_probe(hipStream_t s, const void* src, size_t bytes, unsigned* sink, int grid) {
  hipLaunchKernelGGL(read_kernel, dim3(grid), dim3(256), 0, s, (const u32x4*)src, bytes / 16, sink);
  return hipGetLastError();
}
hipError_t copy_probe(hipStream_t s, void* dst, const void* src, size_t bytes, int grid) {
  hipLaunchKernelGGL(copy_kernel, dim3(grid), dim3(256), 0, s, (uint4*)dst, (const uint4*)src, bytes / 16);
  return hipGetLastError();
}

// ------------------------------------------------------------------ KV pool access (tests, synthetic contexts)
__device__ __forceinline__ void kv_addr(const KvGeom& geo, const int* bt, int pos, int hd, int dd, size_t& ki, size_t& vi) {
  const int page = bt[pos / geo.page_tokens], slot = pos % geo.page_tokens;
  const size_t base = ((size_t)page * geo.n_kv + hd) * geo.head_elems();
  ki = base + (size_t)slot * geo.d + dd;
  vi = base + (size_t)geo.page_tokens * geo.d + (size_t)dd * geo.page_tokens + slot;
}
// Element (pos, head, dd) of K (V) is deviate number ((pos*n_kv + head)*d + dd) of the stream
// keyed by tensor id 0x4B000000 + 2*layer (+1 for V): unit variance, rounded to bf16.
__global__ void kv_fill_kernel(bf16* pool, KvGeom geo, const int* bt, int pos0, int n, uint64_t kbase, uint64_t vbase) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t per = (size_t)geo.n_kv * geo.d;
  if (i >= (size_t)n * per) return;
  const int pos = pos0 + (int)(i / per), hd = (int)(i % per) / geo.d, dd = (int)(i % per) % geo.d;
  const uint64_t e = (uint64_t)pos * per + (i % per);
  size_t ki, vi; kv_addr(geo, bt, pos, hd, dd, ki, vi);
  pool[ki] = f2bf((float)irwin_hall12(kbase, e) * 1.52587890625e-05f);
  pool[vi] = f2bf((float)irwin_hall12(vbase, e) * 1.52587890625e-05f);
}
hipError_t kv_fill_random(hipStream_t s, bf16* pool, KvGeom geo, const int* bt, int pos0, int n, uint64_t seed, int layer) {
  size_t tot = (size_t)n * geo.n_kv * geo.d;
  if (tot == 0) return hipSuccess;
  const uint64_t kb = mix64(seed ^ mix64(0x4B000000ull + 2 * (uint64_t)layer)), vb = mix64(seed ^ mix64(0x4B000000ull + 2 * (uint64_t)layer + 1));
  hipLaunchKernelGGL(kv_fill_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, s, pool, geo, bt, pos0, n, kb, vb);
  return hipGetLastError();
}
__global__ void kv_write_kernel(bf16* pool, KvGeom geo, const int* bt, int pos0, int n, const float* k, const float* v) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t per = (size_t)geo.n_kv * geo.d;
  if (i >= (size_t)n * per) return;
  const int pos = pos0 + (int)(i / per), hd = (int)(i % per) / geo.d, dd = (int)(i % per) % geo.d;
  size_t ki, vi; kv_addr(geo, bt, pos, hd, dd, ki, vi);
  pool[ki] = f2bf(k[i]); pool[vi] = f2bf(v[i]);
}
hipError_t kv_write_tokens(hipStream_t s, bf16* pool, KvGeom geo, const int* bt, int pos0, int n, const float* k, const float* v) {
  size_t tot = (size_t)n * geo.n_kv * geo.d;
  if (tot == 0) return hipSuccess;
  hipLaunchKernelGGL(kv_write_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, s, pool, geo, bt, pos0, n, k, v);
  return hipGetLastError();
}
__global__ void kv_read_kernel(const bf16* pool, KvGeom geo, const int* bt, int pos0, int n, float* k, float* v) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t per = (size_t)geo.n_kv * geo.d;
  if (i >= (size_t)n * per) return;
  const int pos = pos0 + (int)(i / per), hd = (int)(i % per) / geo.d, dd = (int)(i % per) % geo.d;
  size_t ki, vi; kv_addr(geo, bt, pos, hd, dd, ki, vi);
  k[i] = bf2f(pool[ki]); v[i] = bf2f(pool[vi]);
}
hipError_t kv_read_tokens(hipStream_t s, const bf16* pool, KvGeom geo, const int* bt, int pos0, int n, float* k, float* v) {
  size_t tot = (size_t)n * geo.n_kv * geo.d;
  if (tot == 0) return hipSuccess;
  hipLaunchKernelGGL(kv_read_kernel, dim3((unsigned)((tot + 255) / 256)), dim3(256), 0, s, pool, geo, bt, pos0, n, k, v);
  return hipGetLastError();
}

}  // namespace sts
