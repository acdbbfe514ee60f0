// Decode attention over the paged KV cache (one new query token per request), gfx950.
//
// HBM-bound: every K and V byte of a request's context is read exactly once per KV head —
// the G query heads that share a KV head are processed together. Work is split over
// (request, kv head, context chunk of a fixed number of pages) so that a few long contexts
// still fill the CUs while short ones cost few workgroups; a small second kernel merges the
// chunks' (max, sum, weighted V) partials.
//
// Inside a workgroup (4 waves):
//   1. scores: waves take pages in turn, two at a time with the next two already in flight; a lane reads a contiguous 1/4 of one token's K row
//      (64 bytes for d = 128), so a wave reads one 4 KiB page chunk fully coalesced, and
//      accumulates q.k with v_dot2_f32_bf16 (no conversions); 4-lane reduction.
//   2. softmax over the chunk in LDS (exact within the chunk; chunks merge by rescaling).
//   3. P.V: V is stored transposed in a page (d rows of 16 tokens), so a lane owns d rows,
//      reads 32 contiguous bytes per row and dots them with the 16 probabilities.
#include "kernels.h"

namespace sts {

constexpr int MAX_CHUNK_TOKENS = 512;     // tokens per (request, kv head, chunk) workgroup

__device__ __forceinline__ float dot2(unsigned a, unsigned b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}

template <int D, int G>
__global__ void __launch_bounds__(256) attn_decode_kernel(const bf16* __restrict__ q, const DecodeSeq* __restrict__ seqs,
                                                          const AttnItem* __restrict__ items,
                                                          const int* __restrict__ block_tables, const bf16* __restrict__ pool,
                                                          KvGeom geo, int n_q, int chunk_pages, int max_chunks,
                                                          float* __restrict__ ws, float scale_log2e) {
  constexpr int SEG = D / 4;              // K elements per lane (a token's row is split over 4 lanes)
  constexpr int SEGW = SEG / 2;           // ... as packed bf16 pairs
  constexpr int ROWS = D / 64;            // V^T rows per lane
  __shared__ float S[G][MAX_CHUNK_TOKENS];
  __shared__ __align__(16) bf16 P[G][MAX_CHUNK_TOKENS];
  __shared__ float red[4][G][D];
  __shared__ float stat_m[G], stat_l[G];

  const AttnItem item = items[blockIdx.x];          // (request, chunk): only chunks that exist are launched
  const int chunk = item.q0, kvh = blockIdx.y, req = item.seq;
  const DecodeSeq sq = seqs[req];
  const int len = sq.cl + 1;
  const int n_pages = (len + 15) >> 4;
  const int pg0 = chunk * chunk_pages, pg1 = min(n_pages, pg0 + chunk_pages);
  if (pg0 >= pg1) return;                 // this request has fewer chunks (the merge knows)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float* wout = ws + (((size_t)req * geo.n_kv + kvh) * max_chunks + chunk) * G * (D + 2);
  const int t0 = pg0 * 16, nt = min(len, pg1 * 16) - t0;
  const int* bt = block_tables + sq.bt_off;
  const size_t head_elems = geo.head_elems();

  // Page ids of the chunk, one per lane (a chunk has at most 32 pages); the loops below fetch
  // them with a cross-lane read, so no K or V load waits on a block-table load. Indices past the
  // chunk are clamped to its last page: prefetches beyond the end re-read it and are not used.
  const int npg = pg1 - pg0;
  const int wv = __builtin_amdgcn_readfirstlane(wave);
  const int my_page = bt[pg0 + min(lane, npg - 1)];
  auto page_base = [&](int i) -> const bf16* {
    const int page = __builtin_amdgcn_readlane(my_page, __builtin_amdgcn_readfirstlane(min(i, npg - 1)));
    return pool + ((size_t)page * geo.n_kv + kvh) * head_elems;
  };
  // A wave takes the chunk's pages wv, wv+4 (one pair), wv+8, wv+12 (next pair), ...; the next
  // pair is in flight while the current one is consumed.
  const int tok = lane >> 2, seg = lane & 3;
  auto load_k = [&](int i, u32x4 (&kr)[2][SEGW / 4]) {
    const u32x4* p0 = reinterpret_cast<const u32x4*>(page_base(i) + (size_t)tok * D + seg * SEG);
    const u32x4* p1 = reinterpret_cast<const u32x4*>(page_base(i + 4) + (size_t)tok * D + seg * SEG);
#pragma unroll
    for (int x = 0; x < SEGW / 4; x++) { kr[0][x] = p0[x]; kr[1][x] = p1[x]; }
  };
  auto load_v = [&](int i, u32x4 (&vr)[2][ROWS][2]) {
#pragma unroll
    for (int u = 0; u < 2; u++) {
      const bf16* vbase = page_base(i + 4 * u) + (size_t)16 * D;
#pragma unroll
      for (int r = 0; r < ROWS; r++) {
        const u32x4* vp = reinterpret_cast<const u32x4*>(vbase + (size_t)(lane + 64 * r) * 16);
        vr[u][r][0] = vp[0]; vr[u][r][1] = vp[1];
      }
    }
  };

  // ---- 1. scores
  {
    unsigned qr[G][SEGW];
#pragma unroll
    for (int g = 0; g < G; g++) {
      const unsigned* qp = reinterpret_cast<const unsigned*>(q + ((size_t)req * n_q + kvh * G + g) * D + seg * SEG);
#pragma unroll
      for (int i = 0; i < SEGW; i++) qr[g][i] = qp[i];
    }
    auto score = [&](int i, const u32x4 (&kr)[2][SEGW / 4]) {
#pragma unroll
      for (int u = 0; u < 2; u++) {
        if (i + 4 * u >= npg) break;                    // wave-uniform
        float acc[G];
#pragma unroll
        for (int g = 0; g < G; g++) {
          float a = 0.f;
#pragma unroll
          for (int x = 0; x < SEGW / 4; x++) {
            a = dot2(kr[u][x][0], qr[g][4 * x + 0], a);
            a = dot2(kr[u][x][1], qr[g][4 * x + 1], a);
            a = dot2(kr[u][x][2], qr[g][4 * x + 2], a);
            a = dot2(kr[u][x][3], qr[g][4 * x + 3], a);
          }
          a += __shfl_xor(a, 1, 64);
          a += __shfl_xor(a, 2, 64);
          acc[g] = a;
        }
        if (seg == 0) {
          const int t = (i + 4 * u) * 16 + tok;
#pragma unroll
          for (int g = 0; g < G; g++) if (t < nt) S[g][t] = acc[g] * scale_log2e;
        }
      }
    };
    u32x4 ka[2][SEGW / 4], kb[2][SEGW / 4];
    load_k(wv, ka);
    for (int i = wv; i < npg; i += 16) {
      load_k(i + 8, kb);
      score(i, ka);
      load_k(i + 16, ka);
      if (i + 8 < npg) score(i + 8, kb);
    }
  }
  // first V^T pages: in flight during the softmax
  u32x4 va[2][ROWS][2], vb[2][ROWS][2];
  load_v(wv, va);
  __syncthreads();

  // ---- 2. softmax statistics and probabilities (wave w takes heads w, w+4, ...)
  for (int g = wave; g < G; g += 4) {
    float mx = -INFINITY;
    for (int t = lane; t < nt; t += 64) mx = fmaxf(mx, S[g][t]);
    mx = wave_max(mx);
    float sum = 0.f;
    for (int t = lane; t < nt; t += 64) {
      const float p = __builtin_amdgcn_exp2f(S[g][t] - mx);
      sum += p;
      P[g][t] = f2bf(p);
    }
    // zero the tail of the last page so that stale tokens contribute nothing
    for (int t = nt + lane; t < ((nt + 15) & ~15); t += 64) P[g][t] = f2bf(0.f);
    sum = wave_sum(sum);
    if (lane == 0) { stat_m[g] = mx; stat_l[g] = sum; }
  }
  __syncthreads();

  // ---- 3. P.V
  float acc[G][ROWS];
#pragma unroll
  for (int g = 0; g < G; g++)
#pragma unroll
    for (int r = 0; r < ROWS; r++) acc[g][r] = 0.f;
  auto pv = [&](int i, const u32x4 (&vr)[2][ROWS][2]) {
#pragma unroll
    for (int u = 0; u < 2; u++) {
      if (i + 4 * u >= npg) break;                      // wave-uniform
      const int tb = (i + 4 * u) * 16;
#pragma unroll
      for (int g = 0; g < G; g++) {
        const u32x4 p0 = *reinterpret_cast<const u32x4*>(&P[g][tb]);
        const u32x4 p1 = *reinterpret_cast<const u32x4*>(&P[g][tb + 8]);
#pragma unroll
        for (int r = 0; r < ROWS; r++) {
          float a = acc[g][r];
          a = dot2(vr[u][r][0][0], p0[0], a); a = dot2(vr[u][r][0][1], p0[1], a);
          a = dot2(vr[u][r][0][2], p0[2], a); a = dot2(vr[u][r][0][3], p0[3], a);
          a = dot2(vr[u][r][1][0], p1[0], a); a = dot2(vr[u][r][1][1], p1[1], a);
          a = dot2(vr[u][r][1][2], p1[2], a); a = dot2(vr[u][r][1][3], p1[3], a);
          acc[g][r] = a;
        }
      }
    }
  };
  for (int i = wv; i < npg; i += 16) {
    load_v(i + 8, vb);
    pv(i, va);
    load_v(i + 16, va);
    if (i + 8 < npg) pv(i + 8, vb);
  }
#pragma unroll
  for (int g = 0; g < G; g++)
#pragma unroll
    for (int r = 0; r < ROWS; r++) red[wave][g][lane + 64 * r] = acc[g][r];
  __syncthreads();
  for (int i = tid; i < G * D; i += 256) {
    const int g = i / D, dd = i % D;
    wout[g * (D + 2) + dd] = red[0][g][dd] + red[1][g][dd] + red[2][g][dd] + red[3][g][dd];
  }
  if (tid < G) { wout[tid * (D + 2) + D] = stat_m[tid]; wout[tid * (D + 2) + D + 1] = stat_l[tid]; }
}

// Merge the chunks of one (request, query head): out = sum_c o_c 2^(m_c - m) / sum_c l_c 2^(m_c - m).
template <int D>
__global__ void attn_decode_merge_kernel(bf16* __restrict__ out, const float* __restrict__ ws, const DecodeSeq* __restrict__ seqs,
                                         int n_q, int n_kv, int G, int chunk_pages, int max_chunks) {
  const int head = blockIdx.x, req = blockIdx.y, dd = threadIdx.x;
  const int kvh = head / G, g = head % G;
  const int n_pages = (seqs[req].cl + 1 + 15) >> 4;
  const int chunks = (n_pages + chunk_pages - 1) / chunk_pages;
  const float* base = ws + (((size_t)req * n_kv + kvh) * max_chunks) * G * (D + 2) + g * (D + 2);
  const size_t cstride = (size_t)G * (D + 2);
  float m = -INFINITY;
  for (int c = 0; c < chunks; c++) m = fmaxf(m, base[c * cstride + D]);
  float l = 0.f, o = 0.f;
  for (int c = 0; c < chunks; c++) {
    const float w = __builtin_amdgcn_exp2f(base[c * cstride + D] - m);
    l += base[c * cstride + D + 1] * w;
    o += base[c * cstride + dd] * w;
  }
  out[((size_t)req * n_q + head) * D + dd] = f2bf(o / l);
}

int attn_decode_max_chunk_tokens() { return MAX_CHUNK_TOKENS; }
size_t attn_decode_ws_floats(int n, int n_q, int d, int chunks) { return (size_t)n * n_q * chunks * (d + 2); }

template <int D, int G>
static void launch_decode(hipStream_t s, const bf16* q, bf16* out, const DecodeSeq* seqs, const AttnItem* items, int n_items,
                          const int* bt, const bf16* pool, KvGeom geo, int n, int n_q, int chunk_pages, int max_chunks, float* ws, float sc) {
  hipLaunchKernelGGL((attn_decode_kernel<D, G>), dim3(n_items, geo.n_kv), dim3(256), 0, s, q, seqs, items, bt, pool, geo, n_q, chunk_pages, max_chunks, ws, sc);
  hipLaunchKernelGGL(attn_decode_merge_kernel<D>, dim3(n_q, n), dim3(D), 0, s, out, ws, seqs, n_q, geo.n_kv, G, chunk_pages, max_chunks);
}

// q, out: [n, n_q * d] bf16 (q already rotated). A context is cut into chunks of `chunk_pages`
// pages (1..32: at most attn_decode_max_chunk_tokens() tokens); `max_chunks` must be at least
// the chunk count of the longest context. items: one (request, chunk index) record per chunk
// that exists, n_items of them (device memory). ws: attn_decode_ws_floats(n, n_q, d, max_chunks).
hipError_t attn_decode(hipStream_t s, const bf16* q, bf16* out, const DecodeSeq* seqs, const AttnItem* items, int n_items,
                       const int* block_tables, const bf16* pool, KvGeom geo, int n, int n_q, int chunk_pages, int max_chunks, float* ws) {
  if (n == 0 || n_items == 0) return hipSuccess;
  if (geo.page_tokens != 16 || n_q % geo.n_kv != 0 || chunk_pages < 1 || chunk_pages * 16 > MAX_CHUNK_TOKENS || max_chunks < 1) return hipErrorInvalidValue;
  const int G = n_q / geo.n_kv;
  const float sc = 1.4426950408889634f / sqrtf((float)geo.d);
  if (geo.d == 128 && G == 4) launch_decode<128, 4>(s, q, out, seqs, items, n_items, block_tables, pool, geo, n, n_q, chunk_pages, max_chunks, ws, sc);
  else if (geo.d == 128 && G == 8) launch_decode<128, 8>(s, q, out, seqs, items, n_items, block_tables, pool, geo, n, n_q, chunk_pages, max_chunks, ws, sc);
  else if (geo.d == 128 && G == 1) launch_decode<128, 1>(s, q, out, seqs, items, n_items, block_tables, pool, geo, n, n_q, chunk_pages, max_chunks, ws, sc);
  else if (geo.d == 64 && G == 1) launch_decode<64, 1>(s, q, out, seqs, items, n_items, block_tables, pool, geo, n, n_q, chunk_pages, max_chunks, ws, sc);
  else if (geo.d == 64 && G == 4) launch_decode<64, 4>(s, q, out, seqs, items, n_items, block_tables, pool, geo, n, n_q, chunk_pages, max_chunks, ws, sc);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace sts
