// Decode attention over the paged KV cache (one new query token per request), gfx950.
//
// HBM-bound: every K and V byte of a request's context is read exactly once per KV head -- the G
// query heads that share a KV head are processed together. Work is split over (request, KV head,
// context chunk of up to 64 pages) so that a few long contexts still fill the CUs while short ones
// cost few workgroups; a small second kernel merges the chunks' (max, sum, weighted V) partials,
// and a context of a single chunk is finished by the attention kernel itself.
//
// Both contractions run on the matrix cores although the path is memory-bound: with the G query
// heads of a group as MFMA columns the vector ALUs only do the softmax, and the kernel pulls what a
// CU can pull from memory (with dot-product instructions the G * 2 products per key cost about 8
// wave instructions per key and held it well below that).
//
// A wave owns blocks of two pages (32 keys) of the chunk, four blocks apart. Per block:
//   S^T[key, g] = K[key, :] . Q[g, :]       v_mfma_f32_32x32x16_bf16, A = K rows, B = Q rows (columns
//                                           g >= G are zero), so a lane holds one query column and
//                                           the running max / sum need one cross-half exchange
//   O^T[dd, g] += V^T[dd, key] . P^T[key, g]  A = V^T rows straight from global memory (a lane reads the
//                                           16 bytes of 8 consecutive tokens of one d row: a wave
//                                           instruction covers 1 KiB contiguously), B = P^T from the
//                                           S^T accumulator registers
// K rows are fetched global -> LDS without passing through registers, into a buffer private to
// the wave (no workgroup barrier in the key loop, the wave waits on its own vmcnt), two blocks
// deep; the 16-byte chunk c of a row sits at slot c ^ swizzle(row), applied on the global side,
// so the operand reads are conflict free. Row m of a 16-row group of the A operand holds token
// (m & 3) | ((m >> 3) & 1) << 2 | ((m >> 2) & 1) << 3 of the page: with that order the eight
// S^T registers a lane half holds for a page are its tokens 8*half .. 8*half+7, which is the
// order the V^T operand has in memory. Partial (max, sum, O) of the four waves are merged in LDS.
#include <cstdlib>

#include "kernels.h"

namespace sts {

// A context of n_pages is cut into ceil(n_pages / chunk_pages) chunks of EQUAL size (the last may be
// shorter by less than the chunk count) instead of full chunks and a remainder: a workgroup with a
// page or two is bound by the latency of its few dependent loads, and while it waits it holds one
// of the two workgroup slots of its CU.
__device__ __forceinline__ int balanced_chunk_pages(int n_pages, int chunk_pages) {
  const int chunks = (n_pages + chunk_pages - 1) / chunk_pages;
  return (n_pages + chunks - 1) / chunks;
}

__device__ __forceinline__ float half_swap_max_f(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

constexpr int MFMA_LDS_BASE = 1024;                 // buffers filled by direct-to-LDS loads stay clear of address 0
template <int D>
constexpr int attn_decode_mfma_lds() { return MFMA_LDS_BASE + 4 * 2 * 2 * 16 * D * 2; }   // 4 waves x 2 stages x 2 pages of K

template <int D, int G, bool NT>
__global__ void __launch_bounds__(256, 2) attn_decode_mfma_kernel(const bf16* __restrict__ q, bf16* __restrict__ out, const DecodeSeq* __restrict__ seqs,
                                                               const DecodeItem* __restrict__ items,
                                                               const int* __restrict__ block_tables, const bf16* __restrict__ pool,
                                                               KvGeom geo, int n_q, int chunk_pages, int max_chunks,
                                                               float* __restrict__ ws, float scale_log2e) {
  static_assert(G <= 32 && (D == 64 || D == 128), "one 32-column block of query heads; rows of 8 or 16 chunks");
  constexpr int KSTEPS = D / 16, DB = D / 32;
  constexpr int ROWB = D * 2;                        // bytes of a K row
  constexpr int CPR = D / 8;                         // 16-byte chunks per K row
  constexpr int RPI = 64 / CPR;                      // K rows one wave load instruction covers
  constexpr int IPP = 16 / RPI;                      // load instructions per page
  constexpr int PAGE_KB = 16 * ROWB;                 // K bytes of one page and head
  constexpr int STAGE = 2 * PAGE_KB;
  constexpr int LOADS = 2 * IPP + 2 * DB;            // vector-memory loads a wave issues per block (K to LDS + V^T to registers)
  extern __shared__ __align__(16) unsigned char smem[];

  const DecodeItem item = items[blockIdx.x];
  const int chunk = item.chunk, kvh = blockIdx.y, req = item.seq;
  const int len = item.cl + 1;
  const int n_pages = (len + 15) >> 4;
  const int cp = balanced_chunk_pages(n_pages, chunk_pages);
  const int pg0 = chunk * cp, pg1 = min(n_pages, pg0 + cp);
  if (pg0 >= pg1) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, lh = lane >> 5;
  float* wout = ws + (((size_t)req * geo.n_kv + kvh) * max_chunks + chunk) * G * (D + 2);
  const int nt = min(len, pg1 * 16) - pg0 * 16;      // tokens of the chunk
  const int* bt = block_tables + item.bt_off;
  const size_t head_elems = geo.head_elems();
  const int npg = pg1 - pg0, nblk = (npg + 1) >> 1;
  const int wv = __builtin_amdgcn_readfirstlane(wave);
  // page ids of the chunk, one per lane; indices past the chunk repeat its last page (fetched, masked)
  const int my_page = bt[pg0 + min(lane, npg - 1)];
  auto page_base = [&](int i) -> const bf16* {
    const int page = __builtin_amdgcn_readlane(my_page, __builtin_amdgcn_readfirstlane(min(i, npg - 1)));
    return pool + ((size_t)page * geo.n_kv + kvh) * head_elems;
  };
  auto swz = [](int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); };
  unsigned char* kbuf = smem + MFMA_LDS_BASE + wv * 2 * STAGE;

  // lane's part of one K load instruction: row lane / CPR of the RPI rows, the chunk that belongs in slot lane % CPR
  int ksrc[IPP];
#pragma unroll
  for (int j = 0; j < IPP; j++) {
    const int row = j * RPI + lane / CPR;
    ksrc[j] = row * D + ((lane % CPR) ^ swz(row)) * 8;
  }
  auto issue_k = [&](int b, int stage) {
#pragma unroll
    for (int u = 0; u < 2; u++) {
      const bf16* kb = page_base(2 * b + u);
#pragma unroll
      for (int j = 0; j < IPP; j++) {
        if constexpr (NT) load_to_lds16_nt(kb + ksrc[j], kbuf + stage * STAGE + u * PAGE_KB + j * 1024);
        else load_to_lds16(kb + ksrc[j], kbuf + stage * STAGE + u * PAGE_KB + j * 1024);
      }
    }
  };
  auto load_v = [&](int b, u32x4 (&vr)[2][DB]) {
#pragma unroll
    for (int u = 0; u < 2; u++) {
      const bf16* vb = page_base(2 * b + u) + (size_t)16 * D;
#pragma unroll
      for (int bb = 0; bb < DB; bb++) {
        const u32x4* src = reinterpret_cast<const u32x4*>(vb + (bb * 32 + l32) * 16 + lh * 8);
        if constexpr (NT) vr[u][bb] = __builtin_nontemporal_load(src); else vr[u][bb] = *src;
      }
    }
  };

  // Q^T operand: column l32 is query head l32 of the group
  bf16x8 qf[KSTEPS];
#pragma unroll
  for (int kk = 0; kk < KSTEPS; kk++) {
    u32x4 z = {0u, 0u, 0u, 0u};
    if (l32 < G) z = *reinterpret_cast<const u32x4*>(q + ((size_t)req * n_q + kvh * G + l32) * D + kk * 16 + lh * 8);
    qf[kk] = __builtin_bit_cast(bf16x8, z);
  }
  // K operand address of this lane inside a stage: row l32 of the block is token `tok` of page l32 >> 4
  const int tok = (l32 & 3) | (((l32 >> 3) & 1) << 2) | (((l32 >> 2) & 1) << 3);
  const int krow = (l32 >> 4) * PAGE_KB + tok * ROWB;
  int kslot[KSTEPS];
#pragma unroll
  for (int kk = 0; kk < KSTEPS; kk++) kslot[kk] = krow + ((2 * kk + lh) ^ swz(tok)) * 16;

  f32x16 o[DB];
#pragma unroll
  for (int bb = 0; bb < DB; bb++)
#pragma unroll
    for (int r = 0; r < 16; r++) o[bb][r] = 0.f;
  float m_ref = -INFINITY, l_run = 0.f;

  auto scores = [&](int stage, f32x16& s) {
    const unsigned char* kst = kbuf + stage * STAGE;
#pragma unroll
    for (int r = 0; r < 16; r++) s[r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KSTEPS; kk++) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kst + kslot[kk]);
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s, 0, 0, 0);
    }
  };
  auto softmax_pv = [&](int b, f32x16& s, const u32x4 (&vr)[2][DB]) {
    // register r of the block: page r >> 3 of the pair, token 8 * half + (r & 7)
    const int t_base = b * 32 + 8 * lh;
    if (t_base + 23 >= nt) {                         // only a block at the end of the context
#pragma unroll
      for (int r = 0; r < 16; r++)
        if (t_base + (r >> 3) * 16 + (r & 7) >= nt) s[r] = -INFINITY;
    }
    float mx = s[0];
#pragma unroll
    for (int r = 1; r < 16; r++) mx = fmaxf(mx, s[r]);
    mx = half_swap_max_f(mx);
    if (__any(mx > m_ref)) {                         // wave-uniform
      const float m_new = fmaxf(m_ref, mx);
      const float corr = __builtin_amdgcn_exp2f((m_ref - m_new) * scale_log2e);     // 0 on the first block
      m_ref = m_new;
      l_run *= corr;
#pragma unroll
      for (int bb = 0; bb < DB; bb++)
#pragma unroll
        for (int r = 0; r < 16; r++) o[bb][r] *= corr;
    }
    const float nm = -m_ref * scale_log2e;
    float rs = 0.f;
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const float p = __builtin_amdgcn_exp2f(fmaf(s[r], scale_log2e, nm));
      s[r] = p;
      rs += p;
    }
    l_run += rs;
#pragma unroll
    for (int u = 0; u < 2; u++) {
      bf16x8 pb;
#pragma unroll
      for (int e = 0; e < 8; e++) pb[e] = f2bf(s[8 * u + e]);
#pragma unroll
      for (int bb = 0; bb < DB; bb++) o[bb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vr[u][bb]), pb, o[bb], 0, 0, 0);
    }
  };
  // compiler and scheduler fence: no LDS read of a block above the wait for its loads, no refill of
  // a K stage above the reads of the block that used it
  auto fence = [] { __asm__ volatile("" ::: "memory"); __builtin_amdgcn_sched_barrier(0); };
  // The wave's blocks are wv, wv + 4, ...; block i uses K stage i & 1 and V^T registers i & 1.
  // Loads run two blocks ahead: K of block i + 2 goes out as soon as the scores of block i have
  // left its stage, V^T of block i + 2 when block i is finished. Vector-memory loads complete in
  // issue order (K0 V0 K1 V1 K2 V2 ...), so block i has landed once at most the LOADS of block i + 1
  // are outstanding.
  u32x4 va[2][DB], vb[2][DB];
  const int nmine = wv < nblk ? (nblk - wv + 3) >> 2 : 0;
  auto step = [&](int i, int stage, u32x4 (&vr)[2][DB]) {
    const int b = wv + 4 * i;
    if (i + 1 < nmine) wait_vmem<LOADS>(); else wait_vmem<0>();
    fence();
    f32x16 s;
    scores(stage, s);
    if (i + 2 < nmine) {
      __builtin_amdgcn_s_waitcnt(0xC07F);            // lgkmcnt(0): every K operand of this block has been read
      fence();
      issue_k(b + 8, stage);
    }
    softmax_pv(b, s, vr);
    if (i + 2 < nmine) load_v(b + 8, vr);
  };
  if (nmine > 0) {
    issue_k(wv, 0); load_v(wv, va);
    if (nmine > 1) { issue_k(wv + 4, 1); load_v(wv + 4, vb); }
    for (int i = 0; i < nmine; i += 2) {
      step(i, 0, va);
      if (i + 1 < nmine) step(i + 1, 1, vb);
    }
  }
  l_run += __shfl_xor(l_run, 32, 64);

  // ---- merge the four waves (the K buffers are free once every wave is past its loop)
  __syncthreads();
  float* sm = reinterpret_cast<float*>(smem + MFMA_LDS_BASE);            // [4][G] maxima (scaled), then [4][G] sums
  float* sl = sm + 4 * G;
  float* red = sl + 4 * G;                                               // [4][G][D]
  if (lane < G) { sm[wv * G + lane] = m_ref * scale_log2e; sl[wv * G + lane] = l_run; }
  __syncthreads();
  if (l32 < G) {
    float mall = fmaxf(fmaxf(sm[l32], sm[G + l32]), fmaxf(sm[2 * G + l32], sm[3 * G + l32]));
    const float f = (m_ref == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_ref * scale_log2e - mall);
#pragma unroll
    for (int bb = 0; bb < DB; bb++)
#pragma unroll
      for (int r = 0; r < 16; r++) red[(wv * G + l32) * D + bb * 32 + 8 * (r >> 2) + 4 * lh + (r & 3)] = o[bb][r] * f;
  }
  __syncthreads();
  // a context that fits one chunk needs no merge: normalise and store the attention output itself
  const bool single = n_pages <= chunk_pages;
  for (int i = tid; i < G * D; i += 256) {
    const int g = i / D;
    const float o_sum = red[i] + red[G * D + i] + red[2 * G * D + i] + red[3 * G * D + i];
    if (single) {
      const float mall = fmaxf(fmaxf(sm[g], sm[G + g]), fmaxf(sm[2 * G + g], sm[3 * G + g]));
      float l = 0.f;
#pragma unroll
      for (int w = 0; w < 4; w++) l += (sm[w * G + g] == -INFINITY) ? 0.f : sl[w * G + g] * __builtin_amdgcn_exp2f(sm[w * G + g] - mall);
      out[((size_t)req * n_q + kvh * G + g) * D + i % D] = f2bf(o_sum / l);
    } else {
      wout[g * (D + 2) + i % D] = o_sum;
    }
  }
  if (!single && tid < G) {
    const float mall = fmaxf(fmaxf(sm[tid], sm[G + tid]), fmaxf(sm[2 * G + tid], sm[3 * G + tid]));
    float l = 0.f;
#pragma unroll
    for (int w = 0; w < 4; w++) l += (sm[w * G + tid] == -INFINITY) ? 0.f : sl[w * G + tid] * __builtin_amdgcn_exp2f(sm[w * G + tid] - mall);
    wout[tid * (D + 2) + D] = mall;
    wout[tid * (D + 2) + D + 1] = l;
  }
}

// Merge the chunks of one (request, query head): out = sum_c o_c 2^(m_c - m) / sum_c l_c 2^(m_c - m).
template <int D>
__global__ void attn_decode_merge_kernel(bf16* __restrict__ out, const float* __restrict__ ws, const DecodeSeq* __restrict__ seqs,
                                         const int* __restrict__ multi, int n_q, int n_kv, int G, int chunk_pages, int max_chunks) {
  const int head = blockIdx.x, req = multi[blockIdx.y], dd = threadIdx.x;
  const int kvh = head / G, g = head % G;
  const int n_pages = (seqs[req].cl + 1 + 15) >> 4;
  const int chunks = (n_pages + chunk_pages - 1) / chunk_pages;
  if (chunks == 1) return;                         // (not listed by the caller: the attention kernel stored this request's output itself)
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


size_t attn_decode_ws_floats(int n, int n_q, int d, int chunks) { return (size_t)n * n_q * chunks * (d + 2); }

// The kernel keeps a chunk's page ids one per lane: up to 64 pages.
constexpr int MAX_CHUNK_TOKENS = 1024;
int attn_decode_max_chunk_tokens() { return MAX_CHUNK_TOKENS; }

template <int D, int G, bool NT>
static void launch_decode_kernel(hipStream_t s, const bf16* q, bf16* out, const DecodeSeq* seqs, const DecodeItem* items, int n_items,
                                 const int* bt, const bf16* pool, KvGeom geo, int n_q, int chunk_pages, int max_chunks, float* ws, float sc) {
  constexpr int lds = attn_decode_mfma_lds<D>();
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_decode_mfma_kernel<D, G, NT>), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  (void)attr;
  hipLaunchKernelGGL((attn_decode_mfma_kernel<D, G, NT>), dim3(n_items, geo.n_kv), dim3(256), lds, s, q, out, seqs, items, bt, pool, geo, n_q, chunk_pages, max_chunks, ws, sc);
}

template <int D, int G>
static void launch_decode(hipStream_t s, const bf16* q, bf16* out, const DecodeSeq* seqs, const DecodeItem* items, int n_items, const int* multi, int n_multi,
                          const int* bt, const bf16* pool, KvGeom geo, int n_q, int chunk_pages, int max_chunks, float* ws, float sc, bool stream_nt) {
  if (stream_nt) launch_decode_kernel<D, G, true>(s, q, out, seqs, items, n_items, bt, pool, geo, n_q, chunk_pages, max_chunks, ws, sc);
  else launch_decode_kernel<D, G, false>(s, q, out, seqs, items, n_items, bt, pool, geo, n_q, chunk_pages, max_chunks, ws, sc);
  if (n_multi > 0)
    hipLaunchKernelGGL(attn_decode_merge_kernel<D>, dim3(n_q, n_multi), dim3(D), 0, s, out, ws, seqs, multi, n_q, geo.n_kv, G, chunk_pages, max_chunks);
}

// q, out: [n, n_q * d] bf16 (q already rotated). A context is cut into chunks of `chunk_pages`
// pages (at most attn_decode_max_chunk_tokens() tokens); `max_chunks` must be at least
// the chunk count of the longest context. items: one (request, chunk index) record per chunk
// that exists, n_items of them (device memory). multi: the n_multi requests whose context has more than
// one chunk (device memory; only these need the merge kernel, and with none of them it is not launched).
// ws: attn_decode_ws_floats(n, n_q, d, max_chunks). stream_nt: fetch K and V with the non-temporal hint.
hipError_t attn_decode(hipStream_t s, const bf16* q, bf16* out, const DecodeSeq* seqs, const DecodeItem* items, int n_items, const int* multi, int n_multi,
                       const int* block_tables, const bf16* pool, KvGeom geo, int n, int n_q, int chunk_pages, int max_chunks, float* ws, bool stream_nt) {
  if (n == 0 || n_items == 0) return hipSuccess;
  if (n_multi < 0 || n_multi > n || (n_multi > 0 && !multi)) return hipErrorInvalidValue;
  if (geo.page_tokens != 16 || n_q % geo.n_kv != 0 || chunk_pages < 1 || chunk_pages * 16 > attn_decode_max_chunk_tokens() || max_chunks < 1) return hipErrorInvalidValue;
  const int G = n_q / geo.n_kv;
  const float sc = 1.4426950408889634f / sqrtf((float)geo.d);
  if (geo.d == 128 && G == 4) launch_decode<128, 4>(s, q, out, seqs, items, n_items, multi, n_multi, block_tables, pool, geo, n_q, chunk_pages, max_chunks, ws, sc, stream_nt);
  else if (geo.d == 128 && G == 8) launch_decode<128, 8>(s, q, out, seqs, items, n_items, multi, n_multi, block_tables, pool, geo, n_q, chunk_pages, max_chunks, ws, sc, stream_nt);
  else if (geo.d == 128 && G == 1) launch_decode<128, 1>(s, q, out, seqs, items, n_items, multi, n_multi, block_tables, pool, geo, n_q, chunk_pages, max_chunks, ws, sc, stream_nt);
  else if (geo.d == 64 && G == 1) launch_decode<64, 1>(s, q, out, seqs, items, n_items, multi, n_multi, block_tables, pool, geo, n_q, chunk_pages, max_chunks, ws, sc, stream_nt);
  else if (geo.d == 64 && G == 4) launch_decode<64, 4>(s, q, out, seqs, items, n_items, multi, n_multi, block_tables, pool, geo, n_q, chunk_pages, max_chunks, ws, sc, stream_nt);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace sts
