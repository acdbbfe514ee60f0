// Causal flash-style attention for prefill chunks on gfx950, reading K and V from the paged
// cache (the chunk's own K,V are written there first, so a chunk appended after p cached
// tokens needs no separate path).
//
// A workgroup of 4 waves owns 128 consecutive query rows of one head of one sequence; each
// wave owns 32 of them. Per 64-key tile staged through LDS:
//   S^T[key, q] = K[key, :] . Q[q, :]          v_mfma_f32_32x32x16_bf16, A = K rows, B = Q rows
//   online softmax down the key axis: a lane holds one query column (16 keys per 32x32
//   block per lane half), so the running max/sum need one cross-half shuffle only
//   O^T[dd, q] += V^T[dd, key] . P^T[key, q]   A = V^T rows (token-contiguous in a page),
//   B = P^T taken straight from the S^T accumulator registers (no LDS round trip).
// The k index inside one MFMA is a free permutation as long as A and B agree: for P^T the
// eight values a lane already holds (registers 8j..8j+7 of a block) are keys
// {16j + 4*half + 0..3} and {16j + 8 + 4*half + 0..3}; the V^T operand is read from LDS in
// that same order (two 8-byte reads).
#include "kernels.h"

namespace sts {

constexpr int BQ = 128, BKV = 64;

template <int D>
__global__ void __launch_bounds__(256) attn_prefill_kernel(const bf16* __restrict__ qkv, int ld, bf16* __restrict__ out, int ldo,
                                                           const PrefillSeq* __restrict__ seqs, const AttnItem* __restrict__ items,
                                                           const int* __restrict__ block_tables, const bf16* __restrict__ pool,
                                                           KvGeom geo, int n_q, float scale_log2e) {
  constexpr int KS = D + 8;       // K tile row stride (elements): 16-byte reads, conflict free
  constexpr int VS = BKV + 4;     // V^T tile row stride: 8-byte reads, conflict free
  constexpr int KSTEPS = D / 16, DB = D / 32;
  __shared__ __align__(16) bf16 Ks[BKV * KS];
  __shared__ __align__(16) bf16 Vs[D * VS];

  const int head = blockIdx.x % n_q;
  const AttnItem it = items[blockIdx.x / n_q];
  const PrefillSeq sq = seqs[it.seq];
  const int kvh = head / (n_q / geo.n_kv);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, lh = lane >> 5;
  const int* bt = block_tables + sq.bt_off;
  const size_t head_elems = geo.head_elems();

  const int qloc = it.q0 + wave * 32 + l32;              // row inside the chunk
  const bool q_valid = qloc < sq.sl;
  const int qpos = sq.p + qloc;                          // absolute position (causal limit)
  const bf16* qp = qkv + (size_t)(sq.row0 + min(qloc, sq.sl - 1)) * ld + head * D + 8 * lh;
  bf16x8 qf[KSTEPS];
#pragma unroll
  for (int j = 0; j < KSTEPS; j++) qf[j] = *reinterpret_cast<const bf16x8*>(qp + 16 * j);

  const int wave_min_qpos = sq.p + it.q0 + wave * 32;
  const int wave_max_qpos = wave_min_qpos + 31;
  const int k_end = sq.p + min(it.q0 + BQ, sq.sl);       // keys [0, k_end) are needed by this workgroup
  const int n_tiles = (k_end + BKV - 1) / BKV;

  f32x16 o[DB];
#pragma unroll
  for (int b = 0; b < DB; b++)
#pragma unroll
    for (int r = 0; r < 16; r++) o[b][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  for (int kt = 0; kt < n_tiles; kt++) {
    __syncthreads();                                      // everyone is done with the previous tile
    // ---- stage K tile [64 keys][D] and V^T tile [D][64 keys]
    constexpr int KCH = BKV * D / 8;                      // 16-byte chunks in the K tile
#pragma unroll
    for (int c = tid; c < KCH; c += 256) {
      const int key = c / (D / 8), cc = c % (D / 8);
      const int kpos = kt * BKV + key, pg = kpos / 16;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (pg < sq.n_pages)
        v = *reinterpret_cast<const uint4*>(pool + ((size_t)bt[pg] * geo.n_kv + kvh) * head_elems + (size_t)(kpos % 16) * D + cc * 8);
      *reinterpret_cast<uint4*>(Ks + key * KS + cc * 8) = v;
    }
    constexpr int VCH = D * BKV / 8;
#pragma unroll
    for (int c = tid; c < VCH; c += 256) {
      const int pgl = c / (D * 2), rem = c % (D * 2), dd = rem >> 1, hf = rem & 1;
      const int pg = kt * (BKV / 16) + pgl;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (pg < sq.n_pages)
        v = *reinterpret_cast<const uint4*>(pool + ((size_t)bt[pg] * geo.n_kv + kvh) * head_elems + (size_t)16 * D + dd * 16 + hf * 8);
      uint2* dst = reinterpret_cast<uint2*>(Vs + dd * VS + pgl * 16 + hf * 8);
      dst[0] = make_uint2(v.x, v.y);
      dst[1] = make_uint2(v.z, v.w);
    }
    __syncthreads();
    if (kt * BKV > wave_max_qpos) continue;               // wave-uniform: every key of the tile is masked

    // ---- S^T = K Q^T  (two 32-key blocks)
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; kb++) {
#pragma unroll
      for (int r = 0; r < 16; r++) s[kb][r] = 0.f;
#pragma unroll
      for (int j = 0; j < KSTEPS; j++) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(Ks + (kb * 32 + l32) * KS + j * 16 + 8 * lh);
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[j], s[kb], 0, 0, 0);
      }
    }
    // ---- scale, causal mask, online softmax
    const bool need_mask = kt * BKV + BKV - 1 > wave_min_qpos;
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        float v = s[kb][r] * scale_log2e;
        if (need_mask) {
          const int key = kt * BKV + kb * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
          if (key > qpos) v = -INFINITY;
        }
        s[kb][r] = v;
        mx = fmaxf(mx, v);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float corr = __builtin_amdgcn_exp2f(m_run - m_use);
    float rs = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const float p = __builtin_amdgcn_exp2f(s[kb][r] - m_use);
        s[kb][r] = p;
        rs += p;
      }
    rs += __shfl_xor(rs, 32, 64);
    l_run = l_run * corr + rs;
    m_run = m_new;
#pragma unroll
    for (int b = 0; b < DB; b++)
#pragma unroll
      for (int r = 0; r < 16; r++) o[b][r] *= corr;

    // ---- O^T += V^T P^T
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int j2 = 0; j2 < 2; j2++) {
        bf16x8 pb;
#pragma unroll
        for (int e = 0; e < 8; e++) pb[e] = f2bf(s[kb][8 * j2 + e]);
#pragma unroll
        for (int b = 0; b < DB; b++) {
          const bf16* vrow = Vs + (b * 32 + l32) * VS + kb * 32 + 16 * j2 + 4 * lh;
          const bf16x4 v0 = *reinterpret_cast<const bf16x4*>(vrow);
          const bf16x4 v1 = *reinterpret_cast<const bf16x4*>(vrow + 8);
          bf16x8 a;
#pragma unroll
          for (int e = 0; e < 4; e++) { a[e] = v0[e]; a[e + 4] = v1[e]; }
          o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, o[b], 0, 0, 0);
        }
      }
  }

  if (!q_valid) return;
  const float inv_l = 1.f / l_run;
  bf16* orow = out + (size_t)(sq.row0 + qloc) * ldo + head * D + 4 * lh;
#pragma unroll
  for (int b = 0; b < DB; b++)
#pragma unroll
    for (int r4 = 0; r4 < 4; r4++) {
      bf16x4 v;
#pragma unroll
      for (int e = 0; e < 4; e++) v[e] = f2bf(o[b][4 * r4 + e] * inv_l);
      *reinterpret_cast<bf16x4*>(orow + b * 32 + 8 * r4) = v;
    }
}

int attn_prefill_tile_q() { return BQ; }

// qkv: packed [rows, ld] with Q of head h at columns [h*d, (h+1)*d), already rotated.
// out: [rows, ldo], head h at the same columns. items: query tiles (sequence, first row);
// one workgroup per (item, head). Requires page_tokens == 16 and d in {64, 128}.
hipError_t attn_prefill(hipStream_t s, const bf16* qkv, int ld, bf16* out, int ldo, const PrefillSeq* seqs,
                        const AttnItem* items, int n_items, const int* block_tables, const bf16* pool,
                        KvGeom geo, int n_q) {
  if (n_items == 0) return hipSuccess;
  if (geo.page_tokens != 16 || n_q % geo.n_kv != 0) return hipErrorInvalidValue;
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)geo.d);
  dim3 grid((unsigned)n_items * n_q), block(256);
  if (geo.d == 128)
    hipLaunchKernelGGL(attn_prefill_kernel<128>, grid, block, 0, s, qkv, ld, out, ldo, seqs, items, block_tables, pool, geo, n_q, scale_log2e);
  else if (geo.d == 64)
    hipLaunchKernelGGL(attn_prefill_kernel<64>, grid, block, 0, s, qkv, ld, out, ldo, seqs, items, block_tables, pool, geo, n_q, scale_log2e);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace sts
