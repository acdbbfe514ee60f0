// Causal flash-style attention for prefill chunks on gfx950, reading K and V from the paged
// cache (the chunk's own K,V are written there first, so a chunk appended after p cached
// tokens needs no separate path).
//
// A workgroup of 4 waves owns 128 consecutive query rows of one head of one sequence; each
// wave owns 32 of them. A window of the block table and the Q tile sit in LDS; the
// next 64-key K/V tile is fetched into registers while the current one is consumed, then
// written to the (single) LDS tile buffers between two barriers. Per 64-key tile:
//   S^T[key, q] = K[key, :] . Q[q, :]          v_mfma_f32_32x32x16_bf16, A = K rows, B = Q rows
//   online softmax down the key axis: a lane holds one query column (16 keys per 32x32
//   block per lane half), so the running max/sum need one cross-half shuffle only
//   O^T[dd, q] += V^T[dd, key] . P^T[key, q]   A = V^T rows (token-contiguous in a page),
//   B = P^T taken straight from the S^T accumulator registers (no LDS round trip).
// The k index inside one MFMA is a free permutation as long as A and B agree: for P^T the
// eight values a lane already holds (registers 8j..8j+7 of a block) are keys
// {16j + 4*half + 0..3} and {16j + 8 + 4*half + 0..3}; the V^T tile is laid out in LDS in
// that same order, so the operand is one 16-byte read.
#include "kernels.h"

namespace sts {

constexpr int BQ = 128, BKV = 64;

constexpr float RESCALE_LOG2 = 8.f;
constexpr int BT_CACHE = 1024;   // block-table window kept in LDS (16384 tokens), refilled as the key loop crosses it

// max over a lane and its partner 32 lanes away (v_permlane32_swap: the upper half of the first
// operand trades places with the lower half of the second)
__device__ __forceinline__ float half_swap_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

template <int D>
__global__ void __launch_bounds__(256, 2) attn_prefill_kernel(const bf16* __restrict__ qkv, int ld, bf16* __restrict__ out, int ldo,
                                                           const PrefillSeq* __restrict__ seqs, const AttnItem* __restrict__ items,
                                                           const int* __restrict__ block_tables, const bf16* __restrict__ pool,
                                                           KvGeom geo, int n_q, float scale_log2e) {
  constexpr int KS = D + 8;       // K and Q tile row stride (elements): 16-byte reads, conflict free
  constexpr int VS = BKV + 8;     // V^T tile row stride; inside each 16-key group the keys are stored in the
                                  // order 0-3, 8-11, 4-7, 12-15 so that a lane's MFMA operand is one 16-byte read
  constexpr int KSTEPS = D / 16, DB = D / 32;
  constexpr int KCH = BKV * D / 8 / 256;                  // 16-byte chunks of the K tile per thread
  constexpr int VCH = D * BKV / 8 / 256;                  // ... of the V^T tile
  __shared__ __align__(16) bf16 Qs[BQ * KS];
  __shared__ __align__(16) bf16 Ks[BKV * KS];
  __shared__ __align__(16) bf16 Vs[D * VS];
  __shared__ int bts[BT_CACHE];

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
  const int wave_min_qpos = sq.p + it.q0 + wave * 32;
  const int wave_max_qpos = wave_min_qpos + 31;
  const int k_end = sq.p + min(it.q0 + BQ, sq.sl);       // keys [0, k_end) are needed by this workgroup
  const int n_tiles = (k_end + BKV - 1) / BKV;
  const int pages_needed = min(sq.n_pages, (k_end + 15) / 16);

  // ---- stage a window of the block table and the Q tile (rows past the chunk repeat its last row).
  // Window entries past the last needed page repeat that page: the K/V loads are then
  // unconditional, and what they fetch for positions beyond the context is causally masked
  // (the pool only ever holds finite values, so 0 * V stays 0).
  auto fill_bt_window = [&](int first) {
    const int n = min(BT_CACHE, (pages_needed - first + 3) & ~3);
    for (int i = tid; i < n; i += 256) bts[i] = bt[min(first + i, pages_needed - 1)];
  };
  fill_bt_window(0);
  for (int c = tid; c < BQ * (D / 8); c += 256) {
    const int row = c / (D / 8), cc = c % (D / 8);
    const bf16* src = qkv + (size_t)(sq.row0 + min(it.q0 + row, sq.sl - 1)) * ld + head * D + cc * 8;
    *reinterpret_cast<u32x4*>(Qs + row * KS + cc * 8) = *reinterpret_cast<const u32x4*>(src);
  }
  __syncthreads();

  // global -> register staging of one K/V tile. A tile spans 4 pages; chunk j of a thread lies in
  // page slot j * (4 / KCH) + a per-thread constant, at a per-thread constant offset inside the page.
  const size_t page_stride = (size_t)geo.n_kv * head_elems;
  const bf16* pool_h = pool + (size_t)kvh * head_elems;
  const int kslot0 = (tid / (D / 8)) >> 4, vslot0 = tid / (2 * D);
  const int koff = ((tid / (D / 8)) & 15) * D + (tid % (D / 8)) * 8;
  const int voff = 16 * D + ((tid % (2 * D)) >> 1) * 16 + (tid & 1) * 8;
  u32x4 kreg[KCH], vreg[VCH];
  auto load_tile = [&](int kt) {
    const i32x4 pg = *reinterpret_cast<const i32x4*>(bts + (kt * 4) % BT_CACHE);
#pragma unroll
    for (int j = 0; j < KCH; j++) {
      int page;
      if constexpr (D == 128) page = pg[j];
      else page = kslot0 ? pg[2 * j + 1] : pg[2 * j];
      kreg[j] = *reinterpret_cast<const u32x4*>(pool_h + (size_t)page * page_stride + koff);
    }
#pragma unroll
    for (int j = 0; j < VCH; j++) {
      int page;
      if constexpr (D == 128) page = pg[j];
      else page = vslot0 ? pg[2 * j + 1] : pg[2 * j];
      vreg[j] = *reinterpret_cast<const u32x4*>(pool_h + (size_t)page * page_stride + voff);
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int j = 0; j < KCH; j++) {
      const int c = tid + j * 256, key = c / (D / 8), cc = c % (D / 8);
      *reinterpret_cast<u32x4*>(Ks + key * KS + cc * 8) = kreg[j];
    }
#pragma unroll
    for (int j = 0; j < VCH; j++) {
      const int c = tid + j * 256, pgl = c / (D * 2), rem = c % (D * 2), dd = rem >> 1, hf = rem & 1;
      bf16* dst = Vs + dd * VS + pgl * 16 + hf * 4;       // keys 8hf..8hf+3 -> slot 4hf, keys 8hf+4..8hf+7 -> slot 8+4hf
      *reinterpret_cast<u32x2*>(dst) = u32x2{vreg[j][0], vreg[j][1]};
      *reinterpret_cast<u32x2*>(dst + 8) = u32x2{vreg[j][2], vreg[j][3]};
    }
  };

  f32x16 o[DB];
#pragma unroll
  for (int b = 0; b < DB; b++)
#pragma unroll
    for (int r = 0; r < 16; r++) o[b][r] = 0.f;
  float m_ref = -INFINITY, l_run = 0.f;

  load_tile(0);
  store_tile();
  __syncthreads();

  const bf16* qrow = Qs + (wave * 32 + l32) * KS + 8 * lh;
  for (int kt = 0; kt < n_tiles; kt++) {
    const bool more = kt + 1 < n_tiles;                   // uniform
    if (more) {
      if (((kt + 1) * 4) % BT_CACHE == 0) {               // uniform: slide the block-table window
        __syncthreads();
        fill_bt_window((kt + 1) * 4);
        __syncthreads();
      }
      load_tile(kt + 1);                                  // in flight while this tile is consumed
    }

    if (kt * BKV <= wave_max_qpos) {                      // wave-uniform: otherwise every key of the tile is masked
      // ---- S^T = K Q^T  (two 32-key blocks); operand fragments of step j+1 are read from LDS
      // while the MFMAs of step j run
      f32x16 s[2];
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int r = 0; r < 16; r++) s[kb][r] = 0.f;
      __builtin_amdgcn_sched_barrier(0);
      {
        bf16x8 qf[2], kf[2][2];
        const bf16* krow = Ks + l32 * KS + 8 * lh;
        qf[0] = *reinterpret_cast<const bf16x8*>(qrow);
        kf[0][0] = *reinterpret_cast<const bf16x8*>(krow);
        kf[0][1] = *reinterpret_cast<const bf16x8*>(krow + 32 * KS);
#pragma unroll
        for (int j = 0; j < KSTEPS; j++) {
          const int c = j & 1, n = c ^ 1;
          if (j + 1 < KSTEPS) {
            qf[n] = *reinterpret_cast<const bf16x8*>(qrow + 16 * (j + 1));
            kf[n][0] = *reinterpret_cast<const bf16x8*>(krow + 16 * (j + 1));
            kf[n][1] = *reinterpret_cast<const bf16x8*>(krow + 32 * KS + 16 * (j + 1));
          }
          s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[c][0], qf[c], s[0], 0, 0, 0);
          s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[c][1], qf[c], s[1], 0, 0, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
#pragma unroll
        for (int j = 0; j + 1 < KSTEPS; j++) {
          __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      // first V^T operands: in flight during the softmax arithmetic
      bf16x8 vf[2][DB];
      const bf16* vrow = Vs + l32 * VS + 8 * lh;
#pragma unroll
      for (int b = 0; b < DB; b++) vf[0][b] = *reinterpret_cast<const bf16x8*>(vrow + b * 32 * VS);
      __builtin_amdgcn_sched_barrier(0);
      // ---- causal mask and online softmax on the raw scores; the scale rides in the exponent's
      // fused multiply-add. The reference maximum m_ref is only moved when the tile maximum
      // exceeds it by more than 2^RESCALE_LOG2 (probabilities then stay below that factor, far
      // inside fp32/bf16 range), so the rescale of O and l is skipped on most tiles.
      if (kt * BKV + BKV - 1 > wave_min_qpos) {
#pragma unroll
        for (int kb = 0; kb < 2; kb++)
#pragma unroll
          for (int r = 0; r < 16; r++) {
            const int key = kt * BKV + kb * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
            if (key > qpos) s[kb][r] = -INFINITY;
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int r = 0; r < 16; r++) mx = fmaxf(mx, s[kb][r]);
      mx = half_swap_max(mx);
      const bool grow = (mx - m_ref) * scale_log2e > RESCALE_LOG2;     // false when both are -inf (NaN)
      if (__any(grow)) {                                               // wave-uniform
        const float m_upd = grow ? mx : m_ref;
        const float corr = (m_upd == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f((m_ref - m_upd) * scale_log2e);
        m_ref = m_upd;
        l_run *= corr;
#pragma unroll
        for (int b = 0; b < DB; b++)
#pragma unroll
          for (int r = 0; r < 16; r++) o[b][r] *= corr;
      }
      const float nm = (m_ref == -INFINITY) ? 0.f : -m_ref * scale_log2e;
      float rs = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[kb][r], scale_log2e, nm));
          s[kb][r] = p;
          rs += p;
        }
      l_run += rs;                                                      // this half's keys; halves are added at the end

      // ---- O^T += V^T P^T, four groups of 16 keys; the next group's V^T operands are read
      // while the current group's MFMAs run
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < 4; g++) {
        const int c = g & 1, n = c ^ 1;
        if (g + 1 < 4) {
#pragma unroll
          for (int b = 0; b < DB; b++) vf[n][b] = *reinterpret_cast<const bf16x8*>(vrow + b * 32 * VS + 16 * (g + 1));
        }
        bf16x8 pb;
#pragma unroll
        for (int e = 0; e < 8; e++) pb[e] = f2bf(s[g >> 1][8 * (g & 1) + e]);
#pragma unroll
        for (int b = 0; b < DB; b++) o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[c][b], pb, o[b], 0, 0, 0);
      }
#pragma unroll
      for (int g = 0; g + 1 < 4; g++) {
        __builtin_amdgcn_sched_group_barrier(0x100, DB, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, DB, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, DB, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();                                      // everyone is done reading this tile
    if (more) store_tile();
    __syncthreads();
  }

  if (!q_valid) return;
  l_run += __shfl_xor(l_run, 32, 64);
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
