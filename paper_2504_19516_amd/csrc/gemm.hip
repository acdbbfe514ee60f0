// bf16 MFMA GEMM for gfx950:  C[M,N] (+)= A[M,K] * W[N,K]^T, fp32 accumulation.
//
// Both operands are K-contiguous, which is the layout v_mfma_f32_32x32x16_bf16 wants: a lane
// holds 8 consecutive k of one A row (or one W row). A workgroup owns a BM x BN tile and each of
// its waves accumulates a (BM/WGM) x (BN/WGN) sub-tile in 32x32 MFMA blocks.
//
// Three main loops. gemm_dl_kernel: K tiles of 64 of both operands go global -> LDS directly (no
// staging registers, no LDS store instructions): activations into 128-byte rows whose 16-byte chunks
// are XOR-swizzled so that the 16-byte operand reads are bank-conflict free, packed weights as the
// operand-order blocks they are in memory; two or three LDS stages;
// operand reads of the next 16-wide step are slotted between the MFMAs of the current one. It runs
// the 128x128 tiles with 4 waves (two workgroups per CU) for prefill, the 64x128 (4 waves, two per
// CU) and 64x256 (8 waves) tiles with split-K for decode batches, and row-major W of callers that
// bring their own weights. gemm_wreg_kernel: the 256x256 (8 waves) and 128x256 (4 waves) prefill tiles;
// only the activation tile goes through LDS, the W operands go from the packed weight layout straight
// into registers. gemm_skinny_kernel: the same for decode batches of up to 64 rows -- tiles of 256 to 512
// columns, the W operands three K tiles deep in registers.
// Epilogues: bf16 store, fp32 store (split-K partial sums), fp32 residual add, SwiGLU on interleaved
// gate/up rows.
//
// Wave quantisation (paper Section 2.2.1) is met in the launch: the tiles of a partly filled last
// wave of workgroups are cut along K into pieces that fill the partition (gemm_tail_plan), the
// pieces leave fp32 partial tiles, and gemm_tail_fixup sums them in a fixed order and applies the
// epilogue.
//
// Lane layout of the 32x32 accumulator block (register r of lane l):
//   row = 8*(r/4) + 4*(l/32) + r%4,  col = l%32.
#include <atomic>
#include <type_traits>

#include "kernels.h"

namespace sts {

constexpr int GEMM_DL_LDS_BASE = 1024;   // the direct-to-LDS arena stays clear of LDS address 0
#ifndef GEMM_SKINNY_PD
#define GEMM_SKINNY_PD 3                 // K tiles of W operands a wave of gemm_skinny_kernel keeps in flight
#endif

struct GemmArgs {
  const bf16* A; const bf16* W; void* C;
  int lda, ldw, ldc;
  int M, N, K;
  int w_packed;               // W in the packed block layout (weight_packed_index) instead of row-major
  int stream_nt;              // skinny tiles: fetch W with the non-temporal hint
  int tiles_m, tiles_n, group_m;
  int k_per_split;            // K range handled by one blockIdx.y
  long long split_stride;     // elements between consecutive split-K partial outputs
  // Tail splitting. Tiles [0, n_full) are computed whole. The remaining tiles -- the last,
  // partly filled wave of workgroups on the partition -- are cut along K into tail_f pieces each,
  // so that wave takes 1/tail_f of a tile time; pieces leave fp32 partial tiles in tail_ws and a
  // second small kernel adds them up in a fixed order and applies the epilogue.
  int n_full, full_per_xcd, tail_f, n_pieces, piece_per_xcd;
  float* tail_ws;
};

// tile index -> tile coordinates: tiles are walked in groups of group_m tile rows so that
// workgroups resident together share operand rows in L2
__device__ __forceinline__ void tile_coords(const GemmArgs& g, int v, int* tm, int* tn) {
  const int gsz = g.group_m * g.tiles_n;
  const int first_m = (v / gsz) * g.group_m;
  const int gm = min(g.tiles_m - first_m, g.group_m);
  *tm = first_m + (v % gsz) % gm;
  *tn = (v % gsz) / gm;
}

// Workgroups are dealt round-robin to the 8 XCDs, in order: each XCD first gets a contiguous
// run of whole tiles (neighbours share operands in its L2), then its share of the tail pieces.
// Returns false for a padding workgroup. piece < 0 for a whole tile.
template <int BK>
__device__ __forceinline__ bool block_work(const GemmArgs& g, int* v, int* kbeg, int* kend, int* piece) {
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  *piece = -1;
  if (local < g.full_per_xcd) {
    *v = xcd * g.full_per_xcd + local;
    if (*v >= g.n_full) return false;
    *kbeg = blockIdx.y * g.k_per_split;
    *kend = min(g.K, *kbeg + g.k_per_split);
  } else {
    *piece = xcd * g.piece_per_xcd + (local - g.full_per_xcd);
    if (*piece >= g.n_pieces) return false;
    *v = g.n_full + *piece / g.tail_f;
    const int z = *piece % g.tail_f, ksteps = g.K / BK;
    *kbeg = (int)((long long)ksteps * z / g.tail_f) * BK;
    *kend = (int)((long long)ksteps * (z + 1) / g.tail_f) * BK;
  }
  return true;
}

// Epilogue of one workgroup tile (or the partial-tile store of a tail piece).
template <int BM, int BN, int WGM, int WGN, int EPI>
__device__ __forceinline__ void store_tile(const GemmArgs& g, f32x16 (&acc)[BM / WGM / 32][BN / WGN / 32], int m0, int n0, int piece,
                                           int wm, int wn, int l32, int lh) {
  constexpr int WTM = BM / WGM, WTN = BN / WGN, TM = WTM / 32, TN = WTN / 32;
  // a tail piece stores its partial tile, row-major [BM][BN]
  if (piece >= 0) {
    float* part = g.tail_ws + (size_t)piece * (BM * BN) + (size_t)(wm * WTM + 4 * lh) * BN + wn * WTN + l32;
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int r = 0; r < 16; r++)
#pragma unroll
        for (int j = 0; j < TN; j++) part[(size_t)(i * 32 + 8 * (r >> 2) + (r & 3)) * BN + j * 32] = acc[i][j][r];
    return;
  }

  // ---- epilogue
  const int rbase = m0 + wm * WTM + 4 * lh;
  const int cbase = n0 + wn * WTN + l32;
#pragma unroll
  for (int i = 0; i < TM; i++) {
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int row = rbase + i * 32 + 8 * (r >> 2) + (r & 3);
      if (row >= g.M) continue;
      if constexpr (EPI == EPI_SWIGLU_BF16) {
        bf16* out = reinterpret_cast<bf16*>(g.C) + (size_t)row * g.ldc + ((n0 + wn * WTN) >> 1) + l32;
#pragma unroll
        for (int j = 0; j < TN; j += 2) {
          const float gate = acc[i][j][r], up = acc[i][j + 1][r];
          out[(j >> 1) * 32] = f2bf(gate / (1.f + __expf(-gate)) * up);
        }
      } else {
#pragma unroll
        for (int j = 0; j < TN; j++) {
          const size_t idx = (size_t)row * g.ldc + cbase + j * 32;
          if constexpr (EPI == EPI_BF16) reinterpret_cast<bf16*>(g.C)[idx] = f2bf(acc[i][j][r]);
          else if constexpr (EPI == EPI_F32)
            reinterpret_cast<float*>(g.C)[(size_t)blockIdx.y * g.split_stride + idx] = acc[i][j][r];
          else reinterpret_cast<float*>(g.C)[idx] += acc[i][j][r];
        }
      }
    }
  }
}

// ---- direct-to-LDS main loop ---------------------------------------------------------------
// Tiles go global -> LDS without passing through registers (no staging VGPRs, no LDS store
// instructions). A tile row is 128 bytes (BK = 64) and unpadded; the 16-byte K-chunk c of row r
// is stored at slot c ^ ((r >> 1) & 7), which keeps the 16-byte operand reads bank-conflict
// free. One wave instruction fills 64 consecutive slots (8 rows), so the swizzle is applied on
// the global side: each lane fetches the chunk that belongs in its slot.
//
// Schedule of one K tile (four 16-wide steps): steps 0-2 run from the current LDS buffer; then
// the wave waits for its own loads of the next tile and meets the others at the barrier, which
// both publishes the next tile and retires the current buffer (the operands of step 3 are
// already in registers); the loads of the tile after next go out right behind the barrier, a
// whole iteration ahead of their use; step 3 runs while the first operands of the next tile
// are read. The LDS arena starts 1 KB above address 0.
template <int BM, int BN, int WGM, int WGN, int EPI, int NS, bool WPACK = true>
__global__ void __launch_bounds__(WGM* WGN * 64) gemm_dl_kernel(GemmArgs g) {
  constexpr int BK = 64, NT = WGM * WGN * 64;
  static_assert(NS >= 2 && (NS - 2) * (BM + BN) * 8 / NT < 64, "stages: at least two, outstanding loads within vmcnt's range");
  constexpr int WTM = BM / WGM, WTN = BN / WGN, TM = WTM / 32, TN = WTN / 32;
  constexpr int ROWB = BK * 2;                               // bytes per tile row
  constexpr int A_CH = BM * 8 / NT, B_CH = BN * 8 / NT;      // 16-byte chunks per thread
  constexpr int STAGE = (BM + BN) * ROWB;
  static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/thread mismatch");
  static_assert(EPI != EPI_SWIGLU_BF16 || TN % 2 == 0, "swiglu needs gate/up block pairs");
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* arena = smem + GEMM_DL_LDS_BASE;

  int v, kbeg, kend, piece;
  if (!block_work<BK>(g, &v, &kbeg, &kend, &piece)) return;
  int tm, tn;
  tile_coords(g, v, &tm, &tn);
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  const int wm = wave / WGN, wn = wave % WGN;

  // slot q = j * NT + tid of a tile: row q / 8, holds K-chunk (q % 8) ^ ((row >> 1) & 7). A lane keeps
  // the 32-bit byte offset of its chunk from the tile's first row; the tile bases are wave-uniform
  // and advance along K in scalar registers, and so do the LDS destinations (the wave index is read
  // into a scalar once): queuing a load takes no vector ALU work and sends 4 address bytes per lane.
  const int swave = __builtin_amdgcn_readfirstlane(wave);
  const unsigned char* a_base = reinterpret_cast<const unsigned char*>(g.A + (size_t)m0 * g.lda);
  // W: row-major (its tile is laid out in LDS like the A tile), or (WPACK) 32 x 64 blocks of 4 KiB in matrix-core operand
  // order (weight_packed_index), copied to LDS as they are.
  const unsigned char* b_base = WPACK ? reinterpret_cast<const unsigned char*>(g.W) + (size_t)(n0 >> 5) * (g.K >> 6) * 4096
                                      : reinterpret_cast<const unsigned char*>(g.W + (size_t)n0 * g.ldw);
  unsigned a_off[A_CH], b_off[B_CH];
#pragma unroll
  for (int j = 0; j < A_CH; j++) {
    const int q = j * NT + tid, row = q >> 3, ch = (q & 7) ^ ((row >> 1) & 7);
    a_off[j] = (unsigned)(min(m0 + row, g.M - 1) - m0) * (unsigned)g.lda * 2u + ch * 16;
  }
#pragma unroll
  for (int j = 0; j < B_CH; j++) {
    const int q = j * NT + tid, row = q >> 3, ch = (q & 7) ^ ((row >> 1) & 7);
    // packed: slot q is the q-th 16-byte piece of the tile's 4 KiB blocks for this K step, so a wave's load reads 1 KiB of
    // consecutive memory
    b_off[j] = WPACK ? (unsigned)(q >> 8) * (unsigned)(g.K >> 6) * 4096u + (unsigned)(q & 255) * 16u
                     : (unsigned)row * (unsigned)g.ldw * 2u + ch * 16;
  }
  auto issue_a = [&](int stage, int k) {
    unsigned char* sa = arena + stage * STAGE + swave * 1024;
    const unsigned char* ak = a_base + (size_t)k * 2;
#pragma unroll
    for (int j = 0; j < A_CH; j++) lds_dma16(ak, a_off[j], sa + j * NT * 16);
  };
  auto issue_b = [&](int stage, int k) {
    unsigned char* sb = arena + stage * STAGE + swave * 1024 + BM * ROWB;
    const unsigned char* bk = b_base + (WPACK ? (size_t)(k >> 6) * 4096 : (size_t)k * 2);
#pragma unroll
    for (int j = 0; j < B_CH; j++) lds_dma16(bk, b_off[j], sb + j * NT * 16);
  };
  auto issue = [&](int stage, int k) { issue_a(stage, k); issue_b(stage, k); };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

  // byte offset of this lane's operand chunk inside its row, for each of the four K steps
  // and of its W operand: the same for a row-major W tile; a packed W tile is in LDS what it is in memory, 1 KiB per
  // 32-row block and step with lane l's operand at byte 16 l
  int koff[4], kboff[4];
#pragma unroll
  for (int kk = 0; kk < 4; kk++) {
    koff[kk] = ((kk * 2 + lh) ^ ((l32 >> 1) & 7)) * 16;
    kboff[kk] = WPACK ? kk * 1024 : koff[kk];
  }
  const int a_row = (wm * WTM + l32) * ROWB;
  const int b_row = BM * ROWB + (WPACK ? wn * WTN * ROWB + lane * 16 : (wn * WTN + l32) * ROWB);

  constexpr int MPR = (TM * TN) / (TM + TN) > 0 ? (TM * TN) / (TM + TN) : 1;       // MFMAs per LDS read
  constexpr int REST = TM * TN > MPR * (TM + TN) ? TM * TN - MPR * (TM + TN) : 0;

  // NS LDS stages: tile t lives in stage t % NS; while tile t is consumed, tiles t+1 .. t+NS-1
  // are landing or on their way.
  constexpr int LOADS = A_CH + B_CH;                         // loads per thread and tile
  const int nk = (kend - kbeg) / BK;
#pragma unroll
  for (int t = 0; t < NS; t++)
    if (t < nk) issue(t, kbeg + t * BK);
  if (nk >= NS) wait_vmem<(NS - 1) * LOADS>(); else wait_vmem<0>();
  __syncthreads();
  bf16x8 af[2][TM], bfr[2][TN];
#pragma unroll
  for (int i = 0; i < TM; i++) af[0][i] = *reinterpret_cast<const bf16x8*>(arena + a_row + i * 32 * ROWB + koff[0]);
#pragma unroll
  for (int j = 0; j < TN; j++) bfr[0][j] = *reinterpret_cast<const bf16x8*>(arena + b_row + j * 32 * ROWB + kboff[0]);

  int cur = 0;                                               // stage of tile t
  for (int t = 0; t < nk; t++) {
    const int nxt = cur + 1 == NS ? 0 : cur + 1;
    const unsigned char* Ac = arena + cur * STAGE + a_row;
    const unsigned char* Bc = arena + cur * STAGE + b_row;
    const unsigned char* An = arena + nxt * STAGE + a_row;
    const unsigned char* Bn = arena + nxt * STAGE + b_row;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < 3; kk++) {
#pragma unroll
      for (int i = 0; i < TM; i++) af[(kk + 1) & 1][i] = *reinterpret_cast<const bf16x8*>(Ac + i * 32 * ROWB + koff[kk + 1]);
#pragma unroll
      for (int j = 0; j < TN; j++) bfr[(kk + 1) & 1][j] = *reinterpret_cast<const bf16x8*>(Bc + j * 32 * ROWB + kboff[kk + 1]);
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j], acc[i][j], 0, 0, 0);
    }
#pragma unroll
    for (int kk = 0; kk < 3; kk++) {
#pragma unroll
      for (int x = 0; x < TM + TN; x++) {
        __builtin_amdgcn_sched_group_barrier(0x008, MPR, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      if (REST > 0) __builtin_amdgcn_sched_group_barrier(0x008, REST, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    // tile t+1 must have landed; the NS-2 tiles issued after it may still be in flight
    if (t + NS - 1 < nk) wait_vmem<(NS - 2) * LOADS>(); else wait_vmem<0>();
    __syncthreads();
    // the tile after the ones in flight goes into the stage just retired
    if (t + NS < nk) issue(cur, kbeg + (t + NS) * BK);
    __builtin_amdgcn_sched_barrier(0);
    if (t + 1 < nk) {
#pragma unroll
      for (int i = 0; i < TM; i++) af[0][i] = *reinterpret_cast<const bf16x8*>(An + i * 32 * ROWB + koff[0]);
#pragma unroll
      for (int j = 0; j < TN; j++) bfr[0][j] = *reinterpret_cast<const bf16x8*>(Bn + j * 32 * ROWB + kboff[0]);
    }
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[1][i], bfr[1][j], acc[i][j], 0, 0, 0);
#pragma unroll
    for (int x = 0; x < TM + TN; x++) {
      __builtin_amdgcn_sched_group_barrier(0x008, MPR, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    if (REST > 0) __builtin_amdgcn_sched_group_barrier(0x008, REST, 0);
    __builtin_amdgcn_sched_barrier(0);
    cur = nxt;
  }
  store_tile<BM, BN, WGM, WGN, EPI>(g, acc, m0, n0, piece, wm, wn, l32, lh);
}

// ---- main loop of the 256-column prefill tiles: W operands straight from global memory -----------
// (WGM = 2: 256 x 256, eight waves; WGM = 1: 128 x 256, four waves with the same 128 x 64 wave tiles, where no W
// block is shared by two waves and the activation stages are 16 KB)
// With both operands staged through LDS the 256 x 256 tile moves 256 KB through LDS per 64-wide K tile
// (64 KB written by the tile loads, 192 KB read as operands by the 8 waves), which at 128 bytes per cycle
// is as long as the tile's matrix-core work: the loop ran at the LDS's pace, not the MFMAs'. Here only the
// activation tile goes through LDS (three stages of 32 KB, loaded as above). Each wave reads its W
// operands -- 64 columns, so two 32-row blocks of the packed layout -- directly into registers, one
// 16-byte load per lane and 16-wide step from 1 KiB of consecutive memory. One register set serves: the
// operands of step kk of the next K tile are requested right after step kk of this one has used them, a
// whole iteration before they are needed. The two waves of a 256 x 256 tile that share a column block load
// it twice; those bytes come from L2.
//
// A wave's vector-memory operations complete in order, and in iteration t it queues: the A loads of tile
// t + 2 (4), then after each step kk the two W loads of (tile t + 1, step kk). When step kk of tile t waits
// for its operands, the operations queued after them are the W loads of the later steps of tile t, the A
// loads of tile t + 2 and the W loads of the earlier steps of tile t + 1: 10 in the steady state, fewer in
// the last two iterations. The A tile of iteration t + 1 was queued before the operands step 2 waits for,
// so it has landed when the wave reaches the barrier. The W loads are written in assembly, so the compiler
// does not know when their registers are valid; the wait names them as in/out operands, which keeps every
// use behind it.
template <bool NT = false>
__device__ __forceinline__ void load_w16(bf16x8& dst, const unsigned char* base, unsigned lane_off, int step) {
#if defined(__HIP_DEVICE_COMPILE__)
  if constexpr (NT) {   // the same loads with the non-temporal hint
    switch (step) {
      case 0: asm volatile("global_load_dwordx4 %0, %1, %2 nt" : "=v"(dst) : "v"(lane_off), "s"(base) : "memory"); break;
      case 1: asm volatile("global_load_dwordx4 %0, %1, %2 offset:1024 nt" : "=v"(dst) : "v"(lane_off), "s"(base) : "memory"); break;
      case 2: asm volatile("global_load_dwordx4 %0, %1, %2 offset:2048 nt" : "=v"(dst) : "v"(lane_off), "s"(base) : "memory"); break;
      default: asm volatile("global_load_dwordx4 %0, %1, %2 offset:3072 nt" : "=v"(dst) : "v"(lane_off), "s"(base) : "memory"); break;
    }
    return;
  }
  switch (step) {   // the step's 1 KiB piece is addressed by the instruction's immediate offset
    case 0: asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(dst) : "v"(lane_off), "s"(base) : "memory"); break;
    case 1: asm volatile("global_load_dwordx4 %0, %1, %2 offset:1024" : "=v"(dst) : "v"(lane_off), "s"(base) : "memory"); break;
    case 2: asm volatile("global_load_dwordx4 %0, %1, %2 offset:2048" : "=v"(dst) : "v"(lane_off), "s"(base) : "memory"); break;
    default: asm volatile("global_load_dwordx4 %0, %1, %2 offset:3072" : "=v"(dst) : "v"(lane_off), "s"(base) : "memory"); break;
  }
#endif
}
// Wait until at most N vector-memory operations of this wave are outstanding; a and b are valid afterwards.
template <int N>
__device__ __forceinline__ void wait_vmem_for(bf16x8& a, bf16x8& b) {
#if defined(__HIP_DEVICE_COMPILE__)
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N) : "memory");
#endif
}

template <int EPI, int WGM>
__global__ void __launch_bounds__(WGM * 256, 2) gemm_wreg_kernel(GemmArgs g) {
  constexpr int BM = WGM * 128, BN = 256, WGN = 4, BK = 64, NT = WGM * 256, NS = 3;
  constexpr int WTM = BM / WGM, WTN = BN / WGN, TM = WTM / 32, TN = WTN / 32;
  constexpr int ROWB = BK * 2, A_CH = BM * 8 / NT, STAGE = BM * ROWB;
  static_assert(TN == 2 && A_CH == 4, "the waits below count 4 A loads per tile and 2 W loads per step");
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* arena = smem + GEMM_DL_LDS_BASE;

  int v, kbeg, kend, piece;
  if (!block_work<BK>(g, &v, &kbeg, &kend, &piece)) return;
  int tm, tn;
  tile_coords(g, v, &tm, &tn);
  const int m0 = tm * BM, n0 = tn * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  const int swave = __builtin_amdgcn_readfirstlane(wave);
  const int wm = swave / WGN, wn = swave % WGN;

  const unsigned char* a_base = reinterpret_cast<const unsigned char*>(g.A + (size_t)m0 * g.lda);
  unsigned a_off[A_CH];
#pragma unroll
  for (int j = 0; j < A_CH; j++) {
    const int q = j * NT + tid, row = q >> 3, ch = (q & 7) ^ ((row >> 1) & 7);
    a_off[j] = (unsigned)(min(m0 + row, g.M - 1) - m0) * (unsigned)g.lda * 2u + ch * 16;
  }
  auto issue_a = [&](int stage, int k) {
    unsigned char* sa = arena + stage * STAGE + swave * 1024;
    const unsigned char* ak = a_base + (size_t)k * 2;
#pragma unroll
    for (int j = 0; j < A_CH; j++) lds_dma16(ak, a_off[j], sa + j * NT * 16);
  };
  // this wave's two 32-row blocks of W: 4 KiB per K tile each, the blocks of one row K / 64 * 4 KiB apart
  const size_t wrow = (size_t)(g.K >> 6) * 4096;
  const unsigned char* w_base = reinterpret_cast<const unsigned char*>(g.W) + (size_t)((n0 >> 5) + wn * TN) * wrow;
  const unsigned w_lane = (unsigned)lane * 16u;
  bf16x8 w[TN][4];
#pragma unroll
  for (int j = 0; j < TN; j++)
#pragma unroll
    for (int kk = 0; kk < 4; kk++)
#pragma unroll
      for (int e = 0; e < 8; e++) w[j][kk][e] = 0;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

  int koff[4];
#pragma unroll
  for (int kk = 0; kk < 4; kk++) koff[kk] = ((kk * 2 + lh) ^ ((l32 >> 1) & 7)) * 16;
  const int a_row = (wm * WTM + l32) * ROWB;

  const int nk = (kend - kbeg) / BK;
  // Every iteration queues the same operations, also the last ones, whose loads have no tile left to fetch and
  // re-read the last K tile into a stage (or registers) nobody uses any more: the waits then count alike throughout.
  auto tile_k = [&](int t) { return kbeg + min(t, nk - 1) * BK; };
  // prologue: A(0), A(1), then W(0) step by step; A(0) has landed once at most A(1) and W(0) are outstanding
  issue_a(0, tile_k(0));
  issue_a(1, tile_k(1));
  {
    const unsigned char* wk = w_base + (size_t)(tile_k(0) >> 6) * 4096;
#pragma unroll
    for (int kk = 0; kk < 4; kk++)
#pragma unroll
      for (int j = 0; j < TN; j++) load_w16(w[j][kk], wk + j * wrow, w_lane, kk);
  }
  wait_vmem<A_CH + 4 * TN>();
  __syncthreads();
  bf16x8 af[2][TM];
#pragma unroll
  for (int i = 0; i < TM; i++) af[0][i] = *reinterpret_cast<const bf16x8*>(arena + a_row + i * 32 * ROWB + koff[0]);

  int cur = 0;
  for (int t = 0; t < nk; t++) {
    const int nxt = cur + 1 == NS ? 0 : cur + 1;
    const int nx2 = nxt + 1 == NS ? 0 : nxt + 1;
    const unsigned char* Ac = arena + cur * STAGE + a_row;
    const unsigned char* An = arena + nxt * STAGE + a_row;
    const unsigned char* wk = w_base + (size_t)(tile_k(t + 1) >> 6) * 4096;       // W of tile t + 1
    __builtin_amdgcn_sched_barrier(0);
    // tile t + 2 goes into the stage that tile t - 1 left at the last barrier
    issue_a(nx2, tile_k(t + 2));
    auto step = [&](auto kk_c) {
      constexpr int kk = decltype(kk_c)::value;
      __builtin_amdgcn_sched_barrier(0);
      // queued after these operands: the W loads of the later steps of this tile (6 - 2 kk), the A loads of tile
      // t + 2 (4), the W loads of the earlier steps of the next tile (2 kk)
      wait_vmem_for<2 * TN + A_CH + 2>(w[0][kk], w[1][kk]);
      if constexpr (kk == 3) {
        // every wave's A loads of tile t + 1 landed before its step-2 operands did: publish the tile, retire this one
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < TM; i++) af[0][i] = *reinterpret_cast<const bf16x8*>(An + i * 32 * ROWB + koff[0]);
      } else {
#pragma unroll
        for (int i = 0; i < TM; i++) af[(kk + 1) & 1][i] = *reinterpret_cast<const bf16x8*>(Ac + i * 32 * ROWB + koff[kk + 1]);
      }
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], w[j][kk], acc[i][j], 0, 0, 0);
#pragma unroll
      for (int x = 0; x < TM; x++) {
        __builtin_amdgcn_sched_group_barrier(0x008, TN, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < TN; j++) load_w16(w[j][kk], wk + j * wrow, w_lane, kk);
    };
    step(std::integral_constant<int, 0>{});
    step(std::integral_constant<int, 1>{});
    step(std::integral_constant<int, 2>{});
    step(std::integral_constant<int, 3>{});
    cur = nxt;
  }
  // the surplus loads of the last iterations must not land in registers the epilogue reuses
  wait_vmem_for<0>(w[0][0], w[1][0]);
  wait_vmem_for<0>(w[0][1], w[1][1]);
  wait_vmem_for<0>(w[0][2], w[1][2]);
  wait_vmem_for<0>(w[0][3], w[1][3]);
  if constexpr ((EPI == EPI_BF16 || EPI == EPI_SWIGLU_BF16) && WGM == 2) {
    // bf16 outputs leave through LDS: a lane holds one column of its accumulator blocks, so stored directly a wave
    // instruction writes 64-byte pieces of rows; staged as a [rows][columns] image in the (now free) A stages, every
    // lane stores 16 bytes and a row of the tile goes out as whole 128-byte lines.
    if (piece < 0) {
      constexpr bool SW = EPI == EPI_SWIGLU_BF16;
      constexpr int OC = SW ? BN / 2 : BN;                    // output columns of the tile
      constexpr int PR = 64 * 1024 / (OC * 2);                // rows per pass: 64 KB of LDS
      constexpr int PASSES = BM / PR;                         // SwiGLU: all 256 rows at once; bf16 store: the two wave rows in turn
      static_assert(PR % WTM == 0 && 3 * STAGE >= 64 * 1024, "a pass holds whole wave rows and fits the A stages");
      bf16* img = reinterpret_cast<bf16*>(arena);
      bf16* outp = reinterpret_cast<bf16*>(g.C);
      const int oc0 = SW ? (n0 >> 1) : n0;
#pragma unroll
      for (int pass = 0; pass < PASSES; pass++) {
        __syncthreads();                                      // the stage reads of the main loop (or the last pass's copy) are done
        if (wm * WTM / PR == pass) {
          const int rb = wm * WTM % PR + 4 * lh;
#pragma unroll
          for (int i = 0; i < TM; i++)
#pragma unroll
            for (int r = 0; r < 16; r++) {
              bf16* dst = img + (size_t)(rb + i * 32 + 8 * (r >> 2) + (r & 3)) * OC;
              if constexpr (SW) {
                const float gate = acc[i][0][r], up = acc[i][1][r];
                dst[wn * (WTN / 2) + l32] = f2bf(gate / (1.f + __expf(-gate)) * up);
              } else {
#pragma unroll
                for (int j = 0; j < TN; j++) dst[wn * WTN + j * 32 + l32] = f2bf(acc[i][j][r]);
              }
            }
        }
        __syncthreads();
        constexpr int CPRW = OC / 8;                          // 16-byte chunks per row
#pragma unroll
        for (int c = 0; c < PR * CPRW / NT; c++) {
          const int q = c * NT + tid, row = q / CPRW, cc = q % CPRW;
          const int grow = m0 + pass * PR + row;
          if (grow < g.M)
            *reinterpret_cast<u32x4*>(outp + (size_t)grow * g.ldc + oc0 + cc * 8) = *reinterpret_cast<const u32x4*>(img + (size_t)row * OC + cc * 8);
        }
      }
      return;
    }
  }
  store_tile<BM, BN, WGM, WGN, EPI>(g, acc, m0, n0, piece, wm, wn, l32, lh);
}

// ---- decode batches (up to 64 rows per tile): weights streamed through registers, several K tiles deep ----
// A decode GEMM reads every weight byte once and runs at the rate at which its CUs pull bytes from memory; what
// a workgroup reads beside its weights -- the 64 activation rows of its K range, again for every workgroup --
// comes out of that rate. A workgroup here is 4 to 8 waves (the launch's block size; a tile is 64 columns per
// wave wide), so that a width can be chosen that divides N into whole rounds of workgroups on the partition
// while the activation tile is shared by as many waves as possible. A wave reads the W operands of its 64
// columns (two 32-row blocks of the packed layout) straight into registers and keeps PD K tiles of them -- 8 PD
// loads of 1 KiB -- under way. Only the activation tile passes through LDS (PD + 2 stages of 8 KB, fetched by
// the first four waves as in the loops above).
//
// Order of a wave's vector-memory operations (they complete in order): iteration t queues the A loads of
// tile t + PD + 1 (2), then after each step kk the two W loads of (tile t + PD, step kk) into the registers
// that step just used; the prologue queues A(0) and then, for s < PD, A(s + 1) and W(s) in the same order.
// When step kk of tile t waits for its operands, 10 PD - 2 operations were queued after them (the W loads
// of the later steps of tile t: 6 - 2 kk; A and W of the PD - 1 tiles between: 10 each; this iteration's A
// loads: 2; its W loads so far: 2 kk), in every iteration: the last ones re-read the last K tile into
// registers and stages nobody uses. A(t + 1) was queued before the operands step 3 of tile t waits for, so
// it has landed at the barrier there, which also retires the stage of tile t for the A loads of iteration
// t + 1.
template <int EPI, int PD, bool NT>
__global__ void __launch_bounds__(512, 2) gemm_skinny_kernel(GemmArgs g) {
  constexpr int BM = 64, BK = 64, NS = PD + 2, DUTY = 4;     // DUTY waves load the A tile
  constexpr int TM = 2, TN = 2, ROWB = BK * 2, A_CH = BM * 8 / (DUTY * 64), STAGE = BM * ROWB;
  constexpr int WAIT = 10 * PD - 2;
  static_assert(A_CH == 2 && WAIT < 64, "the waits count 2 A loads per tile and 2 W loads per step, within vmcnt's range");
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* arena = smem + GEMM_DL_LDS_BASE;

  int v, kbeg, kend, piece;
  if (!block_work<BK>(g, &v, &kbeg, &kend, &piece)) return;
  int tm, tn;
  tile_coords(g, v, &tm, &tn);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  const int swave = __builtin_amdgcn_readfirstlane(wave);
  const int wn = swave;
  const int m0 = tm * BM, n0 = tn * (int)(blockDim.x >> 6) * 64;     // a tile is 64 columns per wave wide

  const unsigned char* a_base = reinterpret_cast<const unsigned char*>(g.A + (size_t)m0 * g.lda);
  // The first DUTY waves fetch the A tile. The others queue as many 16-byte loads of the tile's first bytes into a
  // spare KB behind the stages, so that every wave's queue has the same shape and the waits below count alike.
  const bool duty = swave < DUTY;
  unsigned a_off[A_CH];
#pragma unroll
  for (int j = 0; j < A_CH; j++) {
    const int q = j * (DUTY * 64) + (tid & (DUTY * 64 - 1)), row = q >> 3, ch = (q & 7) ^ ((row >> 1) & 7);
    a_off[j] = duty ? (unsigned)(min(m0 + row, g.M - 1) - m0) * (unsigned)g.lda * 2u + ch * 16 : 0u;
  }
  auto issue_a = [&](int stage, int k) {
    unsigned char* sa = duty ? arena + stage * STAGE + swave * 1024 : arena + NS * STAGE;
    const unsigned char* ak = a_base + (size_t)k * 2;
#pragma unroll
    for (int j = 0; j < A_CH; j++) lds_dma16(ak, a_off[j], duty ? sa + j * (DUTY * 64) * 16 : sa);
  };
  const size_t wrow = (size_t)(g.K >> 6) * 4096;
  const unsigned char* w_base = reinterpret_cast<const unsigned char*>(g.W) + (size_t)((n0 >> 5) + wn * TN) * wrow;
  const unsigned w_lane = (unsigned)lane * 16u;
  bf16x8 w[PD][TN][4];
#pragma unroll
  for (int s = 0; s < PD; s++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int kk = 0; kk < 4; kk++)
#pragma unroll
        for (int e = 0; e < 8; e++) w[s][j][kk][e] = 0;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

  int koff[4];
#pragma unroll
  for (int kk = 0; kk < 4; kk++) koff[kk] = ((kk * 2 + lh) ^ ((l32 >> 1) & 7)) * 16;
  const int a_row = l32 * ROWB;

  const int nk = (kend - kbeg) / BK;
  auto tile_k = [&](int t) { return kbeg + min(t, nk - 1) * BK; };
  issue_a(0, tile_k(0));
#pragma unroll
  for (int s = 0; s < PD; s++) {
    issue_a(s + 1, tile_k(s + 1));
    const unsigned char* wk = w_base + (size_t)(tile_k(s) >> 6) * 4096;
#pragma unroll
    for (int kk = 0; kk < 4; kk++)
#pragma unroll
      for (int j = 0; j < TN; j++) load_w16<NT>(w[s][j][kk], wk + j * wrow, w_lane, kk);
  }
  wait_vmem<10 * PD>();                                      // A(0) has landed
  __syncthreads();
  bf16x8 af[2][TM];
#pragma unroll
  for (int i = 0; i < TM; i++) af[0][i] = *reinterpret_cast<const bf16x8*>(arena + a_row + i * 32 * ROWB + koff[0]);

  int cur = 0;                                               // stage of tile t
  int ahead = PD + 1;                                        // stage of tile t + PD + 1
  for (int t0 = 0; t0 < nk; t0 += PD) {
    auto tile = [&](auto s_c) {
      constexpr int s = decltype(s_c)::value;                // register set of tile t: t % PD
      const int t = t0 + s;
      const bool live = t < nk;                              // the surplus tiles of the last round only keep the queue's shape
      const int nxt = cur + 1 == NS ? 0 : cur + 1;
      const unsigned char* Ac = arena + cur * STAGE + a_row;
      const unsigned char* An = arena + nxt * STAGE + a_row;
      const unsigned char* wk = w_base + (size_t)(tile_k(t + PD) >> 6) * 4096;
      __builtin_amdgcn_sched_barrier(0);
      issue_a(ahead, tile_k(t + PD + 1));
      auto step = [&](auto kk_c) {
        constexpr int kk = decltype(kk_c)::value;
        __builtin_amdgcn_sched_barrier(0);
        wait_vmem_for<WAIT>(w[s][0][kk], w[s][1][kk]);
        if constexpr (kk == 3) {
          __syncthreads();
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int i = 0; i < TM; i++) af[0][i] = *reinterpret_cast<const bf16x8*>(An + i * 32 * ROWB + koff[0]);
        } else {
#pragma unroll
          for (int i = 0; i < TM; i++) af[(kk + 1) & 1][i] = *reinterpret_cast<const bf16x8*>(Ac + i * 32 * ROWB + koff[kk + 1]);
        }
        if (live) {
#pragma unroll
          for (int i = 0; i < TM; i++)
#pragma unroll
            for (int j = 0; j < TN; j++)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], w[s][j][kk], acc[i][j], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < TN; j++) load_w16<NT>(w[s][j][kk], wk + j * wrow, w_lane, kk);
      };
      step(std::integral_constant<int, 0>{});
      step(std::integral_constant<int, 1>{});
      step(std::integral_constant<int, 2>{});
      step(std::integral_constant<int, 3>{});
      cur = nxt;
      ahead = ahead + 1 == NS ? 0 : ahead + 1;
    };
    tile(std::integral_constant<int, 0>{});
    if constexpr (PD > 1) tile(std::integral_constant<int, 1>{});
    if constexpr (PD > 2) tile(std::integral_constant<int, 2>{});
    if constexpr (PD > 3) tile(std::integral_constant<int, 3>{});
    if constexpr (PD > 4) tile(std::integral_constant<int, 4>{});
    if constexpr (PD > 5) tile(std::integral_constant<int, 5>{});
  }
  // the surplus loads of the last iterations must not land in registers the epilogue reuses
#pragma unroll
  for (int s = 0; s < PD; s++)
#pragma unroll
    for (int kk = 0; kk < 4; kk++) wait_vmem_for<0>(w[s][0][kk], w[s][1][kk]);
  // a wave's 64 x 64 block: the tile store of a four-wave row, placed by the wave's index
  store_tile<BM, 256, 1, 4, EPI>(g, acc, m0, n0, piece, 0, wn, l32, lh);
}

// Adds the tail pieces of each split tile in piece order and applies the epilogue. One thread per
// four consecutive columns.
template <int BM, int BN, int EPI>
__global__ void __launch_bounds__(256) gemm_tail_fixup(GemmArgs g) {
  const int t = blockIdx.x;                                   // tail tile
  const int e = blockIdx.y * 256 + threadIdx.x;
  const int r = e / (BN / 4), c = (e % (BN / 4)) * 4;
  int tm, tn;
  tile_coords(g, g.n_full + t, &tm, &tn);
  const int row = tm * BM + r;
  if (row >= g.M) return;
  if (EPI == EPI_SWIGLU_BF16 && ((c >> 5) & 1)) return;      // "up" columns are consumed by their gate thread
  const float* p = g.tail_ws + (size_t)t * g.tail_f * (BM * BN) + (size_t)r * BN + c;
  f32x4 sum = *reinterpret_cast<const f32x4*>(p), up = {0.f, 0.f, 0.f, 0.f};
  if (EPI == EPI_SWIGLU_BF16) up = *reinterpret_cast<const f32x4*>(p + 32);
  for (int z = 1; z < g.tail_f; z++) {
    sum += *reinterpret_cast<const f32x4*>(p + (size_t)z * (BM * BN));
    if (EPI == EPI_SWIGLU_BF16) up += *reinterpret_cast<const f32x4*>(p + (size_t)z * (BM * BN) + 32);
  }
  const int col = tn * BN + c;
  if constexpr (EPI == EPI_SWIGLU_BF16) {
    bf16x4 o;
#pragma unroll
    for (int i = 0; i < 4; i++) o[i] = f2bf(sum[i] / (1.f + __expf(-sum[i])) * up[i]);
    const int ocol = ((tn * BN + (c & ~63)) >> 1) + (c & 31);
    *reinterpret_cast<bf16x4*>(reinterpret_cast<bf16*>(g.C) + (size_t)row * g.ldc + ocol) = o;
  } else if constexpr (EPI == EPI_BF16) {
    bf16x4 o;
#pragma unroll
    for (int i = 0; i < 4; i++) o[i] = f2bf(sum[i]);
    *reinterpret_cast<bf16x4*>(reinterpret_cast<bf16*>(g.C) + (size_t)row * g.ldc + col) = o;
  } else {
    f32x4* dst = reinterpret_cast<f32x4*>(reinterpret_cast<float*>(g.C) + (size_t)row * g.ldc + col);
    if constexpr (EPI == EPI_RESID_F32) *dst += sum;
    else *dst = sum;
  }
}

// How the tiles of one launch are divided when the partition holds `slots` workgroups of this
// configuration at once: n_full tiles run whole (complete waves), the `rest` tiles of the last
// wave are cut into f pieces (f = 1: no cut). rest * f pieces take ceil(rest * f / slots) rounds
// of 1/f tile time each; every piece also pays a fixed start-up and partial-store cost, taken as
// 3 % of a tile time. The cut is made only if it saves at least a tenth of a tile time.
void gemm_tail_plan(int tiles, int ksteps, int slots, long long max_pieces, int* n_full, int* f) {
  *n_full = tiles; *f = 1;
  if (slots <= 0) return;
  const int full = tiles / slots * slots, rest = tiles - full;
  if (rest == 0) return;
  int best = 1; double best_t = 1.0;
  for (int cut = 2; cut <= std::min(ksteps / 4, 16); cut++) {
    if ((long long)rest * cut > max_pieces) break;               // partial tiles must fit the scratch buffer
    const int rounds = (rest * cut + slots - 1) / slots;
    const double t = rounds * (1.0 / cut + 0.03);
    if (t < best_t - 1e-9) { best_t = t; best = cut; }
  }
  if (best_t > 0.9) return;
  *n_full = full; *f = best;
}

// NS: LDS stages of the main loop.
template <int BM, int BN, int WGM, int WGN, int EPI, int NS>
static hipError_t launch_cfg(hipStream_t s, GemmArgs g, int splits, const GemmTail* tail) {
  constexpr int NT = WGM * WGN * 64, BK = 64;
  constexpr size_t lds_dl = GEMM_DL_LDS_BASE + NS * (size_t)(BM + BN) * BK * sizeof(bf16);
  constexpr size_t lds_wreg = GEMM_DL_LDS_BASE + 3 * (size_t)BM * BK * sizeof(bf16);    // gemm_wreg_kernel: three stages of the A tile
  // packed W: tiles of 256 columns with wave tiles of 128 x 64 take their W operands straight from global memory
  constexpr bool WREG = BN == 256 && WGN == 4 && BM == WGM * 128;
  // decode batches: 64-row tiles, 64 columns per wave, the W operands GEMM_SKINNY_PD tiles deep in registers
  constexpr bool SKINNY = BM == 64 && WGM == 1 && BN == WGN * 64;
  constexpr size_t lds_skinny = GEMM_DL_LDS_BASE + (size_t)(GEMM_SKINNY_PD + 2) * BM * BK * sizeof(bf16) + 1024;
  void (*kern)(GemmArgs) = nullptr;
  void (*kern_rowmajor)(GemmArgs) = nullptr;       // row-major W: the fp32-store epilogue only (callers that bring their own weights)
  if constexpr (WREG) kern = gemm_wreg_kernel<EPI, WGM>;
  else if constexpr (SKINNY) kern = g.stream_nt ? gemm_skinny_kernel<EPI, GEMM_SKINNY_PD, true> : gemm_skinny_kernel<EPI, GEMM_SKINNY_PD, false>;
  else kern = gemm_dl_kernel<BM, BN, WGM, WGN, EPI, NS>;
  if constexpr (EPI == EPI_F32 && !SKINNY) kern_rowmajor = gemm_dl_kernel<BM, BN, WGM, WGN, EPI, NS, false>;
  if (!g.w_packed && !kern_rowmajor) return hipErrorInvalidValue;
  constexpr size_t lds_packed = WREG ? lds_wreg : SKINNY ? lds_skinny : lds_dl;
  const size_t lds = !g.w_packed ? lds_dl : lds_packed;
  static std::atomic<bool> attr_set{false};        // the two phases' control threads may launch the same shape
  if (!attr_set.load()) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_packed);
    if constexpr (SKINNY) {      // both forms of the kernel, whichever this call takes
      void (*other)(GemmArgs) = g.stream_nt ? gemm_skinny_kernel<EPI, GEMM_SKINNY_PD, false> : gemm_skinny_kernel<EPI, GEMM_SKINNY_PD, true>;
      if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void*>(other), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_packed);
    }
    if (e == hipSuccess && kern_rowmajor) e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern_rowmajor), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_dl);
    if (e != hipSuccess) return e;
    attr_set.store(true);
  }
  g.tiles_m = (g.M + BM - 1) / BM;
  g.tiles_n = g.N / BN;
  const int tiles = g.tiles_m * g.tiles_n;
  g.group_m = 8;
  const int ksteps = g.K / BK;
  g.n_full = tiles; g.tail_f = 1; g.n_pieces = 0; g.piece_per_xcd = 0; g.tail_ws = nullptr;
  if (tail && tail->ws && splits == 1 && g.ldc % 4 == 0) {
    int n_full, f;
    gemm_tail_plan(tiles, ksteps, tail->slots, (long long)(tail->ws_bytes / (BM * BN * sizeof(float))), &n_full, &f);
    if (f > 1) {
      g.n_full = n_full; g.tail_f = f; g.n_pieces = (tiles - n_full) * f;
      g.piece_per_xcd = (g.n_pieces + 7) / 8;
      g.tail_ws = tail->ws;
    }
  }
  g.full_per_xcd = (g.n_full + 7) / 8;
  const int per = (ksteps + splits - 1) / splits;
  g.k_per_split = per * BK;
  const int ny = (ksteps + per - 1) / per;
  if (!g.w_packed) kern = kern_rowmajor;
  hipLaunchKernelGGL(kern, dim3((g.full_per_xcd + g.piece_per_xcd) * 8, ny), dim3(NT), lds, s, g);
  if constexpr (!SKINNY) {
    if (g.n_pieces > 0)
      hipLaunchKernelGGL((gemm_tail_fixup<BM, BN, EPI>), dim3(tiles - g.n_full, BM * BN / 1024), dim3(256), 0, s, g);
  }
  return hipGetLastError();
}

template <int EPI>
static hipError_t launch_epi(hipStream_t s, int cfg, const GemmArgs& g, int splits, const GemmTail* tail) {
  switch (cfg) {
    case GEMM_128x128: return launch_cfg<128, 128, 2, 2, EPI, 2>(s, g, splits, tail);
    case GEMM_64x256: return launch_cfg<64, 256, 1, 8, EPI, 3>(s, g, splits, tail);
    case GEMM_64x128: return launch_cfg<64, 128, 1, 4, EPI, 3>(s, g, splits, tail);
    case GEMM_256x256: return launch_cfg<256, 256, 2, 4, EPI, 2>(s, g, splits, tail);
    case GEMM_128x256: return launch_cfg<128, 256, 1, 4, EPI, 2>(s, g, splits, tail);
    case GEMM_64x256S: return launch_cfg<64, 256, 1, 4, EPI, 3>(s, g, splits, nullptr);
    case GEMM_64x320S: return launch_cfg<64, 320, 1, 5, EPI, 3>(s, g, splits, nullptr);
    case GEMM_64x384S: return launch_cfg<64, 384, 1, 6, EPI, 3>(s, g, splits, nullptr);
    case GEMM_64x448S: return launch_cfg<64, 448, 1, 7, EPI, 3>(s, g, splits, nullptr);
    case GEMM_64x512S: return launch_cfg<64, 512, 1, 8, EPI, 3>(s, g, splits, nullptr);
    default: return hipErrorInvalidValue;
  }
}

int gemm_tile_n(int cfg) {
  if (cfg >= GEMM_64x256S && cfg <= GEMM_64x512S) return 256 + 64 * (cfg - GEMM_64x256S);
  return cfg == GEMM_256x256 || cfg == GEMM_64x256 || cfg == GEMM_128x256 ? 256 : 128;
}
int gemm_tile_m(int cfg) { return cfg == GEMM_256x256 ? 256 : cfg == GEMM_128x128 || cfg == GEMM_128x256 ? 128 : 64; }
// Workgroups per CU the launch plan counts: the 8-wave tiles fill a CU, the 4-wave tiles share it in pairs. The 128x256
// tile (4 waves, wave tiles of 128 x 64) is planned one per CU although two fit: it is the shape for launches with little
// more than one tile per CU, where the whole tiles take one slot of every CU and the K pieces of the surplus tiles run
// beside them in the second.
int gemm_wgs_per_cu(int cfg) { return cfg == GEMM_256x256 || cfg == GEMM_64x256 || cfg == GEMM_128x256 || cfg > GEMM_64x256S ? 1 : 2; }

// C = A * W^T with the chosen tile configuration and epilogue. Requirements (checked):
// K % 64 == 0, N % tile_n == 0, leading dimensions multiples of 8 elements, M >= 1; W packed (ldw == K) or,
// for the fp32-store epilogue, row-major.
// With splits > 1 (EPI_F32 only) partial sums go to C + z * split_stride. With `tail` (splits == 1)
// the tiles of the last, partly filled wave of workgroups are cut along K (see GemmArgs).
hipError_t gemm_bf16(hipStream_t s, int cfg, int epi, const bf16* A, int lda, const bf16* W, int ldw,
                     void* C, int ldc, int M, int N, int K, int splits, long long split_stride, const GemmTail* tail, bool w_packed, bool stream_nt) {
  if (M < 1 || K % 64 != 0 || N % gemm_tile_n(cfg) != 0 || lda % 8 != 0 || ldw % 8 != 0) return hipErrorInvalidValue;
  if (w_packed && ldw != K) return hipErrorInvalidValue;          // packed blocks are addressed by K alone
  if (splits < 1 || (splits > 1 && epi != EPI_F32)) return hipErrorInvalidValue;
  if (cfg == GEMM_256x256 && (epi == EPI_BF16 || epi == EPI_SWIGLU_BF16) && ldc % 8 != 0) return hipErrorInvalidValue;   // 16-byte output stores
  if (epi == EPI_SWIGLU_BF16 && cfg == GEMM_64x256) return hipErrorInvalidValue;   // its wave tile is one 32-column block, not a gate/up pair
  if (epi == EPI_SWIGLU_BF16 && cfg == GEMM_128x256) return hipErrorInvalidValue;  // not instantiated: the shape serves the O and down projections
  GemmArgs g{};
  g.A = A; g.W = W; g.C = C; g.lda = lda; g.ldw = ldw; g.ldc = ldc; g.M = M; g.N = N; g.K = K;
  g.split_stride = split_stride; g.w_packed = w_packed ? 1 : 0; g.stream_nt = stream_nt ? 1 : 0;
  switch (epi) {
    case EPI_BF16: return launch_epi<EPI_BF16>(s, cfg, g, splits, tail);
    case EPI_F32: return launch_epi<EPI_F32>(s, cfg, g, splits, tail);
    case EPI_RESID_F32: return launch_epi<EPI_RESID_F32>(s, cfg, g, splits, tail);
    case EPI_SWIGLU_BF16:
      switch (cfg) {   // instantiated only where the wave tile holds gate/up block pairs
        case GEMM_256x256: return launch_cfg<256, 256, 2, 4, EPI_SWIGLU_BF16, 2>(s, g, 1, tail);
        case GEMM_128x128: return launch_cfg<128, 128, 2, 2, EPI_SWIGLU_BF16, 2>(s, g, 1, tail);
        case GEMM_64x256S: return launch_cfg<64, 256, 1, 4, EPI_SWIGLU_BF16, 3>(s, g, 1, nullptr);
        case GEMM_64x320S: return launch_cfg<64, 320, 1, 5, EPI_SWIGLU_BF16, 3>(s, g, 1, nullptr);
        case GEMM_64x384S: return launch_cfg<64, 384, 1, 6, EPI_SWIGLU_BF16, 3>(s, g, 1, nullptr);
        case GEMM_64x448S: return launch_cfg<64, 448, 1, 7, EPI_SWIGLU_BF16, 3>(s, g, 1, nullptr);
        case GEMM_64x512S: return launch_cfg<64, 512, 1, 8, EPI_SWIGLU_BF16, 3>(s, g, 1, nullptr);
        case GEMM_64x128: return launch_cfg<64, 128, 2, 2, EPI_SWIGLU_BF16, 3>(s, g, 1, tail);    // wave tiles of 32 x 64: one gate/up pair
        default: return hipErrorInvalidValue;
      }
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sts
