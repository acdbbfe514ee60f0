// bf16 MFMA GEMM for gfx950:  C[M,N] (+)= A[M,K] * W[N,K]^T, fp32 accumulation.
//
// Both operands are K-contiguous, which is the layout v_mfma_f32_32x32x16_bf16 wants: a lane
// holds 8 consecutive k of one A row (or one W row). A workgroup owns a BM x BN tile; tiles of
// A and W are staged global -> registers -> LDS (double buffered, rows padded by 16 bytes so
// the 16-byte operand reads are bank-conflict free) and each wave accumulates a
// (BM/WGM) x (BN/WGN) sub-tile in 32x32 MFMA blocks.
//
// Lane layout of the 32x32 accumulator block (register r of lane l):
//   row = 8*(r/4) + 4*(l/32) + r%4,  col = l%32.
#include "kernels.h"

namespace sts {

struct GemmArgs {
  const bf16* A; const bf16* W; void* C;
  int lda, ldw, ldc;
  int M, N, K;
  int tiles_m, tiles_n, per_xcd, group_m;
  int k_per_split;            // K range handled by one blockIdx.y
  long long split_stride;     // elements between consecutive split-K partial outputs
};

template <int BM, int BN, int BK, int WGM, int WGN, int EPI>
__global__ void __launch_bounds__(WGM* WGN * 64) gemm_kernel(GemmArgs g) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int WTM = BM / WGM, WTN = BN / WGN, TM = WTM / 32, TN = WTN / 32;
  constexpr int LS = BK + 8;                       // LDS row stride in elements
  constexpr int CPR = BK / 8;                      // 16-byte chunks per tile row
  constexpr int A_CH = BM * CPR / NT, B_CH = BN * CPR / NT;
  static_assert(BM * CPR % NT == 0 && BN * CPR % NT == 0, "tile/thread mismatch");
  static_assert(EPI != EPI_SWIGLU_BF16 || TN % 2 == 0, "swiglu needs gate/up block pairs");
  extern __shared__ __align__(16) unsigned char smem[];
  bf16* As = reinterpret_cast<bf16*>(smem);        // [2][BM][LS]
  bf16* Bs = As + 2 * BM * LS;                     // [2][BN][LS]

  const int v = xcd_contiguous(blockIdx.x, g.per_xcd);
  if (v >= g.tiles_m * g.tiles_n) return;
  const int gsz = g.group_m * g.tiles_n;
  const int first_m = (v / gsz) * g.group_m;
  const int gm = min(g.tiles_m - first_m, g.group_m);
  const int tm = first_m + (v % gsz) % gm, tn = (v % gsz) / gm;
  const int m0 = tm * BM, n0 = tn * BN;
  const int kbeg = blockIdx.y * g.k_per_split, kend = min(g.K, kbeg + g.k_per_split);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lh = lane >> 5;
  const int wm = wave / WGN, wn = wave % WGN;

  const bf16* a_src[A_CH];
  const bf16* b_src[B_CH];
  int a_dst[A_CH], b_dst[B_CH];
#pragma unroll
  for (int j = 0; j < A_CH; j++) {
    int c = tid + j * NT, row = c / CPR, cc = c % CPR;
    a_src[j] = g.A + (size_t)min(m0 + row, g.M - 1) * g.lda + cc * 8;
    a_dst[j] = row * LS + cc * 8;
  }
#pragma unroll
  for (int j = 0; j < B_CH; j++) {
    int c = tid + j * NT, row = c / CPR, cc = c % CPR;
    b_src[j] = g.W + (size_t)(n0 + row) * g.ldw + cc * 8;
    b_dst[j] = row * LS + cc * 8;
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

  u32x4 ra[A_CH], rb[B_CH];
#pragma unroll
  for (int j = 0; j < A_CH; j++) ra[j] = *reinterpret_cast<const u32x4*>(a_src[j] + kbeg);
#pragma unroll
  for (int j = 0; j < B_CH; j++) rb[j] = *reinterpret_cast<const u32x4*>(b_src[j] + kbeg);
#pragma unroll
  for (int j = 0; j < A_CH; j++) *reinterpret_cast<u32x4*>(As + a_dst[j]) = ra[j];
#pragma unroll
  for (int j = 0; j < B_CH; j++) *reinterpret_cast<u32x4*>(Bs + b_dst[j]) = rb[j];
  __syncthreads();

  int cur = 0;
  for (int k = kbeg; k < kend; k += BK) {
    // Prefetch the next K tile into registers while this one is consumed from LDS. The last
    // iteration re-reads its own tile (in bounds, never used) so the loop body has no branch.
    const int kn = min(k + BK, kend - BK);
#pragma unroll
    for (int j = 0; j < A_CH; j++) ra[j] = *reinterpret_cast<const u32x4*>(a_src[j] + kn);
#pragma unroll
    for (int j = 0; j < B_CH; j++) rb[j] = *reinterpret_cast<const u32x4*>(b_src[j] + kn);
    __builtin_amdgcn_sched_barrier(0);     // keep the loads ahead of the MFMA block (the scheduler would sink them)
    const bf16* Ac = As + cur * BM * LS + (wm * WTM + l32) * LS + 8 * lh;
    const bf16* Bc = Bs + cur * BN * LS + (wn * WTN + l32) * LS + 8 * lh;
    // operand fragments are double buffered in registers: the LDS reads of step kk+1 are in
    // flight while the MFMAs of step kk issue
    bf16x8 af[2][TM], bfr[2][TN];
#pragma unroll
    for (int i = 0; i < TM; i++) af[0][i] = *reinterpret_cast<const bf16x8*>(Ac + i * 32 * LS);
#pragma unroll
    for (int j = 0; j < TN; j++) bfr[0][j] = *reinterpret_cast<const bf16x8*>(Bc + j * 32 * LS);
#pragma unroll
    for (int kk = 0; kk < BK / 16; kk++) {
      if (kk + 1 < BK / 16) {
#pragma unroll
        for (int i = 0; i < TM; i++) af[(kk + 1) & 1][i] = *reinterpret_cast<const bf16x8*>(Ac + i * 32 * LS + (kk + 1) * 16);
#pragma unroll
        for (int j = 0; j < TN; j++) bfr[(kk + 1) & 1][j] = *reinterpret_cast<const bf16x8*>(Bc + j * 32 * LS + (kk + 1) * 16);
      }
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j], acc[i][j], 0, 0, 0);
    }
    // scheduling recipe: first the TM+TN fragment reads of step 0, then per step one LDS read
    // slotted between every MPR MFMAs, the last step pure MFMA
    {
      constexpr int MPR = (TM * TN + TM + TN - 1) / (TM + TN);
      __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);
#pragma unroll
      for (int kk = 0; kk + 1 < BK / 16; kk++)
#pragma unroll
        for (int x = 0; x < TM + TN; x++) {
          __builtin_amdgcn_sched_group_barrier(0x008, MPR, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
      __builtin_amdgcn_sched_group_barrier(0x008, TM * TN, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    bf16* An = As + (cur ^ 1) * BM * LS;
    bf16* Bn = Bs + (cur ^ 1) * BN * LS;
#pragma unroll
    for (int j = 0; j < A_CH; j++) *reinterpret_cast<u32x4*>(An + a_dst[j]) = ra[j];
#pragma unroll
    for (int j = 0; j < B_CH; j++) *reinterpret_cast<u32x4*>(Bn + b_dst[j]) = rb[j];
    __syncthreads();
    cur ^= 1;
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

template <int BM, int BN, int BK, int WGM, int WGN, int EPI>
static hipError_t launch_cfg(hipStream_t s, GemmArgs g, int splits) {
  constexpr int NT = WGM * WGN * 64;
  constexpr size_t lds = 2 * (size_t)(BM + BN) * (BK + 8) * sizeof(bf16);
  auto kern = gemm_kernel<BM, BN, BK, WGM, WGN, EPI>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  g.tiles_m = (g.M + BM - 1) / BM;
  g.tiles_n = g.N / BN;
  const int tiles = g.tiles_m * g.tiles_n;
  g.per_xcd = (tiles + 7) / 8;
  g.group_m = 8;
  const int ksteps = g.K / BK;
  const int per = (ksteps + splits - 1) / splits;
  g.k_per_split = per * BK;
  const int ny = (ksteps + per - 1) / per;
  hipLaunchKernelGGL(kern, dim3(g.per_xcd * 8, ny), dim3(NT), lds, s, g);
  return hipGetLastError();
}

template <int EPI>
static hipError_t launch_epi(hipStream_t s, int cfg, const GemmArgs& g, int splits) {
  switch (cfg) {
    case GEMM_256x256: return launch_cfg<256, 256, 64, 2, 2, EPI>(s, g, splits);
    case GEMM_128x128: return launch_cfg<128, 128, 64, 2, 2, EPI>(s, g, splits);
    case GEMM_256x128: return launch_cfg<256, 128, 64, 2, 2, EPI>(s, g, splits);
    case GEMM_64x256: return launch_cfg<64, 256, 64, 1, 4, EPI>(s, g, splits);
    case GEMM_32x256: return launch_cfg<32, 256, 64, 1, 4, EPI>(s, g, splits);
    case GEMM_64x128: return launch_cfg<64, 128, 64, 1, 4, EPI>(s, g, splits);
    case GEMM_64x64: return launch_cfg<64, 64, 64, 2, 2, EPI>(s, g, splits);
    case GEMM_256x256_W8: return launch_cfg<256, 256, 64, 2, 4, EPI>(s, g, splits);
    default: return hipErrorInvalidValue;
  }
}

int gemm_tile_n(int cfg) {
  switch (cfg) {
    case GEMM_256x256: case GEMM_256x256_W8: case GEMM_64x256: case GEMM_32x256: return 256;
    case GEMM_64x64: return 64;
    default: return 128;
  }
}
int gemm_tile_m(int cfg) {
  switch (cfg) {
    case GEMM_256x256: case GEMM_256x256_W8: case GEMM_256x128: return 256;
    case GEMM_128x128: return 128;
    case GEMM_32x256: return 32;
    default: return 64;
  }
}

// C = A * W^T with the chosen tile configuration and epilogue. Requirements (checked):
// K % 64 == 0, N % tile_n == 0, leading dimensions multiples of 8 elements, M >= 1.
// With splits > 1 (EPI_F32 only) partial sums go to C + z * split_stride.
hipError_t gemm_bf16(hipStream_t s, int cfg, int epi, const bf16* A, int lda, const bf16* W, int ldw,
                     void* C, int ldc, int M, int N, int K, int splits, long long split_stride) {
  if (M < 1 || K % 64 != 0 || N % gemm_tile_n(cfg) != 0 || lda % 8 != 0 || ldw % 8 != 0) return hipErrorInvalidValue;
  if (splits < 1 || (splits > 1 && epi != EPI_F32)) return hipErrorInvalidValue;
  if (epi == EPI_SWIGLU_BF16 && (cfg == GEMM_64x128 || cfg == GEMM_64x64)) return hipErrorInvalidValue;   // wave tile of one block
  GemmArgs g{};
  g.A = A; g.W = W; g.C = C; g.lda = lda; g.ldw = ldw; g.ldc = ldc; g.M = M; g.N = N; g.K = K;
  g.split_stride = split_stride;
  switch (epi) {
    case EPI_BF16: return launch_epi<EPI_BF16>(s, cfg, g, splits);
    case EPI_F32: return launch_epi<EPI_F32>(s, cfg, g, splits);
    case EPI_RESID_F32: return launch_epi<EPI_RESID_F32>(s, cfg, g, splits);
    case EPI_SWIGLU_BF16:
      switch (cfg) {   // instantiated only where the wave tile holds gate/up block pairs
        case GEMM_256x256: return launch_cfg<256, 256, 64, 2, 2, EPI_SWIGLU_BF16>(s, g, 1);
        case GEMM_256x256_W8: return launch_cfg<256, 256, 64, 2, 4, EPI_SWIGLU_BF16>(s, g, 1);
        case GEMM_128x128: return launch_cfg<128, 128, 64, 2, 2, EPI_SWIGLU_BF16>(s, g, 1);
        case GEMM_256x128: return launch_cfg<256, 128, 64, 2, 2, EPI_SWIGLU_BF16>(s, g, 1);
        case GEMM_64x256: return launch_cfg<64, 256, 64, 1, 4, EPI_SWIGLU_BF16>(s, g, 1);
        case GEMM_32x256: return launch_cfg<32, 256, 64, 1, 4, EPI_SWIGLU_BF16>(s, g, 1);
        default: return hipErrorInvalidValue;
      }
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sts
