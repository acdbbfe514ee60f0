// Internal (C++) interface between the engine and the gfx950 kernels. Not part of the C ABI.
#pragma once
#include "common.h"

namespace sts {

// ---- GEMM -------------------------------------------------------------------------------
enum GemmEpilogue { EPI_BF16 = 0, EPI_F32 = 1, EPI_RESID_F32 = 2, EPI_SWIGLU_BF16 = 3 };
// the same numbering as STS_GEMM_* in sts.h
enum GemmConfig { GEMM_128x128 = 0, GEMM_64x256 = 1, GEMM_64x128 = 2, GEMM_256x256 = 3, GEMM_128x256 = 4, GEMM_64x256S = 5, GEMM_64x320S = 6, GEMM_64x384S = 7,
                  GEMM_64x448S = 8, GEMM_64x512S = 9, GEMM_NCFG = 10 };
int gemm_tile_m(int cfg);
int gemm_tile_n(int cfg);
int gemm_wgs_per_cu(int cfg);                       // resident workgroups per CU of this configuration
// Tail splitting: `slots` = workgroups the stream's CU partition holds at once, `ws` = fp32 scratch.
struct GemmTail { int slots; float* ws; size_t ws_bytes; };
void gemm_tail_plan(int tiles, int ksteps, int slots, long long max_pieces, int* n_full, int* f);
// W is either row-major [N, ldw] or (w_packed, the engine's weights; needs ldw == K) in
// the packed layout below. The row-major form exists for the fp32-store epilogue only.
hipError_t gemm_bf16(hipStream_t s, int cfg, int epi, const bf16* A, int lda, const bf16* W, int ldw,
                     void* C, int ldc, int M, int N, int K, int splits, long long split_stride,
                     const GemmTail* tail = nullptr, bool w_packed = true, bool stream_nt = false);

// Packed GEMM weights: blocks of 32 rows x 64 columns (4 KiB), stored one after the other along K, then
// along N. A block is laid out the way the matrix cores take a W operand: four pieces of 1 KiB, one per
// 16-column step, each holding for lane l = 32 * h + n of a wave the 8 consecutive elements
// W[row n][16 * step + 8 * h .. + 8). A wave therefore loads an operand straight into registers with one
// 16-byte load per lane from 1 KiB of consecutive memory (the large prefill tile does that, and keeps W
// out of LDS), and the direct-to-LDS loads of the other tiles gather the same bytes in whole 128-byte
// pieces (8 rows of one half-step). A tile's share of a K step is whole 4 KiB blocks instead of one
// 128-byte piece out of each of its rows (rows are K * 2 bytes apart), which is what HBM-bound decode
// GEMMs want. N must be a multiple of 32 and K of 64.
__host__ __device__ __forceinline__ size_t weight_packed_index(int row, int col, int ld) {
  const size_t block = (size_t)(row >> 5) * (ld >> 6) + (col >> 6);
  return block * 2048 + (size_t)((col & 63) >> 4) * 512 + (size_t)((((col >> 3) & 1) << 5) + (row & 31)) * 8 + (col & 7);
}

// ---- paged KV layout ----------------------------------------------------------------------
// One layer's pool is [n_pages][n_kv_heads][ K: page_tokens x d | V^T: d x page_tokens ] bf16.
// V is kept transposed inside a page so that the P*V contraction (over tokens) reads
// token-contiguous operands, as the MFMA operand layout wants.
struct KvGeom {
  int n_kv, d, page_tokens;
  __host__ __device__ size_t head_elems() const { return (size_t)2 * page_tokens * d; }
  __host__ __device__ size_t page_elems() const { return head_elems() * n_kv; }
};

// Per-sequence metadata of one prefill launch (device array, one entry per sequence).
struct PrefillSeq {
  int row0;        // first row of this sequence in the packed activation buffers
  int sl;          // new tokens
  int p;           // tokens already cached (positions 0..p-1)
  int bt_off;      // offset of this sequence's block table in the block-table buffer
  int n_pages;     // valid entries in that block table
};
struct AttnItem { int seq; int q0; };   // one query tile of one sequence

// Per-request metadata of one decode step.
struct DecodeSeq {
  int cl;          // tokens already cached; the new token sits at position cl
  int bt_off;
  int n_pages;     // pages covering positions 0..cl
};

// One context chunk of one decode request, with what its workgroup needs to start: a single
// 16-byte load instead of a chain through the per-request record.
struct DecodeItem { int seq; int chunk; int cl; int bt_off; };

// ---- element-wise / small kernels ---------------------------------------------------------
hipError_t init_weight(hipStream_t s, bf16* dst, int ld, uint64_t seed, uint64_t tensor_id, int rows, int cols,
                       int row_offset, int interleave_block, int interleave_phase, int packed);
hipError_t convert_weight(hipStream_t s, bf16* dst, int ld, const float* src, int rows, int cols,
                          int row_offset, int interleave_block, int interleave_phase, int packed);
hipError_t export_weight(hipStream_t s, float* dst, const bf16* src, int ld, int rows, int cols,
                         int row_offset, int interleave_block, int interleave_phase, int packed);
hipError_t fill_f32(hipStream_t s, float* dst, float v, size_t n);
hipError_t embed_rows(hipStream_t s, float* X, const bf16* emb, const int* tokens, int n, int h);
// embedding rows into the fp32 residual stream X and, in the same pass, their RMSNorm into out (bf16); h <= 8192
hipError_t embed_norm_rows(hipStream_t s, float* X, bf16* out, const bf16* emb, const int* tokens, const float* gain, float eps, int n, int h);
hipError_t rmsnorm_rows(hipStream_t s, bf16* out, const float* X, const float* gain, float eps, int n, int h);
hipError_t gather_rows_f32(hipStream_t s, float* dst, const float* src, const int* rows, int n, int h);
hipError_t rope_kv_write_prefill(hipStream_t s, bf16* qkv, int ld, const PrefillSeq* seqs, int n_seqs,
                                 const int* block_tables, const double* inv_freq, bf16* pool, KvGeom geo,
                                 int n_rows, int n_q);
hipError_t decode_qkv_finish(hipStream_t s, const float* partials, int splits, long long split_stride, int ld,
                             const DecodeSeq* seqs, const int* block_tables, const double* inv_freq,
                             bf16* q_out, bf16* pool, KvGeom geo, int n, int n_q);
hipError_t reduce_resid_norm(hipStream_t s, float* X, const float* partials, int splits, long long split_stride,
                             bf16* out_norm, const float* gain, float eps, int n, int h);
hipError_t reduce_swiglu(hipStream_t s, bf16* H, const float* partials, int splits, long long split_stride,
                         int n, int mlp);
hipError_t reduce_f32(hipStream_t s, float* out, const float* partials, int splits, long long split_stride, size_t n);
hipError_t argmax_rows(hipStream_t s, int* out, const float* logits, int n, int vocab);
hipError_t copy_probe(hipStream_t s, void* dst, const void* src, size_t bytes, int grid);
hipError_t read_probe(hipStream_t s, const void* src, size_t bytes, unsigned* sink, int grid);    // the read half alone; sink: 4 bytes of device memory
hipError_t kv_fill_random(hipStream_t s, bf16* pool, KvGeom geo, const int* block_table, int pos0, int n,
                          uint64_t seed, int layer);
hipError_t kv_write_tokens(hipStream_t s, bf16* pool, KvGeom geo, const int* block_table, int pos0, int n,
                           const float* k, const float* v);
hipError_t kv_read_tokens(hipStream_t s, const bf16* pool, KvGeom geo, const int* block_table, int pos0, int n,
                          float* k, float* v);

// ---- attention ----------------------------------------------------------------------------
hipError_t attn_prefill(hipStream_t s, const bf16* qkv, int ld, bf16* out, int ldo, const PrefillSeq* seqs,
                        const AttnItem* items, int n_items, const int* block_tables, const bf16* pool,
                        KvGeom geo, int n_q);
int attn_prefill_tile_q();
size_t attn_decode_ws_floats(int n, int n_q, int d, int max_chunks);
hipError_t attn_decode(hipStream_t s, const bf16* q, bf16* out, const DecodeSeq* seqs, const DecodeItem* items, int n_items, const int* multi, int n_multi,
                       const int* block_tables, const bf16* pool, KvGeom geo, int n, int n_q, int chunk_pages, int max_chunks, float* ws,
                       bool stream_nt = false);
int attn_decode_max_chunk_tokens();

}  // namespace sts
