/* libsts — spatial-temporal prefill/decode sharing on one MI355X (gfx950): C ABI.
 *
 * The calls follow the serving method of arXiv 2504.19516: a transformer step in which a
 * compute-bound prefill pass and a memory-bound decode pass run at the same time on disjoint
 * compute-unit (CU) partitions of one GPU (Sections 3.1, 3.4, 3.5), a performance estimator
 * (the SM-scaling roofline model, Section 3.2) that predicts each phase's latency on its
 * partition, and an SLO-aware scheduler (Section 3.3, Algorithm 1) that picks the prefill
 * batch, the layer slice and the CU split for each step.
 *
 * Conventions
 *   - Every function returns 0 (STS_OK) or a negative STS_E* code; sts_strerror() names it.
 *     STS_EHIP means a HIP runtime call failed: sts_last_hip_error() returns its code.
 *   - Pointers are HOST pointers unless a parameter says "device". Host buffers are owned by
 *     the caller and are only read or written during the call. All device memory, streams
 *     and KV pages are owned by the library (allocated in sts_init, released in sts_destroy).
 *   - Calls are synchronous: outputs are complete when the call returns.
 *   - One control thread per phase may call concurrently (sts_prefill_* next to
 *     sts_decode_step) as long as they touch disjoint sequences; page allocation is
 *     serialised internally (Section 3.5.1). Everything else is single-threaded.
 *   - sts_profile_*, sts_latency_*, sts_wave_quant, sts_sched_* touch no GPU state and work on
 *     a host without a GPU.
 *   - Without a usable GPU sts_init fails with STS_EHIP; there is no CPU fallback.
 */
#ifndef STS_H
#define STS_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

enum { STS_OK = 0, STS_EINVAL = -1, STS_ENOMEM = -2, STS_ESTATE = -3, STS_EHIP = -4, STS_EIO = -5 };
const char* sts_strerror(int code);
int sts_last_hip_error(void);

typedef struct sts_ctx sts_ctx;
typedef struct sts_profile sts_profile;

/* Model shape: Llama-style decoder blocks (Section 2.1: QKV projection, self-attention,
 * output projection, MLP, element-wise operations between them) with RMSNorm, rotary
 * embedding (half-split pairing), grouped-query attention, SwiGLU, no biases.
 * Requirements: head_dim 64 or 128; page_tokens 16; hidden, mlp multiples of 64;
 * (n_q_heads + 2 n_kv_heads) * head_dim, hidden, 2*mlp and vocab multiples of 128. */
typedef struct {
  int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, mlp, vocab, page_tokens;
  float rope_theta, rms_eps;
} sts_model_desc;

typedef struct {
  uint64_t weight_seed;        /* seed of the on-device weight generator */
  int32_t init_weights;        /* 1: generate N(0,0.02)-like weights on device (norm gains = 1);
                                  0: leave weights zero, caller uses sts_load_weights */
  int32_t kv_pool_pages;       /* pages in the shared KV pool; a page holds page_tokens tokens of every layer */
  int32_t max_prefill_tokens;  /* rows of the prefill activation workspace (sum over a batch) */
  int32_t max_prefill_seqs;    /* sequences per prefill batch */
  int32_t max_decode_batch;    /* requests per decode step */
  int32_t max_seqs;            /* live sequences */
  int32_t max_pages_per_seq;   /* block-table length; at most sts_max_pages_per_seq_limit(page_tokens) */
} sts_init_params;

/* ---- lifetime (Section 3.5.1: weights and the KV pool are allocated once, before serving,
 *      and shared by both phases) */
int sts_init(const sts_model_desc* desc, const sts_init_params* params, sts_ctx** out);
/* Waits for everything the ctx queued (on every partition's stream it ever selected and on the
 * null stream), then releases its memory. The CU-masked streams themselves belong to the process
 * and stay. */
int sts_destroy(sts_ctx* ctx);
/* Optional, as the last call of a process: waits on and destroys the process-wide CU-masked streams
 * (Section 3.5.2's partitions are streams with a CU mask; the library creates one per side and CU
 * count on first use and otherwise keeps them until the process ends). STS_ESTATE while any ctx is
 * alive; afterwards sts_init returns STS_ESTATE (masked streams are not created a second time in one
 * process). For programs that load the HIP runtime late (an interpreter) and run under a profiler
 * whose exit handler walks the queues still open: a masked stream left open there has ended such
 * runs with a fault after all output was written. Destroying a masked stream after work has run on it
 * has twice been seen not to return on this software stack: call this only where a kill timer guards
 * the process (profiler runs); a program that simply exits needs no call. */
int sts_release_streams(void);
/* Longest block table sts_init accepts: decode attention cuts a context into at most 128 chunks of
 * at most 64 pages (Section 3.5.1's pool is shared, a sequence's share of it is bounded by this). */
int sts_max_pages_per_seq_limit(int32_t page_tokens);
/* Host only, no GPU state: how a decode step over contexts of n_pages[i] pages is cut into chunks on
 * a partition of `cus` CUs (pages per chunk, chunks of the longest context), next to the chunk count
 * the engine allocates its merge workspace and work list for when max_pages_per_seq is the bound.
 * max_chunks <= allocated_chunks holds for every input sts_init accepts. */
int sts_decode_chunk_plan(const int32_t* n_pages, int32_t n, int32_t n_kv_heads, int32_t cus, int32_t page_tokens,
                          int32_t max_pages_per_seq, int32_t* chunk_pages, int32_t* max_chunks, int32_t* allocated_chunks);

/* Host only, no GPU state: tile configuration (STS_GEMM_*) and split along K the engine gives a decode-side GEMM of m rows
 * (one token per request), n weight rows and k columns on a partition of `cus` CUs. Up to 64 rows the GEMM streams its
 * weights once and is planned by an estimate of rounds of workgroups and bytes per CU over the 64x128 tile and the skinny tiles
 * whose width divides n (Section 2.1: decode is bound by memory bandwidth; Section 3.2.1: what a partition can pull grows with
 * its CUs only up to a point); above that it takes a prefill tile shape. may_split: a split along K is allowed (its fp32 partial
 * sums are reduced by the caller's next kernel); partials: the output leaves as fp32 partial sums even when unsplit (0 = the
 * GEMM's own epilogue finishes it, as the fused SwiGLU of an unsplit gate/up GEMM does). gemm_rate_256 and partial_bw_cu: the
 * tile model's values (see sts_set_tile_model); stream_bw_cu and stream_bw_gpu: the stream model's (sts_set_stream_model).
 * est_ns (may be NULL): the estimate behind the choice. n: a multiple of 128, k: a multiple of 64, else STS_EINVAL. */
int sts_decode_gemm_plan(int32_t m, int32_t n, int32_t k, int32_t cus, int32_t may_split, int32_t partials, int64_t gemm_rate_256,
                         int64_t partial_bw_cu, int64_t stream_bw_cu, int64_t stream_bw_gpu, int32_t* tile_cfg, int32_t* split_k,
                         int64_t* est_ns);

/* Weights. `name`: "emb", "lm" (layer ignored), "wq","wk","wv","wo","wg","wu","wd" (matrices,
 * row-major [out_features, in_features] fp32, rounded to bf16 on upload) or "g1","g2","gf"
 * (gains, fp32 [hidden]). `count` = number of fp32 elements and must match the tensor. */
int sts_load_weights(sts_ctx* ctx, int32_t layer, const char* name, const float* host, size_t count);
int sts_read_weights(sts_ctx* ctx, int32_t layer, const char* name, float* host, size_t count);

/* ---- sequences and the paged KV cache (Section 3.5.1). Token t of a sequence lives in page
 *      block_table[t / page_tokens], slot t % page_tokens, in every layer. */
int sts_seq_create(sts_ctx* ctx, int32_t* seq_out);
int sts_seq_free(sts_ctx* ctx, int32_t seq);                       /* pages return to the pool; STS_ESTATE while the sequence is part of
                                                                      a layer-sliced prefill batch or of a launch whose finish is due */
int sts_seq_length(sts_ctx* ctx, int32_t seq, int32_t* len_out);
/* Drop the tokens from position new_len on (a rollback: the cache entries before it stay as they are, the pages stay with
 * the sequence). STS_EINVAL if new_len exceeds the length, STS_ESTATE as for sts_seq_free. */
int sts_seq_truncate(sts_ctx* ctx, int32_t seq, int32_t new_len);
int sts_seq_reserve(sts_ctx* ctx, int32_t seq, int32_t n_tokens);  /* make pages cover n_tokens; STS_ENOMEM leaves state unchanged */
int sts_pages_free(sts_ctx* ctx, int32_t* n_out);
/* Test hooks. set_block_table: give an EMPTY sequence these pool pages, in this order (they are
 * taken from the free list; STS_EINVAL if any is in use). get_block_table copies up to cap entries. */
int sts_seq_set_block_table(sts_ctx* ctx, int32_t seq, const int32_t* pages, int32_t n);
int sts_seq_get_block_table(sts_ctx* ctx, int32_t seq, int32_t* pages, int32_t cap, int32_t* n_out);
/* Write / read K and V of positions [pos0, pos0+n) of one layer, fp32 [n, n_kv_heads, head_dim]
 * (rounded to bf16 on write). kv_write extends the sequence length to pos0+n if shorter.
 * kv_fill_random fills positions [0, n) of EVERY layer with unit-variance deviates of the
 * library's counter-based generator (synthetic contexts) and sets the length to n. */
int sts_kv_write(sts_ctx* ctx, int32_t layer, int32_t seq, int32_t pos0, int32_t n, const float* k, const float* v);
int sts_kv_read(sts_ctx* ctx, int32_t layer, int32_t seq, int32_t pos0, int32_t n, float* k, float* v);
int sts_kv_fill_random(sts_ctx* ctx, int32_t seq, int32_t n, uint64_t seed);

/* ---- the step (Sections 3.3.1 and 3.5.2)
 * Prefill: append lens[i] new tokens to sequence seqs[i] (after whatever it already caches)
 * and run layers [layer_begin, layer_end) — the layer slice the scheduler launches per step.
 * Slices of one batch must be issued in order, starting at 0, with the same batch; the hidden
 * state stays on the device in between (STS_ESTATE otherwise). When layer_end == n_layers the
 * sequences' lengths grow and, if `logits` is not NULL, the last token's logits of each
 * sequence are written to logits[n_seqs, vocab] (fp32). tokens: all sequences' new tokens
 * concatenated. STS_ENOMEM (pool exhausted) leaves every sequence unchanged. */
int sts_prefill_batch(sts_ctx* ctx, int32_t n_seqs, const int32_t* seqs, const int32_t* lens, const int32_t* tokens,
                      int32_t layer_begin, int32_t layer_end, float* logits);
int sts_prefill_append(sts_ctx* ctx, int32_t seq, const int32_t* tokens, int32_t n_tokens,
                       int32_t layer_begin, int32_t layer_end, float* logits);
/* The same two calls split into launch / poll / finish, so that one control thread can keep a
 * prefill slice and a decode step in flight at once and react to whichever ends first
 * (Section 3.3.1: the two phases advance independently). A phase has at most one launch
 * outstanding (STS_ESTATE otherwise); the blocking calls and sts_step_concurrent refuse to run
 * while one is. *_finish waits for the launch, updates sequence lengths and copies the outputs
 * that the launch asked for (pass NULL for the others). */
int sts_prefill_launch(sts_ctx* ctx, int32_t n_seqs, const int32_t* seqs, const int32_t* lens, const int32_t* tokens,
                       int32_t layer_begin, int32_t layer_end, int32_t want_logits);
int sts_decode_launch(sts_ctx* ctx, const int32_t* seqs, const int32_t* in_tokens, int32_t n, int32_t want_logits, int32_t want_next);
int sts_phase_done(sts_ctx* ctx, int32_t phase /*0 prefill, 1 decode*/, int32_t* done);
int sts_prefill_finish(sts_ctx* ctx, float* logits);
int sts_decode_finish(sts_ctx* ctx, float* logits, int32_t* next_tokens);
/* Drop the in-flight layer-sliced batch, if any: its sequences keep their old lengths (the pages
 * reserved for the new tokens stay with them until they are freed). */
int sts_prefill_abort(sts_ctx* ctx);
/* Decode: one new token per request through all layers; request i feeds in_tokens[i] at
 * position length(seqs[i]) and attends to everything cached plus itself; lengths grow by 1.
 * logits [n, vocab] and next_tokens [n] (greedy, lowest index wins ties) may each be NULL;
 * with both NULL the LM head is skipped. */
int sts_decode_step(sts_ctx* ctx, const int32_t* seqs, const int32_t* in_tokens, int32_t n,
                    float* logits, int32_t* next_tokens);
/* Both at once: the prefill slice on the prefill partition's stream and the decode step on the
 * decode partition's stream, launched back to back with no synchronisation between them, one
 * join at the end (Section 3.3.1). The two must touch disjoint sequences. Either side may be
 * empty (n == 0). Both sides are validated and the pages of both are reserved before anything is
 * queued: STS_EINVAL, STS_ESTATE or STS_ENOMEM from either side leaves every sequence unchanged
 * and nothing launched. */
int sts_step_concurrent(sts_ctx* ctx,
                        int32_t n_pseqs, const int32_t* pseqs, const int32_t* plens, const int32_t* ptokens,
                        int32_t layer_begin, int32_t layer_end, float* plogits,
                        const int32_t* dseqs, const int32_t* dtokens, int32_t n_decode,
                        float* dlogits, int32_t* dnext);
/* Device time of the last call's prefill part and decode part (HIP events on their own
 * streams), and the wall-clock span of the call. A part that did not run, or whose launch is
 * still in flight (sts_*_launch without its finish), reports 0. */
int sts_last_timing(sts_ctx* ctx, int64_t* prefill_ns, int64_t* decode_ns, int64_t* wall_ns);
/* Test hook: hidden state (residual stream) after the last call of a phase, fp32 [rows, hidden];
 * phase 0 = prefill batch rows, 1 = decode rows. */
int sts_read_hidden(sts_ctx* ctx, int32_t phase, float* out, int32_t rows);

/* ---- CU partition (Section 3.4). prefill_cus / decode_cus: CUs given to each phase, each a
 * multiple of 8 (every XCD must keep a CU of a partition) in [8, total], or 0 = phase
 * suspended. Prefill takes CU-mask bits [0, prefill_cus), decode takes the top decode_cus
 * bits; they are disjoint when prefill_cus + decode_cus <= total. prefill_cus == decode_cus
 * == total is the time-multiplexed configuration (both phases see the whole GPU). -1 leaves
 * that phase as it is; a phase with a launch outstanding cannot be changed (STS_ESTATE).
 * Takes effect for the next call; masked streams are created on first use and cached. */
int sts_set_partition(sts_ctx* ctx, int32_t prefill_cus, int32_t decode_cus);
int sts_get_partition(sts_ctx* ctx, int32_t* prefill_cus, int32_t* decode_cus, int32_t* total_cus);

/* ---- measurement hooks
 * Per-kernel timing: when on, every kernel launch of both phases is bracketed by HIP events on
 * its stream (this serialises nothing but adds event overhead; leave off when timing steps).
 * kernel_times returns, per phase and kernel kind (STS_K_*), accumulated device ns and launch
 * counts since the last reset. */
enum { STS_K_EMBED = 0, STS_K_NORM, STS_K_QKV, STS_K_ROPE, STS_K_ATTN, STS_K_ATTN_MERGE, STS_K_O, STS_K_GATEUP,
       STS_K_SWIGLU, STS_K_DOWN, STS_K_REDUCE, STS_K_HEAD, STS_K_SAMPLE, STS_K_COUNT };
int sts_kernel_timing(sts_ctx* ctx, int32_t on);
int sts_kernel_times(sts_ctx* ctx, int32_t phase, int64_t* ns /*[STS_K_COUNT]*/, int64_t* launches /*[STS_K_COUNT]*/, int32_t reset);
const char* sts_kernel_name(int32_t kind);
/* Copy-kernel bandwidth on `cus` CUs of a phase's partition side (0 = prefill side, 1 = decode
 * side): the memory-copy probe of Section 3.2.2. Moves `bytes` (read + written = 2*bytes) per
 * iteration; returns device ns for `iters` iterations. */
int sts_probe_copy(sts_ctx* ctx, int32_t side, int32_t cus, size_t bytes, int32_t iters, int64_t* ns_out);
/* The same probe without the writes: a read-only stream over `bytes` per iteration (non-temporal loads). What a decode
 * partition can pull at best; the offline profiler stores its rate per CU at 32 CUs and on the whole GPU in the profile
 * (stream_bw_cu, stream_bw_gpu) for the decode GEMM planner. */
int sts_probe_read(sts_ctx* ctx, int32_t side, int32_t cus, size_t bytes, int32_t iters, int64_t* ns_out);

/* One of the prefill side's GEMMs (layer 0's weights, whatever the workspace holds as activations; the residual
 * stream of the workspace is overwritten) with a given tile configuration on `cus` CUs, whole tiles only: m rows
 * (<= max_prefill_tokens) and n weight rows (a multiple of the tile width). product 0: gate/up with its SwiGLU
 * epilogue, K = hidden, n <= 2 * mlp (not for the tile shapes without a SwiGLU form); 1: the O projection, K = the
 * query width, n <= hidden, residual epilogue; 2: the down projection, K = mlp, n <= hidden, residual epilogue.
 * Returns device ns for `iters` launches. The offline profiler (Section 3.2.4) times the tile shapes with it. */
int sts_probe_gemm(sts_ctx* ctx, int32_t cus, int32_t tile_cfg, int32_t product, int32_t m, int32_t n, int32_t iters, int64_t* ns_out);
/* What the engine's choice of GEMM tile and of the cut of a partly filled last wave (Section 2.2.1) assumes about
 * the part: GFLOP/s per busy CU of the 128x128 tiles (two workgroups per CU), of the 256x256 tiles (one) and of the
 * 128x256 tiles (planned one per CU, for the projections with a residual epilogue; their start-up and epilogue are
 * not hidden behind a second workgroup, so a tile costs gemm_fixed_128x256 ns plus its flops at the rate), and MB/s
 * per CU for partial tiles written and read back. The offline profiler measures them and stores them in the
 * profile (sts_profile_tile_model reads them back); until set, figures measured on the 8B shape apply. Takes
 * effect for the next launch; STS_ESTATE while a launch is outstanding. */
int sts_set_tile_model(sts_ctx* ctx, int64_t gemm_rate_128, int64_t gemm_rate_256, int64_t gemm_rate_128x256, int64_t gemm_fixed_128x256,
                       int64_t partial_bw_cu);
/* What the planner of the decode GEMMs (sts_decode_gemm_plan) assumes about the memory system: MB/s a read-only stream reaches
 * per CU of a 32-CU partition, and on the whole GPU (sts_probe_read measures both; the profile keeps them, see
 * sts_profile_stream_model). Until set, figures measured on one MI355X apply (59000, 6400000). stream_bw_gpu >= stream_bw_cu. */
int sts_set_stream_model(sts_ctx* ctx, int64_t stream_bw_cu, int64_t stream_bw_gpu);

/* ---- single operations on host data, for per-kernel parity tests. Inputs are fp32 and are
 * rounded to bf16 on upload; outputs are the kernel's fp32 accumulators (or its bf16 result
 * widened). They use the default stream and their own temporary device buffers. */
/* Host-only: element index of W[row][col] (ld = K columns, a multiple of 64) in the packed layout the GEMM weights are
 * kept in -- blocks of 32 rows x 64 columns, each four 1 KiB pieces in the order the matrix cores take a W operand
 * (lane 32 h + n of a wave holds W[row n][16 step + 8 h .. + 8)). -1 for arguments out of range. Needs no GPU. */
int64_t sts_weight_packed_index(int32_t row, int32_t col, int32_t ld);

/* C[M,N] = A[M,K] * W[N,K]^T. tile_cfg: STS_GEMM_*; epilogue 0 = bf16 store, 1 = fp32 store
 * (split_k >= 1 partial sums are added up on the device), 2 = C += (C given in c_inout),
 * 3 = SwiGLU: W holds gate rows then up rows ([2*N2, K]); output [M, N2].
 * tail_slots > 0 (needs split_k == 1): launch as on a partition that holds tail_slots
 * workgroups at once -- the tiles of the last, partly filled wave (Section 2.2.1) are cut along
 * K into pieces that fill the wave, and a second kernel sums the pieces. 0 = whole tiles only. */
enum { STS_GEMM_128x128 = 0 /* 4 waves, two workgroups per CU */, STS_GEMM_64x256 /* 8 waves */, STS_GEMM_64x128 /* 4 waves, two per CU */,
       STS_GEMM_256x256 /* 8 waves */, STS_GEMM_128x256 /* 4 waves, planned one per CU; no SwiGLU epilogue */,
       /* decode batches: 64-row tiles of 4 to 8 waves, 64 columns per wave, the weights of the library's packed
          layout streamed straight into registers (no row-major form: sts_op_gemm_noalloc rejects them; whole tiles
          only: tail_slots is ignored) */
       STS_GEMM_64x256S /* two workgroups per CU */, STS_GEMM_64x320S, STS_GEMM_64x384S, STS_GEMM_64x448S, STS_GEMM_64x512S };
int sts_op_gemm(const float* a, const float* w, float* c_inout, int32_t m, int32_t n, int32_t k,
                int32_t tile_cfg, int32_t epilogue, int32_t split_k, int32_t tail_slots);
/* sts_op_gemm's fp32-store form (epilogue 1) for callers that cannot allocate -- code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc. a_dev [m, k] and w_dev [n, k]
 * are DEVICE pointers to bf16 (row-major, K contiguous), c_dev [m, n] a DEVICE pointer to fp32; all
 * three are the caller's and must stay valid until the work has run. The kernels are queued on
 * `stream` (a hipStream_t, NULL = the null stream) and the call returns without waiting for them.
 * The split-K partial sums (split_k > 1) or the partial tiles of a cut last wave (tail_slots > 0,
 * needs split_k == 1) go to a fixed device array of STS_NOALLOC_SCRATCH_BYTES that every GPU running
 * this library holds until the process ends; a call whose scratch need (split_k * m * n floats, or
 * tail_slots tiles of the configuration's size) exceeds it returns STS_EINVAL, as do k % 64 != 0 and
 * n not a multiple of the tile width. Nothing in the array has to start at zero (every element read
 * was written by the same call), and its contents after the call are unspecified. All calls on one
 * GPU share the array: calls that may overlap on one GPU (different streams, or different threads)
 * race and must be serialised by the caller. No hipMalloc, hipFree or other allocating routine runs. */
#define STS_NOALLOC_SCRATCH_BYTES ((size_t)32 << 20)
int sts_op_gemm_noalloc(const void* a_dev, const void* w_dev, float* c_dev, int32_t m, int32_t n, int32_t k,
                        int32_t tile_cfg, int32_t split_k, int32_t tail_slots, void* stream);
/* Causal attention of a chunk: q [t, n_q, d], k and v [prior + t, n_kv, d]; query i sits at
 * position prior + i. K,V go through a paged pool with the given page order (pages[] of
 * ceil((prior+t)/16) distinct ids < n_pool_pages). out [t, n_q, d]. */
int sts_op_attn_prefill(const float* q, const float* k, const float* v, float* out, int32_t t, int32_t prior,
                        int32_t n_q, int32_t n_kv, int32_t d, const int32_t* pages, int32_t n_pool_pages);
/* Decode attention: q [n, n_q, d]; request r has ctx[r] cached tokens given in k,v (concatenated
 * over requests, [sum ctx, n_kv, d]) and attends to all of them. A context is cut into
 * ceil(pages / chunk_pages) equal chunks (chunk_pages 1..64) whose partial results are merged; a
 * context of one chunk is finished by the attention kernel itself. out [n, n_q, d].
 * STS_EINVAL for a chunk size out of range. */
int sts_op_attn_decode(const float* q, const float* k, const float* v, float* out, int32_t n, const int32_t* ctx,
                       int32_t n_q, int32_t n_kv, int32_t d, int32_t chunk_pages);

/* ---- performance estimator (Section 3.2) — host only, integer arithmetic.
 * Wave quantisation (Section 2.2.1): g workgroups on n units, b workgroups per unit. */
int sts_wave_quant(int64_t g, int64_t n, int64_t b, int64_t* waves, int64_t* tail, int64_t* idle_num, int64_t* idle_den);

/* Profile = hardware constants (C_peak flop/ns, D_peak bytes/ns, inflection N_d, tile sizes)
 * plus sample grids: bw (D_{p,sl}: decode CUs x co-running prefill tokens -> bytes/ns),
 * alpha_prefill (CUs x tokens -> alpha ppm), alpha_decode (CUs x batch x mean context per request -> ppm),
 * and optionally prefill_corun (decode CUs beside the slice -> slowdown ppm of a prefill slice that shares
 * the memory system with a decode step on a disjoint CU set; Section 3.2.3 treats this direction of the
 * contention as small, a measured table keeps it where it is not). Text format: see sts_profile_dump. */
int sts_profile_parse(const char* text, sts_profile** out);
int sts_profile_load(const char* path, sts_profile** out);
int sts_profile_dump(const sts_profile* p, char* buf, size_t cap, size_t* needed);
int sts_profile_free(sts_profile* p);
/* The profile's tile-model entries (see sts_set_tile_model); each output may be NULL. */
int sts_profile_tile_model(const sts_profile* p, int64_t* gemm_rate_128, int64_t* gemm_rate_256, int64_t* gemm_rate_128x256,
                           int64_t* gemm_fixed_128x256, int64_t* partial_bw_cu);
/* The profile's stream-model entries (see sts_set_stream_model); each output may be NULL. */
int sts_profile_stream_model(const sts_profile* p, int64_t* stream_bw_cu, int64_t* stream_bw_gpu);

/* Execution state ES (Section 3.2.1): prefill lengths sl_i with their cached contexts, prefill
 * CUs pm, decode contexts cl_i (batch size = n_decode), decode CUs dm; plus the layer slice. */
typedef struct {
  int32_t n_prefill; const int32_t* prefill_len; const int32_t* prefill_ctx;
  int32_t n_decode; const int32_t* decode_ctx;
  int32_t prefill_cus, decode_cus;
  int32_t layer_begin, n_layers_step;
} sts_exec_state;
#define STS_INF_NS ((int64_t)1 << 60)
/* Eq. 1 summed over the kernels of the slice (prefill) / the whole step (decode), times the
 * interpolated alpha of Eq. 2. A phase with work but zero CUs gets STS_INF_NS; no work -> 0.
 * When es holds a decode batch on CUs disjoint from the prefill CUs (prefill_cus + decode_cus within
 * the CU count), the prefill figure also carries the profile's prefill_corun factor at decode_cus. */
int sts_latency_query(const sts_profile* p, const sts_model_desc* desc, const sts_exec_state* es,
                      int64_t* prefill_ns, int64_t* decode_ns);
/* Online recalibration (Section 3.2.4): feed one measured prefill slice and/or decode step at
 * execution state es back into the profile. Eq. 2 gives alpha_obs = measured / T' at es; every
 * alpha sample the interpolation at es reads moves by weight_ppm/1e6 * (alpha_obs /
 * alpha_predicted - 1) of its value, so the prediction at es moves that share of the way.
 * A measurement <= 0 skips that phase. Integer arithmetic; not thread-safe against queries on the
 * same profile. */
int sts_profile_observe(sts_profile* p, const sts_model_desc* desc, const sts_exec_state* es,
                        int64_t measured_prefill_ns, int64_t measured_decode_ns, int64_t weight_ppm);
/* The uncalibrated roofline sums T'_{p,ES} (alpha not applied): what a measurement is divided by
 * to obtain alpha (Eq. 2). */
int sts_latency_roofline(const sts_profile* p, const sts_model_desc* desc, const sts_exec_state* es,
                         int64_t* prefill_ns, int64_t* decode_ns);

/* ---- SLO-aware scheduler (Section 3.3, Algorithm 1) — host only, deterministic.
 * Replays an arrival trace in simulated time (the clock advances by the estimator's
 * predictions), logging one decision record per scheduling cycle. */
typedef struct {
  int64_t ttft_slo_ns, tpot_slo_ns;   /* Gamma_p, Gamma_d */
  int32_t layers_per_step;            /* L_step */
  int32_t max_batch_tokens;           /* prefill workspace rows */
  int32_t max_decode_batch;
  int32_t kv_pool_pages;
  int32_t mode;                       /* 0 concurrent + Algorithm 1; 1 time-multiplexed (full GPU, serialised);
                                         2 concurrent, fixed disjoint split (fixed_prefill_cus / rest);
                                         ablations of Section 4.5: 3 Naive (both phases on every CU, arrival
                                         order, decode never delayed), 4 w/Partition (split search only:
                                         arrival order, decode never suspended), 5 w/Scheduler (reordering
                                         and delayed decode only, both phases on every CU); 6 Section 4.4:
                                         prefill on fixed_prefill_cus, decode on every CU. Modes 3, 5, 6
                                         overlap the two CU sets; the replay's simulated durations ignore
                                         that contention, so their timing is meaningful on the GPU only */
  int32_t fixed_prefill_cus;
  int32_t decode_boost_cus;           /* end-of-prefill boost (Section 3.3.1): while the final slice of a prefill
                                         batch runs, decode gets this many extra CUs (a multiple of the granule,
                                         0 = off; modes 0, 2, 4, only when decode runs). The prefill set is kept,
                                         so the two CU sets intersect for that slice; the simulated durations
                                         ignore the contention */
  int32_t min_batch_tokens;           /* batching floor, not in the paper: a new prefill batch keeps taking queued
                                         requests until it holds this many tokens, also past the roofline ridge at
                                         which Algorithm 1 stops batching (0 = the paper's rule alone) */
} sts_sched_config;
typedef struct {                      /* one scheduling cycle of the prefill scheduler */
  int64_t t_ns;                       /* simulated time of the decision */
  int32_t n_tasks;                    /* requests in next_tasks */
  int32_t first_req;                  /* lowest request id in next_tasks, -1 if none */
  int64_t tasks_hash;                 /* order-sensitive hash of the request ids in next_tasks */
  int32_t layer_begin, layer_end;     /* L_exe, L_exe + L_step */
  int32_t prefill_cus, decode_cus;    /* the split chosen */
  int32_t branch;                     /* 0 none, 1 SetBalancedSM, 2 ReduceDecodeSM, 3 ReducePrefillSM */
  int32_t decode_batch;               /* decode batch size seen */
  int64_t predicted_ns;               /* predicted duration of the slice */
} sts_decision;
typedef struct {
  int64_t n_requests, n_finished;
  int64_t out_tokens, makespan_ns;
  int64_t ttft_sum_ns, tpot_sum_ns, n_tpot;
  int64_t n_slo_ok;                   /* TTFT <= Gamma_p and mean TPOT <= Gamma_d */
  int64_t n_decisions;
} sts_replay_stats;
/* One scheduling cycle of Algorithm 1 on a caller-maintained system state S = (ES, PS, RS)
 * (Section 3.3.2), for serving loops that run the real kernels. queue: Q in arrival order;
 * inflight: P with layers_done = L_exe; decode: the running decode batch followed by the requests
 * prefilled but not merged yet. The choice lists next_tasks (ids, in batch order), the queue
 * that remains (reordered ids), whether next_tasks were newly admitted from the queue (the caller
 * then reserves ceil((in_len + out_len) / 16) KV pages for each), the layer slice and the split.
 * n_tasks == 0 means nothing can be admitted yet (KV pool full) or there is no prefill work. */
typedef struct { int32_t id; int32_t in_len, out_len; int64_t arrival_ns; } sts_sched_req;
typedef struct { int32_t in_len, n_dec; int64_t first_token_ns; } sts_sched_dec;
typedef struct {
  int64_t now_ns;
  int32_t n_queue; const sts_sched_req* queue;
  int32_t n_inflight; const sts_sched_req* inflight; int32_t layers_done;
  int32_t n_decode; const sts_sched_dec* decode;
  int32_t pages_free;
  int32_t cur_prefill_cus, cur_decode_cus;      /* the split in force (0/total before the first decision) */
} sts_sched_state;
typedef struct {
  int32_t cap_tasks; int32_t* task_ids;        /* caller's arrays */
  int32_t cap_queue; int32_t* queue_ids;       /* cap_queue >= n_queue */
  int32_t n_tasks, n_queue, admitted;
  int32_t layer_begin, layer_end, prefill_cus, decode_cus, branch;
  int64_t predicted_ns;
} sts_sched_choice;
int sts_sched_decide(const sts_profile* p, const sts_model_desc* desc, const sts_sched_config* cfg,
                     const sts_sched_state* state, sts_sched_choice* choice);

/* trace: n rows of (arrival_ns, in_len, out_len). decisions: caller's array of cap records (may
 * be NULL with cap 0); the first min(cap, n_decisions) are written. */
int sts_sched_replay(const sts_profile* p, const sts_model_desc* desc, const sts_sched_config* cfg,
                     const int64_t* trace, int64_t n, sts_decision* decisions, int64_t cap, sts_replay_stats* stats);

#ifdef __cplusplus
}
#endif
#endif
