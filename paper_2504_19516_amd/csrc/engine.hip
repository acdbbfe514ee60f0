// Concurrent execution engine: owns weights, the shared paged KV pool, the per-phase
// workspaces and the CU-masked streams, and drives the kernels of a prefill layer slice and of
// a decode step (paper Sections 3.4 and 3.5). Everything here is host code; the kernels live in
// gemm.hip, attn_prefill.hip, attn_decode.hip and elementwise.hip.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "kernels.h"
#include "sts.h"

using namespace sts;

static std::atomic<int> g_hip_err{0};   // either phase's control thread may record an error
#define HIPCK(x)                                                 \
  do {                                                           \
    hipError_t e_ = (x);                                         \
    if (e_ != hipSuccess) { g_hip_err = (int)e_; return STS_EHIP; } \
  } while (0)
#define STSCK(x) do { int r_ = (x); if (r_ != STS_OK) return r_; } while (0)

extern "C" const char* sts_strerror(int code) {
  switch (code) {
    case STS_OK: return "ok";
    case STS_EINVAL: return "invalid argument";
    case STS_ENOMEM: return "KV page pool or workspace exhausted";
    case STS_ESTATE: return "call out of order for the current state";
    case STS_EHIP: return "HIP runtime error (see sts_last_hip_error)";
    case STS_EIO: return "file or parse error";
    default: return "unknown error";
  }
}
extern "C" int sts_last_hip_error(void) { return g_hip_err.load(); }

static const char* kKernelNames[STS_K_COUNT] = {"embed", "norm", "qkv", "rope", "attn", "attn_merge", "o", "gateup",
                                                "swiglu", "down", "reduce", "head", "sample"};
extern "C" const char* sts_kernel_name(int32_t kind) { return (kind >= 0 && kind < STS_K_COUNT) ? kKernelNames[kind] : "?"; }

namespace {

struct LayerW { bf16 *wqkv, *wo, *wgu, *wd; float *g1, *g2; };

struct Seq { bool used = false; int len = 0; std::vector<int> pages; };

struct Phase {
  int side = 0;
  int cus = 0;
  hipStream_t stream = nullptr;
  hipEvent_t ev0 = nullptr, ev1 = nullptr;
  bool ran = false;
  // device workspace
  float* X = nullptr; bf16* Xn = nullptr; bf16* QKV = nullptr; bf16* A = nullptr; bf16* H = nullptr;
  float* part = nullptr; float* attn_ws = nullptr; bf16* Q = nullptr;
  float* tail_ws = nullptr; size_t tail_ws_bytes = 0;         // prefill GEMM tail pieces
  float* Xlast = nullptr; bf16* Xlast_n = nullptr; float* logits = nullptr; int* next = nullptr;
  // Per-call metadata (sequence records, block tables, work items, token ids) is packed into one
  // pinned block and reaches the device in a single copy; the pointers below are views into the
  // two blocks, laid out afresh by every launch.
  unsigned char* h_meta = nullptr; unsigned char* d_meta = nullptr; size_t meta_bytes = 0, meta_used = 0;
  int* d_tokens = nullptr; int* d_bt = nullptr; int* d_rows = nullptr;
  PrefillSeq* d_pseq = nullptr; DecodeSeq* d_dseq = nullptr; AttnItem* d_items = nullptr; DecodeItem* d_ditems = nullptr;
  // pinned staging
  int* h_tokens = nullptr; int* h_bt = nullptr; int* h_rows = nullptr;
  PrefillSeq* h_pseq = nullptr; DecodeSeq* h_dseq = nullptr; AttnItem* h_items = nullptr; DecodeItem* h_ditems = nullptr;
  float* h_logits = nullptr; int* h_next = nullptr;
  int rows = 0;                               // rows of the last call
  // per-kernel timing
  std::vector<hipEvent_t> kev; std::vector<int> kkind; size_t kused = 0;
  int64_t kns[STS_K_COUNT] = {0}, kcnt[STS_K_COUNT] = {0};
};

}  // namespace

struct sts_ctx {
  sts_model_desc d;
  sts_init_params p;
  int n_cu = 0;
  int qd = 0, kvd = 0, qkvn = 0;
  KvGeom geo;
  bf16 *emb = nullptr, *lm = nullptr; float* gf = nullptr;
  std::vector<LayerW> layers;
  bf16* pool = nullptr; size_t pool_layer_elems = 0;
  double* inv_freq = nullptr;
  std::mutex alloc_mu;                         // serialises page allocation / release
  std::mutex state_mu;                         // guards the in-flight prefill batch description
  std::mutex part_mu;                          // serialises repartitioning (one control thread per phase may call it)
  std::vector<int> free_pages; std::vector<char> page_used;
  std::vector<Seq> seqs;
  Phase ph[2];
  int part_cus[2] = {0, 0};
  bool ktiming = false;
  // in-flight layer-sliced prefill batch
  bool pf_active = false; int pf_next_layer = 0; std::vector<int> pf_seqs, pf_lens;
  int64_t last_wall_ns = 0;
  // launches whose finish call is still due (non-blocking API)
  std::atomic<bool> pend_prefill{false}, pend_decode{false};    // a launch of that phase is in flight (each set by its own control thread)
  std::vector<int> pend_pseqs, pend_plens, pend_dseqs; int pend_le = 0;
  void* probe_src = nullptr; void* probe_dst = nullptr; size_t probe_bytes = 0;
  std::vector<void*> allocs;
  std::vector<hipStream_t> used_streams;       // every pooled stream this ctx ever selected (guarded by part_mu)
  // what the tile choice of the prefill GEMMs assumes about the part (sts_set_tile_model): TFLOP/s per busy CU of
  // the 128x128 tiles (two workgroups per CU) and of the 256x256 tiles (one), bytes/s per CU for partial tiles
  double rate_128 = 3.5, rate_256 = 4.8, rate_128x256 = 5.0, fixed_128x256 = 25e-6, partial_bw = 20e9;
  double stream_bw_cu = 59e9, stream_bw_gpu = 6.4e12;          // read-only streams: bytes/s per CU of a 32-CU partition, bytes/s of the whole GPU
};

namespace {

template <typename T>
int dev_alloc(sts_ctx* c, T** out, size_t count) {
  void* p = nullptr;
  HIPCK(hipMalloc(&p, std::max<size_t>(count, 1) * sizeof(T)));
  c->allocs.push_back(p);
  *out = reinterpret_cast<T*>(p);
  return STS_OK;
}
// Next 256-byte aligned view of `count` elements in a phase's metadata blocks.
template <typename T>
void meta_take(Phase& ph, T** host, T** dev, size_t count);

template <typename T>
int host_alloc(T** out, size_t count) {
  void* p = nullptr;
  HIPCK(hipHostMalloc(&p, std::max<size_t>(count, 1) * sizeof(T), hipHostMallocDefault));
  *out = reinterpret_cast<T*>(p);
  return STS_OK;
}

template <typename T>
void meta_take(Phase& ph, T** host, T** dev, size_t count) {
  const size_t off = (ph.meta_used + 255) & ~(size_t)255;
  *host = reinterpret_cast<T*>(ph.h_meta + off);
  *dev = reinterpret_cast<T*>(ph.d_meta + off);
  ph.meta_used = off + count * sizeof(T);
}

// CU-masked streams are a process-wide pool: one stream per (side, CU count), created on first
// use and kept until the process ends. Repartitioning is then a pointer switch, engines that
// come and go reuse the same hardware queues, and no masked queue is ever torn down.
std::mutex g_stream_mu;
std::map<std::pair<int, int>, hipStream_t> g_streams;
std::atomic<int> g_live_ctx{0};            // engines alive in this process (sts_release_streams refuses while any is)
std::atomic<bool> g_streams_released{false};   // set by sts_release_streams: the process is ending, no further engine is created

void trace(const char* what) {
  static const bool on = std::getenv("STS_TRACE") != nullptr;
  if (on) { std::fprintf(stderr, "[sts] %s\n", what); std::fflush(stderr); }
}

int get_stream(sts_ctx* c, int side, int cus, hipStream_t* out) {
  std::lock_guard<std::mutex> g(g_stream_mu);
  auto key = std::make_pair(side, cus);
  auto it = g_streams.find(key);
  if (it != g_streams.end()) { *out = it->second; return STS_OK; }
  // A mask that leaves some XCD without a CU makes stream creation fail (and crashes some
  // runtime versions): contiguous runs of >= 8 bits always cover all 8 XCDs because mask bit i
  // belongs to XCD i % 8.
  if (cus < 8 || cus > c->n_cu || cus % 8 != 0) return STS_EINVAL;
  const int words = (c->n_cu + 31) / 32;
  std::vector<uint32_t> mask(words, 0);
  const int lo = side == 0 ? 0 : c->n_cu - cus;
  for (int b = lo; b < lo + cus; b++) mask[b / 32] |= 1u << (b % 32);
  hipStream_t s = nullptr;
  HIPCK(hipExtStreamCreateWithCUMask(&s, words, mask.data()));
  g_streams[key] = s;
  *out = s;
  return STS_OK;
}

// Caller holds part_mu (or is the only user of the ctx).
void remember_stream(sts_ctx* c, hipStream_t s) {
  if (s && std::find(c->used_streams.begin(), c->used_streams.end(), s) == c->used_streams.end()) c->used_streams.push_back(s);
}

int select_streams(sts_ctx* c) {
  for (int side = 0; side < 2; side++) {
    Phase& ph = c->ph[side];
    if (c->part_cus[side] == 0) { ph.stream = nullptr; ph.cus = 0; continue; }
    STSCK(get_stream(c, side, c->part_cus[side], &ph.stream));
    remember_stream(c, ph.stream);
    ph.cus = c->part_cus[side];
  }
  return STS_OK;
}

// ---- per-kernel timing
int k_begin(sts_ctx* c, Phase& ph, int kind) {
  if (!c->ktiming) return STS_OK;
  if (ph.kused + 2 > ph.kev.size()) {
    for (int i = 0; i < 256; i++) { hipEvent_t e; HIPCK(hipEventCreate(&e)); ph.kev.push_back(e); }
  }
  ph.kkind.push_back(kind);
  HIPCK(hipEventRecord(ph.kev[ph.kused], ph.stream));
  return STS_OK;
}
int k_end(sts_ctx* c, Phase& ph) {
  if (!c->ktiming) return STS_OK;
  HIPCK(hipEventRecord(ph.kev[ph.kused + 1], ph.stream));
  ph.kused += 2;
  return STS_OK;
}
int k_collect(sts_ctx* c, Phase& ph) {
  if (!c->ktiming) return STS_OK;
  for (size_t i = 0; i < ph.kkind.size(); i++) {
    float ms = 0.f;
    HIPCK(hipEventElapsedTime(&ms, ph.kev[2 * i], ph.kev[2 * i + 1]));
    ph.kns[ph.kkind[i]] += (int64_t)(ms * 1e6);
    ph.kcnt[ph.kkind[i]] += 1;
  }
  ph.kkind.clear(); ph.kused = 0;
  return STS_OK;
}
#define KL(ph, kind, expr)                \
  do {                                    \
    STSCK(k_begin(c, ph, kind));          \
    HIPCK(expr);                          \
    STSCK(k_end(c, ph));                  \
  } while (0)

int pick_cfg(int m, int n, int k, int cus) {
  // up to 64 rows: 64x128 tiles, two workgroups (8 waves) per CU streaming weights (decode GEMMs whose N allows
  // it take the skinny tiles instead, see pick_decode_gemm)
  if (m <= 64) return GEMM_64x128;
  // up to 128 rows: one row of 128x128 tiles, two workgroups per CU. Above that both shapes compute
  // 256 rows and the 256x256 tile's larger wave tiles run the MFMAs faster; a large decode batch
  // on a small partition is compute-bound (Section 2.1). One 256x256 workgroup fills a CU, so the
  // shape is taken only when its tiles times the deepest split-K still cover the partition.
  const bool covers = (long long)(n / 256) * std::min(8, std::max(1, k / 512)) >= cus;
  return (m <= 128 || n % 256 != 0 || !covers) ? GEMM_128x128 : GEMM_256x256;
}
// Prefill GEMM tile choice for a partition of `cus` CUs: the candidate with the smallest
// estimated time, which is where wave quantisation (paper Section 2.2.1) enters -- complete
// waves of workgroups at the tile's busy-CU rate, then the last wave, whole or cut along K.
// Rates are measured busy-CU throughputs in TFLOP/s per CU: 128x128 tiles run two workgroups
// per CU, 256x256 (8 waves) one.
int pick_prefill_cfg(const sts_ctx* ctx, int epi, int m, int n, int k, int cus, size_t tail_ws_bytes) {
  if (m <= 64) return GEMM_64x128;
  struct Cand { int cfg; double rate; };
  const Cand cands[3] = {{GEMM_128x128, ctx->rate_128}, {GEMM_256x256, ctx->rate_256}, {GEMM_128x256, ctx->rate_128x256}};
  int best = GEMM_128x128; double best_cost = 1e300;
  for (const Cand& c : cands) {
    // 128x256: planned one tile per CU although two fit, so the pieces of a cut last wave run in the second slot beside
    // the whole tiles; the shape of the O and down projections (a little more than one such tile per CU), instantiated
    // for their residual epilogue
    if (c.cfg == GEMM_128x256 && epi != EPI_RESID_F32) continue;
    const int tm = gemm_tile_m(c.cfg), tn = gemm_tile_n(c.cfg), per_cu = gemm_wgs_per_cu(c.cfg);
    if (n % tn != 0) continue;
    const int tiles = ((m + tm - 1) / tm) * (n / tn);
    const int slots = per_cu * std::max(cus, 8);
    int n_full, f;
    gemm_tail_plan(tiles, k / 64, slots, (long long)(tail_ws_bytes / ((size_t)tm * tn * sizeof(float))), &n_full, &f);
    // in units of this configuration's tile time: complete waves, then the last wave -- whole, or
    // in rounds of 1/f with a start-up charge per round, plus the partial tiles written and read
    // back (4 bytes out, 4 in per element and piece, at the measured per-CU rate)
    // one 128x256 tile per CU: start-up and epilogue are exposed, a measured fixed time on top of the flops
    const double tile_s = 2.0 * tm * tn * k / (c.rate * 1e12 / per_cu) + (c.cfg == GEMM_128x256 ? ctx->fixed_128x256 : 0.0);
    double t;
    if (f > 1) {
      const int rest = tiles - n_full, rounds = (rest * f + slots - 1) / slots;
      t = (n_full / slots + rounds * (1.0 / f + 0.03)) * tile_s + (double)rest * f * tm * tn * 8.0 / (std::max(cus, 8) * ctx->partial_bw) + 6e-6;
    } else {
      t = (double)((tiles + slots - 1) / slots) * tile_s;
    }
    const double cost = t;
    if (cost < best_cost) { best_cost = cost; best = c.cfg; }
  }
  return best;
}
// A prefill GEMM on the phase's partition: tile choice, and the last wave of tiles cut along K.
hipError_t prefill_gemm(const sts_ctx* ctx, Phase& ph, int epi, const bf16* A, int lda, const bf16* W, int ldw, void* C, int ldc, int m, int n, int k) {
  int cfg = pick_prefill_cfg(ctx, epi, m, n, k, ph.cus, ph.tail_ws_bytes);
  const GemmTail tail{gemm_wgs_per_cu(cfg) * ph.cus, ph.tail_ws, ph.tail_ws_bytes};
  return gemm_bf16(ph.stream, cfg, epi, A, lda, W, ldw, C, ldc, m, n, k, 1, 0, &tail);
}
int plan_splits(double rate_256, double partial_bw, int cfg, int m, int n, int k, int cus);
int pick_splits(const sts_ctx* ctx, int cfg, int m, int n, int k, int cus) { return plan_splits(ctx->rate_256, ctx->partial_bw, cfg, m, n, k, cus); }
int plan_splits(double rate_256, double partial_bw, int cfg, int m, int n, int k, int cus) {
  const int tiles = ((m + gemm_tile_m(cfg) - 1) / gemm_tile_m(cfg)) * (n / gemm_tile_n(cfg));
  const int slots = gemm_wgs_per_cu(cfg) * std::max(cus, 8);
  const int s_max = std::min(8, std::max(1, k / 512));            // at least 8 K-steps per slice
  if (gemm_wgs_per_cu(cfg) == 1 && gemm_tile_m(cfg) >= 256) {
    // one workgroup owns a CU, so rounds of workgroups are strict: estimated time of s slices =
    // ceil(tiles * s / slots) rounds of a 1/s tile at the measured rate of that tile, plus the fp32
    // partial sums written and read back at the measured per-CU rate; the cheapest s wins
    const double tile_s = 2.0 * gemm_tile_m(cfg) * gemm_tile_n(cfg) * k / (rate_256 * 1e12);
    const double part_s = 8.0 * m * n / (std::max(cus, 8) * partial_bw);
    int best = 1; double best_t = 1e300;
    for (int s = 1; s <= s_max; s++) {
      const double t = (double)(((long long)tiles * s + slots - 1) / slots) * tile_s / s + s * part_s;
      if (t < best_t - 1e-9) { best_t = t; best = s; }
    }
    return best;
  }
  const int s = (slots + tiles - 1) / tiles;                        // fill the partition's workgroup slots
  return std::max(1, std::min(s, s_max));
}

// Tile shape and split-K of one decode GEMM. Above 64 rows: the prefill shapes (pick_cfg) with a split that
// fills the partition. Up to 64 rows the GEMM streams its weights once and runs at the pace at which the
// partition's CUs pull bytes, and everything a workgroup reads counts: its K range of the W columns and, beside
// them, the 64 activation rows of that range again for every workgroup. The candidates are the 64x128 tiles
// through LDS and the skinny tiles of 4 to 8 waves (256 to 512 columns, 64 per wave; the four-wave tiles run two
// workgroups per CU) whose width divides N, each with 1 .. 8 slices along K, and the estimate is
//   rounds of workgroups x (bytes of the workgroups a CU holds / per-CU streaming rate + a start-up time),
// not less than the weight bytes at the rate the memory system gives a whole GPU, plus -- when the output
// leaves as fp32 partial sums for a reduce kernel -- those partial sums written and read back. A wide tile reads
// the activations less often (a small partition is bound by what its CUs can pull); a narrow one, or a deeper
// split, makes more workgroups (a large partition needs them all busy) and fills the last round better: with
// 7 x 2^k columns (the MLP width of the Llama shapes) on 32 or 64 CUs only the 7-wave tile comes out in whole
// rounds.
// `partials`: the output goes through fp32 partial sums (a split needs that; the caller's next kernel reads them).
// Returns the estimated seconds.
struct StreamRates { double rate_256, partial_bw, stream_bw_cu, stream_bw_gpu; };
double plan_decode_gemm(const StreamRates& r, int m, int n, int k, int cus, bool may_split, bool partials, int* cfg, int* splits);
double pick_decode_gemm(const sts_ctx* ctx, int m, int n, int k, int cus, bool may_split, bool partials, int* cfg, int* splits) {
  return plan_decode_gemm(StreamRates{ctx->rate_256, ctx->partial_bw, ctx->stream_bw_cu, ctx->stream_bw_gpu}, m, n, k, cus, may_split, partials, cfg, splits);
}
// r: measured on the part by the offline profiler -- rate_256 (TFLOP/s per busy CU of the 256x256 tile) and partial_bw (bytes/s
// per CU for partial sums) of the tile model; stream_bw_cu and stream_bw_gpu, what a plain read-only stream reaches per CU of a
// 32-CU partition and on the whole GPU. A GEMM's weight stream gets 0.93 and 0.85 of those (its loads share the CU with the
// operand reads and the matrix cores; the best decode GEMMs measured 55 of 58-59 GB/s per CU and 5.1 of 6 TB/s).
double plan_decode_gemm(const StreamRates& r, int m, int n, int k, int cus, bool may_split, bool partials, int* cfg, int* splits) {
  const int c = std::max(cus, 8);
  const double rate_256 = r.rate_256, partial_bw = r.partial_bw;
  const double cu_rate = 0.93 * r.stream_bw_cu;      // bytes/s one CU pulls from memory for a GEMM's streams
  const double mem_rate = 0.85 * r.stream_bw_gpu;    // bytes/s the memory system gives a full GPU of such streams
  constexpr double start_s = 2.5e-6;                 // a workgroup's first loads and its epilogue
  auto estimate = [&](int cand, int s) {
    const int bn = gemm_tile_n(cand), bm = gemm_tile_m(cand), per_cu = gemm_wgs_per_cu(cand);
    const long long wgs = (long long)((m + bm - 1) / bm) * (n / bn) * s, slots = (long long)c * per_cu;
    const long long rounds = (wgs + slots - 1) / slots, last = wgs - (rounds - 1) * slots;
    const double wg_bytes = 2.0 * (k / s) * (bn + bm);
    // one workgroup alone pulls what its loads in flight allow: on a busy memory system a wave of a skinny tile a
    // sixth of the CU's rate (10 GB/s), the four waves of a tile staged through LDS 0.6 of it (34 GB/s)
    const double wg_rate = cand >= GEMM_64x256S ? std::min(cu_rate, cu_rate / 5.5 * (bn / 64)) : 0.62 * cu_rate;
    auto cu_time = [&](long long held) { return std::max(held * wg_bytes / cu_rate, wg_bytes / wg_rate); };
    // complete rounds hold per_cu workgroups on every CU; the last round what is left, dealt over the CUs
    double t = (rounds - 1) * cu_time(per_cu) + cu_time((last + c - 1) / c);
    t = std::max(t, 2.0 * n * k / mem_rate) + rounds * start_s;
    if (partials) t += 8.0 * s * m * n / (c * partial_bw);
    return t;
  };
  if (m > 64 || n % 128 != 0) {
    *cfg = pick_cfg(m, n, k, cus);
    *splits = may_split ? plan_splits(rate_256, partial_bw, *cfg, m, n, k, cus) : 1;
    return estimate(*cfg, *splits);
  }
  const int s_max = may_split ? std::min(8, std::max(1, k / 512)) : 1;
  double best_t = 1e300;
  *cfg = GEMM_64x128; *splits = 1;
  const int cands[6] = {GEMM_64x256S, GEMM_64x320S, GEMM_64x384S, GEMM_64x448S, GEMM_64x512S, GEMM_64x128};
  for (int cand : cands) {
    if (n % gemm_tile_n(cand) != 0) continue;
    // a GEMM that keeps its output (no partial sums) may carry the SwiGLU epilogue, and the 64x128 tile's form of it
    // (wave tiles of 32 x 64) is slow when a CU holds one workgroup: taken only if no skinny width divides N
    if (!partials && cand == GEMM_64x128 && best_t < 1e300) continue;
    for (int s = 1; s <= s_max; s++) {
      const double t = estimate(cand, s);
      if (t < best_t - 1e-12) { best_t = t; *cfg = cand; *splits = s; }
    }
  }
  return best_t;
}

int64_t now_ns();

// Wait for a stream with a short busy poll before blocking: a layer slice or a decode step lasts
// around a millisecond, and the wake-up latency of a blocking wait would be a visible share of it.
hipError_t wait_stream(hipStream_t st) {
  const int64_t t0 = now_ns();
  for (;;) {
    const hipError_t e = hipStreamQuery(st);
    if (e != hipErrorNotReady) return e;                     // done, or a real error
    if (now_ns() - t0 > 20000000) return hipStreamSynchronize(st);
#if defined(__x86_64__)
    __builtin_ia32_pause();
#endif
  }
}

bool valid_seq(sts_ctx* c, int s) { return s >= 0 && s < (int)c->seqs.size() && c->seqs[s].used; }

// Make `seq` own enough pages for n_tokens; caller holds no lock.
int reserve_pages(sts_ctx* c, const std::vector<std::pair<int, int>>& wants) {   // (seq, tokens)
  std::lock_guard<std::mutex> g(c->alloc_mu);
  size_t need = 0;
  for (auto& w : wants) {
    const int np = (w.second + c->geo.page_tokens - 1) / c->geo.page_tokens;
    if (np > c->p.max_pages_per_seq) return STS_EINVAL;
    need += std::max(0, np - (int)c->seqs[w.first].pages.size());
  }
  if (need > c->free_pages.size()) return STS_ENOMEM;
  for (auto& w : wants) {
    const int np = (w.second + c->geo.page_tokens - 1) / c->geo.page_tokens;
    Seq& s = c->seqs[w.first];
    while ((int)s.pages.size() < np) {
      const int pg = c->free_pages.back(); c->free_pages.pop_back();
      c->page_used[pg] = 1; s.pages.push_back(pg);
    }
  }
  return STS_OK;
}

bf16* layer_pool(sts_ctx* c, int l) { return c->pool + (size_t)l * c->pool_layer_elems; }

// ------------------------------------------------------------------------------------ prefill
// Checks of a prefill slice that touch no state: arguments, the order of layer slices, and the
// pages the batch will need (appended to `wants` for slice 0). Nothing is launched or reserved.
int prefill_validate(sts_ctx* c, int n_seqs, const int32_t* seqs, const int32_t* lens, const int32_t* tokens, int lb, int le,
                     std::vector<std::pair<int, int>>* wants) {
  Phase& ph = c->ph[0];
  const sts_model_desc& d = c->d;
  if (n_seqs < 1 || n_seqs > c->p.max_prefill_seqs || !seqs || !lens) return STS_EINVAL;
  if (lb < 0 || le <= lb || le > d.n_layers) return STS_EINVAL;
  if (ph.stream == nullptr) return STS_ESTATE;               // prefill suspended (0 CUs)
  int rows = 0;
  for (int i = 0; i < n_seqs; i++) {
    if (!valid_seq(c, seqs[i]) || lens[i] < 1) return STS_EINVAL;
    for (int j = 0; j < i; j++) if (seqs[j] == seqs[i]) return STS_EINVAL;
    rows += lens[i];
    if (rows > c->p.max_prefill_tokens) return STS_EINVAL;
  }
  std::lock_guard<std::mutex> g(c->state_mu);
  for (int i = 0; i < n_seqs; i++) for (int s : c->pend_dseqs) if (s == seqs[i]) return STS_EINVAL;   // a request is in one phase only
  if (lb == 0) {
    if (!tokens) return STS_EINVAL;
    for (int i = 0; i < rows; i++) if (tokens[i] < 0 || tokens[i] >= d.vocab) return STS_EINVAL;
    if (c->pf_active) return STS_ESTATE;
    for (int i = 0; i < n_seqs; i++) {
      const int total = c->seqs[seqs[i]].len + lens[i];
      if ((total + c->geo.page_tokens - 1) / c->geo.page_tokens > c->p.max_pages_per_seq) return STS_EINVAL;
      wants->push_back({seqs[i], total});
    }
  } else {
    if (!c->pf_active || lb != c->pf_next_layer || (int)c->pf_seqs.size() != n_seqs) return STS_ESTATE;
    for (int i = 0; i < n_seqs; i++) if (c->pf_seqs[i] != seqs[i] || c->pf_lens[i] != lens[i]) return STS_ESTATE;
  }
  return STS_OK;
}

// Queues a validated slice whose pages are reserved. A failure in here (a HIP error) leaves the
// batch description as it was before the call.
int prefill_launch_checked(sts_ctx* c, int n_seqs, const int32_t* seqs, const int32_t* lens, const int32_t* tokens,
                           int lb, int le, bool want_logits);

int prefill_enqueue(sts_ctx* c, int n_seqs, const int32_t* seqs, const int32_t* lens, const int32_t* tokens,
                    int lb, int le, bool want_logits) {
  std::vector<std::pair<int, int>> wants;
  STSCK(prefill_validate(c, n_seqs, seqs, lens, tokens, lb, le, &wants));
  STSCK(reserve_pages(c, wants));
  return prefill_launch_checked(c, n_seqs, seqs, lens, tokens, lb, le, want_logits);
}

int prefill_launch_body(sts_ctx* c, int n_seqs, const int32_t* seqs, const int32_t* lens, const int32_t* tokens,
                        int lb, int le, bool want_logits);

int prefill_launch_checked(sts_ctx* c, int n_seqs, const int32_t* seqs, const int32_t* lens, const int32_t* tokens,
                           int lb, int le, bool want_logits) {
  if (lb == 0) {
    std::lock_guard<std::mutex> g(c->state_mu);
    c->pf_active = true; c->pf_next_layer = 0;
    c->pf_seqs.assign(seqs, seqs + n_seqs); c->pf_lens.assign(lens, lens + n_seqs);
  }
  const int rc = prefill_launch_body(c, n_seqs, seqs, lens, tokens, lb, le, want_logits);
  if (rc != STS_OK && lb == 0) {                             // the batch never started: later prefills are not blocked
    std::lock_guard<std::mutex> g(c->state_mu);
    c->pf_active = false; c->pf_seqs.clear(); c->pf_lens.clear();
  }
  return rc;
}

int prefill_launch_body(sts_ctx* c, int n_seqs, const int32_t* seqs, const int32_t* lens, const int32_t* tokens,
                        int lb, int le, bool want_logits) {
  Phase& ph = c->ph[0];
  const sts_model_desc& d = c->d;
  int rows = 0;
  for (int i = 0; i < n_seqs; i++) rows += lens[i];
  // ---- stage metadata
  const int mp = c->p.max_pages_per_seq, bq = attn_prefill_tile_q();
  ph.meta_used = 0;
  meta_take(ph, &ph.h_pseq, &ph.d_pseq, n_seqs);
  meta_take(ph, &ph.h_rows, &ph.d_rows, n_seqs);
  meta_take(ph, &ph.h_items, &ph.d_items, rows / bq + n_seqs);
  meta_take(ph, &ph.h_tokens, &ph.d_tokens, lb == 0 ? rows : 0);
  size_t bt_entries = 0;                                     // block tables are packed back to back
  for (int i = 0; i < n_seqs; i++) bt_entries += c->seqs[seqs[i]].pages.size();
  meta_take(ph, &ph.h_bt, &ph.d_bt, bt_entries);
  if (ph.meta_used > ph.meta_bytes) return STS_EINVAL;
  int r0 = 0, n_items = 0, bt_off = 0;
  for (int i = 0; i < n_seqs; i++) {
    const Seq& s = c->seqs[seqs[i]];
    ph.h_pseq[i] = PrefillSeq{r0, lens[i], s.len, bt_off, (int)s.pages.size()};
    std::memcpy(ph.h_bt + bt_off, s.pages.data(), s.pages.size() * sizeof(int));
    bt_off += (int)s.pages.size();
    for (int q0 = 0; q0 < lens[i]; q0 += bq) ph.h_items[n_items++] = AttnItem{i, q0};
    ph.h_rows[i] = r0 + lens[i] - 1;
    r0 += lens[i];
  }
  // heaviest query tiles first: the tail of the launch is then made of short ones
  std::stable_sort(ph.h_items, ph.h_items + n_items, [&](const AttnItem& a, const AttnItem& b) {
    return ph.h_pseq[a.seq].p + a.q0 > ph.h_pseq[b.seq].p + b.q0;
  });
  hipStream_t st = ph.stream;
  HIPCK(hipEventRecord(ph.ev0, st));
  if (lb == 0) std::memcpy(ph.h_tokens, tokens, rows * sizeof(int));
  HIPCK(hipMemcpyAsync(ph.d_meta, ph.h_meta, ph.meta_used, hipMemcpyHostToDevice, st));
  const int h = d.hidden;
  const bool fused_embed = lb == 0 && h <= 8192;             // the embedding kernel also writes layer 0's normalised rows
  if (fused_embed) KL(ph, STS_K_EMBED, embed_norm_rows(st, ph.X, ph.Xn, c->emb, ph.d_tokens, c->layers[0].g1, d.rms_eps, rows, h));
  else if (lb == 0) KL(ph, STS_K_EMBED, embed_rows(st, ph.X, c->emb, ph.d_tokens, rows, h));
  for (int l = lb; l < le; l++) {
    const LayerW& w = c->layers[l];
    if (!(fused_embed && l == 0)) KL(ph, STS_K_NORM, rmsnorm_rows(st, ph.Xn, ph.X, w.g1, d.rms_eps, rows, h));
    KL(ph, STS_K_QKV, prefill_gemm(c, ph, EPI_BF16, ph.Xn, h, w.wqkv, h, ph.QKV, c->qkvn, rows, c->qkvn, h));
    KL(ph, STS_K_ROPE, rope_kv_write_prefill(st, ph.QKV, c->qkvn, ph.d_pseq, n_seqs, ph.d_bt, c->inv_freq, layer_pool(c, l), c->geo, rows, d.n_q_heads));
    KL(ph, STS_K_ATTN, attn_prefill(st, ph.QKV, c->qkvn, ph.A, c->qd, ph.d_pseq, ph.d_items, n_items, ph.d_bt, layer_pool(c, l), c->geo, d.n_q_heads));
    KL(ph, STS_K_O, prefill_gemm(c, ph, EPI_RESID_F32, ph.A, c->qd, w.wo, c->qd, ph.X, h, rows, h, c->qd));
    KL(ph, STS_K_NORM, rmsnorm_rows(st, ph.Xn, ph.X, w.g2, d.rms_eps, rows, h));
    KL(ph, STS_K_GATEUP, prefill_gemm(c, ph, EPI_SWIGLU_BF16, ph.Xn, h, w.wgu, h, ph.H, d.mlp, rows, 2 * d.mlp, h));
    KL(ph, STS_K_DOWN, prefill_gemm(c, ph, EPI_RESID_F32, ph.H, d.mlp, w.wd, d.mlp, ph.X, h, rows, h, d.mlp));
  }
  if (le == d.n_layers && want_logits) {
    KL(ph, STS_K_HEAD, gather_rows_f32(st, ph.Xlast, ph.X, ph.d_rows, n_seqs, h));
    KL(ph, STS_K_NORM, rmsnorm_rows(st, ph.Xlast_n, ph.Xlast, c->gf, d.rms_eps, n_seqs, h));
    int head_cfg, head_splits;
    pick_decode_gemm(c, n_seqs, d.vocab, h, ph.cus, false, false, &head_cfg, &head_splits);
    KL(ph, STS_K_HEAD, gemm_bf16(st, head_cfg, EPI_F32, ph.Xlast_n, h, c->lm, h, ph.logits, d.vocab, n_seqs, d.vocab, h, 1, 0));
    HIPCK(hipMemcpyAsync(ph.h_logits, ph.logits, (size_t)n_seqs * d.vocab * sizeof(float), hipMemcpyDeviceToHost, st));
  }
  HIPCK(hipEventRecord(ph.ev1, st));
  ph.ran = true; ph.rows = rows;
  return STS_OK;
}

int prefill_finish(sts_ctx* c, int n_seqs, const int32_t* seqs, const int32_t* lens, int le, float* logits) {
  Phase& ph = c->ph[0];
  HIPCK(wait_stream(ph.stream));
  STSCK(k_collect(c, ph));
  c->pf_next_layer = le;
  if (le == c->d.n_layers) {
    for (int i = 0; i < n_seqs; i++) c->seqs[seqs[i]].len += lens[i];
    { std::lock_guard<std::mutex> g(c->state_mu); c->pf_active = false; }
    if (logits) std::memcpy(logits, ph.h_logits, (size_t)n_seqs * c->d.vocab * sizeof(float));
  }
  return STS_OK;
}

// ------------------------------------------------------------------------------------ decode
// Context chunks of at most chunk_pages pages: the largest of 64/32/16/8 that still yields about
// four workgroups per CU of the partition (8 pages keep the four waves of a workgroup busy with
// one two-page block each), never more than 128 chunks for the longest context.
void decode_chunk_plan(const int* n_pages, int n, int n_kv, int cus, int page_tokens, int* chunk_pages_out, int* max_chunks_out) {
  int max_pages = 1;
  for (int i = 0; i < n; i++) max_pages = std::max(max_pages, n_pages[i]);
  int chunk_pages = attn_decode_max_chunk_tokens() / page_tokens;
  const int floor_pages = std::max(8, (max_pages + 127) / 128);
  while (chunk_pages / 2 >= floor_pages) {
    long long wgs = 0;
    for (int i = 0; i < n; i++) wgs += (n_pages[i] + chunk_pages - 1) / chunk_pages;
    if (wgs * n_kv >= 4LL * cus) break;
    chunk_pages /= 2;
  }
  *chunk_pages_out = chunk_pages;
  *max_chunks_out = (max_pages + chunk_pages - 1) / chunk_pages;
}
// Chunks per context the merge workspace and the work list are allocated for: chunks hold at least
// 8 pages (fewer than one chunk per 4 pages), and never more than 128 per context.
int decode_max_chunks(int max_pages_per_seq) { return (int)std::min<size_t>(128, ((size_t)max_pages_per_seq + 3) / 4); }

// Checks of a decode step that touch no state; the page each request needs for its new token is
// appended to `wants`.
int decode_validate(sts_ctx* c, const int32_t* seqs, const int32_t* in_tokens, int n, std::vector<std::pair<int, int>>* wants) {
  Phase& ph = c->ph[1];
  const sts_model_desc& d = c->d;
  if (n < 1 || n > c->p.max_decode_batch || !seqs || !in_tokens) return STS_EINVAL;
  if (ph.stream == nullptr) return STS_ESTATE;               // decode suspended (0 CUs)
  for (int i = 0; i < n; i++) {
    if (!valid_seq(c, seqs[i]) || in_tokens[i] < 0 || in_tokens[i] >= d.vocab) return STS_EINVAL;
    for (int j = 0; j < i; j++) if (seqs[j] == seqs[i]) return STS_EINVAL;
    if ((c->seqs[seqs[i]].len + 1 + c->geo.page_tokens - 1) / c->geo.page_tokens > c->p.max_pages_per_seq) return STS_EINVAL;
  }
  {
    std::lock_guard<std::mutex> g(c->state_mu);                                        // a request is in one phase only
    if (c->pf_active) for (int i = 0; i < n; i++) for (int s : c->pf_seqs) if (s == seqs[i]) return STS_EINVAL;
  }
  for (int i = 0; i < n; i++) wants->push_back({seqs[i], c->seqs[seqs[i]].len + 1});
  return STS_OK;
}

int decode_launch_checked(sts_ctx* c, const int32_t* seqs, const int32_t* in_tokens, int n, bool want_logits, bool want_next);

int decode_enqueue(sts_ctx* c, const int32_t* seqs, const int32_t* in_tokens, int n, bool want_logits, bool want_next) {
  std::vector<std::pair<int, int>> wants;
  STSCK(decode_validate(c, seqs, in_tokens, n, &wants));
  STSCK(reserve_pages(c, wants));
  return decode_launch_checked(c, seqs, in_tokens, n, want_logits, want_next);
}

int decode_launch_checked(sts_ctx* c, const int32_t* seqs, const int32_t* in_tokens, int n, bool want_logits, bool want_next) {
  Phase& ph = c->ph[1];
  const sts_model_desc& d = c->d;
  const int mp = c->p.max_pages_per_seq, pt = c->geo.page_tokens;
  ph.meta_used = 0;
  meta_take(ph, &ph.h_dseq, &ph.d_dseq, n);
  meta_take(ph, &ph.h_tokens, &ph.d_tokens, n);
  size_t bt_entries = 0;                                     // block tables are packed back to back
  for (int i = 0; i < n; i++) bt_entries += (c->seqs[seqs[i]].len + 1 + pt - 1) / pt;
  meta_take(ph, &ph.h_bt, &ph.d_bt, bt_entries);
  if (ph.meta_used > ph.meta_bytes) return STS_EINVAL;
  int max_pages = 1, bt_off = 0;
  for (int i = 0; i < n; i++) {
    const Seq& s = c->seqs[seqs[i]];
    const int np = (s.len + 1 + pt - 1) / pt;
    ph.h_dseq[i] = DecodeSeq{s.len, bt_off, np};
    std::memcpy(ph.h_bt + bt_off, s.pages.data(), np * sizeof(int));
    bt_off += np;
    max_pages = std::max(max_pages, np);
    ph.h_tokens[i] = in_tokens[i];
  }
  std::vector<int> np_list(n);
  for (int i = 0; i < n; i++) np_list[i] = ph.h_dseq[i].n_pages;
  int chunk_pages, max_chunks;
  decode_chunk_plan(np_list.data(), n, d.n_kv_heads, ph.cus, pt, &chunk_pages, &max_chunks);
  if (max_chunks > decode_max_chunks(mp)) return STS_EINVAL;   // cannot happen within sts_init's bound on max_pages_per_seq
  // one attention workgroup row per context chunk that exists
  int n_items = 0;
  for (int i = 0; i < n; i++) n_items += (ph.h_dseq[i].n_pages + chunk_pages - 1) / chunk_pages;
  meta_take(ph, &ph.h_ditems, &ph.d_ditems, n_items);
  if (ph.meta_used > ph.meta_bytes) return STS_EINVAL;
  n_items = 0;
  for (int i = 0; i < n; i++)
    for (int ch = 0; ch < (ph.h_dseq[i].n_pages + chunk_pages - 1) / chunk_pages; ch++) ph.h_ditems[n_items++] = DecodeItem{i, ch, ph.h_dseq[i].cl, ph.h_dseq[i].bt_off};
  // longest chunks first (a context's chunks are equal, so its chunk length is pages / chunks): the workgroups
  // that finish the launch are then the short ones
  {
    auto chunk_len = [&](const DecodeItem& it) {
      const int np = ph.h_dseq[it.seq].n_pages, chunks = (np + chunk_pages - 1) / chunk_pages;
      return (np + chunks - 1) / chunks;
    };
    std::stable_sort(ph.h_ditems, ph.h_ditems + n_items, [&](const DecodeItem& a, const DecodeItem& b) { return chunk_len(a) > chunk_len(b); });
  }
  // requests whose context has more than one chunk: only they need the merge kernel
  int *h_multi = nullptr, *d_multi = nullptr, n_multi = 0;
  meta_take(ph, &h_multi, &d_multi, (size_t)n);
  if (ph.meta_used > ph.meta_bytes) return STS_EINVAL;
  for (int i = 0; i < n; i++) if (ph.h_dseq[i].n_pages > chunk_pages) h_multi[n_multi++] = i;
  hipStream_t st = ph.stream;
  HIPCK(hipEventRecord(ph.ev0, st));
  HIPCK(hipMemcpyAsync(ph.d_meta, ph.h_meta, ph.meta_used, hipMemcpyHostToDevice, st));
  const int h = d.hidden;
  if (h <= 8192) {
    KL(ph, STS_K_EMBED, embed_norm_rows(st, ph.X, ph.Xn, c->emb, ph.d_tokens, c->layers[0].g1, d.rms_eps, n, h));
  } else {
    KL(ph, STS_K_EMBED, embed_rows(st, ph.X, c->emb, ph.d_tokens, n, h));
    KL(ph, STS_K_NORM, rmsnorm_rows(st, ph.Xn, ph.X, c->layers[0].g1, d.rms_eps, n, h));
  }
  // On a large partition the decode streams (K and V, the weights of the skinny tiles) are fetched with the non-temporal
  // hint: measured on a 6-layer model, the layer-step is 6 % shorter on 256 CUs (attention 72 -> 63 us), 3 % on 128,
  // and no different on 32, where the same hint cost a prefill slice running beside it 0.5 %.
  const bool nt_attn = ph.cus >= 128, nt_w = nt_attn;
  auto skinny = [&](int kind, const bf16* A, int lda, const bf16* W, int N, int K, int* splits_out, long long* stride_out) -> int {
    const long long stride = (long long)n * N;
    *stride_out = stride;
    int cfg, splits;
    pick_decode_gemm(c, n, N, K, ph.cus, true, true, &cfg, &splits);
    *splits_out = splits;
    KL(ph, kind, gemm_bf16(st, cfg, EPI_F32, A, lda, W, K, ph.part, N, n, N, K, splits, stride, nullptr, true, nt_w));
    return STS_OK;
  };
  for (int l = 0; l < d.n_layers; l++) {
    const LayerW& w = c->layers[l];
    int sp; long long ss;
    STSCK(skinny(STS_K_QKV, ph.Xn, h, w.wqkv, c->qkvn, h, &sp, &ss));
    KL(ph, STS_K_ROPE, decode_qkv_finish(st, ph.part, sp, ss, c->qkvn, ph.d_dseq, ph.d_bt, c->inv_freq, ph.Q, layer_pool(c, l), c->geo, n, d.n_q_heads));
    KL(ph, STS_K_ATTN, attn_decode(st, ph.Q, ph.A, ph.d_dseq, ph.d_ditems, n_items, d_multi, n_multi, ph.d_bt, layer_pool(c, l), c->geo, n, d.n_q_heads, chunk_pages, max_chunks, ph.attn_ws, nt_attn));
    STSCK(skinny(STS_K_O, ph.A, c->qd, w.wo, h, c->qd, &sp, &ss));
    KL(ph, STS_K_REDUCE, reduce_resid_norm(st, ph.X, ph.part, sp, ss, ph.Xn, w.g2, d.rms_eps, n, h));
    {
      // gate/up: SwiGLU is the GEMM's epilogue unless cutting K, with its partial sums and the kernel that reduces them
      // (taken as 4 us of launch and start-up), is estimated faster
      int gu_cfg, gu_splits, fu_cfg, fu_splits;
      const double t_split = pick_decode_gemm(c, n, 2 * d.mlp, h, ph.cus, true, true, &gu_cfg, &gu_splits) + 4e-6;
      const double t_fused = pick_decode_gemm(c, n, 2 * d.mlp, h, ph.cus, false, false, &fu_cfg, &fu_splits);
      const bool can_fuse = fu_cfg == GEMM_64x128 || (fu_cfg >= GEMM_64x256S && fu_cfg <= GEMM_64x512S);
      if (can_fuse && (t_fused <= t_split || gu_splits == 1)) {
        KL(ph, STS_K_GATEUP, gemm_bf16(st, fu_cfg, EPI_SWIGLU_BF16, ph.Xn, h, w.wgu, h, ph.H, d.mlp, n, 2 * d.mlp, h, 1, 0, nullptr, true, nt_w));
      } else {
        STSCK(skinny(STS_K_GATEUP, ph.Xn, h, w.wgu, 2 * d.mlp, h, &sp, &ss));
        KL(ph, STS_K_SWIGLU, reduce_swiglu(st, ph.H, ph.part, sp, ss, n, d.mlp));
      }
    }
    STSCK(skinny(STS_K_DOWN, ph.H, d.mlp, w.wd, h, d.mlp, &sp, &ss));
    const float* next_gain = (l + 1 < d.n_layers) ? c->layers[l + 1].g1 : c->gf;
    KL(ph, STS_K_REDUCE, reduce_resid_norm(st, ph.X, ph.part, sp, ss, ph.Xn, next_gain, d.rms_eps, n, h));
  }
  if (want_logits || want_next) {
    int head_cfg, head_splits;
    pick_decode_gemm(c, n, d.vocab, h, ph.cus, false, false, &head_cfg, &head_splits);
    KL(ph, STS_K_HEAD, gemm_bf16(st, head_cfg, EPI_F32, ph.Xn, h, c->lm, h, ph.logits, d.vocab, n, d.vocab, h, 1, 0, nullptr, true, nt_w));
    if (want_next) {
      KL(ph, STS_K_SAMPLE, argmax_rows(st, ph.next, ph.logits, n, d.vocab));
      HIPCK(hipMemcpyAsync(ph.h_next, ph.next, n * sizeof(int), hipMemcpyDeviceToHost, st));
    }
    if (want_logits) HIPCK(hipMemcpyAsync(ph.h_logits, ph.logits, (size_t)n * d.vocab * sizeof(float), hipMemcpyDeviceToHost, st));
  }
  HIPCK(hipEventRecord(ph.ev1, st));
  ph.ran = true; ph.rows = n;
  return STS_OK;
}

int decode_finish(sts_ctx* c, const int32_t* seqs, int n, float* logits, int32_t* next) {
  Phase& ph = c->ph[1];
  HIPCK(wait_stream(ph.stream));
  STSCK(k_collect(c, ph));
  for (int i = 0; i < n; i++) c->seqs[seqs[i]].len += 1;
  if (logits) std::memcpy(logits, ph.h_logits, (size_t)n * c->d.vocab * sizeof(float));
  if (next) std::memcpy(next, ph.h_next, n * sizeof(int));
  return STS_OK;
}

int64_t now_ns() {
  return std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

int alloc_phase(sts_ctx* c, int side) {
  Phase& ph = c->ph[side];
  ph.side = side;
  const sts_model_desc& d = c->d;
  const size_t rows = side == 0 ? c->p.max_prefill_tokens : c->p.max_decode_batch;
  const size_t nseq = side == 0 ? c->p.max_prefill_seqs : c->p.max_decode_batch;
  const size_t mp = c->p.max_pages_per_seq;
  HIPCK(hipEventCreate(&ph.ev0)); HIPCK(hipEventCreate(&ph.ev1));
  STSCK(dev_alloc(c, &ph.X, rows * d.hidden));
  STSCK(dev_alloc(c, &ph.Xn, rows * d.hidden));
  STSCK(dev_alloc(c, &ph.A, rows * c->qd));
  STSCK(dev_alloc(c, &ph.H, rows * d.mlp));
  STSCK(dev_alloc(c, &ph.Xlast, nseq * d.hidden));
  STSCK(dev_alloc(c, &ph.Xlast_n, nseq * d.hidden));
  STSCK(dev_alloc(c, &ph.logits, nseq * d.vocab));
  STSCK(dev_alloc(c, &ph.next, nseq));
  {
    const size_t items = rows / attn_prefill_tile_q() + nseq + 1;
    // decode attention items: a context has at most 128 chunks, and fewer than one per 4 pages (chunks hold >= 8)
    const size_t dec_items = side == 1 ? nseq * (size_t)decode_max_chunks((int)mp) : 0;
    ph.meta_bytes = nseq * (sizeof(PrefillSeq) + sizeof(DecodeSeq) + 2 * sizeof(int)) + items * sizeof(AttnItem) + dec_items * sizeof(DecodeItem) +
                    rows * sizeof(int) + nseq * mp * sizeof(int) + 8 * 256;
    STSCK(dev_alloc(c, &ph.d_meta, ph.meta_bytes));
    STSCK(host_alloc(&ph.h_meta, ph.meta_bytes));
  }
  STSCK(host_alloc(&ph.h_logits, nseq * d.vocab));
  STSCK(host_alloc(&ph.h_next, nseq));
  if (side == 0) {
    STSCK(dev_alloc(c, &ph.QKV, rows * c->qkvn));
    const size_t tail_floats = (size_t)c->n_cu * 256 * 256;   // one wave of partial tiles at the largest tile on every CU
    STSCK(dev_alloc(c, &ph.tail_ws, tail_floats));
    ph.tail_ws_bytes = tail_floats * sizeof(float);
  } else {
    const size_t widest = std::max<size_t>(std::max(c->qkvn, 2 * d.mlp), d.hidden);
    const size_t max_chunks = decode_max_chunks((int)mp);
    STSCK(dev_alloc(c, &ph.part, 8 * rows * widest));
    STSCK(dev_alloc(c, &ph.Q, rows * c->qd));
    STSCK(dev_alloc(c, &ph.attn_ws, attn_decode_ws_floats((int)rows, d.n_q_heads, d.head_dim, (int)max_chunks)));
  }
  return STS_OK;
}

// packed: the tensor is a GEMM weight kept in the packed block layout; the embedding table, read by rows, is row-major
struct TensorRef { bf16* w = nullptr; float* g = nullptr; int ld = 0, rows = 0, cols = 0, row_off = 0, ib = 0, phase = 0; uint64_t tid = 0; int packed = 1; };

int find_tensor(sts_ctx* c, int layer, const char* name, TensorRef* t) {
  const sts_model_desc& d = c->d;
  const std::string n(name ? name : "");
  if (n == "emb") { *t = TensorRef{c->emb, nullptr, d.hidden, d.vocab, d.hidden, 0, 0, 0, 0, 0}; return STS_OK; }
  if (n == "lm") { *t = TensorRef{c->lm, nullptr, d.hidden, d.vocab, d.hidden, 0, 0, 0, 1}; return STS_OK; }
  if (n == "gf") { *t = TensorRef{nullptr, c->gf, 0, 1, d.hidden}; return STS_OK; }
  if (layer < 0 || layer >= d.n_layers) return STS_EINVAL;
  LayerW& w = c->layers[layer];
  const uint64_t base = (uint64_t)(layer + 1) * 16;
  if (n == "g1") { *t = TensorRef{nullptr, w.g1, 0, 1, d.hidden}; return STS_OK; }
  if (n == "g2") { *t = TensorRef{nullptr, w.g2, 0, 1, d.hidden}; return STS_OK; }
  if (n == "wq") { *t = TensorRef{w.wqkv, nullptr, d.hidden, c->qd, d.hidden, 0, 0, 0, base + 0}; return STS_OK; }
  if (n == "wk") { *t = TensorRef{w.wqkv, nullptr, d.hidden, c->kvd, d.hidden, c->qd, 0, 0, base + 1}; return STS_OK; }
  if (n == "wv") { *t = TensorRef{w.wqkv, nullptr, d.hidden, c->kvd, d.hidden, c->qd + c->kvd, 0, 0, base + 2}; return STS_OK; }
  if (n == "wo") { *t = TensorRef{w.wo, nullptr, c->qd, d.hidden, c->qd, 0, 0, 0, base + 3}; return STS_OK; }
  if (n == "wg") { *t = TensorRef{w.wgu, nullptr, d.hidden, d.mlp, d.hidden, 0, 32, 0, base + 4}; return STS_OK; }
  if (n == "wu") { *t = TensorRef{w.wgu, nullptr, d.hidden, d.mlp, d.hidden, 0, 32, 1, base + 5}; return STS_OK; }
  if (n == "wd") { *t = TensorRef{w.wd, nullptr, d.mlp, d.hidden, d.mlp, 0, 0, 0, base + 6}; return STS_OK; }
  return STS_EINVAL;
}

}  // namespace

// ======================================================================================= C ABI
extern "C" int sts_init(const sts_model_desc* desc, const sts_init_params* params, sts_ctx** out) {
  if (!desc || !params || !out) return STS_EINVAL;
  const sts_model_desc& d = *desc;
  if (d.n_layers < 1 || d.hidden < 64 || d.hidden % 128 || d.mlp % 64 || (2 * d.mlp) % 128 || d.vocab % 128) return STS_EINVAL;
  if ((d.head_dim != 64 && d.head_dim != 128) || d.page_tokens != 16) return STS_EINVAL;
  if (d.n_kv_heads < 1 || d.n_q_heads % d.n_kv_heads) return STS_EINVAL;
  const int grp = d.n_q_heads / d.n_kv_heads;
  if (!(grp == 1 || grp == 4 || (grp == 8 && d.head_dim == 128))) return STS_EINVAL;
  if (((d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim) % 128 || (d.n_q_heads * d.head_dim) % 64 || d.mlp % 32) return STS_EINVAL;
  if (params->kv_pool_pages < 1 || params->max_prefill_tokens < 1 || params->max_prefill_seqs < 1 ||
      params->max_decode_batch < 1 || params->max_seqs < 1 || params->max_pages_per_seq < 1) return STS_EINVAL;
  // decode attention cuts a context into at most 128 chunks (the merge workspace and the work list are sized for that)
  if (params->max_pages_per_seq > sts_max_pages_per_seq_limit(d.page_tokens)) return STS_EINVAL;
  if (g_streams_released.load()) return STS_ESTATE;
  int ndev = 0;
  HIPCK(hipGetDeviceCount(&ndev));
  if (ndev < 1) { g_hip_err = (int)hipErrorNoDevice; return STS_EHIP; }
  HIPCK(hipSetDevice(0));
  hipDeviceProp_t prop;
  HIPCK(hipGetDeviceProperties(&prop, 0));
  sts_ctx* c = new sts_ctx();
  g_live_ctx++;
  c->d = d; c->p = *params; c->n_cu = prop.multiProcessorCount;
  c->qd = d.n_q_heads * d.head_dim; c->kvd = d.n_kv_heads * d.head_dim; c->qkvn = c->qd + 2 * c->kvd;
  c->geo = KvGeom{d.n_kv_heads, d.head_dim, d.page_tokens};
  auto fail = [&](int rc) { sts_destroy(c); return rc; };
  int rc;
  // weights
  if ((rc = dev_alloc(c, &c->emb, (size_t)d.vocab * d.hidden)) || (rc = dev_alloc(c, &c->lm, (size_t)d.vocab * d.hidden)) ||
      (rc = dev_alloc(c, &c->gf, d.hidden))) return fail(rc);
  c->layers.resize(d.n_layers);
  for (auto& w : c->layers) {
    if ((rc = dev_alloc(c, &w.wqkv, (size_t)c->qkvn * d.hidden)) || (rc = dev_alloc(c, &w.wo, (size_t)d.hidden * c->qd)) ||
        (rc = dev_alloc(c, &w.wgu, (size_t)2 * d.mlp * d.hidden)) || (rc = dev_alloc(c, &w.wd, (size_t)d.hidden * d.mlp)) ||
        (rc = dev_alloc(c, &w.g1, d.hidden)) || (rc = dev_alloc(c, &w.g2, d.hidden))) return fail(rc);
  }
  // KV pool
  c->pool_layer_elems = (size_t)params->kv_pool_pages * c->geo.page_elems();
  if ((rc = dev_alloc(c, &c->pool, c->pool_layer_elems * d.n_layers))) return fail(rc);
  if (hipMemset(c->pool, 0, c->pool_layer_elems * d.n_layers * sizeof(bf16)) != hipSuccess) return fail(STS_EHIP);
  c->page_used.assign(params->kv_pool_pages, 0);
  for (int pg = params->kv_pool_pages - 1; pg >= 0; pg--) c->free_pages.push_back(pg);   // pop_back hands out page 0 first
  c->seqs.resize(params->max_seqs);
  // rotary frequencies theta^(-2i/d), in double
  {
    std::vector<double> f(d.head_dim / 2);
    for (int i = 0; i < d.head_dim / 2; i++) f[i] = std::pow((double)d.rope_theta, -2.0 * i / d.head_dim);
    if ((rc = dev_alloc(c, &c->inv_freq, f.size()))) return fail(rc);
    if (hipMemcpy(c->inv_freq, f.data(), f.size() * sizeof(double), hipMemcpyHostToDevice) != hipSuccess) return fail(STS_EHIP);
  }
  for (int side = 0; side < 2; side++) if ((rc = alloc_phase(c, side))) return fail(rc);
  // gains = 1, weights generated or zero
  auto ones = [&](float* g) { return fill_f32(nullptr, g, 1.0f, d.hidden) == hipSuccess ? STS_OK : STS_EHIP; };
  if ((rc = ones(c->gf))) return fail(rc);
  for (auto& w : c->layers) if ((rc = ones(w.g1)) || (rc = ones(w.g2))) return fail(rc);
  const char* mats[] = {"emb", "lm", "wq", "wk", "wv", "wo", "wg", "wu", "wd"};
  for (int l = 0; l < d.n_layers; l++) {
    for (const char* name : mats) {
      const bool global = !std::strcmp(name, "emb") || !std::strcmp(name, "lm");
      if (global && l > 0) continue;
      TensorRef t;
      if ((rc = find_tensor(c, l, name, &t))) return fail(rc);
      hipError_t e;
      if (params->init_weights) e = init_weight(nullptr, t.w, t.ld, params->weight_seed, t.tid, t.rows, t.cols, t.row_off, t.ib, t.phase, t.packed);
      else e = hipMemset(t.w + (size_t)(t.ib ? 0 : t.row_off) * t.ld, 0, (size_t)(t.ib ? 2 * t.rows : t.rows) * t.ld * sizeof(bf16));
      if (e != hipSuccess) { g_hip_err = (int)e; return fail(STS_EHIP); }
    }
  }
  if (hipDeviceSynchronize() != hipSuccess) return fail(STS_EHIP);
  // default partition: the whole GPU for both phases (time-multiplexed) until told otherwise
  c->part_cus[0] = c->part_cus[1] = c->n_cu;
  if ((rc = select_streams(c))) return fail(rc);
  *out = c;
  return STS_OK;
}

extern "C" int sts_max_pages_per_seq_limit(int32_t page_tokens) {
  return page_tokens > 0 ? 128 * (attn_decode_max_chunk_tokens() / page_tokens) : 0;
}
extern "C" int sts_decode_gemm_plan(int32_t m, int32_t n, int32_t k, int32_t cus, int32_t may_split, int32_t partials, int64_t gemm_rate_256,
                                    int64_t partial_bw_cu, int64_t stream_bw_cu, int64_t stream_bw_gpu, int32_t* tile_cfg, int32_t* split_k, int64_t* est_ns) {
  if (m < 1 || n < 128 || n % 128 != 0 || k < 64 || k % 64 != 0 || cus < 1 || gemm_rate_256 < 1 || partial_bw_cu < 1 || stream_bw_cu < 1 ||
      stream_bw_gpu < 1 || !tile_cfg || !split_k) return STS_EINVAL;
  int cfg = 0, splits = 1;
  const StreamRates r{gemm_rate_256 * 1e-3, partial_bw_cu * 1e6, stream_bw_cu * 1e6, stream_bw_gpu * 1e6};
  const double t = plan_decode_gemm(r, m, n, k, cus, may_split != 0, partials != 0, &cfg, &splits);
  *tile_cfg = cfg; *split_k = splits;
  if (est_ns) *est_ns = (int64_t)(t * 1e9);
  return STS_OK;
}
extern "C" int sts_decode_chunk_plan(const int32_t* n_pages, int32_t n, int32_t n_kv_heads, int32_t cus, int32_t page_tokens,
                                     int32_t max_pages_per_seq, int32_t* chunk_pages, int32_t* max_chunks, int32_t* allocated_chunks) {
  if (!n_pages || n < 1 || n_kv_heads < 1 || cus < 1 || page_tokens < 1 || !chunk_pages || !max_chunks || !allocated_chunks) return STS_EINVAL;
  for (int i = 0; i < n; i++) if (n_pages[i] < 1 || n_pages[i] > max_pages_per_seq) return STS_EINVAL;
  decode_chunk_plan(n_pages, n, n_kv_heads, cus, page_tokens, chunk_pages, max_chunks);
  *allocated_chunks = decode_max_chunks(max_pages_per_seq);
  return STS_OK;
}

extern "C" int sts_destroy(sts_ctx* c) {
  if (!c) return STS_EINVAL;
  // Everything this ctx ever queued must have drained before its buffers go: the pooled streams of
  // every partition it selected (they outlive the ctx), and the null stream used by the weight
  // loaders and the KV test hooks.
  trace("destroy: sync every stream this ctx used");
  for (hipStream_t s : c->used_streams) (void)hipStreamSynchronize(s);
  (void)hipStreamSynchronize(nullptr);
  trace("destroy: events and pinned buffers");
  for (int side = 0; side < 2; side++) {
    Phase& ph = c->ph[side];
    if (ph.ev0) (void)hipEventDestroy(ph.ev0);
    if (ph.ev1) (void)hipEventDestroy(ph.ev1);
    for (hipEvent_t e : ph.kev) (void)hipEventDestroy(e);
    void* hosts[] = {ph.h_meta, ph.h_logits, ph.h_next};
    for (void* p : hosts) if (p) (void)hipHostFree(p);
  }
  trace("destroy: device memory");
  for (void* p : c->allocs) (void)hipFree(p);
  if (c->probe_src) (void)hipFree(c->probe_src);
  if (c->probe_dst) (void)hipFree(c->probe_dst);
  delete c;
  g_live_ctx--;
  trace("destroy: done");
  return STS_OK;
}

extern "C" int sts_release_streams(void) {
  std::lock_guard<std::mutex> g(g_stream_mu);
  if (g_live_ctx.load() != 0) return STS_ESTATE;
  g_streams_released.store(true);
  for (auto& kv : g_streams) (void)hipStreamSynchronize(kv.second);
  while (!g_streams.empty()) {
    hipStream_t s = g_streams.begin()->second;
    g_streams.erase(g_streams.begin());
    HIPCK(hipStreamDestroy(s));
  }
  return STS_OK;
}

extern "C" int sts_load_weights(sts_ctx* c, int32_t layer, const char* name, const float* host, size_t count) {
  if (!c || !host) return STS_EINVAL;
  TensorRef t;
  STSCK(find_tensor(c, layer, name, &t));
  if (count != (size_t)t.rows * t.cols) return STS_EINVAL;
  if (t.g) { HIPCK(hipMemcpy(t.g, host, count * sizeof(float), hipMemcpyHostToDevice)); return STS_OK; }
  float* tmp = nullptr;
  HIPCK(hipMalloc(&tmp, count * sizeof(float)));
  hipError_t e = hipMemcpy(tmp, host, count * sizeof(float), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = convert_weight(nullptr, t.w, t.ld, tmp, t.rows, t.cols, t.row_off, t.ib, t.phase, t.packed);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  (void)hipFree(tmp);
  HIPCK(e);
  return STS_OK;
}

extern "C" int sts_read_weights(sts_ctx* c, int32_t layer, const char* name, float* host, size_t count) {
  if (!c || !host) return STS_EINVAL;
  TensorRef t;
  STSCK(find_tensor(c, layer, name, &t));
  if (count != (size_t)t.rows * t.cols) return STS_EINVAL;
  if (t.g) { HIPCK(hipMemcpy(host, t.g, count * sizeof(float), hipMemcpyDeviceToHost)); return STS_OK; }
  float* tmp = nullptr;
  HIPCK(hipMalloc(&tmp, count * sizeof(float)));
  hipError_t e = export_weight(nullptr, tmp, t.w, t.ld, t.rows, t.cols, t.row_off, t.ib, t.phase, t.packed);
  if (e == hipSuccess) e = hipMemcpy(host, tmp, count * sizeof(float), hipMemcpyDeviceToHost);
  (void)hipFree(tmp);
  HIPCK(e);
  return STS_OK;
}

// ---- sequences
extern "C" int sts_seq_create(sts_ctx* c, int32_t* seq_out) {
  if (!c || !seq_out) return STS_EINVAL;
  std::lock_guard<std::mutex> g(c->alloc_mu);
  for (size_t i = 0; i < c->seqs.size(); i++)
    if (!c->seqs[i].used) { c->seqs[i] = Seq(); c->seqs[i].used = true; *seq_out = (int)i; return STS_OK; }
  return STS_ENOMEM;
}
extern "C" int sts_seq_free(sts_ctx* c, int32_t seq) {
  if (!c || !valid_seq(c, seq)) return STS_EINVAL;
  {
    // a sequence of the layer-sliced batch or of a launch still in flight keeps its pages: kernels
    // may be reading and writing them
    std::lock_guard<std::mutex> g(c->state_mu);
    if (c->pf_active) for (int s : c->pf_seqs) if (s == seq) return STS_ESTATE;
    for (int s : c->pend_pseqs) if (s == seq) return STS_ESTATE;
    for (int s : c->pend_dseqs) if (s == seq) return STS_ESTATE;
  }
  std::lock_guard<std::mutex> g(c->alloc_mu);
  for (int pg : c->seqs[seq].pages) { c->page_used[pg] = 0; c->free_pages.push_back(pg); }
  c->seqs[seq] = Seq();
  return STS_OK;
}
extern "C" int sts_seq_length(sts_ctx* c, int32_t seq, int32_t* len_out) {
  if (!c || !valid_seq(c, seq) || !len_out) return STS_EINVAL;
  *len_out = c->seqs[seq].len;
  return STS_OK;
}
extern "C" int sts_seq_truncate(sts_ctx* c, int32_t seq, int32_t new_len) {
  if (!c || !valid_seq(c, seq) || new_len < 0) return STS_EINVAL;
  {
    std::lock_guard<std::mutex> g(c->state_mu);      // not under kernels that append to it or read its length
    if (c->pf_active) for (int s : c->pf_seqs) if (s == seq) return STS_ESTATE;
    for (int s : c->pend_pseqs) if (s == seq) return STS_ESTATE;
    for (int s : c->pend_dseqs) if (s == seq) return STS_ESTATE;
  }
  std::lock_guard<std::mutex> g(c->alloc_mu);
  if (new_len > c->seqs[seq].len) return STS_EINVAL;
  c->seqs[seq].len = new_len;
  return STS_OK;
}
extern "C" int sts_seq_reserve(sts_ctx* c, int32_t seq, int32_t n_tokens) {
  if (!c || !valid_seq(c, seq) || n_tokens < 0) return STS_EINVAL;
  return reserve_pages(c, {{seq, n_tokens}});
}
extern "C" int sts_pages_free(sts_ctx* c, int32_t* n_out) {
  if (!c || !n_out) return STS_EINVAL;
  std::lock_guard<std::mutex> g(c->alloc_mu);
  *n_out = (int)c->free_pages.size();
  return STS_OK;
}
extern "C" int sts_seq_set_block_table(sts_ctx* c, int32_t seq, const int32_t* pages, int32_t n) {
  if (!c || !valid_seq(c, seq) || !pages || n < 0 || n > c->p.max_pages_per_seq) return STS_EINVAL;
  std::lock_guard<std::mutex> g(c->alloc_mu);
  Seq& s = c->seqs[seq];
  if (s.len != 0 || !s.pages.empty()) return STS_ESTATE;
  for (int i = 0; i < n; i++) {
    if (pages[i] < 0 || pages[i] >= c->p.kv_pool_pages || c->page_used[pages[i]]) return STS_EINVAL;
    for (int j = 0; j < i; j++) if (pages[j] == pages[i]) return STS_EINVAL;
  }
  for (int i = 0; i < n; i++) {
    c->page_used[pages[i]] = 1;
    c->free_pages.erase(std::find(c->free_pages.begin(), c->free_pages.end(), pages[i]));
    s.pages.push_back(pages[i]);
  }
  return STS_OK;
}
extern "C" int sts_seq_get_block_table(sts_ctx* c, int32_t seq, int32_t* pages, int32_t cap, int32_t* n_out) {
  if (!c || !valid_seq(c, seq) || !n_out) return STS_EINVAL;
  const Seq& s = c->seqs[seq];
  *n_out = (int)s.pages.size();
  for (int i = 0; i < std::min<int>(cap, (int)s.pages.size()); i++) pages[i] = s.pages[i];
  return STS_OK;
}

namespace {
int upload_bt(sts_ctx* c, const Seq& s, int** d_bt) {
  HIPCK(hipMalloc(d_bt, std::max<size_t>(1, s.pages.size()) * sizeof(int)));
  HIPCK(hipMemcpy(*d_bt, s.pages.data(), s.pages.size() * sizeof(int), hipMemcpyHostToDevice));
  return STS_OK;
}
}  // namespace

extern "C" int sts_kv_write(sts_ctx* c, int32_t layer, int32_t seq, int32_t pos0, int32_t n, const float* k, const float* v) {
  if (!c || !valid_seq(c, seq) || layer < 0 || layer >= c->d.n_layers || pos0 < 0 || n < 1 || !k || !v) return STS_EINVAL;
  STSCK(reserve_pages(c, {{seq, pos0 + n}}));
  Seq& s = c->seqs[seq];
  const size_t cnt = (size_t)n * c->kvd;
  int* d_bt = nullptr; float *dk = nullptr, *dv = nullptr;
  STSCK(upload_bt(c, s, &d_bt));
  HIPCK(hipMalloc(&dk, cnt * sizeof(float))); HIPCK(hipMalloc(&dv, cnt * sizeof(float)));
  HIPCK(hipMemcpy(dk, k, cnt * sizeof(float), hipMemcpyHostToDevice));
  HIPCK(hipMemcpy(dv, v, cnt * sizeof(float), hipMemcpyHostToDevice));
  HIPCK(kv_write_tokens(nullptr, layer_pool(c, layer), c->geo, d_bt, pos0, n, dk, dv));
  HIPCK(hipDeviceSynchronize());
  (void)hipFree(d_bt); (void)hipFree(dk); (void)hipFree(dv);
  s.len = std::max(s.len, pos0 + n);
  return STS_OK;
}
extern "C" int sts_kv_read(sts_ctx* c, int32_t layer, int32_t seq, int32_t pos0, int32_t n, float* k, float* v) {
  if (!c || !valid_seq(c, seq) || layer < 0 || layer >= c->d.n_layers || pos0 < 0 || n < 1 || !k || !v) return STS_EINVAL;
  Seq& s = c->seqs[seq];
  if ((size_t)(pos0 + n + c->geo.page_tokens - 1) / c->geo.page_tokens > s.pages.size()) return STS_EINVAL;
  const size_t cnt = (size_t)n * c->kvd;
  int* d_bt = nullptr; float *dk = nullptr, *dv = nullptr;
  STSCK(upload_bt(c, s, &d_bt));
  HIPCK(hipMalloc(&dk, cnt * sizeof(float))); HIPCK(hipMalloc(&dv, cnt * sizeof(float)));
  HIPCK(kv_read_tokens(nullptr, layer_pool(c, layer), c->geo, d_bt, pos0, n, dk, dv));
  HIPCK(hipMemcpy(k, dk, cnt * sizeof(float), hipMemcpyDeviceToHost));
  HIPCK(hipMemcpy(v, dv, cnt * sizeof(float), hipMemcpyDeviceToHost));
  (void)hipFree(d_bt); (void)hipFree(dk); (void)hipFree(dv);
  return STS_OK;
}
extern "C" int sts_kv_fill_random(sts_ctx* c, int32_t seq, int32_t n, uint64_t seed) {
  if (!c || !valid_seq(c, seq) || n < 1) return STS_EINVAL;
  STSCK(reserve_pages(c, {{seq, n}}));
  Seq& s = c->seqs[seq];
  int* d_bt = nullptr;
  STSCK(upload_bt(c, s, &d_bt));
  for (int l = 0; l < c->d.n_layers; l++) HIPCK(kv_fill_random(nullptr, layer_pool(c, l), c->geo, d_bt, 0, n, seed, l));
  HIPCK(hipDeviceSynchronize());
  (void)hipFree(d_bt);
  s.len = n;
  return STS_OK;
}

// ---- the step
extern "C" int sts_prefill_batch(sts_ctx* c, int32_t n_seqs, const int32_t* seqs, const int32_t* lens, const int32_t* tokens,
                                 int32_t lb, int32_t le, float* logits) {
  if (!c) return STS_EINVAL;
  if (c->pend_prefill) return STS_ESTATE;
  const int64_t t0 = now_ns();
  STSCK(prefill_enqueue(c, n_seqs, seqs, lens, tokens, lb, le, logits != nullptr));
  STSCK(prefill_finish(c, n_seqs, seqs, lens, le, logits));
  c->last_wall_ns = now_ns() - t0;
  return STS_OK;
}
extern "C" int sts_prefill_append(sts_ctx* c, int32_t seq, const int32_t* tokens, int32_t n_tokens, int32_t lb, int32_t le, float* logits) {
  return sts_prefill_batch(c, 1, &seq, &n_tokens, tokens, lb, le, logits);
}
// ---- the same step, split into launch / poll / finish for serving loops that keep both phases in
// flight from one control thread
extern "C" int sts_prefill_launch(sts_ctx* c, int32_t n_seqs, const int32_t* seqs, const int32_t* lens, const int32_t* tokens,
                                  int32_t lb, int32_t le, int32_t want_logits) {
  if (!c) return STS_EINVAL;
  if (c->pend_prefill) return STS_ESTATE;
  STSCK(prefill_enqueue(c, n_seqs, seqs, lens, tokens, lb, le, want_logits != 0));
  std::lock_guard<std::mutex> g(c->state_mu);
  c->pend_prefill = true; c->pend_le = le;
  c->pend_pseqs.assign(seqs, seqs + n_seqs); c->pend_plens.assign(lens, lens + n_seqs);
  return STS_OK;
}
extern "C" int sts_decode_launch(sts_ctx* c, const int32_t* seqs, const int32_t* in_tokens, int32_t n, int32_t want_logits, int32_t want_next) {
  if (!c) return STS_EINVAL;
  if (c->pend_decode) return STS_ESTATE;
  {
    // the batch is listed before anything is queued, so that from this moment neither a prefill of
    // one of its sequences nor sts_seq_free gets through
    std::lock_guard<std::mutex> g(c->state_mu);
    c->pend_dseqs.assign(seqs, seqs + std::max(n, 0));
  }
  const int rc = decode_enqueue(c, seqs, in_tokens, n, want_logits != 0, want_next != 0);
  if (rc != STS_OK) { std::lock_guard<std::mutex> g(c->state_mu); c->pend_dseqs.clear(); return rc; }
  c->pend_decode = true;
  return STS_OK;
}
extern "C" int sts_phase_done(sts_ctx* c, int32_t phase, int32_t* done) {
  if (!c || phase < 0 || phase > 1 || !done) return STS_EINVAL;
  if (!(phase == 0 ? c->pend_prefill : c->pend_decode)) return STS_ESTATE;
  const hipError_t e = hipEventQuery(c->ph[phase].ev1);
  if (e == hipSuccess) *done = 1;
  else if (e == hipErrorNotReady) *done = 0;
  else { g_hip_err = (int)e; return STS_EHIP; }
  return STS_OK;
}
extern "C" int sts_prefill_finish(sts_ctx* c, float* logits) {
  if (!c) return STS_EINVAL;
  if (!c->pend_prefill) return STS_ESTATE;
  const std::vector<int> seqs = c->pend_pseqs, lens = c->pend_plens;
  const int rc = prefill_finish(c, (int)seqs.size(), seqs.data(), lens.data(), c->pend_le, logits);
  std::lock_guard<std::mutex> g(c->state_mu);
  c->pend_prefill = false; c->pend_pseqs.clear(); c->pend_plens.clear();
  return rc;
}
extern "C" int sts_decode_finish(sts_ctx* c, float* logits, int32_t* next) {
  if (!c) return STS_EINVAL;
  if (!c->pend_decode) return STS_ESTATE;
  const std::vector<int> seqs = c->pend_dseqs;
  const int rc = decode_finish(c, seqs.data(), (int)seqs.size(), logits, next);
  std::lock_guard<std::mutex> g(c->state_mu);
  c->pend_decode = false; c->pend_dseqs.clear();
  return rc;
}
extern "C" int sts_prefill_abort(sts_ctx* c) {
  if (!c) return STS_EINVAL;
  std::lock_guard<std::mutex> g(c->state_mu);
  c->pf_active = false; c->pf_next_layer = 0; c->pf_seqs.clear(); c->pf_lens.clear();
  return STS_OK;
}
extern "C" int sts_decode_step(sts_ctx* c, const int32_t* seqs, const int32_t* in_tokens, int32_t n, float* logits, int32_t* next) {
  if (!c) return STS_EINVAL;
  if (c->pend_decode) return STS_ESTATE;
  const int64_t t0 = now_ns();
  STSCK(decode_enqueue(c, seqs, in_tokens, n, logits != nullptr, next != nullptr));
  STSCK(decode_finish(c, seqs, n, logits, next));
  c->last_wall_ns = now_ns() - t0;
  return STS_OK;
}
extern "C" int sts_step_concurrent(sts_ctx* c, int32_t n_pseqs, const int32_t* pseqs, const int32_t* plens, const int32_t* ptokens,
                                   int32_t lb, int32_t le, float* plogits, const int32_t* dseqs, const int32_t* dtokens,
                                   int32_t n_decode, float* dlogits, int32_t* dnext) {
  if (!c || n_pseqs < 0 || n_decode < 0 || (n_pseqs == 0 && n_decode == 0)) return STS_EINVAL;
  if (c->pend_prefill || c->pend_decode) return STS_ESTATE;
  for (int i = 0; i < n_pseqs; i++) for (int j = 0; j < n_decode; j++) if (pseqs && dseqs && pseqs[i] == dseqs[j]) return STS_EINVAL;
  const int64_t t0 = now_ns();
  c->ph[0].ran = c->ph[1].ran = false;
  // Both sides are checked and the pages of both are reserved in one step before anything is
  // queued: an invalid argument or an exhausted pool on either side leaves every sequence as it was.
  std::vector<std::pair<int, int>> wants;
  if (n_pseqs > 0) STSCK(prefill_validate(c, n_pseqs, pseqs, plens, ptokens, lb, le, &wants));
  if (n_decode > 0) STSCK(decode_validate(c, dseqs, dtokens, n_decode, &wants));
  STSCK(reserve_pages(c, wants));
  if (n_pseqs > 0) STSCK(prefill_launch_checked(c, n_pseqs, pseqs, plens, ptokens, lb, le, plogits != nullptr));
  const int64_t t1 = now_ns();
  int rc = STS_OK;
  if (n_decode > 0) rc = decode_launch_checked(c, dseqs, dtokens, n_decode, dlogits != nullptr, dnext != nullptr);
  const int64_t t2 = now_ns();
  if (rc != STS_OK) {
    // only a HIP failure can get here; the prefill slice already queued is waited for and dropped
    if (n_pseqs > 0) { (void)wait_stream(c->ph[0].stream); (void)k_collect(c, c->ph[0]); (void)sts_prefill_abort(c); }
    return rc;
  }
  if (n_pseqs > 0) STSCK(prefill_finish(c, n_pseqs, pseqs, plens, le, plogits));
  const int64_t t3 = now_ns();
  if (n_decode > 0) STSCK(decode_finish(c, dseqs, n_decode, dlogits, dnext));
  c->last_wall_ns = now_ns() - t0;
  if (getenv("STS_PROF")) fprintf(stderr, "[sts prof] prefill_enqueue %lld decode_enqueue %lld prefill_wait %lld decode_finish %lld us\n",
                                  (long long)(t1 - t0) / 1000, (long long)(t2 - t1) / 1000, (long long)(t3 - t2) / 1000, (long long)(now_ns() - t3) / 1000);
  return STS_OK;
}
extern "C" int sts_last_timing(sts_ctx* c, int64_t* prefill_ns, int64_t* decode_ns, int64_t* wall_ns) {
  if (!c) return STS_EINVAL;
  int64_t t[2] = {0, 0};
  for (int side = 0; side < 2; side++) {
    if (!c->ph[side].ran) continue;
    float ms = 0.f;
    const hipError_t e = hipEventElapsedTime(&ms, c->ph[side].ev0, c->ph[side].ev1);
    if (e == hipErrorNotReady) { (void)hipGetLastError(); continue; }   // that phase has a launch in flight: reported as 0
    HIPCK(e);
    t[side] = (int64_t)((double)ms * 1e6);
  }
  if (prefill_ns) *prefill_ns = t[0];
  if (decode_ns) *decode_ns = t[1];
  if (wall_ns) *wall_ns = c->last_wall_ns;
  return STS_OK;
}
extern "C" int sts_read_hidden(sts_ctx* c, int32_t phase, float* out, int32_t rows) {
  if (!c || phase < 0 || phase > 1 || !out || rows < 1 || rows > c->ph[phase].rows) return STS_EINVAL;
  HIPCK(hipMemcpy(out, c->ph[phase].X, (size_t)rows * c->d.hidden * sizeof(float), hipMemcpyDeviceToHost));
  return STS_OK;
}

// ---- partition
extern "C" int sts_set_partition(sts_ctx* c, int32_t prefill_cus, int32_t decode_cus) {
  if (!c) return STS_EINVAL;
  std::lock_guard<std::mutex> g(c->part_mu);
  const int old[2] = {c->part_cus[0], c->part_cus[1]};
  if (prefill_cus == -1) prefill_cus = old[0];
  if (decode_cus == -1) decode_cus = old[1];
  const int v[2] = {prefill_cus, decode_cus};
  for (int x : v) if (x != 0 && (x < 8 || x > c->n_cu || x % 8 != 0)) return STS_EINVAL;
  if ((prefill_cus != old[0] && c->pend_prefill) || (decode_cus != old[1] && c->pend_decode)) return STS_ESTATE;
  // only a side whose CU count changes is touched: the other side's control thread may be queuing
  // a step on its stream at this moment
  hipStream_t st[2] = {c->ph[0].stream, c->ph[1].stream};
  for (int side = 0; side < 2; side++) {
    if (v[side] == old[side]) continue;
    if (v[side] == 0) { st[side] = nullptr; continue; }
    const int rc = get_stream(c, side, v[side], &st[side]);
    if (rc != STS_OK) return rc;                  // nothing was changed yet
  }
  for (int side = 0; side < 2; side++) {
    if (v[side] == old[side]) continue;
    c->part_cus[side] = v[side]; c->ph[side].stream = st[side]; c->ph[side].cus = v[side];
    remember_stream(c, st[side]);
  }
  return STS_OK;
}
extern "C" int sts_get_partition(sts_ctx* c, int32_t* prefill_cus, int32_t* decode_cus, int32_t* total_cus) {
  if (!c) return STS_EINVAL;
  if (prefill_cus) *prefill_cus = c->part_cus[0];
  if (decode_cus) *decode_cus = c->part_cus[1];
  if (total_cus) *total_cus = c->n_cu;
  return STS_OK;
}

// ---- measurement hooks
extern "C" int sts_kernel_timing(sts_ctx* c, int32_t on) {
  if (!c) return STS_EINVAL;
  c->ktiming = on != 0;
  return STS_OK;
}
extern "C" int sts_kernel_times(sts_ctx* c, int32_t phase, int64_t* ns, int64_t* launches, int32_t reset) {
  if (!c || phase < 0 || phase > 1) return STS_EINVAL;
  Phase& ph = c->ph[phase];
  for (int k = 0; k < STS_K_COUNT; k++) {
    if (ns) ns[k] = ph.kns[k];
    if (launches) launches[k] = ph.kcnt[k];
    if (reset) { ph.kns[k] = 0; ph.kcnt[k] = 0; }
  }
  return STS_OK;
}
extern "C" int sts_set_tile_model(sts_ctx* c, int64_t gemm_rate_128, int64_t gemm_rate_256, int64_t gemm_rate_128x256, int64_t gemm_fixed_128x256,
                                  int64_t partial_bw_cu) {
  if (!c || gemm_rate_128 < 1 || gemm_rate_256 < 1 || gemm_rate_128x256 < 1 || gemm_fixed_128x256 < 0 || partial_bw_cu < 1) return STS_EINVAL;
  if (c->pend_prefill || c->pend_decode) return STS_ESTATE;
  c->rate_128 = gemm_rate_128 * 1e-3; c->rate_256 = gemm_rate_256 * 1e-3; c->rate_128x256 = gemm_rate_128x256 * 1e-3;
  c->fixed_128x256 = gemm_fixed_128x256 * 1e-9; c->partial_bw = partial_bw_cu * 1e6;
  return STS_OK;
}
extern "C" int sts_set_stream_model(sts_ctx* c, int64_t stream_bw_cu, int64_t stream_bw_gpu) {
  if (!c || stream_bw_cu < 1 || stream_bw_gpu < stream_bw_cu) return STS_EINVAL;
  c->stream_bw_cu = stream_bw_cu * 1e6; c->stream_bw_gpu = stream_bw_gpu * 1e6;
  return STS_OK;
}
extern "C" int sts_probe_gemm(sts_ctx* c, int32_t cus, int32_t tile_cfg, int32_t product, int32_t m, int32_t n, int32_t iters, int64_t* ns_out) {
  if (!c || !ns_out || iters < 1 || tile_cfg < 0 || tile_cfg >= GEMM_NCFG || product < 0 || product > 2) return STS_EINVAL;
  const sts_model_desc& d = c->d;
  const int n_max = product == 0 ? 2 * d.mlp : d.hidden;
  if (m < 1 || m > c->p.max_prefill_tokens || n < 64 || n > n_max || n % 64 || n % gemm_tile_n(tile_cfg)) return STS_EINVAL;
  // gate/up runs with its SwiGLU epilogue, which needs gate/up block pairs in a wave tile
  if (product == 0 && (tile_cfg == GEMM_64x256 || tile_cfg == GEMM_128x256)) return STS_EINVAL;
  if (c->pend_prefill) return STS_ESTATE;
  hipStream_t st;
  STSCK(get_stream(c, 0, cus, &st));
  { std::lock_guard<std::mutex> g(c->part_mu); remember_stream(c, st); }
  Phase& ph = c->ph[0];
  struct Events {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ~Events() { if (e0) (void)hipEventDestroy(e0); if (e1) (void)hipEventDestroy(e1); }
  } ev;
  HIPCK(hipEventCreate(&ev.e0)); HIPCK(hipEventCreate(&ev.e1));
  const LayerW& w0 = c->layers[0];
  auto run = [&]() {
    if (product == 1) return gemm_bf16(st, tile_cfg, EPI_RESID_F32, ph.A, c->qd, w0.wo, c->qd, ph.X, d.hidden, m, n, c->qd, 1, 0);
    if (product == 2) return gemm_bf16(st, tile_cfg, EPI_RESID_F32, ph.H, d.mlp, w0.wd, d.mlp, ph.X, d.hidden, m, n, d.mlp, 1, 0);
    return gemm_bf16(st, tile_cfg, EPI_SWIGLU_BF16, ph.Xn, d.hidden, w0.wgu, d.hidden, ph.H, d.mlp, m, n, d.hidden, 1, 0);
  };
  for (int i = 0; i < 2; i++) HIPCK(run());                         // warm-up
  HIPCK(hipEventRecord(ev.e0, st));
  for (int i = 0; i < iters; i++) HIPCK(run());
  HIPCK(hipEventRecord(ev.e1, st));
  HIPCK(hipEventSynchronize(ev.e1));
  float ms = 0.f;
  HIPCK(hipEventElapsedTime(&ms, ev.e0, ev.e1));
  *ns_out = (int64_t)((double)ms * 1e6);
  return STS_OK;
}
static int probe_stream(sts_ctx* c, int32_t side, int32_t cus, size_t bytes, int32_t iters, int64_t* ns_out, bool read_only) {
  if (!c || side < 0 || side > 1 || bytes < 4096 || bytes % 16 || iters < 1 || !ns_out) return STS_EINVAL;
  hipStream_t st;
  STSCK(get_stream(c, side, cus, &st));
  { std::lock_guard<std::mutex> g(c->part_mu); remember_stream(c, st); }
  if (c->probe_bytes < bytes) {
    if (c->probe_src) { (void)hipFree(c->probe_src); (void)hipFree(c->probe_dst); c->probe_src = c->probe_dst = nullptr; c->probe_bytes = 0; }
    HIPCK(hipMalloc(&c->probe_src, bytes)); HIPCK(hipMalloc(&c->probe_dst, bytes));
    HIPCK(hipMemset(c->probe_src, 1, bytes)); HIPCK(hipMemset(c->probe_dst, 0, bytes));
    HIPCK(hipDeviceSynchronize());
    c->probe_bytes = bytes;
  }
  struct Events {                                                   // destroyed on every return path
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ~Events() { if (e0) (void)hipEventDestroy(e0); if (e1) (void)hipEventDestroy(e1); }
  } ev;
  HIPCK(hipEventCreate(&ev.e0)); HIPCK(hipEventCreate(&ev.e1));
  // The copy runs 8 workgroups per CU. The read stream's rate depends on how many workgroups share a CU (on the whole GPU
  // two per CU read a fifth more than eight), and the probe reports what the memory system can give: the best of 2, 4 and 8.
  // Its sink is the first word of the copy's destination buffer.
  float best_ms = 0.f;
  for (int per_cu : {8, 4, 2}) {
    const int grid = cus * per_cu;
    auto launch = [&]() { return read_only ? read_probe(st, c->probe_src, bytes, reinterpret_cast<unsigned*>(c->probe_dst), grid)
                                           : copy_probe(st, c->probe_dst, c->probe_src, bytes, grid); };
    HIPCK(launch());   // warm-up
    HIPCK(hipEventRecord(ev.e0, st));
    for (int i = 0; i < iters; i++) HIPCK(launch());
    HIPCK(hipEventRecord(ev.e1, st));
    HIPCK(hipEventSynchronize(ev.e1));
    float ms = 0.f;
    HIPCK(hipEventElapsedTime(&ms, ev.e0, ev.e1));
    if (best_ms == 0.f || ms < best_ms) best_ms = ms;
    if (!read_only) break;
  }
  *ns_out = (int64_t)((double)best_ms * 1e6);
  return STS_OK;
}
extern "C" int sts_probe_copy(sts_ctx* c, int32_t side, int32_t cus, size_t bytes, int32_t iters, int64_t* ns_out) {
  return probe_stream(c, side, cus, bytes, iters, ns_out, false);
}
extern "C" int sts_probe_read(sts_ctx* c, int32_t side, int32_t cus, size_t bytes, int32_t iters, int64_t* ns_out) {
  return probe_stream(c, side, cus, bytes, iters, ns_out, true);
}
