// Performance estimator (paper Section 3.2): wave quantisation (Section 2.2.1), the SM-scaling
// roofline model (Eq. 1), the calibration factor alpha (Eq. 2) interpolated over sampled
// execution states, and the measured co-run bandwidth D_{p,sl} for decode (Section 3.2.3).
// Host only. Integer arithmetic throughout (ns, flop, bytes, flop/ns, bytes/ns, alpha in ppm,
// floor division), so that scheduling decisions are reproducible bit for bit.
#include "latency.h"

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <sstream>
#include <string>

namespace sts {

using i128 = __int128;

int64_t floor_div(i128 a, i128 b) {
  i128 q = a / b, r = a % b;
  if (r != 0 && ((r < 0) != (b < 0))) q -= 1;
  return (int64_t)q;
}
static inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

void wave_quant(int64_t g, int64_t n, int64_t b, int64_t* w, int64_t* tail) {
  *w = cdiv(g, b * n);
  *tail = cdiv(g - b * n * (*w - 1), b);
}

int64_t Grid::min_value() const { return values.empty() ? 0 : *std::min_element(values.begin(), values.end()); }

// Multilinear interpolation, first axis outermost; outside the grid the nearest segment is
// extended; floor at every stage.
static int64_t interp_rec(const Grid& g, size_t axis, size_t offset, size_t stride, const int64_t* x) {
  if (axis == g.axes.size()) return g.values[offset];
  const std::vector<int64_t>& ax = g.axes[axis];
  const size_t sub = stride / ax.size();
  if (ax.size() == 1) return interp_rec(g, axis + 1, offset, sub, x);
  size_t i = 0;
  while (i + 2 < ax.size() && x[axis] >= ax[i + 1]) i++;
  const int64_t v0 = interp_rec(g, axis + 1, offset + i * sub, sub, x);
  const int64_t v1 = interp_rec(g, axis + 1, offset + (i + 1) * sub, sub, x);
  return v0 + floor_div((i128)(v1 - v0) * (x[axis] - ax[i]), ax[i + 1] - ax[i]);
}
int64_t interp(const Grid& g, const int64_t* x) { return interp_rec(g, 0, 0, g.values.size(), x); }

int64_t alpha_at(const Grid& g, const int64_t* x) {
  return std::max<int64_t>(std::max<int64_t>(interp(g, x), g.min_value() / 2), 1);
}

struct Kern { int64_t flop, mem, g; bool gemm = false; };

static void prefill_kernels(const sts_model_desc& s, const Profile& hw, const int32_t* sl, const int32_t* p, int n,
                            std::vector<Kern>* ks, Kern* head) {
  const int64_t h = s.hidden, d = s.head_dim, qd = (int64_t)s.n_q_heads * d, kvd = (int64_t)s.n_kv_heads * d, qkvn = qd + 2 * kvd;
  const int64_t mlp = s.mlp;
  int64_t t = 0, att_flop = 0, att_mem = 0, att_g = 0;
  for (int i = 0; i < n; i++) {
    const int64_t l = sl[i], c = p[i];
    t += l;
    att_flop += 4 * qd * (l * c + l * (l + 1) / 2);
    att_mem += 2 * (2 * l * qd + 2 * (c + l) * kvd);
    att_g += cdiv(l, hw.tile_q) * s.n_q_heads;
  }
  const int64_t rows = cdiv(t, hw.tile_m), tn = hw.tile_n;
  const int64_t tp = hw.use_waveq ? rows * hw.tile_m : t;      // thread blocks compute whole tiles
  ks->clear();
  ks->push_back({4 * t * h, 4 * t * h, 0});                                                             // norm1
  ks->push_back({2 * tp * h * qkvn, 2 * (h * qkvn + t * h + t * qkvn), rows * cdiv(qkvn, tn), true});    // qkv
  ks->push_back({4 * t * qkvn, 4 * t * qkvn, 0});                                                       // rope
  ks->push_back({att_flop, att_mem, att_g});                                                            // attn
  ks->push_back({2 * tp * qd * h, 2 * (qd * h + t * qd + 2 * t * h), rows * cdiv(h, tn), true});         // o
  ks->push_back({4 * t * h, 4 * t * h, 0});                                                             // norm2
  ks->push_back({4 * tp * h * mlp, 2 * (2 * h * mlp + t * h + t * mlp), rows * cdiv(2 * mlp, tn), true}); // gate/up
  ks->push_back({2 * tp * mlp * h, 2 * (mlp * h + t * mlp + 2 * t * h), rows * cdiv(h, tn), true});      // down
  const int64_t b = n, v = s.vocab;
  *head = Kern{2 * b * h * v, 2 * (h * v + b * h + b * v), 0, false};
}

static void decode_kernels(const sts_model_desc& s, const int32_t* cl, int n, std::vector<Kern>* ks, Kern* head) {
  const int64_t h = s.hidden, d = s.head_dim, qd = (int64_t)s.n_q_heads * d, kvd = (int64_t)s.n_kv_heads * d, qkvn = qd + 2 * kvd;
  const int64_t mlp = s.mlp, b = n, v = s.vocab;
  int64_t ctx = 0;
  for (int i = 0; i < n; i++) ctx += (int64_t)cl[i] + 1;
  ks->clear();
  ks->push_back({4 * b * h, 4 * b * h, 0});
  ks->push_back({2 * b * h * qkvn, 2 * (h * qkvn + b * h + b * qkvn), 0});
  ks->push_back({4 * b * qkvn, 4 * b * qkvn, 0});
  ks->push_back({4 * qd * ctx, 2 * (2 * kvd * ctx + 2 * b * qd), 0});
  ks->push_back({2 * b * qd * h, 2 * (qd * h + b * qd + 2 * b * h), 0});
  ks->push_back({4 * b * h, 4 * b * h, 0});
  ks->push_back({4 * b * h * mlp, 2 * (2 * h * mlp + b * h + b * mlp), 0});
  ks->push_back({2 * b * mlp * h, 2 * (mlp * h + b * mlp + 2 * b * h), 0});
  *head = Kern{2 * b * h * v, 2 * (h * v + b * h + b * v), 0, false};
}

// Eq. 1: T' = flop / min(flop/mem * D_p, C_p) = max(flop / C_p, mem / D_p).
int64_t srm_ns(int64_t flop, int64_t mem, int64_t n_p, const Profile& hw, int64_t d_override) {
  const int64_t t_c = floor_div((i128)flop * hw.n_cu, (i128)hw.c_peak * n_p);
  int64_t t_m;
  if (d_override >= 0) t_m = floor_div(mem, std::max<int64_t>(d_override, 1));
  else t_m = floor_div((i128)mem * hw.n_d, (i128)hw.d_peak * std::min<int64_t>(n_p, hw.n_d));
  return std::max(t_c, t_m);
}

static int64_t waveq_adjust(int64_t t, int64_t g, int64_t n_p, int64_t b) {
  int64_t w, tail;
  wave_quant(g, n_p, b, &w, &tail);
  return floor_div((i128)t * n_p * w, n_p * w - n_p + tail);
}

// The GEMM kernels' remedy for wave quantisation: `full` waves of whole tiles, then the rest
// tiles cut along K into f pieces that take `rounds` rounds of 1/f tile time plus a fixed cost
// per piece (3 % of a tile time); f = 1 when no cut in 2..max_cut saves a tenth of a tile time.
static constexpr int64_t PIECE_COST_PPM = 30000;
static void tail_plan(int64_t g, int64_t slots, int64_t max_cut, int64_t* full, int64_t* f, int64_t* rounds) {
  *full = g / slots;
  const int64_t rest = g - *full * slots;
  *f = 1; *rounds = rest ? 1 : 0;
  if (rest == 0 || max_cut < 2) return;
  int64_t best = 1, best_cost = PPM;
  for (int64_t cut = 2; cut <= max_cut; cut++) {
    const int64_t r = (rest * cut + slots - 1) / slots;
    const int64_t cost = r * (PPM / cut + PIECE_COST_PPM);
    if (cost < best_cost) { best = cut; best_cost = cost; }
  }
  if (best_cost > 900000) return;
  *f = best; *rounds = (rest * best + slots - 1) / slots;
}
static int64_t waveq_tail_adjust(int64_t t, int64_t g, int64_t n_p, int64_t b, int64_t max_cut) {
  const int64_t slots = b * n_p;
  int64_t full, f, rounds;
  tail_plan(g, slots, max_cut, &full, &f, &rounds);
  if (f == 1) return waveq_adjust(t, g, n_p, b);
  const int64_t waves_ppm = full * PPM + rounds * (PPM / f + PIECE_COST_PPM);
  return floor_div((i128)t * waves_ppm * slots, (i128)g * PPM);
}

int64_t prefill_roofline_ns(const sts_model_desc& s, const Profile& hw, const int32_t* sl, const int32_t* p, int n,
                            int pm, int layer_begin, int n_layers_step) {
  std::vector<Kern> ks; Kern head;
  prefill_kernels(s, hw, sl, p, n, &ks, &head);
  int64_t per_layer = 0;
  for (const Kern& k : ks) {
    int64_t t = srm_ns(k.flop, k.mem, pm, hw, -1);
    if (hw.use_waveq && k.g > 0)
      t = hw.tail_cut > 0 && k.gemm ? waveq_tail_adjust(t, k.g, pm, hw.wgs_per_cu, hw.tail_cut) : waveq_adjust(t, k.g, pm, hw.wgs_per_cu);
    per_layer += t;
  }
  int64_t total = per_layer * n_layers_step;
  if (layer_begin + n_layers_step >= s.n_layers) total += srm_ns(head.flop, head.mem, pm, hw, -1);
  return total;
}

int64_t decode_roofline_ns(const sts_model_desc& s, const Profile& hw, const int32_t* cl, int n, int dm, int64_t co_tokens) {
  int64_t d_meas = -1;
  if (!hw.bw.values.empty()) {
    const int64_t x[2] = {dm, co_tokens};
    d_meas = std::max<int64_t>(interp(hw.bw, x), 1);
  }
  std::vector<Kern> ks; Kern head;
  decode_kernels(s, cl, n, &ks, &head);
  int64_t per_layer = 0;
  for (const Kern& k : ks) per_layer += srm_ns(k.flop, k.mem, dm, hw, d_meas);
  return per_layer * s.n_layers + srm_ns(head.flop, head.mem, dm, hw, d_meas);
}

// Slowdown of a prefill slice beside a decode step that runs on co_decode_cus other CUs (1.0 = PPM
// when nothing decodes beside it or no table was measured).
int64_t prefill_corun_ppm(const Profile& hw, int co_decode_cus) {
  if (co_decode_cus <= 0 || hw.prefill_corun.values.empty()) return PPM;
  const int64_t x[1] = {co_decode_cus};
  return alpha_at(hw.prefill_corun, x);
}

int64_t predict_prefill_ns(const sts_model_desc& s, const Profile& hw, const int32_t* sl, const int32_t* p, int n,
                           int pm, int layer_begin, int n_layers_step, int co_decode_cus) {
  if (n <= 0) return 0;
  if (pm <= 0) return INF_NS;
  const int64_t t = prefill_roofline_ns(s, hw, sl, p, n, pm, layer_begin, n_layers_step);
  int64_t tok = 0;
  for (int i = 0; i < n; i++) tok += sl[i];
  const int64_t x[2] = {pm, tok};
  const int64_t alone = floor_div((i128)t * alpha_at(hw.alpha_prefill, x), PPM);
  return floor_div((i128)alone * prefill_corun_ppm(hw, co_decode_cus), PPM);
}

int64_t predict_decode_ns(const sts_model_desc& s, const Profile& hw, const int32_t* cl, int n, int dm, int64_t co_tokens) {
  if (n <= 0) return 0;
  if (dm <= 0) return INF_NS;
  const int64_t t = decode_roofline_ns(s, hw, cl, n, dm, co_tokens);
  int64_t ctx = 0;
  for (int i = 0; i < n; i++) ctx += cl[i];
  const int64_t x[3] = {dm, n, ctx / n};
  return floor_div((i128)t * alpha_at(hw.alpha_decode, x), PPM);
}

// ---- text format -------------------------------------------------------------------------
static bool parse_grid(std::istringstream& in, int nd, Grid* g) {
  g->axes.clear(); g->values.clear();
  std::string line, tok;
  size_t total = 1;
  for (int a = 0; a < nd; a++) {
    if (!std::getline(in, line)) return false;
    std::istringstream ls(line);
    if (!(ls >> tok) || tok != "axis") return false;
    std::vector<int64_t> ax; int64_t v;
    while (ls >> v) ax.push_back(v);
    if (ax.empty()) return false;
    for (size_t i = 1; i < ax.size(); i++) if (ax[i] <= ax[i - 1]) return false;
    total *= ax.size();
    g->axes.push_back(ax);
  }
  if (!std::getline(in, line)) return false;
  std::istringstream ls(line);
  if (!(ls >> tok) || tok != "values") return false;
  int64_t v;
  while (ls >> v) g->values.push_back(v);
  return g->values.size() == total;
}

bool parse_profile(const std::string& text, Profile* hw) {
  *hw = Profile();
  std::istringstream in(text);
  std::string line;
  bool header = false;
  while (std::getline(in, line)) {
    if (line.empty() || line[0] == '#') continue;
    std::istringstream ls(line);
    std::string key; ls >> key;
    if (key.empty()) continue;
    if (!header) { int ver = 0; if (key != "sts-profile" || !(ls >> ver) || ver != 1) return false; header = true; continue; }
    if (key == "grid") {
      std::string name; int nd = 0;
      if (!(ls >> name >> nd) || nd < 1 || nd > 3) return false;
      Grid* g = name == "bw" ? &hw->bw : name == "alpha_prefill" ? &hw->alpha_prefill : name == "alpha_decode" ? &hw->alpha_decode :
                name == "prefill_corun" ? &hw->prefill_corun : nullptr;
      const int want = name == "alpha_decode" ? 3 : name == "prefill_corun" ? 1 : 2;
      if (!g || nd != want || !parse_grid(in, nd, g)) return false;
      continue;
    }
    int64_t v;
    if (!(ls >> v)) return false;
    if (key == "n_cu") hw->n_cu = v; else if (key == "granule") hw->granule = v; else if (key == "c_peak") hw->c_peak = v;
    else if (key == "d_peak") hw->d_peak = v; else if (key == "n_d") hw->n_d = v; else if (key == "tile_m") hw->tile_m = v;
    else if (key == "tile_n") hw->tile_n = v; else if (key == "tile_q") hw->tile_q = v; else if (key == "wgs_per_cu") hw->wgs_per_cu = v; else if (key == "use_waveq") hw->use_waveq = v;
    else if (key == "tail_cut") hw->tail_cut = v;
    else if (key == "gemm_rate_128") hw->gemm_rate_128 = v; else if (key == "gemm_rate_256") hw->gemm_rate_256 = v;
    else if (key == "gemm_rate_128x256") hw->gemm_rate_128x256 = v; else if (key == "gemm_fixed_128x256") hw->gemm_fixed_128x256 = v;
    else if (key == "partial_bw_cu") hw->partial_bw_cu = v;
    else if (key == "stream_bw_cu") hw->stream_bw_cu = v; else if (key == "stream_bw_gpu") hw->stream_bw_gpu = v;
    else return false;
  }
  return header && hw->n_cu > 0 && hw->granule > 0 && hw->c_peak > 0 && hw->d_peak > 0 && hw->n_d > 0 && hw->tile_m > 0 &&
         hw->tile_n > 0 && hw->tile_q > 0 && hw->wgs_per_cu > 0 && hw->tail_cut >= 0 && hw->tail_cut <= 64 &&
         hw->gemm_rate_128 > 0 && hw->gemm_rate_256 > 0 && hw->gemm_rate_128x256 > 0 && hw->gemm_fixed_128x256 >= 0 && hw->partial_bw_cu > 0 &&
         hw->stream_bw_cu > 0 && hw->stream_bw_gpu >= hw->stream_bw_cu;
}

static void dump_grid(std::ostringstream& o, const char* name, const Grid& g) {
  if (g.values.empty()) return;
  o << "grid " << name << " " << g.axes.size() << "\n";
  for (auto& ax : g.axes) { o << "axis"; for (int64_t v : ax) o << " " << v; o << "\n"; }
  o << "values"; for (int64_t v : g.values) o << " " << v; o << "\n";
}
std::string dump_profile(const Profile& hw) {
  std::ostringstream o;
  o << "sts-profile 1\n";
  o << "n_cu " << hw.n_cu << "\ngranule " << hw.granule << "\nc_peak " << hw.c_peak << "\nd_peak " << hw.d_peak << "\nn_d " << hw.n_d
    << "\ntile_m " << hw.tile_m << "\ntile_n " << hw.tile_n << "\ntile_q " << hw.tile_q << "\nwgs_per_cu " << hw.wgs_per_cu << "\nuse_waveq " << hw.use_waveq << "\ntail_cut " << hw.tail_cut
    << "\ngemm_rate_128 " << hw.gemm_rate_128 << "\ngemm_rate_256 " << hw.gemm_rate_256 << "\ngemm_rate_128x256 " << hw.gemm_rate_128x256 << "\ngemm_fixed_128x256 " << hw.gemm_fixed_128x256 << "\npartial_bw_cu " << hw.partial_bw_cu
    << "\nstream_bw_cu " << hw.stream_bw_cu << "\nstream_bw_gpu " << hw.stream_bw_gpu << "\n";
  dump_grid(o, "bw", hw.bw);
  dump_grid(o, "prefill_corun", hw.prefill_corun);
  dump_grid(o, "alpha_prefill", hw.alpha_prefill);
  dump_grid(o, "alpha_decode", hw.alpha_decode);
  return o.str();
}

}  // namespace sts

// ======================================================================================= C ABI
using namespace sts;

struct sts_profile { Profile hw; };

extern "C" int sts_wave_quant(int64_t g, int64_t n, int64_t b, int64_t* waves, int64_t* tail, int64_t* idle_num, int64_t* idle_den) {
  if (g < 1 || n < 1 || b < 1) return STS_EINVAL;
  int64_t w, t;
  wave_quant(g, n, b, &w, &t);
  if (waves) *waves = w;
  if (tail) *tail = t;
  if (idle_num) *idle_num = n - t;
  if (idle_den) *idle_den = n * w;
  return STS_OK;
}
extern "C" int sts_profile_tile_model(const sts_profile* p, int64_t* gemm_rate_128, int64_t* gemm_rate_256, int64_t* gemm_rate_128x256,
                                      int64_t* gemm_fixed_128x256, int64_t* partial_bw_cu) {
  if (!p) return STS_EINVAL;
  if (gemm_rate_128) *gemm_rate_128 = p->hw.gemm_rate_128;
  if (gemm_rate_256) *gemm_rate_256 = p->hw.gemm_rate_256;
  if (gemm_rate_128x256) *gemm_rate_128x256 = p->hw.gemm_rate_128x256;
  if (gemm_fixed_128x256) *gemm_fixed_128x256 = p->hw.gemm_fixed_128x256;
  if (partial_bw_cu) *partial_bw_cu = p->hw.partial_bw_cu;
  return STS_OK;
}
extern "C" int sts_profile_stream_model(const sts_profile* p, int64_t* stream_bw_cu, int64_t* stream_bw_gpu) {
  if (!p) return STS_EINVAL;
  if (stream_bw_cu) *stream_bw_cu = p->hw.stream_bw_cu;
  if (stream_bw_gpu) *stream_bw_gpu = p->hw.stream_bw_gpu;
  return STS_OK;
}
extern "C" int sts_profile_parse(const char* text, sts_profile** out) {
  if (!text || !out) return STS_EINVAL;
  sts_profile* p = new sts_profile();
  if (!parse_profile(text, &p->hw)) { delete p; return STS_EIO; }
  *out = p;
  return STS_OK;
}
extern "C" int sts_profile_load(const char* path, sts_profile** out) {
  if (!path || !out) return STS_EINVAL;
  FILE* f = std::fopen(path, "rb");
  if (!f) return STS_EIO;
  std::string text; char buf[4096]; size_t n;
  while ((n = std::fread(buf, 1, sizeof(buf), f)) > 0) text.append(buf, n);
  std::fclose(f);
  return sts_profile_parse(text.c_str(), out);
}
extern "C" int sts_profile_dump(const sts_profile* p, char* buf, size_t cap, size_t* needed) {
  if (!p) return STS_EINVAL;
  const std::string s = dump_profile(p->hw);
  if (needed) *needed = s.size() + 1;
  if (buf && cap > 0) { const size_t n = std::min(cap - 1, s.size()); std::memcpy(buf, s.data(), n); buf[n] = 0; }
  return STS_OK;
}
extern "C" int sts_profile_free(sts_profile* p) { delete p; return STS_OK; }

const Profile* sts_profile_get(const sts_profile* p) { return &p->hw; }

static int check_es(const sts_profile* p, const sts_model_desc* d, const sts_exec_state* es) {
  if (!p || !d || !es || es->n_prefill < 0 || es->n_decode < 0 || es->prefill_cus < 0 || es->decode_cus < 0) return STS_EINVAL;
  if (es->n_prefill > 0 && (!es->prefill_len || !es->prefill_ctx || es->n_layers_step < 1 || es->layer_begin < 0)) return STS_EINVAL;
  if (es->n_decode > 0 && !es->decode_ctx) return STS_EINVAL;
  for (int i = 0; i < es->n_prefill; i++) if (es->prefill_len[i] < 1 || es->prefill_ctx[i] < 0) return STS_EINVAL;
  for (int i = 0; i < es->n_decode; i++) if (es->decode_ctx[i] < 0) return STS_EINVAL;
  return STS_OK;
}
// The decode CUs a prefill slice of this execution state shares the GPU with: a decode batch on a
// disjoint CU set; 0 when nothing decodes or the two sets overlap.
static int co_decode_cus(const Profile& hw, const sts_exec_state* es) {
  return (es->n_decode > 0 && es->decode_cus > 0 && (int64_t)es->prefill_cus + es->decode_cus <= hw.n_cu) ? es->decode_cus : 0;
}
extern "C" int sts_latency_query(const sts_profile* p, const sts_model_desc* d, const sts_exec_state* es, int64_t* prefill_ns, int64_t* decode_ns) {
  int rc = check_es(p, d, es);
  if (rc) return rc;
  int64_t co = 0;
  if (es->prefill_cus > 0) for (int i = 0; i < es->n_prefill; i++) co += es->prefill_len[i];
  if (prefill_ns) *prefill_ns = predict_prefill_ns(*d, p->hw, es->prefill_len, es->prefill_ctx, es->n_prefill, es->prefill_cus, es->layer_begin,
                                                   es->n_layers_step, co_decode_cus(p->hw, es));
  if (decode_ns) *decode_ns = predict_decode_ns(*d, p->hw, es->decode_ctx, es->n_decode, es->decode_cus, co);
  return STS_OK;
}
// ---- online recalibration (Section 3.2.4): one observation moves every alpha sample that the
// interpolation at the observed execution state reads by weight * (alpha_obs / alpha_predicted - 1)
// of its value.
static void blend(Grid& g, const int64_t* x, int64_t t_measured, int64_t t_roofline, int64_t weight_ppm) {
  const int64_t a_pred = alpha_at(g, x);
  const int64_t a_obs = floor_div((i128)t_measured * PPM, std::max<int64_t>(t_roofline, 1));
  // flat indices of the samples the interpolation at x reads (both ends of each axis's segment)
  std::vector<size_t> corners{0};
  size_t stride = g.values.size();
  for (size_t a = 0; a < g.axes.size(); a++) {
    const std::vector<int64_t>& ax = g.axes[a];
    stride /= ax.size();
    if (ax.size() == 1) continue;
    size_t i = 0;
    while (i + 2 < ax.size() && x[a] >= ax[i + 1]) i++;
    std::vector<size_t> next;
    for (size_t c : corners) { next.push_back(c + i * stride); next.push_back(c + (i + 1) * stride); }
    corners.swap(next);
  }
  for (size_t c : corners) {
    const int64_t old = g.values[c];
    const int64_t target = floor_div((i128)old * a_obs, a_pred);
    g.values[c] = std::max<int64_t>(1, old + floor_div((i128)(target - old) * weight_ppm, PPM));
  }
}
extern "C" int sts_profile_observe(sts_profile* p, const sts_model_desc* d, const sts_exec_state* es, int64_t measured_prefill_ns,
                                   int64_t measured_decode_ns, int64_t weight_ppm) {
  int rc = check_es(p, d, es);
  if (rc) return rc;
  if (weight_ppm < 0 || weight_ppm > PPM) return STS_EINVAL;
  int64_t co = 0;
  if (es->prefill_cus > 0) for (int i = 0; i < es->n_prefill; i++) co += es->prefill_len[i];
  if (measured_prefill_ns > 0 && es->n_prefill > 0 && es->prefill_cus > 0) {
    int64_t roof = prefill_roofline_ns(*d, p->hw, es->prefill_len, es->prefill_ctx, es->n_prefill, es->prefill_cus, es->layer_begin, es->n_layers_step);
    roof = floor_div((i128)roof * prefill_corun_ppm(p->hw, co_decode_cus(p->hw, es)), PPM);      // alpha stays the stand-alone factor
    const int64_t x[2] = {es->prefill_cus, co};
    blend(p->hw.alpha_prefill, x, measured_prefill_ns, roof, weight_ppm);
  }
  if (measured_decode_ns > 0 && es->n_decode > 0 && es->decode_cus > 0) {
    const int64_t roof = decode_roofline_ns(*d, p->hw, es->decode_ctx, es->n_decode, es->decode_cus, co);
    int64_t ctx = 0;
    for (int i = 0; i < es->n_decode; i++) ctx += es->decode_ctx[i];
    const int64_t x[3] = {es->decode_cus, es->n_decode, ctx / es->n_decode};
    blend(p->hw.alpha_decode, x, measured_decode_ns, roof, weight_ppm);
  }
  return STS_OK;
}

extern "C" int sts_latency_roofline(const sts_profile* p, const sts_model_desc* d, const sts_exec_state* es, int64_t* prefill_ns, int64_t* decode_ns) {
  int rc = check_es(p, d, es);
  if (rc) return rc;
  int64_t co = 0;
  if (es->prefill_cus > 0) for (int i = 0; i < es->n_prefill; i++) co += es->prefill_len[i];
  if (prefill_ns) *prefill_ns = (es->n_prefill == 0) ? 0 : (es->prefill_cus <= 0 ? INF_NS :
      prefill_roofline_ns(*d, p->hw, es->prefill_len, es->prefill_ctx, es->n_prefill, es->prefill_cus, es->layer_begin, es->n_layers_step));
  if (decode_ns) *decode_ns = (es->n_decode == 0) ? 0 : (es->decode_cus <= 0 ? INF_NS :
      decode_roofline_ns(*d, p->hw, es->decode_ctx, es->n_decode, es->decode_cus, co));
  return STS_OK;
}
