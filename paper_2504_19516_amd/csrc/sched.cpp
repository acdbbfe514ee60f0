// SLO-aware scheduler (paper Section 3.3, Algorithm 1) and its trace replay in simulated time.
// Host only, integer arithmetic, deterministic: the decisions are a pure function of the
// profile, the trace and the configuration.
//
// Per prefill scheduling cycle: estimate TTFT of the in-flight batch P and of the queue Q under
// the current execution state; reorder Q by least estimated latency unless that would push a
// request past its TTFT SLO; continue P, or batch from Q until the batch's arithmetic intensity
// reaches the roofline ridge; then one of SetBalancedSM / ReduceDecodeSM / ReducePrefillSM picks
// the CU split on the grid {0, g, ..., N-g} of decode CUs; the slice [L_exe, L_exe + L_step) is
// launched. Each decode step merges the newly prefilled requests and runs on the CUs the last
// decision left to decode (all CUs when prefill has no work).
#include <algorithm>
#include <cstdint>
#include <vector>

#include "latency.h"
#include "sts.h"

namespace sts {
namespace {

constexpr int PAGE = 16;

struct QReq { int id; int64_t arrival; int32_t in_len, out_len; };           // a queued or in-flight prefill request
struct DReq { int64_t first_token; int32_t n_dec, in_len; };                  // a decoding (or handed-off) request

struct Decision {
  std::vector<int> tasks;        // ids of next_tasks, in order
  std::vector<int> queue;        // ids of the reordered queue that remains
  std::vector<int64_t> pages;    // pages reserved for each newly admitted task (empty when continuing P)
  int layer_begin = 0, layer_end = 0, pm = 0, dm = 0, branch = 0;
  int64_t predicted_ns = -1;     // -1: nothing could be admitted (KV pool full)
  bool admitted = false;         // tasks were taken from the queue (a new batch starts)
};

int64_t p90(std::vector<int64_t> v) {
  if (v.empty()) return 0;
  std::sort(v.begin(), v.end());
  return v[(9 * v.size() + 9) / 10 - 1];
}

struct Ctx {
  const sts_model_desc& s; const Profile& hw; const sts_sched_config& cfg;
  int n, g;
  // co_dm: CUs of a decode step running beside the slice on the other CUs (0 = prefill runs alone)
  int64_t t_prefill(const std::vector<QReq>& rs, int pm_, int l0, int nl, int co_dm) const {
    std::vector<int32_t> sl(rs.size()), p(rs.size(), 0);
    for (size_t i = 0; i < rs.size(); i++) sl[i] = rs[i].in_len;
    return predict_prefill_ns(s, hw, sl.data(), p.data(), (int)rs.size(), pm_, l0, nl, co_dm);
  }
  int64_t t_decode(const std::vector<DReq>& rs, int dm_, int64_t co) const {
    std::vector<int32_t> cl(rs.size());
    for (size_t i = 0; i < rs.size(); i++) cl[i] = rs[i].in_len + rs[i].n_dec;
    return predict_decode_ns(s, hw, cl.data(), (int)rs.size(), dm_, co);
  }
  // One layer's flop and bytes of the batch (the same closed forms the estimator sums).
  bool intensity_below_ridge(const std::vector<QReq>& rs, int pm_) const {
    const int64_t h = s.hidden, d = s.head_dim, qd = (int64_t)s.n_q_heads * d, kvd = (int64_t)s.n_kv_heads * d, qkvn = qd + 2 * kvd, mlp = s.mlp;
    int64_t t = 0; __int128 flop = 0, mem = 0;
    for (const QReq& r : rs) {
      const int64_t l = r.in_len;
      t += l;
      flop += 4 * qd * (l * (l + 1) / 2);
      mem += 2 * (2 * l * qd + 2 * l * kvd);
    }
    flop += (__int128)4 * t * h + 2 * t * h * qkvn + 4 * t * qkvn + 2 * t * qd * h + 4 * t * h + 4 * t * h * mlp + 2 * t * mlp * h;
    mem += (__int128)4 * t * h + 2 * (h * qkvn + t * h + t * qkvn) + 4 * t * qkvn + 2 * (qd * h + t * qd + 2 * t * h) + 4 * t * h +
           2 * (2 * h * mlp + t * h + t * mlp) + 2 * (mlp * h + t * mlp + 2 * t * h);
    return flop * hw.d_peak * std::min<int64_t>(pm_, hw.n_d) * hw.n_cu < mem * hw.c_peak * pm_ * hw.n_d;
  }
};

// Algorithm 1, one scheduling cycle. Q in arrival order; P the in-flight batch with l_exe layers
// done; dec the decoding requests followed by those handed off but not merged yet.
Decision decide(const Ctx& c, int64_t now, const std::vector<QReq>& Q, const std::vector<QReq>& P, int l_exe,
                const std::vector<DReq>& dec, int64_t pages_free, int pm, int dm) {
  const sts_sched_config& cfg = c.cfg;
  const int n = c.n, g = c.g, n_layers = c.s.n_layers;
  Decision out;
  const int pm_cur = pm > 0 ? pm : n;
  // while requests decode, a prefill slice on pm_c < n CUs has a decode step on the other n - pm_c beside it
  auto co_dm = [&](int pm_c) { return (dec.empty() || pm_c >= n) ? 0 : n - pm_c; };
  const int64_t t_p = P.empty() ? 0 : c.t_prefill(P, pm_cur, l_exe, n_layers - l_exe, co_dm(pm_cur));
  const size_t nq = Q.size();
  std::vector<int64_t> est(nq);
  for (size_t i = 0; i < nq; i++) est[i] = c.t_prefill(std::vector<QReq>{Q[i]}, pm_cur, 0, n_layers, co_dm(pm_cur));
  std::vector<int> fcfs(nq), sjf(nq);
  for (size_t i = 0; i < nq; i++) fcfs[i] = sjf[i] = (int)i;
  std::sort(sjf.begin(), sjf.end(), [&](int a, int b) {
    if (est[a] != est[b]) return est[a] < est[b];
    if (Q[a].arrival != Q[b].arrival) return Q[a].arrival < Q[b].arrival;
    return Q[a].id < Q[b].id;
  });
  std::vector<int64_t> ttft(nq, 0), t_fcfs(nq, 0), t_sjf(nq, 0);
  auto ttfts = [&](const std::vector<int>& order, std::vector<int64_t>& o) {
    int64_t acc = t_p;
    for (int i : order) { acc += est[i]; o[i] = now - Q[i].arrival + acc; }
  };
  ttfts(fcfs, t_fcfs); ttfts(sjf, t_sjf);
  std::vector<char> is_hurt(nq, 0);
  std::vector<int> order;
  const bool reorder = cfg.mode != 3 && cfg.mode != 4;       // the ablations without the scheduler keep arrival order
  if (reorder) {
    for (int i : fcfs) if (t_sjf[i] > cfg.ttft_slo_ns && cfg.ttft_slo_ns >= t_fcfs[i]) { is_hurt[i] = 1; order.push_back(i); }
    for (int i : sjf) if (!is_hurt[i]) order.push_back(i);
  } else {
    order = fcfs;
  }
  ttfts(order, ttft);

  bool satisfy;
  std::vector<QReq> next_tasks;
  size_t taken = 0;
  if (!P.empty()) {
    satisfy = true;
    for (const QReq& r : P) if (now - r.arrival + t_p > cfg.ttft_slo_ns) satisfy = false;
    next_tasks = P;
  } else {
    std::vector<int64_t> qt;
    for (int i : order) qt.push_back(ttft[i]);
    satisfy = p90(qt) <= cfg.ttft_slo_ns;
    int64_t tokens = 0;
    while (taken < order.size() && (next_tasks.empty() || c.intensity_below_ridge(next_tasks, pm_cur) || tokens < cfg.min_batch_tokens)) {
      const QReq& r = Q[order[taken]];
      const int64_t need = ((int64_t)r.in_len + r.out_len + PAGE - 1) / PAGE;
      if (!next_tasks.empty() && tokens + r.in_len > cfg.max_batch_tokens) break;
      if (need > pages_free) break;
      out.pages.push_back(need); pages_free -= need;
      next_tasks.push_back(r); tokens += r.in_len;
      taken++;
    }
    out.admitted = !next_tasks.empty();
    l_exe = 0;
  }
  for (size_t k = taken; k < order.size(); k++) out.queue.push_back(Q[order[k]].id);
  if (next_tasks.empty()) return out;
  const int l_eff = std::min<int>(cfg.layers_per_step, n_layers - l_exe);
  int64_t co = 0;
  for (const QReq& r : next_tasks) co += r.in_len;
  const int half = std::max(g, (n / 2) / g * g);

  auto tpot90 = [&](int dm_c) -> int64_t {
    if (dec.empty()) return 0;
    int64_t extra;
    if (dm_c > 0) extra = c.t_decode(dec, dm_c, co);
    else extra = c.t_prefill(next_tasks, n, l_exe, l_eff, 0) + c.t_decode(dec, half, co);
    std::vector<int64_t> v;
    for (const DReq& r : dec) v.push_back((now - r.first_token + extra) / (r.n_dec + 1));
    return p90(v);
  };
  auto ttft_max = [&](int pm_c) -> int64_t {
    const int64_t t = c.t_prefill(next_tasks, pm_c, l_exe, n_layers - l_exe, co_dm(pm_c));
    int64_t m = INT64_MIN;
    for (const QReq& r : next_tasks) m = std::max(m, now - r.arrival + t);
    return m;
  };
  std::vector<int> grid;
  for (int x = 0; x < n; x += g) grid.push_back(x);

  int branch = 0, pm_new, dm_new;
  if (cfg.mode == 1 || cfg.mode == 3) { pm_new = n; dm_new = n; }
  else if (cfg.mode == 2) { pm_new = cfg.fixed_prefill_cus; dm_new = n - cfg.fixed_prefill_cus; }
  else if (cfg.mode == 6) { pm_new = cfg.fixed_prefill_cus; dm_new = n; }
  else if (cfg.mode == 5) {
    // scheduler without partitioning: both phases see every CU; decode is delayed for this slice
    // when TTFT is at risk and the decoding requests' TPOT can absorb it
    pm_new = n;
    if (!dec.empty() && !satisfy && tpot90(0) <= cfg.tpot_slo_ns) { branch = 2; dm_new = 0; }
    else dm_new = n;
  }
  else {
    const int cur_dm = (pm > 0 && dm < n) ? dm : half;
    const int64_t tp_now = tpot90(cur_dm);
    auto balanced = [&]() -> int {
      bool have = false; __int128 best = 0; int best_dm = dec.empty() ? grid[0] : grid[1];
      for (size_t k = dec.empty() ? 0 : 1; k < grid.size(); k++) {
        const __int128 a = (__int128)ttft_max(n - grid[k]) * cfg.tpot_slo_ns, b = (__int128)tpot90(grid[k]) * cfg.ttft_slo_ns;
        const __int128 v = a > b ? a : b;
        if (!have || v < best) { have = true; best = v; best_dm = grid[k]; }
      }
      return best_dm;
    };
    auto smallest_dm_meeting_tpot = [&]() -> int {
      // decode is suspended (0 CUs) only when TTFT is at risk, or when nothing decodes
      for (size_t k = (dec.empty() || (!satisfy && cfg.mode != 4)) ? 0 : 1; k < grid.size(); k++)
        if (tpot90(grid[k]) <= cfg.tpot_slo_ns) return grid[k];
      return -1;
    };
    if (!satisfy && tp_now > cfg.tpot_slo_ns) { branch = 1; dm_new = balanced(); }
    else if (tp_now <= cfg.tpot_slo_ns) {
      branch = 2; dm_new = smallest_dm_meeting_tpot();
      if (dm_new < 0) dm_new = balanced();
    } else {
      branch = 3; dm_new = smallest_dm_meeting_tpot();
      if (dm_new < 0) {
        for (int k = (int)grid.size() - 1; k >= 0; k--) if (ttft_max(n - grid[k]) <= cfg.ttft_slo_ns) { dm_new = grid[k]; break; }
        if (dm_new < 0) dm_new = balanced();
      }
    }
    pm_new = n - dm_new;
  }
  // End-of-prefill boost (Section 3.3.1): while the batch's final slice runs, decode gets extra CUs
  // so the hand-over to decode-only is smooth. The prefill set stays, so the two sets intersect for
  // that slice instead of the phases synchronising.
  if (cfg.decode_boost_cus > 0 && (cfg.mode == 0 || cfg.mode == 2 || cfg.mode == 4) && !dec.empty() && dm_new > 0 &&
      l_exe + l_eff == n_layers)
    dm_new = std::min(n, dm_new + cfg.decode_boost_cus);
  for (const QReq& r : next_tasks) out.tasks.push_back(r.id);
  out.layer_begin = l_exe; out.layer_end = l_exe + l_eff; out.pm = pm_new; out.dm = dm_new; out.branch = branch;
  out.predicted_ns = c.t_prefill(next_tasks, pm_new, l_exe, l_eff, dm_new > 0 ? co_dm(pm_new) : 0);
  return out;
}

int64_t hash_ids(const std::vector<int>& ids) {
  int64_t h = 0;
  for (int i : ids) h = (int64_t)(((__int128)h * 1000003 + i + 1) % ((__int128)1 << 62));
  return h;
}

struct Req {
  int64_t arrival; int32_t in_len, out_len;
  int32_t pages = 0; int64_t first_token = -1; int32_t n_dec = 0; int64_t finish = -1;
};

struct Replay {
  Ctx c;
  const sts_sched_config& cfg;
  std::vector<Req> reqs;
  int n;
  int64_t now = 0; size_t next_arrival = 0;
  std::vector<int> Q, P, H, D, decode_batch;
  int l_exe = 0; int64_t pages_free;
  int pm, dm;
  int64_t prefill_done_at = -1, decode_done_at = -1;
  bool turn_decode = false;
  std::vector<sts_decision> decisions;

  Replay(const sts_model_desc& s_, const Profile& hw_, const sts_sched_config& c_, const int64_t* trace, int64_t cnt)
      : c{s_, hw_, c_, (int)hw_.n_cu, (int)hw_.granule}, cfg(c_), n((int)hw_.n_cu), pages_free(c_.kv_pool_pages) {
    reqs.resize(cnt);
    for (int64_t i = 0; i < cnt; i++) { reqs[i].arrival = trace[3 * i]; reqs[i].in_len = (int32_t)trace[3 * i + 1]; reqs[i].out_len = (int32_t)trace[3 * i + 2]; }
    if (cfg.mode == 1) { pm = n; dm = n; } else { pm = 0; dm = n; }
  }
  QReq qreq(int i) const { return QReq{i, reqs[i].arrival, reqs[i].in_len, reqs[i].out_len}; }
  DReq dreq(int i) const { return DReq{reqs[i].first_token, reqs[i].n_dec, reqs[i].in_len}; }
  int64_t t_decode_ids(const std::vector<int>& ids, int dm_, int64_t co) const {
    std::vector<DReq> v; for (int i : ids) v.push_back(dreq(i));
    return c.t_decode(v, dm_, co);
  }

  // Returns the predicted duration of the slice it launches, or -1 if nothing can be admitted yet.
  int64_t schedule() {
    std::vector<QReq> q, p; std::vector<DReq> dec;
    for (int i : Q) q.push_back(qreq(i));
    for (int i : P) p.push_back(qreq(i));
    for (int i : D) dec.push_back(dreq(i));
    for (int i : H) dec.push_back(dreq(i));
    const Decision d = decide(c, now, q, p, l_exe, dec, pages_free, pm, dm);
    if (d.admitted) {
      for (size_t k = 0; k < d.tasks.size(); k++) { reqs[d.tasks[k]].pages = (int32_t)d.pages[k]; pages_free -= d.pages[k]; }
      P = d.tasks; l_exe = 0;
    }
    Q = d.queue;
    if (d.tasks.empty()) return -1;
    pm = d.pm; dm = d.dm;
    sts_decision r{};
    r.t_ns = now; r.n_tasks = (int32_t)d.tasks.size();
    r.first_req = *std::min_element(d.tasks.begin(), d.tasks.end());
    r.tasks_hash = hash_ids(d.tasks); r.layer_begin = d.layer_begin; r.layer_end = d.layer_end; r.prefill_cus = pm; r.decode_cus = dm;
    r.branch = d.branch; r.decode_batch = (int32_t)dec.size(); r.predicted_ns = d.predicted_ns;
    decisions.push_back(r);
    return d.predicted_ns;
  }

  void finish(int i) { reqs[i].finish = now; pages_free += reqs[i].pages; }

  void run() {
    const bool serial = cfg.mode == 1;
    for (;;) {
      while (next_arrival < reqs.size() && reqs[next_arrival].arrival <= now) {
        const Req& r = reqs[next_arrival];
        if (((int64_t)r.in_len + r.out_len + PAGE - 1) / PAGE <= cfg.kv_pool_pages && r.in_len <= cfg.max_batch_tokens) Q.push_back((int)next_arrival);
        next_arrival++;
      }
      bool busy = prefill_done_at >= 0 || decode_done_at >= 0;
      if (prefill_done_at < 0 && (!P.empty() || !Q.empty()) && !(serial && (busy || (turn_decode && (!D.empty() || !H.empty()))))) {
        const int64_t dur = schedule();
        if (dur >= 0) { prefill_done_at = now + dur; busy = true; }
      }
      if (decode_done_at < 0 && !(serial && busy)) {
        while (!H.empty() && (int)D.size() < cfg.max_decode_batch) { D.push_back(H.front()); H.erase(H.begin()); }
        if (!D.empty()) {
          const bool prefill_running = prefill_done_at >= 0;
          const int dm_eff = (serial || !prefill_running) ? n : dm;
          if (dm_eff > 0) {
            int64_t co = 0;
            if (prefill_running && !serial) for (int i : P) co += reqs[i].in_len;
            decode_batch = D;
            decode_done_at = now + t_decode_ids(D, dm_eff, co);
          }
        }
      }
      int64_t next = -1;
      auto consider = [&](int64_t t) { if (t >= 0 && (next < 0 || t < next)) next = t; };
      consider(prefill_done_at); consider(decode_done_at);
      if (next_arrival < reqs.size()) consider(reqs[next_arrival].arrival);
      if (next < 0) break;
      now = std::max(now, next);
      if (prefill_done_at >= 0 && prefill_done_at <= now) {
        prefill_done_at = -1; turn_decode = true;
        l_exe = std::min<int>(l_exe + cfg.layers_per_step, c.s.n_layers);
        if (l_exe == c.s.n_layers) {
          for (int i : P) {
            reqs[i].first_token = now;
            if (reqs[i].out_len <= 1) finish(i); else H.push_back(i);
          }
          P.clear(); l_exe = 0;
        }
      }
      if (decode_done_at >= 0 && decode_done_at <= now) {
        decode_done_at = -1; turn_decode = false;
        for (int i : decode_batch) {
          reqs[i].n_dec += 1;
          if (reqs[i].n_dec >= reqs[i].out_len - 1) { finish(i); D.erase(std::find(D.begin(), D.end(), i)); }
        }
      }
    }
  }
};

bool config_ok(const Profile& hw, const sts_sched_config* cfg) {
  if (cfg->layers_per_step < 1 || cfg->max_batch_tokens < 1 || cfg->max_decode_batch < 1 || cfg->kv_pool_pages < 1 ||
      cfg->mode < 0 || cfg->mode > 6 || cfg->ttft_slo_ns < 1 || cfg->tpot_slo_ns < 1) return false;
  if (hw.n_cu % hw.granule != 0 || hw.n_cu / hw.granule < 2) return false;
  if (cfg->decode_boost_cus < 0 || cfg->decode_boost_cus % hw.granule) return false;
  if (cfg->min_batch_tokens < 0) return false;
  if ((cfg->mode == 2 || cfg->mode == 6) && (cfg->fixed_prefill_cus < hw.granule || cfg->fixed_prefill_cus >= hw.n_cu || cfg->fixed_prefill_cus % hw.granule)) return false;
  return true;
}

}  // namespace
}  // namespace sts

extern "C" int sts_sched_decide(const sts_profile* p, const sts_model_desc* desc, const sts_sched_config* cfg,
                                const sts_sched_state* st, sts_sched_choice* out) {
  using namespace sts;
  if (!p || !desc || !cfg || !st || !out) return STS_EINVAL;
  const Profile& hw = *sts_profile_get(p);
  if (!config_ok(hw, cfg)) return STS_EINVAL;
  if (st->n_queue < 0 || st->n_inflight < 0 || st->n_decode < 0 || (st->n_queue > 0 && !st->queue) || (st->n_inflight > 0 && !st->inflight) ||
      (st->n_decode > 0 && !st->decode) || st->layers_done < 0 || st->layers_done >= desc->n_layers) return STS_EINVAL;
  if (out->cap_tasks < 0 || out->cap_queue < st->n_queue || (out->cap_tasks > 0 && !out->task_ids) || (out->cap_queue > 0 && !out->queue_ids)) return STS_EINVAL;
  std::vector<QReq> Q, P; std::vector<DReq> dec;
  for (int i = 0; i < st->n_queue; i++) Q.push_back(QReq{st->queue[i].id, st->queue[i].arrival_ns, st->queue[i].in_len, st->queue[i].out_len});
  for (int i = 0; i < st->n_inflight; i++) P.push_back(QReq{st->inflight[i].id, st->inflight[i].arrival_ns, st->inflight[i].in_len, st->inflight[i].out_len});
  for (int i = 0; i < st->n_decode; i++) dec.push_back(DReq{st->decode[i].first_token_ns, st->decode[i].n_dec, st->decode[i].in_len});
  for (const QReq& r : Q) if (r.in_len < 1 || r.out_len < 1) return STS_EINVAL;
  const Ctx c{*desc, hw, *cfg, (int)hw.n_cu, (int)hw.granule};
  const Decision d = decide(c, st->now_ns, Q, P, st->layers_done, dec, st->pages_free, st->cur_prefill_cus, st->cur_decode_cus);
  if ((int)d.tasks.size() > out->cap_tasks) return STS_EINVAL;
  out->n_tasks = (int32_t)d.tasks.size();
  for (size_t i = 0; i < d.tasks.size(); i++) out->task_ids[i] = d.tasks[i];
  out->n_queue = (int32_t)d.queue.size();
  for (size_t i = 0; i < d.queue.size(); i++) out->queue_ids[i] = d.queue[i];
  out->admitted = d.admitted ? 1 : 0;
  out->layer_begin = d.layer_begin; out->layer_end = d.layer_end; out->prefill_cus = d.pm; out->decode_cus = d.dm;
  out->branch = d.branch; out->predicted_ns = d.predicted_ns;
  return STS_OK;
}

extern "C" int sts_sched_replay(const sts_profile* p, const sts_model_desc* desc, const sts_sched_config* cfg,
                                const int64_t* trace, int64_t n, sts_decision* decisions, int64_t cap, sts_replay_stats* stats) {
  using namespace sts;
  if (!p || !desc || !cfg || (n > 0 && !trace) || n < 0 || cap < 0 || (cap > 0 && !decisions)) return STS_EINVAL;
  const Profile& hw = *sts_profile_get(p);
  if (!config_ok(hw, cfg)) return STS_EINVAL;
  for (int64_t i = 0; i < n; i++) {
    if (trace[3 * i + 1] < 1 || trace[3 * i + 2] < 1 || trace[3 * i] < 0 || (i > 0 && trace[3 * i] < trace[3 * (i - 1)])) return STS_EINVAL;
  }
  Replay r(*desc, hw, *cfg, trace, n);
  r.run();
  for (int64_t i = 0; i < std::min<int64_t>(cap, (int64_t)r.decisions.size()); i++) decisions[i] = r.decisions[i];
  if (stats) {
    sts_replay_stats st{};
    st.n_requests = n; st.n_decisions = (int64_t)r.decisions.size();
    for (const auto& q : r.reqs) {
      if (q.finish < 0) continue;
      st.n_finished++; st.out_tokens += q.out_len; st.makespan_ns = std::max(st.makespan_ns, q.finish);
      st.ttft_sum_ns += q.first_token - q.arrival;
      int64_t tp = 0;
      if (q.n_dec > 0) { tp = (q.finish - q.first_token) / q.n_dec; st.tpot_sum_ns += tp; st.n_tpot++; }
      if (q.first_token - q.arrival <= cfg->ttft_slo_ns && tp <= cfg->tpot_slo_ns) st.n_slo_ok++;
    }
    *stats = st;
  }
  return STS_OK;
}
