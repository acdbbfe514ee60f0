"""Oracle, part 3: the SLO-aware scheduler replayed over an arrival trace.  TEST INFRASTRUCTURE.

Follows the paper's Algorithm 1 ("SLO-aware Scheduling for Prefill") and Section 3.3 in the
paper's order: estimate latencies, publish/read the other phase's estimates, reorder the queue
by least estimated latency, pick next_tasks (continue the in-flight batch, else batch from the
queue until its arithmetic intensity reaches the ridge), then exactly one of SetBalancedSM /
ReduceDecodeSM / ReducePrefillSM, and return (next_tasks, split, L_exe + L_step). The decode
scheduler "follows analogously": every decode step merges newly prefilled requests, predicts
its step latency and runs on whatever CUs the last decision left to decode.

The replay runs in simulated time: each slice or step takes exactly the estimator's prediction,
so every decision is a pure function of (profile, trace, configuration). All arithmetic is
integer. "SM" in the paper is "CU" here.

Readings where the paper is silent (listed in the design document):
  * the empty slot of Algorithm 1's return statement is the chosen split
  * split grid: decode CUs dm in {0, g, 2g, ..., N - g}, prefill gets N - dm
  * ReduceDecodeSM: smallest dm whose predicted P90 TPOT meets the SLO; none -> balanced.
    dm = 0 (decode suspended for this slice) is a candidate only when the TTFT check failed
    ("extreme cases of high request load") or when no request is decoding
  * ReducePrefillSM: the same search; none -> largest dm that keeps every in-flight TTFT within
    its SLO; none -> balanced
  * SetBalancedSM: dm minimising max(TTFT/Gamma_p, TPOT/Gamma_d); ties -> more prefill CUs
  * P90 is nearest-rank: the ceil(0.9 n)-th smallest; of nothing, 0
  * predicted TPOT of a decoding request = (time since its first token + next step) / (tokens + 1);
    with dm = 0 the next step is one prefill slice on all CUs followed by a step on N/2 CUs
  * predicted TTFT = waiting so far + remaining in-flight prefill + queued prefills ahead of it
  * "peak" of the batching loop is the roofline ridge C_p / D_p at the current prefill CUs; at
    least one request is admitted; batching also stops at the workspace token cap and when the
    KV pool cannot hold the next request's input and output
  * queue order: (estimated prefill latency, arrival, id); a request that would miss its TTFT
    SLO under that order but not under arrival order goes to the front (no starvation)
  * when prefill has no work decode runs on all CUs
  * the first output token comes from the prefill; a request decodes out_len - 1 more

Outside the paper, off by default: Config.min_batch_tokens keeps the batching loop of Algorithm 1
going past the ridge until the batch holds that many tokens (queued requests only). With 0 the
loop is the paper's rule exactly.
"""
from __future__ import annotations

from dataclasses import dataclass, field

from . import latency as L

PAGE = 16


@dataclass
class Config:
    ttft_slo_ns: int
    tpot_slo_ns: int
    layers_per_step: int
    max_batch_tokens: int
    max_decode_batch: int
    kv_pool_pages: int
    # 0 Algorithm 1; 1 time-multiplexed; 2 fixed disjoint split; the paper's ablations (Section 4.5):
    # 3 Naive (both phases on every CU, arrival order, no delayed decode), 4 w/Partition (the split
    # search only: arrival order, decode never suspended), 5 w/Scheduler (reordering and delayed
    # decode only: both phases on every CU); 6 the sensitivity study's setting (Section 4.4): prefill
    # on a fixed CU count, decode on every CU
    mode: int = 0
    fixed_prefill_cus: int = 0
    # end-of-prefill boost (Section 3.3.1): extra decode CUs while the final slice of a prefill batch
    # runs; the prefill set is kept, so the two sets intersect for that slice. 0 = off
    decode_boost_cus: int = 0
    # batching floor: keep adding queued requests to a new prefill batch until it holds this many tokens,
    # even past the roofline ridge where Algorithm 1 stops (a batch at the ridge is still small enough
    # for wave quantisation and launch overheads to cost 10-60 %). 0 = the paper's rule alone
    min_batch_tokens: int = 0


def chunked_prefill_iterations(sl, cs, ds):
    """Chunked-prefill accounting (Section 2.2.2): with a token budget cs per hybrid batch of which
    ds go to the running decode requests, a prompt of sl tokens needs N = ceil(sl / (cs - ds))
    iterations, and chunk i (1-based) attends over the i chunks cached so far, N(N+1)/2 chunk
    loads of KV cache in all. Returns (N, N(N+1)/2)."""
    assert cs > ds >= 0 and sl >= 1
    n = -(-sl // (cs - ds))
    return n, n * (n + 1) // 2


@dataclass
class Req:
    rid: int
    arrival: int
    in_len: int
    out_len: int
    pages: int = 0
    first_token: int = -1
    n_dec: int = 0
    finish: int = -1


def p90(values):
    if not values:
        return 0
    s = sorted(values)
    return s[(9 * len(s) + 9) // 10 - 1]


def tasks_hash(ids):
    h = 0
    for i in ids:
        h = (h * 1000003 + i + 1) % (1 << 62)
    return h


class Replay:
    def __init__(self, shape: L.Shape, hw: L.Profile, cfg: Config, trace):
        self.s, self.hw, self.cfg = shape, hw, cfg
        self.reqs = [Req(i, int(a), int(il), int(ol)) for i, (a, il, ol) in enumerate(trace)]
        self.n = hw.n_cu
        self.g = hw.granule
        self.now = 0
        self.next_arrival = 0
        self.Q: list[int] = []
        self.P: list[int] = []
        self.l_exe = 0
        self.H: list[int] = []
        self.D: list[int] = []
        self.pages_free = cfg.kv_pool_pages
        self.pm, self.dm = (self.n, self.n) if cfg.mode == 1 else (0, self.n)
        self.prefill_done_at = -1       # -1: idle
        self.decode_done_at = -1
        self.decode_batch: list[int] = []
        self.turn_decode = False        # time-multiplexed mode: whose turn it is
        self.decisions = []
        self.n_rejected = 0

    # ---------------------------------------------------------------- estimator shorthands
    def t_prefill(self, ids, pm, l0, nl, co_dm):
        """co_dm: CUs of a decode step running beside the slice on the other CUs (0 = prefill alone)."""
        return L.predict_prefill_ns(self.s, self.hw, [(self.reqs[i].in_len, 0) for i in ids], pm, l0, nl, co_dm)

    def t_decode(self, ids, dm, co):
        return L.predict_decode_ns(self.s, self.hw, [self.reqs[i].in_len + self.reqs[i].n_dec for i in ids], dm, co)

    def intensity_below_ridge(self, ids, pm):
        ks, _ = L.prefill_kernels(self.s, self.hw, [(self.reqs[i].in_len, 0) for i in ids], False, whole_tiles=False)
        flop, mem = sum(k[1] for k in ks), sum(k[2] for k in ks)
        hw = self.hw
        return flop * hw.d_peak * min(pm, hw.n_d) * hw.n_cu < mem * hw.c_peak * pm * hw.n_d

    # ---------------------------------------------------------------- Algorithm 1
    def schedule(self):
        cfg, reqs, now = self.cfg, self.reqs, self.now
        n_layers = self.s.n_layers
        pm_cur = self.pm if self.pm > 0 else self.n
        # line 2: estimate latencies of P u Q under the current execution state
        # while requests decode, a prefill slice on pm < n CUs has a decode step on the other n - pm beside it
        # (dec is built below from D and H; the same test is used here)
        co_dm = lambda pm_c: 0 if (not (self.D or self.H) or pm_c >= self.n) else self.n - pm_c
        t_p = self.t_prefill(self.P, pm_cur, self.l_exe, n_layers - self.l_exe, co_dm(pm_cur)) if self.P else 0
        est = {i: self.t_prefill([i], pm_cur, 0, n_layers, co_dm(pm_cur)) for i in self.Q}
        # line 5: sort by least estimated latency, guarded against new SLO violations
        fcfs = list(self.Q)
        sjf = sorted(self.Q, key=lambda i: (est[i], reqs[i].arrival, i))

        def ttfts(order):
            out, acc = {}, t_p
            for i in order:
                acc += est[i]
                out[i] = now - reqs[i].arrival + acc
            return out

        t_fcfs, t_sjf = ttfts(fcfs), ttfts(sjf)
        if cfg.mode in (3, 4):                   # ablations without the scheduler keep arrival order
            self.Q = fcfs
        else:
            hurt = [i for i in fcfs if t_sjf[i] > cfg.ttft_slo_ns >= t_fcfs[i]]
            self.Q = hurt + [i for i in sjf if i not in hurt]
        ttft = ttfts(self.Q)
        for i in self.P:
            ttft[i] = now - reqs[i].arrival + t_p
        # lines 6-13: next_tasks
        if self.P:
            satisfy = all(ttft[i] <= cfg.ttft_slo_ns for i in self.P)
            next_tasks = list(self.P)
        else:
            satisfy = p90([ttft[i] for i in self.Q]) <= cfg.ttft_slo_ns
            next_tasks, tokens = [], 0
            while self.Q and (not next_tasks or self.intensity_below_ridge(next_tasks, pm_cur) or tokens < cfg.min_batch_tokens):
                i = self.Q[0]
                need = (reqs[i].in_len + reqs[i].out_len + PAGE - 1) // PAGE
                if next_tasks and tokens + reqs[i].in_len > cfg.max_batch_tokens:
                    break
                if need > self.pages_free:
                    break
                self.Q.pop(0)
                reqs[i].pages = need
                self.pages_free -= need
                next_tasks.append(i)
                tokens += reqs[i].in_len
            if not next_tasks:
                return None                      # the pool is full: wait for decode to free pages
            self.P = list(next_tasks)
            self.l_exe = 0
        l_eff = min(cfg.layers_per_step, n_layers - self.l_exe)
        # lines 3-4 and 14-20: the decode side's TPOT estimates and the split
        dec = self.D + self.H
        co = sum(reqs[i].in_len for i in next_tasks)

        def tpot90(dm):
            if not dec:
                return 0
            if dm > 0:
                extra = self.t_decode(dec, dm, co)
            else:
                half = max(self.g, (self.n // 2) // self.g * self.g)
                extra = self.t_prefill(next_tasks, self.n, self.l_exe, l_eff, 0) + self.t_decode(dec, half, co)
            return p90([(now - reqs[i].first_token + extra) // (reqs[i].n_dec + 1) for i in dec])

        def ttft_max(pm):
            t = self.t_prefill(next_tasks, pm, self.l_exe, n_layers - self.l_exe, co_dm(pm))
            return max(now - reqs[i].arrival + t for i in next_tasks)

        grid = list(range(0, self.n, self.g))          # candidate decode CUs
        branch = 0
        if cfg.mode in (1, 3):
            pm, dm = self.n, self.n
        elif cfg.mode == 2:
            pm, dm = cfg.fixed_prefill_cus, self.n - cfg.fixed_prefill_cus
        elif cfg.mode == 6:
            pm, dm = cfg.fixed_prefill_cus, self.n
        elif cfg.mode == 5:
            pm = self.n
            if dec and not satisfy and tpot90(0) <= cfg.tpot_slo_ns:
                branch, dm = 2, 0
            else:
                dm = self.n
        else:
            cur_dm = self.dm if (self.pm > 0 and self.dm < self.n) else max(self.g, (self.n // 2) // self.g * self.g)
            tp_now = tpot90(cur_dm)

            def balanced():
                cands = grid if not dec else grid[1:]
                best, best_dm = None, cands[0]
                for dm_c in cands:
                    v = max(ttft_max(self.n - dm_c) * cfg.tpot_slo_ns, tpot90(dm_c) * cfg.ttft_slo_ns)
                    if best is None or v < best:
                        best, best_dm = v, dm_c
                return best_dm

            def smallest_dm_meeting_tpot():
                # decode is suspended (dm = 0) only when TTFT is at risk, or when nothing decodes
                for dm_c in (grid if (not dec or (not satisfy and cfg.mode != 4)) else grid[1:]):
                    if tpot90(dm_c) <= cfg.tpot_slo_ns:
                        return dm_c
                return None

            if not satisfy and tp_now > cfg.tpot_slo_ns:
                branch, dm = 1, balanced()
            elif tp_now <= cfg.tpot_slo_ns:
                branch = 2
                dm = smallest_dm_meeting_tpot()
                if dm is None:
                    dm = balanced()
            else:
                branch = 3
                dm = smallest_dm_meeting_tpot()
                if dm is None:
                    ok = [dm_c for dm_c in grid if ttft_max(self.n - dm_c) <= cfg.ttft_slo_ns]
                    dm = ok[-1] if ok else balanced()
            pm = self.n - dm
        if cfg.decode_boost_cus > 0 and cfg.mode in (0, 2, 4) and dec and dm > 0 and self.l_exe + l_eff == n_layers:
            dm = min(self.n, dm + cfg.decode_boost_cus)
        self.pm, self.dm = pm, dm
        dur = self.t_prefill(next_tasks, pm, self.l_exe, l_eff, co_dm(pm) if dm > 0 else 0)
        self.decisions.append((now, len(next_tasks), min(next_tasks), tasks_hash(next_tasks), self.l_exe, self.l_exe + l_eff,
                               pm, dm, branch, len(dec), dur))
        return dur

    # ---------------------------------------------------------------- event loop
    def finish(self, i):
        r = self.reqs[i]
        r.finish = self.now
        self.pages_free += r.pages

    def run(self):
        reqs, cfg = self.reqs, self.cfg
        guard = 0
        while True:
            guard += 1
            assert guard < 50_000_000
            while self.next_arrival < len(reqs) and reqs[self.next_arrival].arrival <= self.now:
                r = reqs[self.next_arrival]
                if (r.in_len + r.out_len + PAGE - 1) // PAGE > cfg.kv_pool_pages or r.in_len > cfg.max_batch_tokens:
                    self.n_rejected += 1
                else:
                    self.Q.append(r.rid)
                self.next_arrival += 1
            serial = cfg.mode == 1
            busy = self.prefill_done_at >= 0 or self.decode_done_at >= 0
            # prefill engine
            if self.prefill_done_at < 0 and (self.P or self.Q) and not (serial and (busy or (self.turn_decode and (self.D or self.H)))):
                dur = self.schedule()
                if dur is not None:
                    self.prefill_done_at = self.now + dur
                    busy = True
            # decode engine
            if self.decode_done_at < 0 and not (serial and busy):
                while self.H and len(self.D) < cfg.max_decode_batch:
                    self.D.append(self.H.pop(0))
                if self.D:
                    prefill_running = self.prefill_done_at >= 0
                    dm = self.n if (serial or not prefill_running) else self.dm
                    if dm > 0:
                        co = sum(reqs[i].in_len for i in self.P) if (prefill_running and not serial) else 0
                        self.decode_batch = list(self.D)
                        self.decode_done_at = self.now + self.t_decode(self.D, dm, co)
            # next event
            times = [t for t in (self.prefill_done_at, self.decode_done_at) if t >= 0]
            if self.next_arrival < len(reqs):
                times.append(reqs[self.next_arrival].arrival)
            if not times:
                break
            self.now = max(self.now, min(times))
            if self.prefill_done_at >= 0 and self.prefill_done_at <= self.now:
                self.prefill_done_at = -1
                self.turn_decode = True
                self.l_exe = min(self.l_exe + cfg.layers_per_step, self.s.n_layers)
                if self.l_exe == self.s.n_layers:
                    for i in self.P:
                        reqs[i].first_token = self.now
                        if reqs[i].out_len <= 1:
                            self.finish(i)
                        else:
                            self.H.append(i)
                    self.P, self.l_exe = [], 0
            if self.decode_done_at >= 0 and self.decode_done_at <= self.now:
                self.decode_done_at = -1
                self.turn_decode = False
                for i in self.decode_batch:
                    reqs[i].n_dec += 1
                    if reqs[i].n_dec >= reqs[i].out_len - 1:
                        self.finish(i)
                        self.D.remove(i)
        return self.stats()

    def stats(self):
        cfg = self.cfg
        done = [r for r in self.reqs if r.finish >= 0]
        ttft_sum = sum(r.first_token - r.arrival for r in done)
        tpots = [(r.finish - r.first_token) // r.n_dec for r in done if r.n_dec > 0]
        ok = 0
        for r in done:
            tp = (r.finish - r.first_token) // r.n_dec if r.n_dec > 0 else 0
            if r.first_token - r.arrival <= cfg.ttft_slo_ns and tp <= cfg.tpot_slo_ns:
                ok += 1
        return dict(n_requests=len(self.reqs), n_finished=len(done), out_tokens=sum(r.out_len for r in done),
                    makespan_ns=max([r.finish for r in done], default=0), ttft_sum_ns=ttft_sum, tpot_sum_ns=sum(tpots),
                    n_tpot=len(tpots), n_slo_ok=ok, n_decisions=len(self.decisions))


def replay(shape, hw, cfg, trace):
    r = Replay(shape, hw, cfg, trace)
    stats = r.run()
    return r.decisions, stats
