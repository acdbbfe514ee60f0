"""Live serving of an arrival trace on the GPU (paper Sections 3.3 and 3.5.2): one control thread
keeps a layer-sliced prefill batch and a decode step in flight on their CU partitions, asks the
library's Algorithm 1 (`sts_sched_decide`) for the next prefill tasks and CU split at every
prefill cycle, and hands prefilled requests over to the decode batch without moving any KV.

Modes: "concurrent" (Algorithm 1 picks the split), "tm" (time-multiplexed: same kernels, whole
GPU, prefill slices and decode steps strictly alternate), "fixed:<prefill CUs>" (concurrent with
a static split), the paper's ablations "naive", "wpart", "wsched" (Section 4.5) and
"fixedall:<prefill CUs>" (Section 4.4: prefill on a fixed CU count, decode on every CU), and
"chunked:<chunk tokens>", the chunked-prefill baseline (whole GPU, one prompt chunk through all
layers then one decode step, alternating). Arrivals follow the trace in real time. Token values are random (weights are
random too): output lengths come from the trace, so argmax flips cannot change the workload.

    python -m paper_2504_19516_amd.serve --model 8b --rate 8 --window 20 --mode concurrent \
        --profile paper_2504_19516_amd/data/mi355x_llama8b.profile
"""
from __future__ import annotations

import argparse
import json
import sys
import threading
import time

import numpy as np

from . import sts, synth

PAGE = 16


class Req:
    __slots__ = ("rid", "arrival", "in_len", "out_len", "seq", "tokens", "first_token", "n_dec", "finish")

    def __init__(self, rid, arrival, in_len, out_len):
        self.rid, self.arrival, self.in_len, self.out_len = rid, int(arrival), int(in_len), int(out_len)
        self.seq, self.tokens, self.first_token, self.n_dec, self.finish = -1, None, -1, 0, -1


class LiveServer:
    def __init__(self, desc, profile_text, cfg, kv_pool_pages, max_batch_tokens=16384, max_decode_batch=256, max_ctx=10240,
                 sched_slo_ns=None, recalibrate_ppm=0, control_threads=1):
        """cfg carries the SLOs requests are judged by; sched_slo_ns = (ttft, tpot) optionally gives the
        scheduler tighter targets than those (headroom for estimator error and for the running-mean TPOT,
        which Algorithm 1 otherwise steers right onto the limit)."""
        self.desc, self.cfg = desc, dict(cfg)
        self.slo = (cfg["ttft_slo_ns"], cfg["tpot_slo_ns"])
        self.recalibrate_ppm = int(recalibrate_ppm)      # > 0: feed every finished slice and step back into alpha (Section 3.2.4)
        self.control_threads = int(control_threads)      # 2: one control thread per phase, as the paper's two engines (Section 3.5);
                                                         # measured no faster than 1 here (the Python parts of the two loops share the GIL)
        if sched_slo_ns:
            self.cfg.update(ttft_slo_ns=int(sched_slo_ns[0]), tpot_slo_ns=int(sched_slo_ns[1]))
        self.cfg.update(max_batch_tokens=max_batch_tokens, max_decode_batch=max_decode_batch, kv_pool_pages=kv_pool_pages)
        self.profile = sts.Profile(text=profile_text)
        self.eng = sts.Engine(desc, weight_seed=1234, init_weights=True, kv_pool_pages=kv_pool_pages,
                              max_prefill_tokens=max_batch_tokens, max_prefill_seqs=64, max_decode_batch=max_decode_batch,
                              max_seqs=4096, max_pages_per_seq=(max_ctx + PAGE - 1) // PAGE)
        self.eng.set_tile_model(*self.profile.tile_model())      # the GEMM tile choice uses the rates measured for this profile
        self.eng.set_stream_model(*self.profile.stream_model())  # ... and the decode GEMM planner its read-stream rates
        self.n_cu = self.eng.get_partition()[2]
        self.max_ctx = max_ctx
        # Live-mode replay (Algorithm 1's decisions must be reproducible from a per-cycle log): when this is a
        # list, every scheduling cycle appends the exact state handed to sts_sched_decide, the scheduler
        # configuration and the choice that came back, so that a second implementation can re-decide it.
        self.state_log = None

    def decide(self, cfg, now, queue, inflight, layers_done, decode, pages_free, pm, dm):
        ch = self.profile.decide(self.desc, cfg, now, queue, inflight, layers_done, decode, pages_free, pm, dm)
        if self.state_log is not None:
            self.state_log.append(dict(cfg=dict(cfg), now_ns=int(now), queue=[tuple(map(int, q)) for q in queue],
                                       inflight=[tuple(map(int, q)) for q in inflight], layers_done=int(layers_done),
                                       decode=[tuple(map(int, d)) for d in decode], pages_free=int(pages_free),
                                       cur_prefill_cus=int(pm), cur_decode_cus=int(dm), choice=dict(ch)))
        return ch

    def close(self):
        self.eng.close()

    def run_chunked(self, trace, chunk_tokens, seed=0):
        """The chunked-prefill baseline the paper compares against (Sections 2.2.2, 4.1): one engine on the
        whole GPU; every iteration runs one prompt chunk of at most `chunk_tokens` tokens through ALL
        layers (appended after the tokens of that prompt already cached, so its attention re-reads
        them) and then one decode step of the running batch, i.e. the hybrid batch of
        chunk + decode tokens executed back to back. The token budget is shared as in Section 2.2.2:
        the ds running decode requests come first, the prompt gets the remaining cs - ds tokens (at
        least one). Prompts are taken in arrival order."""
        eng, desc = self.eng, self.desc
        n = self.n_cu
        rng = np.random.default_rng(seed)
        reqs = [Req(i, a, il, ol) for i, (a, il, ol) in enumerate(trace)]
        Q, D = [], []
        cur, done_tokens = None, 0
        next_arrival, rejected, chunks = 0, 0, 0
        eng.set_partition(n, n)
        max_batch = self.cfg["max_decode_batch"]
        t0 = time.perf_counter_ns()
        clock = lambda: time.perf_counter_ns() - t0
        while True:
            now = clock()
            while next_arrival < len(reqs) and reqs[next_arrival].arrival <= now:
                r = reqs[next_arrival]
                if r.in_len + r.out_len > self.max_ctx:
                    rejected += 1
                else:
                    Q.append(r)
                next_arrival += 1
            if cur is None and Q and len(D) < max_batch and eng.pages_free() >= (Q[0].in_len + Q[0].out_len + PAGE - 1) // PAGE:
                cur, done_tokens = Q.pop(0), 0
                cur.seq = eng.seq_create()
                eng.seq_reserve(cur.seq, cur.in_len + cur.out_len)
                cur.tokens = rng.integers(0, desc.vocab, cur.in_len, dtype=np.int32)
            if cur is None and not D:
                if next_arrival >= len(reqs) and not Q:
                    break
                if next_arrival < len(reqs):
                    wait = reqs[next_arrival].arrival - clock()
                    if wait > 0:
                        time.sleep(wait * 1e-9)
                continue
            if cur is not None:
                m = min(max(1, chunk_tokens - len(D)), cur.in_len - done_tokens)
                eng.prefill_launch([cur.seq], [cur.tokens[done_tokens:done_tokens + m]], 0, desc.n_layers,
                                   want_logits=(done_tokens + m == cur.in_len))
                eng.prefill_finish()
                done_tokens += m
                chunks += 1
                if done_tokens == cur.in_len:
                    now = clock()
                    cur.first_token = now
                    if cur.out_len <= 1:
                        cur.finish = now
                        eng.seq_free(cur.seq)
                    else:
                        D.append(cur)
                    cur = None
            if D:
                batch = list(D)
                eng.decode_launch([r.seq for r in batch], rng.integers(0, desc.vocab, len(batch), dtype=np.int32), want_next=True)
                eng.decode_finish(len(batch))
                now = clock()
                for r in batch:
                    r.n_dec += 1
                    if r.n_dec >= r.out_len - 1:
                        r.finish = now
                        eng.seq_free(r.seq)
                        D.remove(r)
        cfg = dict(self.cfg, ttft_slo_ns=self.slo[0], tpot_slo_ns=self.slo[1])
        return self.stats(reqs, rejected, cfg), [(0, 0, 0, 0, 0, n, n, 0, 0, 0)] * chunks, []

    def run(self, trace, mode="concurrent", seed=0, log_every=0):
        if mode.startswith("chunked"):
            return self.run_chunked(trace, int(mode.split(":")[1]), seed)
        eng, desc, cfg = self.eng, self.desc, dict(self.cfg)
        serial = mode == "tm"
        name = mode.split(":")[0]
        cfg["mode"] = MODES[name]
        if name == "boost":
            cfg["decode_boost_cus"] = int(mode.split(":")[1])
        elif ":" in mode:
            cfg["fixed_prefill_cus"] = int(mode.split(":")[1])
        if not serial and self.control_threads == 2:
            return self.run_two_threads(trace, cfg, seed)
        n = self.n_cu
        rng = np.random.default_rng(seed)
        reqs = [Req(i, a, il, ol) for i, (a, il, ol) in enumerate(trace)]
        Q, P, H, D = [], [], [], []
        l_exe, pm, dm = 0, (n if serial else 0), n
        prefill_busy = decode_busy = turn_decode = False
        decode_batch, cur_slice = [], None
        next_arrival, rejected = 0, 0
        timeline, decisions = [], []
        # |predicted - measured| / measured of every slice and step, measured on the device (HIP events around
        # the phase's kernels, what the estimator was calibrated on); the host clock, which also sees how late
        # this loop noticed the end of a phase while it was queuing the other one, is kept beside it
        err_p, err_d, err_p_host, err_d_host = [], [], [], []
        eng.set_partition(n, n)
        t0 = time.perf_counter_ns()
        clock = lambda: time.perf_counter_ns() - t0
        next_report = 30_000_000_000

        def finish(r, now):
            r.finish = now
            eng.seq_free(r.seq)

        while True:
            now = clock()
            while next_arrival < len(reqs) and reqs[next_arrival].arrival <= now:
                r = reqs[next_arrival]
                total = r.in_len + r.out_len
                if (total + PAGE - 1) // PAGE > cfg["kv_pool_pages"] or r.in_len > cfg["max_batch_tokens"] or total > self.max_ctx:
                    rejected += 1
                else:
                    Q.append(r)
                next_arrival += 1
            # ---- prefill engine: one scheduling cycle of Algorithm 1
            if not prefill_busy and (P or Q) and not (serial and (decode_busy or (turn_decode and (D or H)))):
                ch = self.decide(cfg, now, [(r.rid, r.arrival, r.in_len, r.out_len) for r in Q],
                                 [(r.rid, r.arrival, r.in_len, r.out_len) for r in P], l_exe,
                                 [(r.first_token, r.n_dec, r.in_len) for r in D + H], eng.pages_free(), pm, dm)
                by_id = {r.rid: r for r in Q}
                Q = [by_id[i] for i in ch["queue"]]
                if ch["tasks"]:
                    if ch["admitted"]:
                        P = [by_id[i] for i in ch["tasks"]]
                        l_exe = 0
                        for r in P:
                            r.seq = eng.seq_create()
                            eng.seq_reserve(r.seq, r.in_len + r.out_len)      # the pages Algorithm 1 accounted for
                            r.tokens = rng.integers(0, desc.vocab, r.in_len, dtype=np.int32)
                    pm, dm = ch["prefill_cus"], ch["decode_cus"]
                    if not serial:
                        eng.set_partition(pm, -1)
                    lb, le = ch["layer_begin"], ch["layer_end"]
                    eng.prefill_launch([r.seq for r in P], [r.tokens for r in P], lb, le, want_logits=(le == desc.n_layers))
                    prefill_busy, cur_slice = True, (now, lb, le, ch["predicted_ns"])
                    # the decode batch beside the slice (the estimator's co-run slowdown applies when one runs on other CUs)
                    slice_es = dict(prefill_len=[r.in_len for r in P], prefill_ctx=[0] * len(P),
                                    decode_ctx=[r.in_len + r.n_dec for r in D + H] if dm > 0 else [], prefill_cus=pm,
                                    decode_cus=dm, layer_begin=lb, n_layers_step=le - lb)
                    decisions.append((now, len(P), sum(r.in_len for r in P), lb, le, pm, dm, ch["branch"], len(D) + len(H), len(Q)))
            # ---- decode engine: merge hand-offs, one step on the CUs left to it
            if not decode_busy and not (serial and prefill_busy):
                while H and len(D) < cfg["max_decode_batch"]:
                    D.append(H.pop(0))
                if D:
                    dm_eff = n if (serial or not prefill_busy) else dm
                    if dm_eff > 0:
                        if not serial:
                            eng.set_partition(-1, dm_eff)
                        decode_batch = list(D)
                        co = [sum(r.in_len for r in P)] if (prefill_busy and not serial and P) else []
                        step_es = dict(prefill_len=co, prefill_ctx=[0] * len(co), decode_ctx=[r.in_len + r.n_dec for r in D],
                                       prefill_cus=pm if co else 0, decode_cus=dm_eff, layer_begin=0, n_layers_step=1)
                        step_pred = self.profile.query(desc, step_es)[1]
                        step_t0 = clock()
                        eng.decode_launch([r.seq for r in D], rng.integers(0, desc.vocab, len(D), dtype=np.int32), want_next=True)
                        decode_busy = True
            # ---- wait for the next event
            if not prefill_busy and not decode_busy:
                if next_arrival >= len(reqs) and not (P or Q or H or D):
                    break
                if next_arrival < len(reqs):
                    wait = reqs[next_arrival].arrival - clock()
                    if wait > 0:
                        time.sleep(wait * 1e-9)
                continue
            pdone = ddone = False
            while True:
                if prefill_busy and eng.phase_done(0):
                    pdone = True
                if decode_busy and eng.phase_done(1):
                    ddone = True
                if pdone or ddone:
                    break
                if next_arrival < len(reqs) and reqs[next_arrival].arrival <= clock() and not (prefill_busy and decode_busy):
                    break
                time.sleep(20e-6)
            now = clock()
            if pdone:
                eng.prefill_finish()
                prefill_busy, turn_decode = False, True
                l_exe = cur_slice[2]
                dev_ns = eng.last_timing()[0] or now - cur_slice[0]
                timeline.append((now, "prefill", pm, sum(r.in_len for r in P), cur_slice[1], cur_slice[2], now - cur_slice[0], cur_slice[3],
                                 dev_ns, len(P), len(D) if decode_busy else 0))
                err_p.append(abs(cur_slice[3] - dev_ns) / max(1, dev_ns))
                err_p_host.append(abs(cur_slice[3] - (now - cur_slice[0])) / max(1, now - cur_slice[0]))
                if self.recalibrate_ppm:
                    self.profile.observe(desc, slice_es, dev_ns, 0, self.recalibrate_ppm)
                if l_exe == desc.n_layers:
                    for r in P:
                        r.first_token = now
                        if r.out_len <= 1:
                            finish(r, now)
                        else:
                            H.append(r)
                    P, l_exe = [], 0
            if ddone:
                eng.decode_finish(len(decode_batch))
                decode_busy, turn_decode = False, False
                dev_ns = eng.last_timing()[1] or now - step_t0
                err_d.append(abs(step_pred - dev_ns) / max(1, dev_ns))
                err_d_host.append(abs(step_pred - (now - step_t0)) / max(1, now - step_t0))
                if self.recalibrate_ppm:
                    self.profile.observe(desc, step_es, 0, dev_ns, self.recalibrate_ppm)
                for r in decode_batch:
                    r.n_dec += 1
                    if r.n_dec >= r.out_len - 1:
                        finish(r, now)
                        D.remove(r)
                if now >= next_report:             # a long run says where it is every 30 s
                    next_report = now + 30_000_000_000
                    print(f"[serve] {mode}: t = {now / 1e9:.0f} s, {sum(r.finish >= 0 for r in reqs)}/{len(reqs)} finished, "
                          f"{len(Q)} queued, {len(D)} decoding", file=sys.stderr, flush=True)
                if log_every and len(timeline) % log_every == 0:
                    timeline.append((now, "decode", eng.get_partition()[1], len(decode_batch)))
        eng.set_partition(n, n)
        st = self.stats(reqs, rejected, dict(cfg, ttft_slo_ns=self.slo[0], tpot_slo_ns=self.slo[1]))
        st["estimator_mape_prefill"] = float(np.mean(err_p)) if err_p else 0.0
        st["estimator_mape_decode"] = float(np.mean(err_d)) if err_d else 0.0
        st["estimator_mape_prefill_host_clock"] = float(np.mean(err_p_host)) if err_p_host else 0.0
        st["estimator_mape_decode_host_clock"] = float(np.mean(err_d_host)) if err_d_host else 0.0
        return st, decisions, timeline

    def run_two_threads(self, trace, cfg, seed=0):
        """The concurrent modes with one control thread per phase (Section 3.5: two engines that run
        autonomously and meet only in shared metadata): the prefill thread admits arrivals, runs
        Algorithm 1 and launches layer slices; the decode thread merges the requests handed over and
        launches decode steps on the CUs the last decision left to it. They share the hand-over list,
        the split in force and the decode status under one lock; the library allows one caller per
        phase. Queuing a decode step (about 1 ms of host time) then does not hold back the next prefill
        slice; measured on the 8B shape the two loops serve no better than the single one."""
        eng, desc, n = self.eng, self.desc, self.n_cu
        reqs = [Req(i, a, il, ol) for i, (a, il, ol) in enumerate(trace)]
        lock, prof_lock = threading.Lock(), threading.Lock()
        sh = dict(H=[], D=[], prefill_busy=False, pm=0, dm=n, co=0, prefill_over=False, error=None)
        decisions, timeline, err_p, err_d = [], [], [], []
        rejected = [0]
        eng.set_partition(n, n)
        t0 = time.perf_counter_ns()
        clock = lambda: time.perf_counter_ns() - t0
        recal = self.recalibrate_ppm

        def prof_call(fn, *a):
            if not recal:
                return fn(*a)
            with prof_lock:                     # observe() rewrites alpha samples that queries read
                return fn(*a)

        def prefill_loop():
            rng = np.random.default_rng(seed)
            Q, P = [], []
            l_exe, pm, dm, nxt = 0, 0, n, 0
            while True:
                now = clock()
                while nxt < len(reqs) and reqs[nxt].arrival <= now:
                    r = reqs[nxt]
                    total = r.in_len + r.out_len
                    if (total + PAGE - 1) // PAGE > cfg["kv_pool_pages"] or r.in_len > cfg["max_batch_tokens"] or total > self.max_ctx:
                        rejected[0] += 1
                    else:
                        Q.append(r)
                    nxt += 1
                launched = False
                if P or Q:
                    with lock:
                        dec = [(r.first_token, r.n_dec, r.in_len) for r in sh["D"] + sh["H"]]
                    ch = prof_call(self.decide, cfg, now, [(r.rid, r.arrival, r.in_len, r.out_len) for r in Q],
                                   [(r.rid, r.arrival, r.in_len, r.out_len) for r in P], l_exe, dec, eng.pages_free(), pm, dm)
                    by_id = {r.rid: r for r in Q}
                    Q = [by_id[i] for i in ch["queue"]]
                    if ch["tasks"]:
                        if ch["admitted"]:
                            P = [by_id[i] for i in ch["tasks"]]
                            l_exe = 0
                            for r in P:
                                r.seq = eng.seq_create()
                                eng.seq_reserve(r.seq, r.in_len + r.out_len)
                                r.tokens = rng.integers(0, desc.vocab, r.in_len, dtype=np.int32)
                        pm, dm = ch["prefill_cus"], ch["decode_cus"]
                        eng.set_partition(pm, -1)
                        lb, le = ch["layer_begin"], ch["layer_end"]
                        with lock:
                            sh.update(prefill_busy=True, pm=pm, dm=dm, co=sum(r.in_len for r in P))
                        eng.prefill_launch([r.seq for r in P], [r.tokens for r in P], lb, le, want_logits=(le == desc.n_layers))
                        launched = True
                        slice_es = dict(prefill_len=[r.in_len for r in P], prefill_ctx=[0] * len(P),
                                        decode_ctx=[in_len + n_dec for _, n_dec, in_len in dec] if dm > 0 else [], prefill_cus=pm,
                                        decode_cus=dm, layer_begin=lb, n_layers_step=le - lb)
                        decisions.append((now, len(P), sum(r.in_len for r in P), lb, le, pm, dm, ch["branch"], len(dec), len(Q)))
                        while not eng.phase_done(0):
                            time.sleep(20e-6)
                        eng.prefill_finish()
                        done = clock()
                        l_exe = le
                        timeline.append((done, "prefill", pm, sum(r.in_len for r in P), lb, le, done - now, ch["predicted_ns"]))
                        err_p.append(abs(ch["predicted_ns"] - (done - now)) / max(1, done - now))
                        if recal:
                            prof_call(self.profile.observe, desc, slice_es, done - now, 0, recal)
                        if l_exe == desc.n_layers:
                            hand = []
                            for r in P:
                                r.first_token = done
                                if r.out_len <= 1:
                                    r.finish = done
                                    eng.seq_free(r.seq)
                                else:
                                    hand.append(r)
                            with lock:
                                sh["H"].extend(hand)
                            P, l_exe = [], 0
                if not launched:
                    # nothing to run (or the KV pool is full): decode gets the whole GPU until the next slice. The flag
                    # stays set between the slices of a batch, so the split of the last decision holds across them.
                    with lock:
                        sh["prefill_busy"] = False
                    if nxt >= len(reqs) and not (P or Q):
                        break
                    wait = (reqs[nxt].arrival - clock()) if (nxt < len(reqs) and not (P or Q)) else 200_000   # KV pool full: retry shortly
                    if wait > 0:
                        time.sleep(min(wait, 2_000_000) * 1e-9)

        def decode_loop():
            rng = np.random.default_rng(seed + 1)
            while True:
                with lock:
                    while sh["H"] and len(sh["D"]) < cfg["max_decode_batch"]:
                        sh["D"].append(sh["H"].pop(0))
                    batch = list(sh["D"])
                    busy, pm, dm, co_tok = sh["prefill_busy"], sh["pm"], sh["dm"], sh["co"]
                    over = sh["prefill_over"] and not sh["H"]
                if not batch:
                    if over:
                        break
                    time.sleep(50e-6)
                    continue
                dm_eff = dm if busy else n
                if dm_eff <= 0:                  # decode is suspended for this slice
                    time.sleep(50e-6)
                    continue
                eng.set_partition(-1, dm_eff)
                co = [co_tok] if busy else []
                step_es = dict(prefill_len=co, prefill_ctx=[0] * len(co), decode_ctx=[r.in_len + r.n_dec for r in batch],
                               prefill_cus=pm if co else 0, decode_cus=dm_eff, layer_begin=0, n_layers_step=1)
                pred = prof_call(self.profile.query, desc, step_es)[1]
                t_start = clock()
                eng.decode_launch([r.seq for r in batch], rng.integers(0, desc.vocab, len(batch), dtype=np.int32), want_next=True)
                while not eng.phase_done(1):
                    time.sleep(20e-6)
                eng.decode_finish(len(batch))
                now = clock()
                err_d.append(abs(pred - (now - t_start)) / max(1, now - t_start))
                if recal:
                    prof_call(self.profile.observe, desc, step_es, 0, now - t_start, recal)
                gone = []
                for r in batch:
                    r.n_dec += 1
                    if r.n_dec >= r.out_len - 1:
                        r.finish = now
                        eng.seq_free(r.seq)
                        gone.append(r)
                if gone:
                    with lock:
                        for r in gone:
                            sh["D"].remove(r)

        def guarded(fn):
            def run():
                try:
                    fn()
                except BaseException as e:      # surfaces in the caller; the other thread is told to stop
                    sh["error"] = e
                finally:
                    if fn is prefill_loop:
                        with lock:
                            sh["prefill_over"] = True
            return run

        tp = threading.Thread(target=guarded(prefill_loop))
        td = threading.Thread(target=guarded(decode_loop))
        tp.start(); td.start()
        tp.join()
        if sh["error"] is not None:             # the decode thread leaves once nothing is handed over any more
            with lock:
                sh["H"].clear(); sh["D"].clear()
        td.join()
        if sh["error"] is not None:
            raise sh["error"]
        eng.set_partition(n, n)
        st = self.stats(reqs, rejected[0], dict(cfg, ttft_slo_ns=self.slo[0], tpot_slo_ns=self.slo[1]))
        st["estimator_mape_prefill"] = float(np.mean(err_p)) if err_p else 0.0
        st["estimator_mape_decode"] = float(np.mean(err_d)) if err_d else 0.0
        return st, decisions, timeline

    @staticmethod
    def stats(reqs, rejected, cfg):
        done = [r for r in reqs if r.finish >= 0]
        ttft = np.array([r.first_token - r.arrival for r in done], dtype=np.float64)
        tpot = np.array([(r.finish - r.first_token) / r.n_dec for r in done if r.n_dec > 0], dtype=np.float64)
        ok = sum(1 for r in done if (r.first_token - r.arrival) <= cfg["ttft_slo_ns"] and
                 (r.n_dec == 0 or (r.finish - r.first_token) / r.n_dec <= cfg["tpot_slo_ns"]))
        span = max((r.finish for r in done), default=0)
        out_tokens = sum(r.out_len for r in done)
        in_tokens = sum(r.in_len for r in done)
        pct = lambda a, q: float(np.percentile(a, q)) / 1e6 if len(a) else 0.0
        return dict(n_requests=len(reqs), n_finished=len(done), rejected=rejected, makespan_s=span / 1e9,
                    out_tokens=out_tokens, in_tokens=in_tokens, out_tokens_per_s=out_tokens / max(span, 1) * 1e9,
                    total_tokens_per_s=(out_tokens + in_tokens) / max(span, 1) * 1e9, requests_per_s=len(done) / max(span, 1) * 1e9,
                    ttft_mean_ms=float(ttft.mean()) / 1e6 if len(ttft) else 0.0, ttft_p90_ms=pct(ttft, 90),
                    tpot_mean_ms=float(tpot.mean()) / 1e6 if len(tpot) else 0.0, tpot_p90_ms=pct(tpot, 90),
                    slo_attainment=ok / max(1, len(reqs)))


# scheduler policies: Algorithm 1, time-multiplexed, fixed disjoint split "fixed:<prefill CUs>", the
# ablations of Section 4.5 (naive, wpart, wsched) and Section 4.4's "fixedall:<prefill CUs>" (prefill
# on a fixed CU count, decode on every CU); "boost:<extra decode CUs>" is Algorithm 1 with the end-of-prefill
# decode boost of Section 3.3.1 (the two CU sets intersect during a batch's final slice)
MODES = {"concurrent": 0, "tm": 1, "fixed": 2, "naive": 3, "wpart": 4, "wsched": 5, "fixedall": 6, "boost": 0}

WORKLOADS = {
    "conversation": (dict(kind="lognormal", median=600, sigma=1.0, cap=8192), dict(kind="lognormal", median=250, sigma=0.9, cap=2048)),
    "long": (dict(kind="uniform", lo=8192, hi=32768), dict(kind="uniform", lo=64, hi=512)),
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--model", default="8b", choices=["8b", "70b", "tiny"])
    ap.add_argument("--layers", type=int, default=0)
    ap.add_argument("--workload", default="conversation", choices=list(WORKLOADS))
    ap.add_argument("--rates", default="4,8")
    ap.add_argument("--window", type=float, default=15.0)
    ap.add_argument("--modes", default="concurrent,tm")
    ap.add_argument("--profile", required=True)
    ap.add_argument("--ttft-ms", type=float, default=1000.0)
    ap.add_argument("--tpot-ms", type=float, default=50.0)
    ap.add_argument("--sched-ttft-ms", type=float, default=0.0, help="TTFT target given to the scheduler (default: the SLO)")
    ap.add_argument("--sched-tpot-ms", type=float, default=0.0, help="TPOT target given to the scheduler (default: the SLO)")
    ap.add_argument("--layers-per-step", type=int, default=4)
    ap.add_argument("--min-batch-tokens", type=int, default=0,
                    help="batching floor: a new prefill batch keeps taking queued requests until it holds this many tokens (0: Algorithm 1's rule alone)")
    ap.add_argument("--recalibrate-ppm", type=int, default=0,
                    help="online alpha recalibration weight (parts per million per observation; 0 = off)")
    ap.add_argument("--control-threads", type=int, default=1, choices=[1, 2],
                    help="1: a single loop drives both phases; 2: one control thread per phase in the concurrent modes")
    ap.add_argument("--pool-pages", type=int, default=40000)
    ap.add_argument("--max-ctx", type=int, default=10240)
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
    make = {"8b": synth.llama8b_model, "70b": synth.llama70b_model}.get(args.model)
    desc = (make(args.layers) if args.layers else make()) if make else synth.tiny_model()
    cfg = dict(ttft_slo_ns=int(args.ttft_ms * 1e6), tpot_slo_ns=int(args.tpot_ms * 1e6), layers_per_step=args.layers_per_step,
               min_batch_tokens=args.min_batch_tokens)
    sched = (int((args.sched_ttft_ms or args.ttft_ms) * 1e6), int((args.sched_tpot_ms or args.tpot_ms) * 1e6))
    srv = LiveServer(desc, open(args.profile).read(), cfg, args.pool_pages, max_ctx=args.max_ctx,
                     max_batch_tokens=max(16384, args.max_ctx if args.workload == "long" else 0), sched_slo_ns=sched,
                     recalibrate_ppm=args.recalibrate_ppm, control_threads=args.control_threads)
    ind, outd = WORKLOADS[args.workload]
    results = []
    for rate in [float(x) for x in args.rates.split(",")]:
        trace = synth.poisson_trace(int(rate * 10) + 1, rate, args.window, ind, outd)
        for mode in args.modes.split(","):
            st, dec, tl = srv.run([tuple(int(x) for x in r) for r in trace], mode)
            splits = {}
            for d in dec:
                splits[d[5]] = splits.get(d[5], 0) + 1
            row = dict(rate=rate, mode=mode, **st, prefill_cus_histogram=splits)
            print(json.dumps(row), flush=True)
            results.append(row)
    if args.out:
        with open(args.out, "w") as f:
            json.dump(results, f, indent=1)
    srv.close()


if __name__ == "__main__":
    main()
