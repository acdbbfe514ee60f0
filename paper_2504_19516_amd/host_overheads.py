"""Host-side cost of the control path (paper Section 4.6 reports 10.2 us per latency prediction and
4.1 us per SM reconfiguration): microseconds per `sts_latency_query`, per `sts_sched_decide`
cycle and per `sts_set_partition` switch, measured through the Python binding (so the ctypes
marshalling is included) and, for the query, also per call of the library alone via a replay.

    python -m paper_2504_19516_amd.host_overheads --profile paper_2504_19516_amd/data/mi355x_llama8b.profile [--gpu]
"""
from __future__ import annotations

import argparse
import time

import numpy as np

from . import sts, synth


def per_call_us(fn, n):
    fn()
    t0 = time.perf_counter_ns()
    for _ in range(n):
        fn()
    return (time.perf_counter_ns() - t0) / n / 1e3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--profile", required=True)
    ap.add_argument("--gpu", action="store_true", help="also time sts_set_partition (needs the GPU)")
    args = ap.parse_args()
    desc = synth.llama8b_model()
    prof = sts.Profile(text=open(args.profile).read())
    ctx = [int(c) for c in synth.lognormal_lengths(2, 64, 1024, 0.8, 8192)]
    es = dict(prefill_len=[2048], prefill_ctx=[0], decode_ctx=ctx, prefill_cus=224, decode_cus=32, layer_begin=0, n_layers_step=4)
    print(f"sts_latency_query (one 2048-token prefill slice of 4 layers + 64 decodes), through the binding: "
          f"{per_call_us(lambda: prof.query(desc, es), 2000):.1f} us per call")
    cfg = dict(ttft_slo_ns=1_000_000_000, tpot_slo_ns=50_000_000, layers_per_step=4, max_batch_tokens=16384, max_decode_batch=256,
               kv_pool_pages=40000, mode=0, fixed_prefill_cus=0)
    rng = np.random.default_rng(3)
    for nq, nd in ((4, 32), (20, 128), (60, 256)):
        queue = [(i, 1000 * i, int(x), 200) for i, x in enumerate(synth.lognormal_lengths(5, nq, 600, 1.0, 8192))]
        dec = [(10_000_000 * int(rng.integers(1, 50)), int(rng.integers(1, 300)), int(rng.integers(50, 2000))) for _ in range(nd)]
        us = per_call_us(lambda: prof.decide(desc, cfg, 2_000_000_000, queue, [], 0, dec, 30000, 224, 32), 300)
        print(f"sts_sched_decide (Algorithm 1, {nq} queued, {nd} decoding; every candidate split is priced with the estimator): {us:.0f} us per cycle")
    # the library alone: a replay makes a few predictions per scheduling cycle and decode step
    trace = synth.poisson_trace(1, 16.0, 10.0, dict(kind="lognormal", median=600, sigma=1.0, cap=8192),
                                dict(kind="lognormal", median=250, sigma=0.9, cap=2048))
    t0 = time.perf_counter_ns()
    dec_log, st = prof.replay(desc, cfg, trace)
    dt = time.perf_counter_ns() - t0
    print(f"sts_sched_replay of a 10 s, 16 req/s trace: {dt / 1e6:.1f} ms for {st['n_decisions']} scheduling cycles "
          f"({dt / 1e3 / max(1, st['n_decisions']):.0f} us per cycle including the decode steps between them)")
    if args.gpu:
        eng = sts.Engine(synth.llama8b_model(1), weight_seed=1, init_weights=False, kv_pool_pages=64, max_prefill_tokens=256, max_prefill_seqs=2,
                         max_decode_batch=8, max_seqs=8, max_pages_per_seq=8)
        n = eng.get_partition()[2]
        for pm in range(32, n, 32):                       # create every masked stream of the grid once
            eng.set_partition(pm, n - pm)
        k = [0]

        def switch():
            k[0] += 1
            pm = 224 if k[0] & 1 else 192
            eng.set_partition(pm, n - pm)
        print(f"sts_set_partition between existing CU sets (a pointer switch in the masked-stream pool): {per_call_us(switch, 5000):.2f} us per call")
        eng.close()


if __name__ == "__main__":
    main()
