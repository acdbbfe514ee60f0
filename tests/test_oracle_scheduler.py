"""Pins of the scheduler oracle: cases whose branch can be read off by inspection, the
nearest-rank percentile, and invariants that hold for any trace."""
import numpy as np
import pytest

from oracle import latency as L
from oracle import scheduler as S
from paper_2504_19516_amd import synth

SHAPE = L.Shape(32, 4096, 32, 8, 128, 14336, 128256)


def profile():
    hw = L.Profile(n_cu=256, granule=32, c_peak=1_000_000, d_peak=4_000, n_d=112, tile_m=128, tile_n=128, tile_q=128)
    hw.alpha_prefill = L.Grid([[32, 256], [256, 8192]], [[1_600_000, 1_300_000], [1_700_000, 1_400_000]])
    hw.alpha_decode = L.Grid([[32, 256], [1, 64], [1024, 131072]], [[[2_500_000, 1_500_000], [2_000_000, 1_400_000]],
                                                                    [[5_000_000, 2_000_000], [3_000_000, 1_800_000]]])
    return hw


def config(**kw):
    c = dict(ttft_slo_ns=1_000_000_000, tpot_slo_ns=50_000_000, layers_per_step=4, max_batch_tokens=16384,
             max_decode_batch=256, kv_pool_pages=40000, mode=0, fixed_prefill_cus=0)
    c.update(kw)
    return S.Config(**c)


def test_chunked_prefill_accounting_by_brute_force():
    """Section 2.2.2: count the iterations and the KV chunk loads by running the lock-step loop."""
    for sl, cs, ds in ((16384, 1024, 0), (16384, 2048, 0), (1000, 512, 12), (513, 512, 0), (5, 512, 500), (4096, 256, 255)):
        left, iters, loads = sl, 0, 0
        while left > 0:
            left -= min(cs - ds, left)
            iters += 1
            loads += iters                      # this chunk's attention reads every chunk cached so far, itself included
        assert S.chunked_prefill_iterations(sl, cs, ds) == (iters, loads)
    assert S.chunked_prefill_iterations(16384, 1024, 0) == (16, 136)


def test_p90_is_nearest_rank():
    assert S.p90([]) == 0 and S.p90([5]) == 5
    assert S.p90(list(range(1, 11))) == 9                 # ceil(0.9 * 10) = 9th smallest
    assert S.p90(list(range(11, 0, -1))) == 10            # ceil(0.9 * 11) = 10th smallest
    assert S.p90([3, 1]) == 3


def test_single_request_gets_whole_gpu_and_layers_in_order():
    dec, st = S.replay(SHAPE, profile(), config(), [(0, 2048, 1)])
    assert [(d[4], d[5]) for d in dec] == [(l, l + 4) for l in range(0, 32, 4)]
    for d in dec:
        assert d[1] == 1 and d[2] == 0            # one task, request 0
        assert (d[6], d[7], d[8]) == (256, 0, 2)  # no decode work: ReduceDecodeSM gives decode nothing
    assert st["n_finished"] == 1 and st["out_tokens"] == 1
    # simulated clock: TTFT is exactly the sum of the predicted slices
    assert st["ttft_sum_ns"] == sum(d[10] for d in dec) == st["makespan_ns"]


def test_decode_is_given_the_minimum_that_meets_tpot():
    """Second request arrives while the first decodes: decode keeps the smallest CU count whose
    predicted P90 TPOT is within the SLO (Section 3.3.1), prefill the rest."""
    hw, cfg = profile(), config()
    dec, st = S.replay(SHAPE, hw, cfg, [(0, 512, 200), (100_000_000, 4096, 4)])
    second = [d for d in dec if d[2] == 1]
    assert second and all(d[8] == 2 for d in second)
    dms = {d[7] for d in second}
    assert dms == {32}                             # a batch of one decodes within 50 ms on the smallest partition
    assert all(d[6] + d[7] == 256 for d in second)
    assert st["n_finished"] == 2 and st["n_slo_ok"] == 2


def test_end_of_prefill_boost_by_inspection():
    """Section 3.3.1: while the final slice of a prefill runs, decode gets extra CUs and the prefill
    set is kept (the sets intersect); every other slice, and every decision without the boost, is
    unchanged because the simulated durations ignore the shared CUs."""
    hw = profile()
    trace = [(0, 512, 200), (100_000_000, 4096, 4)]
    base = S.replay(SHAPE, hw, config(), trace)[0]
    boost = S.replay(SHAPE, hw, config(decode_boost_cus=64), trace)[0]
    assert len(base) == len(boost)
    n_boosted = 0
    for a, b in zip(base, boost):
        assert a[:7] == b[:7] and a[8:] == b[8:]                 # same batch, slice, prefill CUs, branch, duration
        last_with_decode = a[5] == SHAPE.n_layers and a[9] > 0 and a[7] > 0
        assert b[7] == (min(hw.n_cu, a[7] + 64) if last_with_decode else a[7])
        n_boosted += last_with_decode
    assert n_boosted == 1                                        # the second request's last slice, beside request 0's decode
    last = [d for d in boost if d[2] == 1][-1]
    assert (last[6], last[7]) == (224, 96)                       # 224 + 96 > 256: 64 CUs are shared for that slice
    # nothing decodes -> nothing to boost
    solo = S.replay(SHAPE, hw, config(decode_boost_cus=64), [(0, 2048, 1)])[0]
    assert all(d[7] == 0 for d in solo)


def test_tight_tpot_pushes_cus_to_decode_and_overload_balances():
    hw = profile()
    trace = [(0, 256, 400)] * 48 + [(400_000_000 + i, 8000, 8) for i in range(12)]
    loose = S.replay(SHAPE, hw, config(), trace)[0]
    tight = S.replay(SHAPE, hw, config(tpot_slo_ns=12_000_000), trace)[0]
    late_loose = [d for d in loose if d[0] > 400_000_000 and d[9] > 0]
    late_tight = [d for d in tight if d[0] > 400_000_000 and d[9] > 0]
    assert max(d[7] for d in late_tight) > max(d[7] for d in late_loose)
    # impossible SLOs on both sides: every late decision is the balanced branch
    over = S.replay(SHAPE, hw, config(ttft_slo_ns=1_000_000, tpot_slo_ns=1_000_000), trace)[0]
    late_over = [d for d in over if d[0] > 400_000_000 and d[9] > 0]
    assert late_over and all(d[8] == 1 for d in late_over)
    assert all(0 < d[7] < 256 for d in late_over)


def check_invariants(shape, hw, cfg, trace):
    dec, st = S.replay(shape, hw, cfg, trace)
    n = len(trace)
    assert st["n_finished"] == n and st["out_tokens"] == int(sum(t[2] for t in trace))
    started = [d for d in dec if d[4] == 0]
    assert sum(d[1] for d in started) == n                     # every request enters exactly one batch
    by_batch = {}
    for d in dec:
        by_batch.setdefault((d[3], d[2]), []).append((d[4], d[5]))
    for slices in by_batch.values():                           # layers run in order, all of them
        assert slices[0][0] == 0 and slices[-1][1] == shape.n_layers
        assert all(a[1] == b[0] for a, b in zip(slices, slices[1:]))
    for d in dec:
        if cfg.mode in (1, 3):
            assert d[6] == d[7] == hw.n_cu
        elif cfg.mode == 5:
            assert d[6] == hw.n_cu and d[7] in (0, hw.n_cu)
        elif cfg.mode == 6:
            assert d[6] == cfg.fixed_prefill_cus and d[7] == hw.n_cu
        elif cfg.decode_boost_cus and d[5] == shape.n_layers and d[9] > 0 and d[7] > 0:
            assert hw.n_cu < d[6] + d[7] <= hw.n_cu + cfg.decode_boost_cus and d[7] <= hw.n_cu
        else:
            assert d[6] + d[7] == hw.n_cu and d[6] >= hw.granule and d[6] % hw.granule == 0
    assert all(a[0] <= b[0] for a, b in zip(dec, dec[1:]))
    return dec, st


@pytest.mark.parametrize("mode", [0, 1, 2, 3, 4, 5, 6])
@pytest.mark.parametrize("rate", [2.0, 12.0])
def test_invariants_on_poisson_trace(mode, rate):
    trace = synth.poisson_trace(7, rate, 8.0, dict(kind="lognormal", median=600, sigma=1.0, cap=8192),
                                dict(kind="lognormal", median=250, sigma=0.9, cap=2048))
    cfg = config(mode=mode, fixed_prefill_cus=160)
    check_invariants(SHAPE, profile(), cfg, [tuple(int(x) for x in r) for r in trace])


def test_invariants_with_end_of_prefill_boost():
    trace = synth.poisson_trace(7, 12.0, 8.0, dict(kind="lognormal", median=600, sigma=1.0, cap=8192),
                                dict(kind="lognormal", median=250, sigma=0.9, cap=2048))
    for mode in (0, 2, 4):
        dec, _ = check_invariants(SHAPE, profile(), config(mode=mode, fixed_prefill_cus=160, decode_boost_cus=64),
                                  [tuple(int(x) for x in r) for r in trace])
        assert any(d[6] + d[7] > 256 for d in dec)


def test_reorder_does_not_starve_long_request():
    hw = profile()
    trace = [(0, 8000, 2)] + [(1000 + i, 64, 2) for i in range(40)]
    dec, st = check_invariants(SHAPE, hw, config(ttft_slo_ns=2_000_000_000), trace)
    first_batches = [d for d in dec if d[4] == 0]
    assert first_batches[0][2] == 0                           # it arrived alone and starts at once
    # with a long request queued behind many short ones the guard still brings it forward in time
    trace2 = [(0, 64, 2)] + [(10, 8000, 2)] + [(20 + i, 64, 2) for i in range(200)]
    dec2, st2 = check_invariants(SHAPE, hw, config(ttft_slo_ns=400_000_000), trace2)
    start_long = [d[0] for d in dec2 if d[4] == 0 and d[2] <= 1 and d[3] == S.tasks_hash([1])]
    assert start_long and start_long[0] <= 400_000_000


def test_ablation_policies_by_inspection():
    """Section 4.5: Naive and w/Partition keep arrival order; w/Partition never suspends decode while
    requests decode; w/Scheduler reorders like the full design but never splits the CUs."""
    hw = profile()
    # a long request ahead of many short ones: the scheduler policies bring short ones forward
    trace = [(0, 64, 40)] + [(10, 8000, 40)] + [(20 + i, 64, 40) for i in range(30)]

    for mode, reorders in ((0, True), (3, False), (4, False), (5, True)):
        dec, st = S.replay(SHAPE, hw, config(mode=mode, max_batch_tokens=8000), [tuple(t) for t in trace])
        starts = [d for d in dec if d[4] == 0]
        long_pos = next(k for k, d in enumerate(starts) if d[2] == 1)      # the batch whose lowest id is the long request
        assert (long_pos > 1) == reorders, (mode, long_pos)       # in arrival order the long one is second
        if mode == 4:
            assert all(d[7] > 0 for d in dec if d[9] > 0)          # decode batch present -> decode keeps CUs
        if mode in (3, 5):
            assert all(d[6] == hw.n_cu for d in dec)


def test_small_pool_serialises_admission_without_deadlock():
    trace = [(i * 1000, 1000, 50) for i in range(12)]
    dec, st = check_invariants(SHAPE, profile(), config(kv_pool_pages=200), trace)   # three requests fit at a time
    assert st["n_finished"] == 12


def test_time_multiplexed_is_slower_under_load():
    trace = synth.poisson_trace(9, 10.0, 6.0, dict(kind="lognormal", median=600, sigma=1.0, cap=8192),
                                dict(kind="lognormal", median=250, sigma=0.9, cap=2048))
    tr = [tuple(int(x) for x in r) for r in trace]
    a = S.replay(SHAPE, profile(), config(mode=0), tr)[1]
    b = S.replay(SHAPE, profile(), config(mode=1), tr)[1]
    assert a["n_finished"] == b["n_finished"] == len(tr)
    assert a["ttft_sum_ns"] < b["ttft_sum_ns"]


def test_batching_floor_by_inspection():
    """Three 700-token prompts queued at time 0. A 700-token batch is already past the roofline ridge of this
    profile, so Algorithm 1's rule starts one prompt alone; with min_batch_tokens = 1500 the first batch
    keeps taking queued prompts until it holds at least 1500 tokens (three prompts: 700, 1400, 2100), and
    with a floor that a single prompt already meets nothing changes."""
    trace = [(0, 700, 1)] * 3
    first = lambda cfg: S.replay(SHAPE, profile(), cfg, trace)[0][0]
    assert first(config())[1] == 1
    assert first(config(min_batch_tokens=1500))[1] == 3
    assert first(config(min_batch_tokens=1400))[1] == 2
    assert first(config(min_batch_tokens=700))[1] == 1
    # never more than the queue holds, and max_batch_tokens still caps the batch
    assert first(config(min_batch_tokens=100000))[1] == 3
    assert first(config(min_batch_tokens=100000, max_batch_tokens=1400))[1] == 2


# ---------------------------------------------------------------------------------------------
# Algorithm 1, lines 14-20, and the reorder guard of Section 3.3.2 on hand-built states. The
# estimator is replaced by literal tables (milliseconds per layer over the prefill CUs, per step
# over the decode CUs), so every number in the expected decision can be worked out on paper and
# none of it passes through the latency model or the library.
MS = 1_000_000
PREFILL_MS_PER_LAYER = {256: 8, 224: 10, 192: 12, 160: 15, 128: 20, 96: 30, 64: 45, 32: 90}


class TableReplay(S.Replay):
    """Replay whose estimator is two literal tables; the batching loop stops after one request."""

    def __init__(self, cfg, trace, decode_ms, prefill_ms=None):
        super().__init__(SHAPE, profile(), cfg, trace)
        self.decode_ms = decode_ms
        self.prefill_ms = prefill_ms            # per request id: ms for the whole prefill, whatever the CUs

    def t_prefill(self, ids, pm, l0, nl, co_dm):
        if self.prefill_ms is not None:
            return sum(self.prefill_ms[i] for i in ids) * MS * nl // SHAPE.n_layers
        return PREFILL_MS_PER_LAYER[pm] * MS * nl

    def t_decode(self, ids, dm, co):
        return self.decode_ms[dm] * MS

    def intensity_below_ridge(self, ids, pm):
        return False


def inflight_state(decode_ms):
    """Request 0 decodes (first token just now, none generated yet, so its predicted TPOT is the
    next step's latency); request 1 arrived 100 ms ago and has 4 of 32 prefill layers done; the
    split in force is 224 prefill / 32 decode CUs."""
    r = TableReplay(config(), [(0, 512, 200), (0, 4096, 4)], decode_ms)
    r.now = 100 * MS
    r.reqs[0].first_token = r.now
    r.D = [0]
    r.P, r.l_exe = [1], 4
    r.pm, r.dm = 224, 32
    return r


def test_reduce_prefill_sm_takes_smallest_decode_share_that_meets_tpot():
    """In-flight TTFT: 100 ms waited + 28 layers x 10 ms = 380 ms <= 1 s, so `satisfy` holds; TPOT on
    the current 32 decode CUs is 80 ms > 50 ms: neither SetBalancedSM (needs `not satisfy`) nor
    ReduceDecodeSM (needs TPOT within its SLO) applies, Algorithm 1 takes its third branch. Walking
    the decode share upwards, 32 -> 80 ms, 64 -> 60 ms, 96 -> 40 ms: 96 CUs is the first that meets
    50 ms, prefill keeps the other 160; the slice is 4 layers x 15 ms."""
    r = inflight_state({32: 80, 64: 60, 96: 40, 128: 30, 160: 25, 192: 22, 224: 20})
    dur = r.schedule()
    now, n_tasks, first, _, l0, l1, pm, dm, branch, n_dec, pred = r.decisions[-1]
    assert (n_tasks, first, l0, l1) == (1, 1, 4, 8)
    assert (pm, dm, branch, n_dec) == (160, 96, 3, 1)
    assert dur == pred == 4 * 15 * MS


def test_reduce_prefill_sm_falls_back_to_largest_decode_share_that_keeps_ttft():
    """No decode share meets the 50 ms TPOT (the best, 224 CUs, still needs 55 ms). The fallback gives
    decode as much as the in-flight request's TTFT allows: 100 ms waited + 28 layers x t(pm) <= 1000 ms
    needs t <= 32.1 ms per layer, i.e. at least 96 prefill CUs (30 ms; 64 CUs take 45 ms), so decode
    gets 256 - 96 = 160 CUs. The slice is 4 layers x 30 ms."""
    r = inflight_state({32: 90, 64: 85, 96: 80, 128: 75, 160: 70, 192: 60, 224: 55})
    dur = r.schedule()
    _, _, _, _, l0, l1, pm, dm, branch, _, pred = r.decisions[-1]
    assert (l0, l1, pm, dm, branch) == (4, 8, 96, 160, 3)
    assert dur == pred == 4 * 30 * MS


def test_reduce_prefill_sm_without_any_admissible_share_balances():
    """As above, but the in-flight request has already waited 990 ms: no split keeps its TTFT (the
    28 layers left need 224 ms even on every CU) -- yet on the current 224 CUs its estimate is
    990 + 280 = 1270 ms > 1 s, so `satisfy` fails and with TPOT over its SLO Algorithm 1 takes the
    first branch, SetBalancedSM: minimise max(TTFT / 1000 ms, TPOT / 50 ms) over the decode shares
    32..224 (decode is not suspended while a request decodes).
      dm   pm   TTFT = 990 + 28 t(pm)   /1000    TPOT  /50     max
      32   224  1270                    1.270    90    1.80    1.80
      64   192  1326                    1.326    85    1.70    1.70
      96   160  1410                    1.410    80    1.60    1.60
      128  128  1550                    1.550    75    1.50    1.55   <- smallest
      160  96   1830                    1.830    70    1.40    1.83
    so decode gets 128 CUs and the slice is 4 layers x 20 ms."""
    r = inflight_state({32: 90, 64: 85, 96: 80, 128: 75, 160: 70, 192: 60, 224: 55})
    r.now = 990 * MS
    r.reqs[0].first_token = r.now
    dur = r.schedule()
    _, _, _, _, _, _, pm, dm, branch, _, pred = r.decisions[-1]
    assert (pm, dm, branch) == (128, 128, 1)
    assert dur == pred == 4 * 20 * MS


def test_reorder_guard_moves_exactly_the_request_it_would_hurt():
    """Queue in arrival order A, B, C, D (ids 0..3) with whole-prefill estimates 600, 300, 100, 200 ms;
    A has waited 200 ms, the others 50 ms; TTFT SLO 1000 ms; nothing is in flight.
      arrival order:            A 200+600 = 800, B 50+900 = 950, C 50+1000 = 1050, D 50+1200 = 1250
      least-latency order C, D, B, A:  C 50+100 = 150, D 50+300 = 350, B 50+600 = 650, A 200+1200 = 1400
    Only A meets its SLO in arrival order and misses it after the reordering, so only A is moved to
    the front; the rest keep the least-latency order: A, C, D, B. The batching loop (stubbed to stop
    after one request) then starts A and leaves C, D, B queued in that order."""
    cfg = config()
    trace = [(150 * MS, 4000, 2), (300 * MS, 2000, 2), (300 * MS, 700, 2), (300 * MS, 1400, 2)]
    r = TableReplay(cfg, trace, {}, prefill_ms={0: 600, 1: 300, 2: 100, 3: 200})
    r.now = 350 * MS
    r.Q = [0, 1, 2, 3]
    r.schedule()
    assert r.P == [0] and r.Q == [2, 3, 1]
    assert r.decisions[-1][1:4] == (1, 0, S.tasks_hash([0]))
    # without a request that the reordering would push over its SLO the order is least-latency first
    r2 = TableReplay(config(ttft_slo_ns=2000 * MS), trace, {}, prefill_ms={0: 600, 1: 300, 2: 100, 3: 200})
    r2.now = 350 * MS
    r2.Q = [0, 1, 2, 3]
    r2.schedule()
    assert r2.P == [2] and r2.Q == [3, 1, 0]
    # a request that misses its SLO either way is not protected (A has waited 700 ms: 1300 and 1900 ms)
    r3 = TableReplay(cfg, [(-350 * MS, 4000, 2)] + trace[1:], {}, prefill_ms={0: 600, 1: 300, 2: 100, 3: 200})
    r3.now = 350 * MS
    r3.Q = [0, 1, 2, 3]
    r3.schedule()
    assert r3.P == [2] and r3.Q == [3, 1, 0]
