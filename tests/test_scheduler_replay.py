"""The library's scheduler against the independent oracle replay: same profile, same trace,
same configuration -> identical decisions (CU split, batch composition, layer slice, branch,
predicted duration) and identical request statistics, bit for bit."""
import numpy as np
import pytest

from oracle import latency as L
from oracle import scheduler as S
from paper_2504_19516_amd import synth
from tests.test_library import sample_profile, sts  # noqa: F401  (fixture)

IN3 = dict(kind="lognormal", median=600, sigma=1.0, cap=8192)
OUT3 = dict(kind="lognormal", median=250, sigma=0.9, cap=2048)
IN4 = dict(kind="uniform", lo=8192, hi=32768)
OUT4 = dict(kind="uniform", lo=64, hi=512)


def shape_of(desc):
    return L.Shape(desc.n_layers, desc.hidden, desc.n_q_heads, desc.n_kv_heads, desc.head_dim, desc.mlp, desc.vocab)


def run_both(sts, desc, hw, cfg, trace):
    want_dec, want_st = S.replay(shape_of(desc), hw, S.Config(**cfg), [tuple(int(x) for x in r) for r in trace])
    got_dec, got_st = sts.Profile(text=L.dump_profile(hw)).replay(desc, cfg, trace)
    assert got_st == want_st
    assert len(got_dec) == len(want_dec)
    for a, b in zip(got_dec, want_dec):
        assert a == b
    return want_dec, want_st


CFG3 = dict(ttft_slo_ns=1_000_000_000, tpot_slo_ns=50_000_000, layers_per_step=4, max_batch_tokens=16384,
            max_decode_batch=256, kv_pool_pages=60000, mode=0, fixed_prefill_cus=0)


@pytest.mark.parametrize("rate,seed", [(2.0, 1), (8.0, 2), (16.0, 3)])
@pytest.mark.parametrize("mode", [0, 1, 2, 3, 4, 5, 6])
def test_replay_matches_oracle_on_conversational_traces(sts, rate, seed, mode):
    trace = synth.poisson_trace(seed, rate, 6.0, IN3, OUT3)
    cfg = dict(CFG3, mode=mode, fixed_prefill_cus=192)
    dec, st = run_both(sts, synth.llama8b_model(), sample_profile(), cfg, trace)
    assert st["n_finished"] == len(trace)


@pytest.mark.parametrize("mode", [0, 2, 4])
def test_replay_matches_oracle_with_end_of_prefill_boost(sts, mode):
    trace = synth.poisson_trace(8, 12.0, 6.0, IN3, OUT3)
    cfg = dict(CFG3, mode=mode, fixed_prefill_cus=192, decode_boost_cus=64)
    dec, st = run_both(sts, synth.llama8b_model(), sample_profile(), cfg, trace)
    assert any(d[6] + d[7] > 256 for d in dec)
    with pytest.raises(Exception):
        sts.Profile(text=L.dump_profile(sample_profile())).replay(synth.llama8b_model(), dict(cfg, decode_boost_cus=20), trace)


def test_replay_matches_oracle_on_long_prompts_and_70b(sts):
    trace = synth.poisson_trace(4, 1.0, 10.0, IN4, OUT4)
    cfg = dict(CFG3, max_batch_tokens=65536, kv_pool_pages=30000)
    run_both(sts, synth.llama8b_model(), sample_profile(), cfg, trace)
    cfg70 = dict(CFG3, ttft_slo_ns=3_000_000_000, tpot_slo_ns=100_000_000, layers_per_step=8, kv_pool_pages=26000)
    run_both(sts, synth.llama70b_model(), sample_profile(), cfg70, synth.poisson_trace(5, 2.0, 8.0, IN3, OUT3))


def test_replay_matches_oracle_under_pressure(sts):
    """Tight SLOs and a small pool exercise the balanced branch, suspension and admission stalls."""
    trace = synth.poisson_trace(6, 20.0, 3.0, IN3, OUT3)
    hw = sample_profile()
    hw.use_waveq = 0
    for cfg in (dict(CFG3, ttft_slo_ns=200_000_000, tpot_slo_ns=15_000_000), dict(CFG3, kv_pool_pages=2500),
                dict(CFG3, ttft_slo_ns=2_000_000, tpot_slo_ns=2_000_000, max_decode_batch=16)):
        dec, st = run_both(sts, synth.llama8b_model(), hw, cfg, trace)
    assert any(d[8] == 1 for d in dec)


def test_replay_rejects_bad_input(sts):
    p = sts.Profile(text=L.dump_profile(sample_profile()))
    with pytest.raises(sts.StsError):
        p.replay(synth.llama8b_model(), dict(CFG3, layers_per_step=0), np.array([[0, 10, 10]]))
    with pytest.raises(sts.StsError):
        p.replay(synth.llama8b_model(), CFG3, np.array([[5, 10, 10], [1, 10, 10]]))     # arrivals not sorted


def test_single_cycle_decide_matches_oracle_on_built_states(sts):
    """sts_sched_decide on caller-built states against the oracle's schedule() on the same state."""
    desc, hw = synth.llama8b_model(), sample_profile()
    p = sts.Profile(text=L.dump_profile(hw))
    rng = np.random.default_rng(11)
    for case in range(40):
        n = int(rng.integers(2, 30))
        trace = [(int(rng.integers(0, 2_000_000_000)), int(rng.integers(16, 9000)), int(rng.integers(1, 600))) for _ in range(n)]
        trace.sort()
        cfg = dict(CFG3, ttft_slo_ns=int(rng.choice([300_000_000, 1_000_000_000])), tpot_slo_ns=int(rng.choice([8_000_000, 50_000_000])),
                   kv_pool_pages=int(rng.choice([3000, 60000])))
        r = S.Replay(shape_of(desc), hw, S.Config(**cfg), trace)
        ids = list(range(n))
        rng.shuffle(ids)
        n_dec, n_p = int(rng.integers(0, n // 2 + 1)), int(rng.integers(0, 2))
        dec_ids, rest = ids[:n_dec], ids[n_dec:]
        p_ids = sorted(rest[:n_p * int(rng.integers(1, 3))])
        q_ids = sorted(set(rest) - set(p_ids))
        r.now = 2_100_000_000 + int(rng.integers(0, 500_000_000))
        r.D, r.H = dec_ids[: len(dec_ids) // 2], dec_ids[len(dec_ids) // 2:]
        for i in dec_ids:
            r.reqs[i].first_token = r.now - int(rng.integers(1_000_000, 900_000_000))
            r.reqs[i].n_dec = int(rng.integers(0, 300))
        r.P, r.Q = list(p_ids), list(q_ids)
        r.l_exe = int(rng.integers(0, 8)) * 4 if p_ids else 0
        r.pages_free = int(rng.integers(100, cfg["kv_pool_pages"]))
        r.pm, r.dm = [(0, 256), (224, 32), (128, 128), (256, 0)][int(rng.integers(0, 4))]
        args = (r.now, [(i, trace[i][0], trace[i][1], trace[i][2]) for i in r.Q], [(i, trace[i][0], trace[i][1], trace[i][2]) for i in r.P],
                r.l_exe, [(r.reqs[i].first_token, r.reqs[i].n_dec, r.reqs[i].in_len) for i in r.D + r.H], r.pages_free, r.pm, r.dm)
        had_p = bool(r.P)
        got = p.decide(desc, cfg, *args)
        dur = r.schedule()
        assert got["queue"] == r.Q, case
        if dur is None:
            assert got["tasks"] == [] and got["predicted_ns"] == -1
            continue
        d = r.decisions[-1]
        assert got["tasks"] == r.P and got["admitted"] == (not had_p)
        assert (got["layer_begin"], got["layer_end"], got["prefill_cus"], got["decode_cus"], got["branch"], got["predicted_ns"]) == \
               (d[4], d[5], d[6], d[7], d[8], d[10]), case


@pytest.mark.parametrize("mode", [0, 1, 5])
def test_replay_matches_oracle_with_a_batching_floor(sts, mode):
    """min_batch_tokens keeps a new batch taking queued requests past the roofline ridge; the library's
    replay stays equal to the oracle's, and batches do grow."""
    trace = synth.poisson_trace(9, 24.0, 6.0, IN3, OUT3)
    plain, _ = run_both(sts, synth.llama8b_model(), sample_profile(), dict(CFG3, mode=mode), trace)
    floor, st = run_both(sts, synth.llama8b_model(), sample_profile(), dict(CFG3, mode=mode, min_batch_tokens=2048), trace)
    assert st["n_finished"] == len(trace)
    assert max(d[1] for d in floor) > max(d[1] for d in plain)
    with pytest.raises(Exception):
        sts.Profile(text=L.dump_profile(sample_profile())).replay(synth.llama8b_model(), dict(CFG3, min_batch_tokens=-1), trace)
