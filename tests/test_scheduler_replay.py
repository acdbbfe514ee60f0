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
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_replay_matches_oracle_on_conversational_traces(sts, rate, seed, mode):
    trace = synth.poisson_trace(seed, rate, 6.0, IN3, OUT3)
    cfg = dict(CFG3, mode=mode, fixed_prefill_cus=192)
    dec, st = run_both(sts, synth.llama8b_model(), sample_profile(), cfg, trace)
    assert st["n_finished"] == len(trace)


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
