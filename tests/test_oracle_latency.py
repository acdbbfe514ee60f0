"""Pins of the latency-model oracle: the paper's printed wave-quantisation table, the
worked roofline example, Eq. 1's two equivalent forms, and interpolation properties."""
import os
from fractions import Fraction

import pytest

from oracle import latency as L

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_table1():
    rows = []
    for line in open(os.path.join(GOLD, "wave_quant_table1.txt")):
        if line.strip() and not line.startswith("#"):
            seq, kern, g, pct = line.split()
            rows.append((int(seq), kern, [int(x) for x in g.split("+")], pct))
    return rows


def test_wave_quant_reproduces_paper_table1():
    """Table 1 (108 SMs, one block per SM): idle percentages as printed. An MLP cell lists the block
    counts of its two GEMMs (gate/up, down) and is their flop-weighted (2 : 1) mean."""
    rows = read_table1()
    assert sorted({k for _, k, _, _ in rows}) == ["Attn", "MLP", "O", "QKV"] and len(rows) == 16
    for seq, kern, gs, pct in rows:
        idles = [L.wave_quant(g, 108, 1)[2] for g in gs]
        assert len(gs) == (2 if kern == "MLP" else 1)
        idle = (2 * idles[0] + idles[1]) / 3 if kern == "MLP" else idles[0]
        assert f"{float(idle) * 100:.1f}" == pct, (seq, kern, gs, float(idle))


def test_wave_quant_definitions():
    # exact multiple: no idle; one extra block: a whole wave for one unit
    assert L.wave_quant(216, 108) == (2, 108, Fraction(0))
    w, tail, idle = L.wave_quant(217, 108)
    assert (w, tail) == (3, 1) and idle == Fraction(107, 324)
    # b blocks per unit: 2 per SM, 300 blocks on 108 SMs -> 2 waves, tail ceil(300/2 - 108) = 42
    assert L.wave_quant(300, 108, 2)[:2] == (2, 42)
    # the O-projection bound quoted in Section 2.2.2: 100 - idle = 59 % and 79 %
    assert round(100 * (1 - L.wave_quant(64, 108)[2])) == 59
    assert round(100 * (1 - L.wave_quant(256, 108)[2])) == 79


def test_srm_worked_example_section_3_2_2():
    """N = 108, N_d = 30: at 54 SMs bandwidth stays at peak and the plateau halves; at 20
    SMs both drop (slope to 2/3, plateau to 20/108)."""
    hw = L.Profile(n_cu=108, c_peak=1000, d_peak=100, n_d=30)
    big = 10 ** 9
    # memory-bound kernel (no flops): time = mem / D_p
    assert L.srm_ns(0, big, 108, hw) == big // 100
    assert L.srm_ns(0, big, 54, hw) == big // 100
    assert L.srm_ns(0, big, 20, hw) == big * 30 // (100 * 20)
    # compute-bound kernel (no bytes): time = flop / C_p
    assert L.srm_ns(big, 0, 54, hw) == 2 * big // 1000
    assert L.srm_ns(big, 0, 20, hw) == big * 108 // (1000 * 20)


@pytest.mark.parametrize("n_p", [20, 30, 54, 108])
@pytest.mark.parametrize("flop,mem", [(10 ** 12, 10 ** 9), (10 ** 9, 10 ** 9), (5 * 10 ** 10, 3 * 10 ** 9)])
def test_eq1_min_form_equals_max_form(n_p, flop, mem):
    hw = L.Profile(n_cu=108, c_peak=312_000, d_peak=1_555, n_d=30)
    c_p = Fraction(hw.c_peak * n_p, hw.n_cu)
    d_p = Fraction(hw.d_peak) * min(Fraction(1), Fraction(n_p, hw.n_d))
    t_eq1 = Fraction(flop) / min(Fraction(flop, mem) * d_p, c_p)       # Eq. 1 as printed
    assert abs(L.srm_ns(flop, mem, n_p, hw) - t_eq1) < 1


def test_interp_reproduces_samples_and_is_linear_between():
    axes = [[32, 128], [64, 256, 1024]]
    vals = [[1_500_000, 1_300_000, 1_200_000], [1_100_000, 1_050_000, 1_000_000]]
    for i, a in enumerate(axes[0]):
        for j, b in enumerate(axes[1]):
            assert L.interp(axes, vals, [a, b]) == vals[i][j]
    assert L.interp(axes, vals, [32, 160]) == 1_400_000            # midway on the second axis
    assert L.interp(axes, vals, [80, 64]) == 1_300_000             # midway on the first axis
    # two samples along CUs are enough: extrapolation continues the line
    assert L.interp([[64, 128]], [2_000_000, 1_000_000], [192]) == 0
    assert L.interp([[64, 128]], [2_000_000, 1_000_000], [32]) == 2_500_000
    g = L.Grid([[64, 128]], [2_000_000, 1_000_000])
    assert L.alpha_at(g, [192]) == 500_000                          # clamped to half the smallest sample


def test_alpha_roundtrip_eq2():
    s = L.Shape(32, 4096, 32, 8, 128, 14336, 128256)
    hw = L.Profile()
    t = L.prefill_roofline_ns(s, hw, [(2048, 0)], 128, 0, 1)
    a = L.alpha_from_measurement(3 * t // 2, t)
    assert abs(a - 1_500_000) <= 1
    hw.alpha_prefill = L.Grid([[128], [2048]], [[a]])
    assert abs(L.predict_prefill_ns(s, hw, [(2048, 0)], 128, 0, 1) - 3 * t // 2) <= 2


def test_work_counts_against_hand_totals():
    """8B-shaped layer, 2048 new tokens: 893.4 GFLOP of GEMM and 34.4 GFLOP of causal
    attention; decode batch of 64: 436.2 MB of weights per layer."""
    s = L.Shape(1, 4096, 32, 8, 128, 14336, 128256)
    ks, _ = L.prefill_kernels(s, L.Profile(), [(2048, 0)], False)
    d = {k[0]: k for k in ks}
    gemm = sum(d[k][1] for k in ("qkv", "o", "gateup", "down"))
    assert gemm == 2 * 2048 * 218_103_808
    assert abs(d["attn"][1] - 34.4e9) < 0.1e9
    assert d["qkv"][3] == 8 * 24 and d["gateup"][3] == 8 * 112 and d["attn"][3] == 16 * 32
    kd, head = L.decode_kernels(s, [1000] * 64)
    w_bytes = sum(x[2] for x in kd if x[0] in ("qkv", "o", "gateup", "down"))
    assert 436_207_616 <= w_bytes <= 436_207_616 * 1.03
    assert dict((x[0], x[2]) for x in kd)["attn"] >= 64 * 1001 * 4096
    assert head[0][2] >= 2 * 4096 * 128256


def test_prediction_monotone_in_cus_and_inf_when_suspended():
    s = L.Shape(32, 4096, 32, 8, 128, 14336, 128256)
    hw = L.Profile(use_waveq=0)
    prev = None
    for n in range(32, 257, 32):
        t = L.predict_prefill_ns(s, hw, [(2048, 0)], n, 0, 4)
        d = L.predict_decode_ns(s, hw, [1024] * 64, n, 0)
        if prev:
            assert t <= prev[0] and d <= prev[1]
        prev = (t, d)
    assert L.predict_prefill_ns(s, hw, [(2048, 0)], 0, 0, 4) == L.INF_NS
    assert L.predict_decode_ns(s, hw, [1024] * 64, 0, 0) == L.INF_NS
    assert L.predict_decode_ns(s, hw, [], 0, 0) == 0


def test_contention_table_replaces_d_p_for_decode():
    s = L.Shape(1, 4096, 32, 8, 128, 14336, 1024)
    hw = L.Profile()
    hw.bw = L.Grid([[64, 128], [0, 4096]], [[3000, 2000], [5000, 4000]])
    solo = L.decode_roofline_ns(s, hw, [1024] * 64, 64, 0)
    co = L.decode_roofline_ns(s, hw, [1024] * 64, 64, 4096)
    assert 1.45 < co / solo < 1.55                                   # 3000 -> 2000 bytes/ns
    ks, head = L.decode_kernels(s, [1024] * 64)
    assert abs(solo - sum(k[2] for k in ks + head) / 3000) < len(ks) + 2


def test_prefill_corun_table_by_hand():
    """The measured slowdown of a prefill slice beside a decode step multiplies the stand-alone
    prediction: exact at the samples, linear between and beyond them, absent when nothing decodes
    beside the slice or when the two CU sets overlap."""
    s = L.Shape(32, 4096, 32, 8, 128, 14336, 128256)
    hw = L.Profile(use_waveq=0)
    hw.prefill_corun = L.Grid([[0, 32, 64, 128]], [1_000_000, 1_100_000, 1_200_000, 1_400_000])
    alone = L.predict_prefill_ns(s, hw, [(2048, 0)], 224, 0, 4)
    assert L.predict_prefill_ns(s, hw, [(2048, 0)], 224, 0, 4, 0) == alone
    assert L.predict_prefill_ns(s, hw, [(2048, 0)], 224, 0, 4, 32) == alone * 1_100_000 // 1_000_000
    assert L.predict_prefill_ns(s, hw, [(2048, 0)], 192, 0, 4, 48) == L.predict_prefill_ns(s, hw, [(2048, 0)], 192, 0, 4) * 1_150_000 // 1_000_000
    assert L.prefill_corun_ppm(hw, 192) == 1_600_000                  # extrapolated along the last segment
    es = dict(prefill_len=[2048], prefill_ctx=[0], decode_ctx=[1000] * 8, prefill_cus=224, decode_cus=32, layer_begin=0, n_layers_step=4)
    assert L.latency_query(s, hw, es)[0] == alone * 1_100_000 // 1_000_000
    assert L.latency_query(s, hw, dict(es, decode_ctx=[]))[0] == alone                       # nothing decodes
    assert L.latency_query(s, hw, dict(es, decode_cus=64))[0] == alone                       # 224 + 64 > 256: overlapping sets
    hw.prefill_corun = None
    assert L.latency_query(s, hw, es)[0] == alone
    assert L.parse_profile(L.dump_profile(hw)) == hw


def test_wave_quant_adjustment_uses_workgroups_per_cu():
    """224 CUs x 2 resident workgroups: 512 tiles need 2 waves of 448 slots, the second one
    running on 64/2 = 32 CUs -> 1 - idle = (224*2 - 224 + 32) / (224*2)."""
    assert L._waveq_adjust(1_000_000, 512, 224, 2) == 1_000_000 * 448 // 256
    assert L._waveq_adjust(1_000_000, 512, 256, 2) == 1_000_000          # exactly one wave
    assert L._waveq_adjust(1_000_000, 512, 224, 1) == 1_000_000 * 672 // 512


def test_tail_cut_plan_and_adjustment_by_hand():
    """The last, partly filled wave cut along K. Hand cases for 448 slots (224 CUs x 2):
    512 tiles -> one whole wave, 64 tiles left; 7 pieces each fill the 448 slots once, so the
    last wave costs 1/7 + 3 % of a tile time. A brute-force search over the cuts confirms the
    choice; counts that divide evenly, or where no cut saves a tenth of a tile, stay uncut."""
    assert L.tail_plan(512, 448, 16) == (1, 64, 7, 1)
    assert L.tail_plan(896, 448, 16) == (2, 0, 1, 0)
    assert L.tail_plan(512, 320, 16)[:3] == (1, 192, 5)               # 960 pieces = 3 rounds of 1/5
    assert L.tail_plan(430, 448, 16)[2] == 1                          # 430 of 448 slots busy: nothing to gain
    assert L.tail_plan(512, 448, 0)[2] == 1
    for g, slots in [(512, 448), (128, 224), (100, 96), (777, 512), (5, 448)]:
        full, rest, f, rounds = L.tail_plan(g, slots, 16)
        costs = {c: -(-rest * c // slots) * (L.PPM // c + L.PIECE_COST_PPM) for c in range(2, 17)}
        if rest and min(costs.values()) <= 900_000:
            assert costs[f] == min(costs.values()) and rounds == -(-rest * f // slots)
        else:
            assert f == 1
    t = 1_000_000
    want = t * (L.PPM + (L.PPM // 7 + 30_000)) * 448 // (512 * L.PPM)
    assert L._waveq_tail_adjust(t, 512, 224, 2, 16) == want
    assert 1.02 * t < want < 1.03 * t                                 # against 1.75 t uncut
    assert L._waveq_tail_adjust(t, 896, 224, 2, 16) == t
    assert L._waveq_tail_adjust(t, 430, 224, 2, 16) == L._waveq_adjust(t, 430, 224, 2)
    # whole layer, 2048 tokens of the 8B shape on 224 CUs: the O and down GEMMs (512 tiles each)
    # lose their 75 % second-wave penalty, gate/up (3584 = 8 x 448) is unchanged
    s = L.Shape(1, 4096, 32, 8, 128, 14336, 128256)
    hw0, hw1 = L.Profile(tile_m=128, tile_n=128, wgs_per_cu=2), L.Profile(tile_m=128, tile_n=128, wgs_per_cu=2, tail_cut=16)
    cut, whole = L.prefill_roofline_ns(s, hw1, [(2048, 0)], 224, 0, 1), L.prefill_roofline_ns(s, hw0, [(2048, 0)], 224, 0, 1)
    assert 0.8 * whole < cut < 0.9 * whole
    # 512-tile GEMMs fill 256 CUs x 2 exactly; only qkv (768 tiles) still gains
    assert L.prefill_roofline_ns(s, hw1, [(2048, 0)], 256, 0, 1) <= L.prefill_roofline_ns(s, hw0, [(2048, 0)], 256, 0, 1)


def test_profile_text_roundtrip():
    hw = L.Profile(n_d=112, c_peak=1_234_567, wgs_per_cu=2, tail_cut=16)
    hw.bw = L.Grid([[32, 64], [0, 2048, 8192]], [[1600, 1500, 1400], [2700, 2500, 2300]])
    hw.alpha_decode = L.Grid([[32, 256], [8, 64], [1000, 100000]],
                             [[[1, 2], [3, 4]], [[5, 6], [7, 8]]])
    hw2 = L.parse_profile(L.dump_profile(hw))
    assert hw2 == hw


def test_online_recalibration_by_hand():
    """Section 3.2.4 / Eq. 2 on a 2 x 2 alpha grid, every number worked out on paper. Samples over
    (CUs, tokens) = (64 | 192) x (1000 | 3000): 1.0, 1.2 / 1.4, 1.6. The execution state (128 CUs,
    2000 tokens) is the centre of the cell, so the interpolation reads all four and predicts their
    mean, alpha = 1.3. A slice measured at 1.56 times its roofline time gives alpha_obs = 1.56
    (Eq. 2), 1.2 times the prediction. With weight 0.5 every sample the interpolation read moves by
    0.5 x (1.2 - 1) = +10 % of its own value: 1.1, 1.32 / 1.54, 1.76; the prediction at the state
    moves from 1.3 to 1.43, half of the way to 1.56."""
    g = L.Grid([[64, 192], [1000, 3000]], [[1_000_000, 1_200_000], [1_400_000, 1_600_000]])
    assert L.alpha_at(g, [128, 2000]) == 1_300_000
    L._blend(g, [128, 2000], 1_560_000, 1_000_000, 500_000)
    assert g.values == [[1_100_000, 1_320_000], [1_540_000, 1_760_000]]
    assert L.alpha_at(g, [128, 2000]) == 1_430_000
    # weight 1: the prediction at the state lands on the measurement; a state on a grid line reads
    # (and moves) only the two samples of that line
    g = L.Grid([[64, 192], [1000, 3000]], [[1_000_000, 1_200_000], [1_400_000, 1_600_000]])
    L._blend(g, [64, 2000], 2_200_000, 1_000_000, 1_000_000)          # predicted 1.1, observed 2.2: samples double
    assert g.values[0] == [2_000_000, 2_400_000]
    assert L.alpha_at(g, [64, 2000]) == 2_200_000
    # through observe(): the roofline time comes from the model (pinned by the tests above), the
    # measurement is 1.56 times it; only the prefill grid moves, the decode grid is untouched
    s = L.Shape(32, 4096, 32, 8, 128, 14336, 128256)
    hw = L.Profile(use_waveq=0)
    hw.alpha_prefill = L.Grid([[64, 192], [1000, 3000]], [[1_000_000, 1_200_000], [1_400_000, 1_600_000]])
    hw.alpha_decode = L.Grid([[64, 192], [8, 64], [512, 4096]], [[[1_000_000, 1_100_000], [1_200_000, 1_300_000]], [[900_000, 950_000], [1_000_000, 1_050_000]]])
    before_decode = [[list(r) for r in p] for p in hw.alpha_decode.values]
    roof = L.prefill_roofline_ns(s, hw, [(2000, 0)], 128, 4, 4)
    es = dict(prefill_len=[2000], prefill_ctx=[0], decode_ctx=[], prefill_cus=128, decode_cus=0, layer_begin=4, n_layers_step=4)
    L.observe(s, hw, es, roof * 156 // 100, 0, 500_000)
    want = [[1_100_000, 1_320_000], [1_540_000, 1_760_000]]
    for row, wrow in zip(hw.alpha_prefill.values, want):
        for v, wv in zip(row, wrow):
            assert abs(v - wv) <= 2                                     # floor of roof * 1.56 costs at most a ppm or two
    assert hw.alpha_decode.values == before_decode
    # a decode measurement moves the eight samples around (128 CUs, batch 36, mean context 2304) and no prefill sample
    hw.alpha_prefill = L.Grid([[64, 192], [1000, 3000]], [[1_000_000, 1_200_000], [1_400_000, 1_600_000]])
    cls = [2304] * 36
    es = dict(prefill_len=[], prefill_ctx=[], decode_ctx=cls, prefill_cus=0, decode_cus=128, layer_begin=0, n_layers_step=0)
    a_pred = L.alpha_at(hw.alpha_decode, [128, 36, 2304])
    assert a_pred == (1_000_000 + 1_100_000 + 1_200_000 + 1_300_000 + 900_000 + 950_000 + 1_000_000 + 1_050_000) // 8
    droof = L.decode_roofline_ns(s, hw, cls, 128, 0)
    L.observe(s, hw, es, 0, droof * a_pred // 1_000_000 * 2, 1_000_000)     # measured twice the prediction, weight 1
    flat = [v for p in hw.alpha_decode.values for r in p for v in r]
    for v, old in zip(flat, [1_000_000, 1_100_000, 1_200_000, 1_300_000, 900_000, 950_000, 1_000_000, 1_050_000]):
        assert abs(v - 2 * old) <= 4
    assert hw.alpha_prefill.values == [[1_000_000, 1_200_000], [1_400_000, 1_600_000]]
