"""CPU-side checks of the built library: it loads, exports every symbol the header declares,
and its host-only parts (performance estimator) agree with the oracle bit for bit."""
import os
import re

import pytest

from oracle import latency as L
from paper_2504_19516_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sts():
    from paper_2504_19516_amd import sts as m
    if not os.path.exists(m.LIB_PATH):
        from paper_2504_19516_amd import build
        build.build()
    m.lib()
    return m


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "sts.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sts_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(sts):
    names = declared_symbols()
    assert len(names) >= 35
    for n in names:
        assert hasattr(sts.lib(), n), n
    assert sorted(sts.EXPORTS) == names


def test_packed_weight_layout_is_the_documented_operand_order(sts):
    """The packed GEMM weight layout, checked on the host against its definition: 32 x 64 blocks along K then along N,
    a block = four 1 KiB pieces (one per 16-column step), lane 32 h + n of a piece holding the 8 consecutive elements
    W[row n][16 step + 8 h .. + 8) -- and every element has exactly one place."""
    import ctypes as C
    f = sts.lib().sts_weight_packed_index
    f.restype = C.c_int64
    rows, ld = 96, 192
    seen = set()
    for r in range(rows):
        for c in range(ld):
            block = (r // 32) * (ld // 64) + c // 64
            step, h, e = (c % 64) // 16, (c % 16) // 8, c % 8
            lane = 32 * h + r % 32
            want = block * 2048 + step * 512 + lane * 8 + e
            got = f(r, c, ld)
            assert got == want, (r, c, got, want)
            seen.add(got)
    assert seen == set(range(rows * ld))
    assert f(0, ld, ld) == -1 and f(-1, 0, ld) == -1 and f(0, 0, 100) == -1


def test_error_strings(sts):
    assert sts.lib().sts_strerror(0) == b"ok"
    assert b"invalid" in sts.lib().sts_strerror(sts.EINVAL)


@pytest.mark.skipif(os.path.exists("/dev/kfd"), reason="a GPU is present")
def test_init_fails_loudly_without_gpu(sts):
    with pytest.raises(sts.StsError) as e:
        sts.Engine(synth.tiny_model(), kv_pool_pages=8)
    assert e.value.code == sts.EHIP


def test_wave_quant_matches_oracle(sts):
    for g, n, b in [(64, 108, 1), (256, 108, 1), (217, 108, 1), (300, 108, 2), (896, 224, 1), (3584, 512, 1), (5, 256, 3)]:
        w, tail, idle = L.wave_quant(g, n, b)
        cw, ct, num, den = sts.wave_quant(g, n, b)
        assert (cw, ct) == (w, tail) and idle == L.Fraction(num, den)


def sample_profile():
    hw = L.Profile(n_cu=256, granule=32, c_peak=1_000_000, d_peak=5_000, n_d=112, tile_m=128, tile_n=128, tile_q=128, wgs_per_cu=2, use_waveq=1)
    hw.bw = L.Grid([[32, 64, 128, 256], [0, 2048, 8192]],
                   [[1500, 1300, 1200], [2600, 2300, 2100], [4500, 4000, 3700], [5200, 4800, 4400]])
    hw.prefill_corun = L.Grid([[0, 32, 64, 128, 192]], [1_000_000, 1_110_000, 1_190_000, 1_370_000, 1_480_000])
    hw.alpha_prefill = L.Grid([[32, 128, 256], [256, 2048, 16384]],
                              [[2_400_000, 1_900_000, 1_700_000], [2_300_000, 1_800_000, 1_650_000], [2_500_000, 2_000_000, 1_800_000]])
    hw.alpha_decode = L.Grid([[32, 256], [8, 64, 256], [4096, 262144]],
                             [[[3_000_000, 2_000_000], [2_500_000, 1_800_000], [2_200_000, 1_700_000]],
                              [[6_000_000, 3_000_000], [4_000_000, 2_500_000], [3_000_000, 2_100_000]]])
    return hw


def test_profile_text_roundtrip_between_implementations(sts):
    hw = sample_profile()
    text = L.dump_profile(hw)
    p = sts.Profile(text=text)
    assert L.parse_profile(p.dump()) == hw
    with pytest.raises(sts.StsError) as e:
        sts.Profile(text="not a profile")
    assert e.value.code == sts.EIO


@pytest.mark.parametrize("waveq,tail_cut", [(0, 0), (1, 0), (1, 16), (1, 5)])
def test_latency_query_bit_exact_vs_oracle(sts, waveq, tail_cut):
    import numpy as np
    hw = sample_profile()
    hw.use_waveq = waveq
    hw.tail_cut = tail_cut
    p = sts.Profile(text=L.dump_profile(hw))
    rng = np.random.default_rng(5)
    for desc in (synth.llama8b_model(), synth.llama70b_model(), synth.tiny_model()):
        shape = L.Shape(desc.n_layers, desc.hidden, desc.n_q_heads, desc.n_kv_heads, desc.head_dim, desc.mlp, desc.vocab)
        for _ in range(60):
            npre, ndec = int(rng.integers(0, 5)), int(rng.integers(0, 40))
            es = dict(prefill_len=[int(x) for x in rng.integers(1, 20000, npre)],
                      prefill_ctx=[int(x) for x in rng.integers(0, 5000, npre)],
                      decode_ctx=[int(x) for x in rng.integers(0, 30000, ndec)],
                      prefill_cus=int(rng.choice([0, 8, 32, 96, 224, 256])), decode_cus=int(rng.choice([0, 8, 32, 160, 256])),
                      layer_begin=int(rng.integers(0, desc.n_layers)), n_layers_step=int(rng.integers(1, 5)))
            assert p.query(desc, es) == L.latency_query(shape, hw, es), es
            reqs = list(zip(es["prefill_len"], es["prefill_ctx"]))
            if npre and es["prefill_cus"]:
                want = L.prefill_roofline_ns(shape, hw, reqs, es["prefill_cus"], es["layer_begin"], es["n_layers_step"])
                assert p.query(desc, es, roofline=True)[0] == want


def test_latency_query_rejects_bad_state(sts):
    p = sts.Profile(text=L.dump_profile(sample_profile()))
    with pytest.raises(sts.StsError):
        p.query(synth.tiny_model(), dict(prefill_len=[0], prefill_ctx=[0], prefill_cus=32))


def test_online_recalibration_bit_exact_vs_oracle_and_converges(sts):
    """A stream of observations (Eq. 2 applied online, Section 3.2.4) leaves the library's profile and
    the oracle's identical, text for text; and repeated observations of one state pull its
    prediction onto the measurement."""
    import numpy as np
    hw = sample_profile()
    hw.tail_cut = 16
    p = sts.Profile(text=L.dump_profile(hw))
    desc = synth.llama8b_model()
    shape = L.Shape(desc.n_layers, desc.hidden, desc.n_q_heads, desc.n_kv_heads, desc.head_dim, desc.mlp, desc.vocab)
    rng = np.random.default_rng(11)
    for _ in range(200):
        npre, ndec = int(rng.integers(0, 4)), int(rng.integers(0, 30))
        es = dict(prefill_len=[int(x) for x in rng.integers(1, 12000, npre)], prefill_ctx=[int(x) for x in rng.integers(0, 3000, npre)],
                  decode_ctx=[int(x) for x in rng.integers(0, 20000, ndec)], prefill_cus=int(rng.choice([0, 32, 96, 224, 256])),
                  decode_cus=int(rng.choice([0, 32, 160, 256])), layer_begin=int(rng.integers(0, 28)), n_layers_step=4)
        mp, md = int(rng.integers(0, 50_000_000)), int(rng.integers(0, 50_000_000))
        w = int(rng.choice([0, 50_000, 300_000, 1_000_000]))
        p.observe(desc, es, mp, md, w)
        L.observe(shape, hw, es, mp, md, w)
    assert L.parse_profile(p.dump()) == hw
    es = dict(prefill_len=[3000], prefill_ctx=[0], decode_ctx=[1500] * 40, prefill_cus=192, decode_cus=64, layer_begin=0, n_layers_step=4)
    target_p, target_d = 7_000_000, 9_000_000
    for _ in range(60):
        p.observe(desc, es, target_p, target_d, 300_000)
    got = p.query(desc, es)
    assert abs(got[0] - target_p) <= 0.02 * target_p and abs(got[1] - target_d) <= 0.02 * target_d


def test_host_overheads_tool_runs_without_a_gpu(sts, capsys, monkeypatch):
    """The control-path timing tool (latency query, Algorithm 1 cycle, replay) needs no GPU."""
    import os
    import sys
    from paper_2504_19516_amd import host_overheads
    prof = os.path.join(os.path.dirname(host_overheads.__file__), "data", "mi355x_llama8b.profile")
    monkeypatch.setattr(sys, "argv", ["host_overheads", "--profile", prof])
    host_overheads.main()
    out = capsys.readouterr().out
    assert "sts_latency_query" in out and out.count("sts_sched_decide") == 3 and "sts_sched_replay" in out


def test_pmc_traffic_tool_scales_counters_by_the_copy_kernel(tmp_path, capsys, monkeypatch):
    """The counter arithmetic on hand-made rocprofv3 CSVs: the unit of each counter comes from the largest
    copy-kernel launches (512 MiB each way; smaller probe launches are ignored), the gate/up GEMM is the
    SwiGLU instantiation, the decode step sums the decode-only kernels per attention launch, and only the launches on the
    benchmarked partitions' queues count."""
    import sys
    from paper_2504_19516_amd import pmc_traffic
    gateup = "void sts::gemm_wreg_kernel<3, 2>(sts::GemmArgs)"
    other = "void sts::gemm_wreg_kernel<0, 2>(sts::GemmArgs)"
    skinny = "void sts::gemm_dl_kernel<64, 128, 1, 4, 1, 3, true>(sts::GemmArgs)"
    skinny2 = "void sts::gemm_skinny_kernel<1, 3>(sts::GemmArgs)"
    attn = "void sts::attn_decode_mfma_kernel<128, 4>(args)"
    copy = "sts::copy_kernel(a, b, c)"

    def write(name, counter, unit):
        # (kernel, counter value, hardware queue): queue 4 = prefill partition, 5 = decode partition, 2 = the streams of the
        # time-multiplexed reference, whose launches must not enter the figures
        rows = [(copy, (512 << 20) // unit, 1)] * 3 + [(copy, (256 << 20) // unit, 1)] * 5      # reference launches, then probes
        rows += [(gateup, 800_000_000 // unit, 4), (gateup, 780_000_000 // unit, 4), (other, 123, 4), (gateup, 500_000_000 // unit, 2)]
        rows += [(attn, 300_000_000 // unit, 5)] * 2 + [(skinny, 100_000_000 // unit, 5)] * 4 + [(skinny2, 100_000_000 // unit, 5)] * 4   # two decode steps
        rows += [(attn, 900_000_000 // unit, 2), (skinny, 900_000_000 // unit, 2)]
        path = tmp_path / name
        with open(path, "w") as f:
            f.write("Counter_Name,Kernel_Name,Counter_Value,Queue_Id\n")
            for k, v, q in rows:
                f.write(f'{counter},"{k}",{v},{q}\n')
        return str(path)
    fetch, wr = write("fetch.csv", "FETCH_SIZE", 2048), write("write.csv", "WRITE_SIZE", 1024)
    monkeypatch.setattr(sys, "argv", ["pmc_traffic", fetch, wr, "--prefill-cus", "224"])
    pmc_traffic.main()
    out = capsys.readouterr().out
    assert "2048.00 bytes per unit" in out and "1024.00 bytes per unit" in out
    assert "gate/up GEMM HBM traffic per launch: 1580.0 MB (read 790.0, written 790.0)" in out
    assert "decode layer-step HBM traffic (its own kernels, mean of 2 steps): 1400.0 MB (read 700.0, written 700.0)" in out


def test_live_serving_statistics_by_inspection():
    """SLO attainment counts a request only when its TTFT and its mean TPOT are both inside their limits
    (the definition of the paper's Section 4.1); unfinished requests count against it; throughput is over
    the makespan. Four hand-made requests, one per case."""
    from paper_2504_19516_amd import serve
    ms = 1_000_000

    def req(rid, arrival, first, n_dec, finish, in_len=100, out_len=11):
        r = serve.Req(rid, arrival, in_len, out_len)
        r.first_token, r.n_dec, r.finish = first, n_dec, finish
        return r
    reqs = [req(0, 0, 500 * ms, 10, 900 * ms),                 # TTFT 0.5 s, TPOT 40 ms: inside both
            req(1, 100 * ms, 1200 * ms, 10, 1500 * ms),        # TTFT 1.1 s: late first token
            req(2, 200 * ms, 300 * ms, 10, 900 * ms),          # TPOT 60 ms: slow decode
            req(3, 300 * ms, -1, 0, -1)]                       # never finished
    st = serve.LiveServer.stats(reqs, 0, dict(ttft_slo_ns=1000 * ms, tpot_slo_ns=50 * ms))
    assert st["n_requests"] == 4 and st["n_finished"] == 3
    assert st["slo_attainment"] == 0.25
    assert st["makespan_s"] == 1.5 and st["out_tokens"] == 33 and st["in_tokens"] == 300
    assert abs(st["out_tokens_per_s"] - 22.0) < 1e-9 and abs(st["total_tokens_per_s"] - 222.0) < 1e-9
    assert abs(st["ttft_mean_ms"] - (500 + 1100 + 100) / 3) < 1e-9 and abs(st["tpot_mean_ms"] - (40 + 30 + 60) / 3) < 1e-9


def test_decode_chunk_sizing_stays_within_what_the_engine_allocates(sts):
    """Host arithmetic of the decode attention work list: for every block-table bound that sts_init
    accepts and any mix of context lengths and partition sizes, a context is cut into at most as
    many chunks as the merge workspace and the work list are allocated for (at most 128), chunks
    hold 8..64 pages, and the bound itself is 128 chunks of 64 pages."""
    import numpy as np
    limit = sts.max_pages_per_seq_limit(16)
    assert limit == 128 * 64
    rng = np.random.default_rng(5)
    for mp in (1, 3, 8, 64, 513, 520, 2048, 4097, limit):
        for cus in (8, 32, 128, 256):
            for _ in range(6):
                n = int(rng.integers(1, 65))
                pages = rng.integers(1, mp + 1, size=n)
                pages[0] = mp                                     # the longest context the bound allows
                cp, mc, alloc = sts.decode_chunk_plan(pages, 8, cus, 16, mp)
                assert cp in (8, 16, 32, 64)
                assert mc == -(-mp // cp)
                assert mc <= alloc <= 128, (mp, cus, cp, mc, alloc)
    with pytest.raises(sts.StsError):
        sts.decode_chunk_plan([limit + 1], 8, 32, 16, limit)       # a context longer than the block table


def test_decode_gemm_plan_fits_tiles_to_the_partition():
    """Host logic of the decode GEMM planner (no GPU): the tile width divides N, the split stays within what the K extent
    feeds and the library accepts (at most 8 slices of at least 512 columns); a GEMM that has to finish its own output is
    never split; the Llama MLP width (7 * 2^k columns for gate and up together) comes out in whole rounds of 7-wave tiles on
    32 and 64 CUs, where every power-of-two width would leave a last round three quarters full; a whole GPU gets many
    small workgroups instead of a few wide ones; above 64 rows the decode GEMM takes a prefill tile shape."""
    from paper_2504_19516_amd import sts
    width = {"64x128": 128, "64x256s": 256, "64x320s": 320, "64x384s": 384, "64x448s": 448, "64x512s": 512}
    shapes = [(6144, 4096), (4096, 4096), (28672, 4096), (4096, 14336), (128256, 4096), (10240, 8192), (57344, 8192), (8192, 28672),
              (768, 256), (2048, 256), (256, 1024), (1024, 256), (640, 128)]
    for cus in (8, 32, 64, 96, 128, 160, 192, 224, 256):
        for n, k in shapes:
            for m in (1, 8, 37, 64):
                for may_split, partials in ((True, True), (False, False), (False, True)):
                    name, split, ns = sts.decode_gemm_plan(m, n, k, cus, may_split, partials)
                    assert name in width and n % width[name] == 0, (name, n)
                    assert 1 <= split <= max(1, min(8, k // 512)) and ns > 0
                    if not may_split:
                        assert split == 1
    for cus in (32, 64):
        assert sts.decode_gemm_plan(64, 28672, 4096, cus, may_split=False, partials=False)[:2] == ("64x448s", 1)
        assert sts.decode_gemm_plan(64, 57344, 8192, cus, may_split=False, partials=False)[:2] == ("64x448s", 1)
    # one wide tile per CU cannot keep 256 CUs busy with 4096 columns: narrow tiles, split deep
    name, split, _ = sts.decode_gemm_plan(64, 4096, 14336, 256)
    assert name == "64x128" and split >= 4
    # on a small partition the same GEMM takes wide tiles (the activation rows are re-read once per workgroup)
    assert width[sts.decode_gemm_plan(64, 4096, 14336, 32)[0]] >= 384
    # a slower estimate for fewer CUs, and never below the weight bytes at the memory system's rate
    t32, t256 = sts.decode_gemm_plan(64, 28672, 4096, 32)[2], sts.decode_gemm_plan(64, 28672, 4096, 256)[2]
    assert t32 > 2.5 * t256 and t256 >= 2 * 28672 * 4096 / 5.5e12 * 1e9
    assert sts.decode_gemm_plan(200, 28672, 4096, 32)[0] in ("128x128", "256x256")
    # the estimate follows the measured stream rates it is given: half the per-CU rate doubles a small partition's time,
    # and a whole GPU is held to the memory system's rate
    slow = sts.decode_gemm_plan(64, 28672, 4096, 32, stream_bw_cu=29500)[2]
    assert 1.7 * t32 < slow < 2.1 * t32
    assert sts.decode_gemm_plan(64, 28672, 4096, 256, stream_bw_gpu=3200000)[2] > 1.5 * t256
    for bad in ((64, 100, 4096, 32), (64, 4096, 100, 32), (0, 4096, 4096, 32), (64, 4096, 4096, 0)):
        with pytest.raises(sts.StsError) as e:
            sts.decode_gemm_plan(*bad)
        assert e.value.code == sts.EINVAL
    with pytest.raises(sts.StsError):
        sts.decode_gemm_plan(64, 4096, 4096, 32, stream_bw_cu=0)
