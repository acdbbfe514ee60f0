"""Per-kernel parity: each HIP kernel, called through the C ABI's single-operation entry
points, against the CPU oracle fed the same bf16-rounded inputs.

Tolerances (max |gpu - ref| / max |ref| over the compared tensor):
  fp32 accumulator outputs  <= 1e-3   (inputs identical; only summation order differs)
  bf16 outputs              <= 2e-2   (one or two bf16 roundings on the way out)
"""
import numpy as np
import pytest

from oracle import transformer as T
from paper_2504_19516_amd import synth

pytestmark = pytest.mark.gpu

ACC_TOL, BF16_TOL = 1e-3, 2e-2


def rel(a, b):
    return float(np.abs(np.asarray(a, np.float64) - np.asarray(b, np.float64)).max() / np.abs(b).max())


@pytest.fixture(scope="module")
def sts():
    from paper_2504_19516_amd import sts as m
    m.lib()
    return m


@pytest.mark.parametrize("cfg,m", [("256x256", 300), ("128x128", 300), ("64x256", 70), ("64x256", 20), ("64x128", 64), ("128x128", 1),
                                   ("64x128", 50), ("256x256", 513), ("128x256", 129), ("128x256", 300)])
def test_gemm_fp32_accumulators(sts, cfg, m):
    n, k = 512, 320
    a = synth.normal_bf16(1, (m, k))
    w = synth.normal_bf16(2, (n, k), 0.05)
    ref = T.op_linear(a.astype(np.float64), w.astype(np.float64))
    got = sts.op_gemm(a, w, cfg, epilogue=1)
    assert rel(got, ref) <= ACC_TOL
    assert rel(got, ref) <= 1e-5          # in practice fp32 accumulation of 320 terms


@pytest.mark.parametrize("cfg", ["256x256", "128x128", "64x128", "64x256", "128x256"])
@pytest.mark.parametrize("k", [64, 128, 192, 576])
@pytest.mark.parametrize("epilogue", [0, 1])
def test_gemm_short_and_odd_k_extents(sts, cfg, k, epilogue):
    """One, two, three and nine K tiles: the prologue, the steady loop and the surplus loads of the last iterations of every
    main loop (the 256x256 loop keeps three activation stages and requests operands a tile ahead), rows that end inside a tile."""
    m, n = 290, 512
    a = synth.normal_bf16(11, (m, k))
    w = synth.normal_bf16(12, (n, k), 0.1)
    ref = T.op_linear(a.astype(np.float64), w.astype(np.float64))
    got = sts.op_gemm(a, w, cfg, epilogue=epilogue)
    assert rel(got, ref) <= (BF16_TOL if epilogue == 0 else 1e-5)


@pytest.mark.parametrize("cfg,m,split", [("64x256", 64, 4), ("64x256", 8, 8), ("128x128", 130, 2), ("64x128", 33, 3), ("64x128", 64, 8),
                                         ("256x256", 300, 2), ("128x256", 200, 4)])
def test_gemm_split_k(sts, cfg, m, split):
    n, k = 256, 1024
    a = synth.normal_bf16(3, (m, k))
    w = synth.normal_bf16(4, (n, k), 0.05)
    ref = T.op_linear(a.astype(np.float64), w.astype(np.float64))
    assert rel(sts.op_gemm(a, w, cfg, epilogue=1, split_k=split), ref) <= 1e-5


@pytest.mark.parametrize("cfg", ["256x256", "128x128", "64x128", "64x256", "128x256"])
def test_gemm_bf16_store_and_residual(sts, cfg):
    m, n, k = 200, 256, 192
    a = synth.normal_bf16(5, (m, k))
    w = synth.normal_bf16(6, (n, k), 0.05)
    ref = T.op_linear(a.astype(np.float64), w.astype(np.float64))
    got = sts.op_gemm(a, w, cfg, epilogue=0)
    assert rel(got, ref) <= BF16_TOL
    assert np.array_equal(got, synth.to_bf16(got))                   # really bf16 values
    x = np.random.default_rng(7).standard_normal((m, n)).astype(np.float32)
    got2 = sts.op_gemm(a, w, cfg, epilogue=2, c_in=x)
    assert rel(got2, x.astype(np.float64) + ref) <= 1e-5


@pytest.mark.parametrize("cfg,m", [("256x256", 260), ("128x128", 100), ("128x128", 5), ("256x256", 513), ("64x128", 64), ("64x128", 37),
                                   ("64x128", 130)])
def test_gemm_swiglu_epilogue(sts, cfg, m):
    n2, k = 256, 448
    a = synth.normal_bf16(8, (m, k))
    wg = synth.normal_bf16(9, (n2, k), 0.2)
    wu = synth.normal_bf16(10, (n2, k), 0.2)
    a64 = a.astype(np.float64)
    ref = T.silu(T.op_linear(a64, wg.astype(np.float64))) * T.op_linear(a64, wu.astype(np.float64))
    got = sts.op_gemm(a, np.concatenate([wg, wu]), cfg, epilogue=3)
    assert rel(got, ref) <= BF16_TOL


SKINNY = [("64x256s", 256), ("64x320s", 320), ("64x384s", 384), ("64x448s", 448), ("64x512s", 512)]


@pytest.mark.parametrize("cfg,width", SKINNY)
@pytest.mark.parametrize("m,k,split", [(64, 64, 1), (37, 128, 1), (1, 192, 1), (64, 256, 1), (130, 576, 1), (64, 1024, 4), (50, 1088, 3), (8, 2048, 8)])
def test_gemm_skinny_tiles_fp32(sts, cfg, width, m, k, split):
    """The decode tiles (64 rows, 64 columns per wave, weights streamed into registers three K tiles deep): fewer K tiles than
    the pipeline is deep, a K extent that leaves surplus iterations in its last round, rows that end inside a tile and more
    than one tile of rows, slices along K of unequal length."""
    n = 2 * width
    a = synth.normal_bf16(21, (m, k))
    w = synth.normal_bf16(22, (n, k), 0.05)
    ref = T.op_linear(a.astype(np.float64), w.astype(np.float64))
    assert rel(sts.op_gemm(a, w, cfg, epilogue=1, split_k=split), ref) <= 1e-5


@pytest.mark.parametrize("cfg,width", SKINNY)
@pytest.mark.parametrize("m,k", [(64, 448), (29, 128)])
def test_gemm_skinny_tiles_epilogues(sts, cfg, width, m, k):
    n = 2 * width
    a = synth.normal_bf16(23, (m, k))
    a64 = a.astype(np.float64)
    w = synth.normal_bf16(24, (n, k), 0.1)
    ref = T.op_linear(a64, w.astype(np.float64))
    got = sts.op_gemm(a, w, cfg, epilogue=0)
    assert rel(got, ref) <= BF16_TOL and np.array_equal(got, synth.to_bf16(got))
    x = np.random.default_rng(25).standard_normal((m, n)).astype(np.float32)
    assert rel(sts.op_gemm(a, w, cfg, epilogue=2, c_in=x), x.astype(np.float64) + ref) <= 1e-5
    wg, wu = w[:width], w[width:]
    ref3 = T.silu(T.op_linear(a64, wg.astype(np.float64))) * T.op_linear(a64, wu.astype(np.float64))
    assert rel(sts.op_gemm(a, w, cfg, epilogue=3), ref3) <= BF16_TOL


@pytest.mark.parametrize("cfg,m,n,slots", [("128x128", 300, 512, 8), ("128x128", 300, 512, 10), ("128x128", 300, 512, 40),
                                           ("128x128", 300, 512, 16), ("256x256", 513, 512, 4), ("256x256", 513, 512, 15),
                                           ("64x128", 64, 640, 4), ("128x256", 300, 768, 7), ("128x256", 513, 512, 8)])
@pytest.mark.parametrize("epilogue", [0, 1, 2, 3])
def test_gemm_tail_wave_split(sts, cfg, m, n, slots, epilogue):
    """The tiles of the last, partly filled wave of workgroups (Section 2.2.1) are cut along K and
    summed by a second kernel: same results as whole tiles, for every epilogue."""
    if epilogue == 3 and cfg == "128x256":
        pytest.skip("the 128x256 tile has no SwiGLU form (it serves the projections with a residual epilogue)")
    k = 1024
    a = synth.normal_bf16(40, (m, k))
    a64 = a.astype(np.float64)
    if epilogue == 3:
        wg = synth.normal_bf16(41, (n // 2, k), 0.05)
        wu = synth.normal_bf16(42, (n // 2, k), 0.05)
        ref = T.silu(T.op_linear(a64, wg.astype(np.float64))) * T.op_linear(a64, wu.astype(np.float64))
        got = sts.op_gemm(a, np.concatenate([wg, wu]), cfg, epilogue=3, tail_slots=slots)
        assert rel(got, ref) <= BF16_TOL
        return
    w = synth.normal_bf16(43, (n, k), 0.05)
    ref = T.op_linear(a64, w.astype(np.float64))
    if epilogue == 2:
        x = np.random.default_rng(44).standard_normal((m, n)).astype(np.float32)
        got = sts.op_gemm(a, w, cfg, epilogue=2, c_in=x, tail_slots=slots)
        assert rel(got, x.astype(np.float64) + ref) <= 1e-5
    else:
        got = sts.op_gemm(a, w, cfg, epilogue=epilogue, tail_slots=slots)
        assert rel(got, ref) <= (BF16_TOL if epilogue == 0 else 1e-5)


def test_gemm_rejects_bad_shapes(sts):
    a = np.zeros((4, 100), np.float32); w = np.zeros((256, 100), np.float32)
    with pytest.raises(sts.StsError) as e:
        sts.op_gemm(a, w, "128x128")          # K not a multiple of 64
    assert e.value.code == sts.EINVAL
    with pytest.raises(sts.StsError):
        sts.op_gemm(np.zeros((4, 64), np.float32), np.zeros((192, 64), np.float32), "256x256")   # N not a multiple of the tile
    with pytest.raises(sts.StsError) as e:
        sts.op_gemm(np.zeros((4, 64), np.float32), np.zeros((512, 64), np.float32), "64x256", epilogue=3)   # no SwiGLU form of this tile
    assert e.value.code == sts.EINVAL
    with pytest.raises(sts.StsError) as e:
        sts.op_gemm(np.zeros((4, 64), np.float32), np.zeros((512, 64), np.float32), "128x256", epilogue=3)  # nor of this one
    assert e.value.code == sts.EINVAL


@pytest.mark.parametrize("t,prior,nq,nkv,d", [(128, 0, 4, 4, 64), (300, 0, 8, 2, 128), (70, 45, 4, 1, 128), (1, 0, 4, 4, 64),
                                              (200, 330, 4, 4, 64), (129, 16, 8, 2, 128),
                                              (130, 16500, 4, 1, 128),      # context beyond one block-table window (16384 tokens)
                                              (40, 33000, 4, 1, 64)])       # ... beyond two
def test_prefill_attention(sts, t, prior, nq, nkv, d):
    q = synth.normal_bf16(11, (t, nq, d))
    k = synth.normal_bf16(12, (prior + t, nkv, d))
    v = synth.normal_bf16(13, (prior + t, nkv, d))
    ref = T.op_causal_attention(q.astype(np.float64), k.astype(np.float64), v.astype(np.float64), prior)
    n_pages = (prior + t + 15) // 16
    pages = synth.page_permutation(14, n_pages + 5)[:n_pages]
    got = sts.op_attn_prefill(q, k, v, prior, pages, n_pages + 5)
    assert rel(got, ref) <= BF16_TOL
    # page order must not matter at all: same kernel, same tiles, only addresses differ
    got2 = sts.op_attn_prefill(q, k, v, prior, np.arange(n_pages, dtype=np.int32), n_pages + 5)
    assert np.array_equal(got, got2)


@pytest.mark.parametrize("nq,nkv,d,ctx,chunks", [(4, 4, 64, [32, 256, 1, 17, 100], 32), (4, 4, 64, [250, 33], 4),
                                                 (32, 8, 128, [1000, 40, 513, 16], 8), (8, 1, 128, [700], 5),
                                                 (32, 8, 128, [2048, 100], 16), (4, 4, 64, [129, 3], 1),
                                                 (32, 8, 128, [3000, 1025, 64], 64), (8, 1, 128, [1500], 33),
                                                 (16, 2, 128, [600, 31], 8), (4, 1, 64, [1100, 15], 64)])
def test_decode_attention(sts, nq, nkv, d, ctx, chunks):
    """`chunks` = pages per context chunk."""
    n = len(ctx)
    q = synth.normal_bf16(15, (n, nq, d))
    k = synth.normal_bf16(16, (sum(ctx), nkv, d))
    v = synth.normal_bf16(17, (sum(ctx), nkv, d))
    got = sts.op_attn_decode(q, k, v, ctx, chunks)
    off = 0
    for r, c in enumerate(ctx):
        kk, vv = k[off:off + c].astype(np.float64), v[off:off + c].astype(np.float64)
        for h in range(nq):
            ref = T.attend_one(q[r, h].astype(np.float64), kk[:, h // (nq // nkv)], vv[:, h // (nq // nkv)])
            assert rel(got[r, h], ref) <= BF16_TOL, (r, h)
        off += c
