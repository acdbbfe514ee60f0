"""Parity at the benchmark's full size and launch configuration (config 2: one 8B-shaped layer,
2048-token prefill concurrent with 64 decodes at lognormal contexts, permuted pages), on
sampled outputs the oracle can compute one by one: a few prefill rows and a few decode requests
of the layer's output hidden state. Tolerance 2e-2 (bf16 path against the fp64 oracle)."""
import numpy as np
import pytest

from oracle import transformer as T
from paper_2504_19516_amd import synth

pytestmark = pytest.mark.gpu
TOL = 2e-2


def rel(a, b):
    return float(np.abs(np.asarray(a, np.float64) - np.asarray(b, np.float64)).max() / np.abs(b).max())


@pytest.fixture(scope="module")
def case():
    import bench
    from paper_2504_19516_amd import sts
    sts.lib()
    wl = bench.Workload(sts)
    desc = wl.desc
    w = synth.make_weights(desc, 1234)              # bf16 model: the values the device generated
    yield wl, desc, w
    wl.eng.close()


def test_weights_match_generator_at_full_size(case):
    wl, desc, w = case
    for name in ("wq", "wd", "wg"):
        got = wl.eng.read_weights(0, name, desc.shape(name))
        assert np.array_equal(got, w["layers"][0][name]), name


@pytest.mark.parametrize("split", [(224, 32), (128, 128), (256, 256)])
def test_sampled_outputs_of_the_benchmark_step(case, split):
    wl, desc, w = case
    eng = wl.eng
    wl.reset_contexts()
    eng.set_partition(*split)
    pseq = eng.seq_create()
    eng.step_concurrent([pseq], [wl.ptokens], 0, 1, wl.dseqs, wl.dtokens, want_plogits=False, want_dlogits=False, want_dnext=False)
    hp = eng.read_hidden(0, 2048)
    hd = eng.read_hidden(1, 64)
    eng.seq_free(pseq)
    assert np.isfinite(hp).all() and np.isfinite(hd).all()

    lw = {k: np.asarray(v, np.float64) for k, v in w["layers"][0].items()}
    emb = np.asarray(w["emb"], np.float64)
    # ---- prefill: K,V of all 2048 tokens, then three sampled rows through the whole layer
    rows = [0, 1000, 2047]
    kv = T.PagedKV(1, 2048 // 16, desc.n_kv_heads, 16, desc.head_dim)
    kv.add_sequence(0, list(range(2048 // 16)))
    ref = T.layer_chunk(desc, lw, 0, kv, 0, 0, emb[wl.ptokens], np.float64, rows=rows)
    assert rel(hp[rows], ref) <= TOL
    # ---- decode: the shortest, the longest and one other request
    ctx = [int(c) for c in wl.ctx]
    picks = sorted({int(np.argmin(ctx)), int(np.argmax(ctx)), 7})
    for r in picks:
        c = ctx[r]
        n_pages = (c + 16) // 16
        kvd = T.PagedKV(1, n_pages, desc.n_kv_heads, 16, desc.head_dim)
        kvd.add_sequence(0, list(range(n_pages)), c)
        k = synth.kv_values(1000 + r, 0, "k", 0, c, desc.n_kv_heads, desc.head_dim)
        v = synth.kv_values(1000 + r, 0, "v", 0, c, desc.n_kv_heads, desc.head_dim)
        for t in range(c):
            kvd.write(0, 0, t, k[t], v[t])
        refd = T.layer_chunk(desc, lw, 0, kvd, 0, c, emb[[wl.dtokens[r]]], np.float64)
        assert rel(hd[r], refd[0]) <= TOL, (r, c)


def test_sampled_outputs_of_a_70b_shaped_layer():
    """The wide shape of config 5 (hidden 8192, 64 query heads on 8 KV heads of 128: groups of 8) on
    one layer, MLP cut to a quarter to keep the oracle's weights small: a 700-token prefill beside
    the decode of 12 requests, sampled rows against the oracle. Covers the K = 8192 GEMM shapes, the
    group-of-8 decode attention and chunked contexts at this width."""
    from paper_2504_19516_amd import sts
    sts.lib()
    desc = synth.ModelDesc(1, 8192, 64, 8, 128, 7168, 1024, 16, 5.0e5, 1.0e-5, "bf16")
    ctx = [int(c) for c in synth.lognormal_lengths(9, 12, 900, 0.8, 3000)]
    pages = sum((c + 32 + 15) // 16 for c in ctx) + 700 // 16 + 8
    eng = sts.Engine(desc, weight_seed=77, init_weights=True, kv_pool_pages=pages + 16, max_prefill_tokens=1024, max_prefill_seqs=1,
                     max_decode_batch=16, max_seqs=20, max_pages_per_seq=(3000 + 64) // 16)
    w = synth.make_weights(desc, 77)
    dseqs = []
    for i, c in enumerate(ctx):
        s_ = eng.seq_create()
        eng.kv_fill_random(s_, c, 2000 + i)
        eng.seq_reserve(s_, c + 16)
        dseqs.append(s_)
    ptok = synth.tokens(21, 700, desc.vocab)
    dtok = synth.tokens(22, len(ctx), desc.vocab)
    eng.set_partition(192, 64)
    pseq = eng.seq_create()
    eng.step_concurrent([pseq], [ptok], 0, 1, dseqs, dtok, want_plogits=False, want_dlogits=False, want_dnext=False)
    hp = eng.read_hidden(0, 700)
    hd = eng.read_hidden(1, len(ctx))
    eng.close()
    assert np.isfinite(hp).all() and np.isfinite(hd).all()
    lw = {k: np.asarray(v, np.float64) for k, v in w["layers"][0].items()}
    emb = np.asarray(w["emb"], np.float64)
    rows = [0, 333, 699]
    kv = T.PagedKV(1, 700 // 16 + 1, desc.n_kv_heads, 16, desc.head_dim)
    kv.add_sequence(0, list(range(700 // 16 + 1)))
    ref = T.layer_chunk(desc, lw, 0, kv, 0, 0, emb[ptok], np.float64, rows=rows)
    assert rel(hp[rows], ref) <= TOL
    for r in sorted({int(np.argmin(ctx)), int(np.argmax(ctx)), 5}):
        c = ctx[r]
        n_pages = (c + 16) // 16
        kvd = T.PagedKV(1, n_pages, desc.n_kv_heads, 16, desc.head_dim)
        kvd.add_sequence(0, list(range(n_pages)), c)
        k = synth.kv_values(2000 + r, 0, "k", 0, c, desc.n_kv_heads, desc.head_dim)
        v = synth.kv_values(2000 + r, 0, "v", 0, c, desc.n_kv_heads, desc.head_dim)
        for t in range(c):
            kvd.write(0, 0, t, k[t], v[t])
        refd = T.layer_chunk(desc, lw, 0, kvd, 0, c, emb[[dtok[r]]], np.float64)
        assert rel(hd[r], refd[0]) <= TOL, (r, c)
