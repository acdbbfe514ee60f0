"""Parity at the benchmark's full size and launch configuration (config 2: one 8B-shaped layer,
2048-token prefill concurrent with 64 decodes at lognormal contexts, permuted pages). At the
split the benchmark times (224 prefill / 32 decode CUs) every one of the 2048 prefill rows and
every one of the 64 decode requests is compared with the oracle; at the other splits a sample of
rows and requests. Further cases at full width: the LM head and greedy sampling at the real
vocabulary of 128256, and one layer of the 70B shape with its real MLP width of 28672.
Tolerance 2e-2 (bf16 path against the fp64 oracle)."""
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


def decode_reference(desc, lw, emb, ctx_len, seed, token):
    """One request of the decode batch through the oracle's layer: its synthetic cached K,V (the
    recipe of the library's random fill) and the new token at position ctx_len."""
    n_pages = (ctx_len + 16) // 16
    kvd = T.PagedKV(1, n_pages, desc.n_kv_heads, 16, desc.head_dim)
    kvd.add_sequence(0, list(range(n_pages)), ctx_len)
    k = synth.kv_values(seed, 0, "k", 0, ctx_len, desc.n_kv_heads, desc.head_dim)
    v = synth.kv_values(seed, 0, "v", 0, ctx_len, desc.n_kv_heads, desc.head_dim)
    for t in range(ctx_len):
        kvd.write(0, 0, t, k[t], v[t])
    return T.layer_chunk(desc, lw, 0, kvd, 0, ctx_len, emb[[token]], np.float64)[0]


@pytest.mark.timeout(900)
def test_every_output_of_the_benchmark_step_at_the_timed_split(case):
    """The step bench.py times (224 / 32 CUs): all 2048 prefill rows -- every tile of every GEMM, the
    cut last wave and its fix-up included -- and all 64 decode requests, against the oracle."""
    wl, desc, w = case
    eng = wl.eng
    wl.reset_contexts()
    eng.set_partition(224, 32)
    pseq = eng.seq_create()
    eng.step_concurrent([pseq], [wl.ptokens], 0, 1, wl.dseqs, wl.dtokens, want_plogits=False, want_dlogits=False, want_dnext=False)
    hp = eng.read_hidden(0, 2048)
    hd = eng.read_hidden(1, 64)
    eng.seq_free(pseq)
    lw = {k: np.asarray(v, np.float64) for k, v in w["layers"][0].items()}
    emb = np.asarray(w["emb"], np.float64)
    kv = T.PagedKV(1, 2048 // 16, desc.n_kv_heads, 16, desc.head_dim)
    kv.add_sequence(0, list(range(2048 // 16)))
    ref = T.layer_chunk(desc, lw, 0, kv, 0, 0, emb[wl.ptokens], np.float64)
    assert ref.shape == hp.shape == (2048, desc.hidden)
    scale = np.abs(ref).max()
    row_err = np.abs(hp - ref).max(axis=1) / scale
    assert row_err.max() <= TOL, (int(row_err.argmax()), float(row_err.max()))
    ctx = [int(c) for c in wl.ctx]
    refd = np.stack([decode_reference(desc, lw, emb, ctx[r], 1000 + r, wl.dtokens[r]) for r in range(64)])
    req_err = np.abs(hd - refd).max(axis=1) / np.abs(refd).max()
    assert req_err.max() <= TOL, (int(req_err.argmax()), float(req_err.max()))


@pytest.mark.parametrize("split", [(128, 128), (256, 256), (32, 224)])
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
        refd = decode_reference(desc, lw, emb, ctx[r], 1000 + r, wl.dtokens[r])
        assert rel(hd[r], refd) <= TOL, (r, ctx[r])


@pytest.mark.timeout(900)
def test_lm_head_and_greedy_sampling_at_the_real_vocabulary():
    """Final norm, LM head (N = 128256) and greedy sampling of a decode step: one 8B-shaped layer,
    64 requests, weights loaded from the host. Logits of every request against the oracle, and the
    sampled token: it is the argmax of the device's own logits (lowest index on ties), and its
    reference logit is within the tolerance of the reference maximum."""
    from paper_2504_19516_amd import sts
    sts.lib()
    desc = synth.llama8b_model(n_layers=1, vocab=128256)
    w = synth.normal_weights(desc, 31, emb_block_rows=1024)
    ctx = [int(c) for c in synth.lognormal_lengths(4, 64, 200, 0.8, 1500)]
    pages = sum((c + 1 + 15) // 16 for c in ctx)
    eng = sts.Engine(desc, weight_seed=0, init_weights=False, kv_pool_pages=pages + 16, max_prefill_tokens=128, max_prefill_seqs=1,
                     max_decode_batch=64, max_seqs=70, max_pages_per_seq=(1500 + 32) // 16)
    eng.load_all(w)
    dseqs = []
    for i, c in enumerate(ctx):
        s_ = eng.seq_create()
        eng.kv_fill_random(s_, c, 3000 + i)
        dseqs.append(s_)
    dtok = synth.tokens(23, 64, desc.vocab)
    eng.set_partition(192, 64)
    got, nxt = eng.decode_step(dseqs, dtok)
    eng.close()
    assert got.shape == (64, 128256) and np.isfinite(got).all()
    lw = {k: np.asarray(v, np.float64) for k, v in w["layers"][0].items()}
    emb = np.asarray(w["emb"][:1024], np.float64)
    x = np.stack([decode_reference(desc, lw, emb, ctx[r], 3000 + r, int(dtok[r]) % 1024) for r in range(64)])
    del lw
    lm = np.asarray(w["lm"], np.float64)
    ref = (lm @ T.rmsnorm(x, np.asarray(w["gf"], np.float64), desc.rms_eps).T).T       # Oracle.logits, all requests at once
    assert rel(got, ref) <= TOL
    scale = np.abs(ref).max()
    for r in range(64):
        assert nxt[r] == T.greedy(got[r]), r
        assert ref[r, nxt[r]] >= ref[r].max() - TOL * scale, r


@pytest.mark.timeout(900)
def test_sampled_outputs_of_a_70b_shaped_layer():
    """One layer of the config-5 shape at its real widths (hidden 8192, 64 query heads on 8 KV heads of
    128: groups of 8, MLP 28672: the N = 57344 gate/up and K = 28672 down products), weights loaded
    from the host: a 700-token prefill beside the decode of 12 requests, sampled rows and requests
    against the oracle."""
    from paper_2504_19516_amd import sts
    sts.lib()
    desc = synth.llama70b_model(n_layers=1, vocab=1024)
    ctx = [int(c) for c in synth.lognormal_lengths(9, 12, 900, 0.8, 3000)]
    pages = sum((c + 32 + 15) // 16 for c in ctx) + 700 // 16 + 8
    eng = sts.Engine(desc, weight_seed=0, init_weights=False, kv_pool_pages=pages + 16, max_prefill_tokens=1024, max_prefill_seqs=1,
                     max_decode_batch=16, max_seqs=20, max_pages_per_seq=(3000 + 64) // 16)
    w = synth.normal_weights(desc, 77)
    eng.load_all(w)
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
    rows = [0, 127, 128, 333, 511, 512, 699]
    kv = T.PagedKV(1, 700 // 16 + 1, desc.n_kv_heads, 16, desc.head_dim)
    kv.add_sequence(0, list(range(700 // 16 + 1)))
    ref = T.layer_chunk(desc, lw, 0, kv, 0, 0, emb[ptok], np.float64, rows=rows)
    assert rel(hp[rows], ref) <= TOL
    for r in sorted({int(np.argmin(ctx)), int(np.argmax(ctx)), 5}):
        refd = decode_reference(desc, lw, emb, ctx[r], 2000 + r, dtok[r])
        assert rel(hd[r], refd) <= TOL, (r, ctx[r])
