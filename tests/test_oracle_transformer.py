"""Pins of the transformer oracle against things other than itself: library routines,
closed forms, invariants and a brute-force formulation."""
import numpy as np
import pytest
import torch

from oracle import transformer as T
from paper_2504_19516_amd import synth


def small_desc(**kw):
    d = dict(n_layers=2, hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=16, mlp=96, vocab=50,
             page_tokens=4, rope_theta=1.0e4, rms_eps=1e-5, dtype="fp32")
    d.update(kw)
    return synth.ModelDesc(**d)


def make(desc, seed=5, n_pages=32, dtype=np.float64, scale=8.0):
    w = synth.make_weights(desc, seed)
    # N(0, 0.02) at hidden 64 gives nearly uniform attention; scale up so every term matters
    for lw in w["layers"]:
        for k in synth.SLOT:
            lw[k] = lw[k] * np.float32(scale)
    w["emb"] = w["emb"] * np.float32(40.0)
    return T.Oracle(desc, w, n_pages, dtype), w


# ------------------------------------------------------------------ element-wise closed forms
def test_rmsnorm_matches_library_routine():
    x = np.random.default_rng(0).standard_normal((5, 32))
    g = np.random.default_rng(1).standard_normal(32)
    ref = torch.nn.functional.rms_norm(torch.tensor(x), (32,), torch.tensor(g), 1e-5).numpy()
    assert np.allclose(T.rmsnorm(x, g, 1e-5), ref, rtol=1e-12, atol=1e-12)


def test_silu_matches_library_routine():
    x = np.linspace(-8, 8, 101)
    assert np.allclose(T.silu(x), torch.nn.functional.silu(torch.tensor(x)).numpy(), rtol=1e-12)


def test_rope_hand_values_and_pairing():
    # d = 4, theta = 1e4, pos = 3: pair (0,2) turns by 3 rad, pair (1,3) by 3 * 1e4^(-1/2) = 0.03 rad
    x = np.array([[1.0, 2.0, 3.0, 4.0]])
    y = T.rope(x, 3, 1.0e4)[0]
    c0, s0, c1, s1 = np.cos(3.0), np.sin(3.0), np.cos(0.03), np.sin(0.03)
    assert np.allclose(y, [1 * c0 - 3 * s0, 2 * c1 - 4 * s1, 1 * s0 + 3 * c0, 2 * s1 + 4 * c1], atol=1e-14)
    assert np.array_equal(T.rope(x, 0, 1.0e4), x)          # position 0 is the identity


def test_rope_preserves_norm_and_is_relative():
    rng = np.random.default_rng(2)
    q, k = rng.standard_normal((1, 32)), rng.standard_normal((1, 32))
    assert np.allclose(np.linalg.norm(T.rope(q, 17, 5e5)), np.linalg.norm(q))
    d1 = T.rope(q, 40, 5e5)[0] @ T.rope(k, 33, 5e5)[0]
    d2 = T.rope(q, 107, 5e5)[0] @ T.rope(k, 100, 5e5)[0]
    assert np.allclose(d1, d2, rtol=1e-10)
    assert not np.allclose(d1, T.rope(q, 40, 5e5)[0] @ T.rope(k, 30, 5e5)[0])


# ------------------------------------------------------------------ attention
def brute_force_attention(q, k, v, prior):
    """Explicit score matrix with a -inf mask above the causal diagonal."""
    t, nq, d = q.shape
    n, nkv, _ = k.shape
    out = np.zeros_like(q)
    for h in range(nq):
        kk, vv = k[:, h // (nq // nkv)], v[:, h // (nq // nkv)]
        s = q[:, h] @ kk.T / np.sqrt(d)                               # [t, n]
        mask = np.arange(n)[None, :] > (prior + np.arange(t))[:, None]
        s = np.where(mask, -np.inf, s)
        e = np.exp(s - s.max(axis=1, keepdims=True))
        out[:, h] = (e / e.sum(axis=1, keepdims=True)) @ vv
    return out


@pytest.mark.parametrize("prior", [0, 5])
def test_causal_attention_equals_brute_force_and_sdpa(prior):
    rng = np.random.default_rng(3)
    t, nq, nkv, d = 7, 4, 2, 8
    q = rng.standard_normal((t, nq, d)) * 2
    k = rng.standard_normal((prior + t, nkv, d)) * 2
    v = rng.standard_normal((prior + t, nkv, d))
    got = T.op_causal_attention(q, k, v, prior)
    assert np.allclose(got, brute_force_attention(q, k, v, prior), rtol=1e-12, atol=1e-13)
    if prior == 0:   # library routine: torch's scaled_dot_product_attention with a causal mask
        tq = torch.tensor(q).permute(1, 0, 2)[None]
        tk = torch.tensor(np.repeat(k, nq // nkv, axis=1)).permute(1, 0, 2)[None]
        tv = torch.tensor(np.repeat(v, nq // nkv, axis=1)).permute(1, 0, 2)[None]
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0]
        assert np.allclose(got, ref.permute(1, 0, 2).numpy(), rtol=1e-10, atol=1e-12)


def test_zero_query_gives_running_mean_of_values():
    rng = np.random.default_rng(4)
    v = rng.standard_normal((9, 1, 4))
    k = rng.standard_normal((9, 1, 4))
    out = T.op_causal_attention(np.zeros((9, 2, 4)), k, v, 0)
    want = np.cumsum(v[:, 0], axis=0) / np.arange(1, 10)[:, None]
    assert np.allclose(out[:, 0], want) and np.allclose(out[:, 1], want)


# ------------------------------------------------------------------ whole model vs an independent library model
def hf_llama(desc, w):
    from transformers import LlamaConfig, LlamaForCausalLM
    cfg = LlamaConfig(vocab_size=desc.vocab, hidden_size=desc.hidden, intermediate_size=desc.mlp,
                      num_hidden_layers=desc.n_layers, num_attention_heads=desc.n_q_heads,
                      num_key_value_heads=desc.n_kv_heads, head_dim=desc.head_dim,
                      rms_norm_eps=desc.rms_eps, rope_theta=desc.rope_theta, attention_bias=False,
                      mlp_bias=False, tie_word_embeddings=False, max_position_embeddings=4096,
                      attn_implementation="eager")
    m = LlamaForCausalLM(cfg).double().eval()
    sd = {"model.embed_tokens.weight": w["emb"], "lm_head.weight": w["lm"], "model.norm.weight": w["gf"]}
    names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj",
             "wo": "self_attn.o_proj", "wg": "mlp.gate_proj", "wu": "mlp.up_proj", "wd": "mlp.down_proj"}
    for l, lw in enumerate(w["layers"]):
        for k, n in names.items():
            sd[f"model.layers.{l}.{n}.weight"] = lw[k]
        sd[f"model.layers.{l}.input_layernorm.weight"] = lw["g1"]
        sd[f"model.layers.{l}.post_attention_layernorm.weight"] = lw["g2"]
    m.load_state_dict({k: torch.tensor(np.asarray(v, dtype=np.float64)) for k, v in sd.items()}, strict=True)
    return m


def test_prefill_logits_match_library_llama():
    desc = small_desc()
    orc, w = make(desc)
    # non-trivial gains so a dropped gain would show
    rng = np.random.default_rng(6)
    w["gf"] = (1 + 0.3 * rng.standard_normal(desc.hidden)).astype(np.float32)
    for lw in w["layers"]:
        lw["g1"] = (1 + 0.3 * rng.standard_normal(desc.hidden)).astype(np.float32)
        lw["g2"] = (1 + 0.3 * rng.standard_normal(desc.hidden)).astype(np.float32)
    orc = T.Oracle(desc, w, 32)
    toks = synth.tokens(1, 13, desc.vocab)
    orc.kv.add_sequence(0, [7, 2, 9, 4])
    got = orc.prefill_append(0, toks)
    with torch.no_grad():
        ref = hf_llama(desc, w)(torch.tensor(toks[None].astype(np.int64))).logits[0].numpy()
    assert np.abs(ref[-1]).max() > 0.1
    # the library computes its rotary angles in float32 even in a float64 model: agreement is ~1e-7
    assert np.allclose(got, ref[-1], rtol=1e-5, atol=2e-6)
    # the tiny parity configuration's own shape (head_dim 64, MHA) as well
    desc2 = synth.tiny_model()
    w2 = synth.make_weights(desc2, 1234)
    o2 = T.Oracle(desc2, w2, 8)
    o2.kv.add_sequence(0, [3, 1])
    t2 = synth.tokens(2, 20, desc2.vocab)
    with torch.no_grad():
        r2 = hf_llama(desc2, w2)(torch.tensor(t2[None].astype(np.int64))).logits[0, -1].numpy()
    assert np.abs(r2).max() > 0.01
    assert np.allclose(o2.prefill_append(0, t2), r2, rtol=1e-5, atol=1e-7)


# ------------------------------------------------------------------ invariants of the paged step
def test_decode_equals_row_of_full_recompute():
    desc = small_desc()
    toks = synth.tokens(3, 12, desc.vocab)
    a, _ = make(desc)
    a.kv.add_sequence(0, [0, 1, 2])
    a.prefill_append(0, toks[:11])
    dec = a.decode_step([0], [toks[11]])[0]
    b, _ = make(desc)
    b.kv.add_sequence(0, [0, 1, 2])
    full = b.prefill_append(0, toks)
    assert np.allclose(dec, full, rtol=1e-10, atol=1e-12)
    assert a.kv.length[0] == 12


def test_page_order_does_not_change_result_bitwise():
    desc = small_desc()
    toks = synth.tokens(4, 14, desc.vocab)
    outs = []
    for pages in ([0, 1, 2, 3], [11, 3, 30, 7]):
        o, _ = make(desc)
        o.kv.add_sequence(5, pages)
        o.prefill_append(5, toks[:10])
        outs.append(o.decode_step([5], [toks[10]])[0])
    assert np.array_equal(outs[0], outs[1])


def test_chunked_and_layer_sliced_prefill_equal_whole():
    desc = small_desc()
    toks = synth.tokens(5, 15, desc.vocab)
    whole, _ = make(desc)
    whole.kv.add_sequence(0, [0, 1, 2, 3])
    ref = whole.prefill_append(0, toks)
    ch, _ = make(desc)
    ch.kv.add_sequence(0, [0, 1, 2, 3])
    assert ch.prefill_append(0, toks[:6]) is not None
    got = ch.prefill_append(0, toks[6:])
    assert np.allclose(got, ref, rtol=1e-10, atol=1e-12)
    sl, _ = make(desc)
    sl.kv.add_sequence(0, [0, 1, 2, 3])
    assert sl.prefill_append(0, toks, 0, 1) is None
    got2 = sl.prefill_append(0, toks, 1, 2)
    assert np.array_equal(got2, ref)
    with pytest.raises(AssertionError):
        sl2, _ = make(desc)
        sl2.kv.add_sequence(0, [0, 1, 2, 3])
        sl2.prefill_append(0, toks, 1, 2)


def test_row_subset_equals_rows_of_full_layer():
    desc = small_desc()
    o1, w = make(desc)
    o2, _ = make(desc)
    x = np.random.default_rng(7).standard_normal((9, desc.hidden))
    for o in (o1, o2):
        o.kv.add_sequence(0, [4, 5, 6])
    full = T.layer_chunk(desc, o1.w["layers"][0], 0, o1.kv, 0, 0, x, np.float64)
    part = T.layer_chunk(desc, o2.w["layers"][0], 0, o2.kv, 0, 0, x, np.float64, rows=[2, 8])
    assert np.array_equal(part, full[[2, 8]])
    assert np.array_equal(o1.kv.k, o2.kv.k) and np.array_equal(o1.kv.v, o2.kv.v)


def test_fp32_mode_agrees_with_fp64():
    desc = small_desc()
    toks = synth.tokens(6, 12, desc.vocab)
    res = []
    for dt in (np.float64, np.float32):
        o, _ = make(desc, dtype=dt)
        o.kv.add_sequence(0, [0, 1, 2])
        res.append(o.prefill_append(0, toks))
    assert res[1].dtype == np.float32
    assert np.abs(res[0] - res[1]).max() / np.abs(res[0]).max() < 1e-5


def test_greedy_takes_lowest_index_on_ties():
    assert T.greedy(np.array([1.0, 3.0, 3.0, 2.0])) == 1


# ------------------------------------------------------------------ the input generator itself
def test_weight_generator_statistics_and_slicing():
    w = synth.weight_slice(1234, 17, 0, 200000, False)
    assert abs(float(w.mean())) < 2e-4 and abs(float(w.std()) - 0.02) < 2e-4
    assert np.array_equal(synth.weight_slice(1234, 17, 5000, 100, False), w[5000:5100])
    assert not np.array_equal(synth.weight_slice(1234, 18, 0, 100, False), w[:100])
    b = synth.weight_slice(1234, 17, 0, 1000, True)
    assert np.all((b.view(np.uint32) & 0xFFFF) == 0) and np.abs(b - w[:1000]).max() <= 0.02 * 6 * 2 ** -8


def test_bf16_rounding_ties_to_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7], dtype=np.float32)
    assert np.array_equal(synth.to_bf16(x), np.array([1.0, 1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7], dtype=np.float32))
    ref = torch.tensor(np.linspace(-3, 3, 1001, dtype=np.float32)).to(torch.bfloat16).float().numpy()
    assert np.array_equal(synth.to_bf16(np.linspace(-3, 3, 1001, dtype=np.float32)), ref)
