"""Oracle, part 1: the transformer step over a paged KV cache.  TEST INFRASTRUCTURE.

The paper describes the model only as stacked blocks of QKV projection, self
attention, output projection and MLP, with element-wise operations in between
(Section 2.1), prefill building a KV cache that decode then reads (Section 2.1), the
cache being paged and shared by both phases (Section 3.5.1). The concrete block used
here is the Llama-shaped one the workload configurations name: RMSNorm, rotary
position embedding, grouped-query causal attention, SwiGLU MLP, no biases.

Everything is written out directly in numpy, in float64 unless `dtype` says
otherwise: no blocking, no fusion, no online softmax. A matmul is a library step.

Readings where the paper is silent (all listed in the design document):
  * rotary pairing is half-split: element i pairs with i + d/2, angle pos * theta^(-2i/d)
  * RMSNorm: x / sqrt(mean(x^2) + eps) * gain
  * softmax scale 1/sqrt(d); token at absolute position t attends to positions 0..t
  * query head h reads KV head h // (n_q / n_kv)
  * token t of a sequence lives in page block_table[t // page_tokens], slot t % page_tokens
  * a chunk appended after p cached tokens has positions p, p+1, ...
  * running layers [a,b) then [b,c) equals running [a,c): the hidden state is kept
"""
from __future__ import annotations

import numpy as np


class PagedKV:
    """K and V of every layer in fixed-size pages addressed through per-sequence block tables."""

    def __init__(self, n_layers, n_pages, n_kv_heads, page_tokens, head_dim, dtype=np.float64):
        shape = (n_layers, n_pages, page_tokens, n_kv_heads, head_dim)
        self.k = np.zeros(shape, dtype=dtype)
        self.v = np.zeros(shape, dtype=dtype)
        self.page_tokens = page_tokens
        self.block_table: dict[int, list[int]] = {}
        self.length: dict[int, int] = {}

    def add_sequence(self, seq: int, pages: list[int], length: int = 0):
        self.block_table[seq] = list(pages)
        self.length[seq] = length

    def write(self, layer, seq, pos, k, v):
        """Store K,V ([n_kv, d] each) of the token at logical position `pos`."""
        page = self.block_table[seq][pos // self.page_tokens]
        slot = pos % self.page_tokens
        self.k[layer, page, slot] = k
        self.v[layer, page, slot] = v

    def gather(self, layer, seq, n):
        """K,V of logical positions 0..n-1, each [n, n_kv, d]."""
        pt = self.page_tokens
        ks = np.stack([self.k[layer, self.block_table[seq][t // pt], t % pt] for t in range(n)])
        vs = np.stack([self.v[layer, self.block_table[seq][t // pt], t % pt] for t in range(n)])
        return ks, vs


def rmsnorm(x, gain, eps):
    """x: [..., h]."""
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * gain


def rope(x, pos, theta):
    """Rotate x [n_heads, d] for absolute position `pos` (half-split pairing)."""
    d = x.shape[-1]
    half = d // 2
    i = np.arange(half, dtype=x.dtype)
    ang = pos * theta ** (-2.0 * i / d)
    c, s = np.cos(ang), np.sin(ang)
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def attend_one(q, ks, vs):
    """One query vector q [d] against keys/values [n, d]: softmax(q.k / sqrt(d)) v."""
    s = ks @ q / np.sqrt(q.shape[0])
    p = np.exp(s - np.max(s))
    return (p / np.sum(p)) @ vs


def layer_chunk(desc, lw, layer, kv: PagedKV, seq, p, x, dtype, rows=None):
    """One transformer block for a chunk of n tokens at absolute positions p..p+n-1 of `seq`.

    Writes the chunk's K,V into the cache; token i then attends to positions 0..p+i.
    x: [n, h] residual-stream input; returns the block's output [n, h]. A decode step is
    the case n = 1. With `rows` (indices into the chunk) every token's K,V is still
    computed and cached but only those rows are carried through attention, output
    projection and MLP, and only they are returned, [len(rows), h].
    """
    nq, nkv, d = desc.n_q_heads, desc.n_kv_heads, desc.head_dim
    n = x.shape[0]
    a = rmsnorm(x, lw["g1"], desc.rms_eps)
    k = (a @ lw["wk"].T).reshape(n, nkv, d)
    v = (a @ lw["wv"].T).reshape(n, nkv, d)
    for i in range(n):
        kv.write(layer, seq, p + i, rope(k[i], p + i, desc.rope_theta), v[i])
    rows = list(range(n)) if rows is None else list(rows)
    x = x[rows]
    q = (a[rows] @ lw["wq"].T).reshape(len(rows), nq, d)
    ks, vs = kv.gather(layer, seq, p + n)
    group = nq // nkv
    o = np.empty((len(rows), nq, d), dtype=dtype)
    for j, i in enumerate(rows):
        qi = rope(q[j], p + i, desc.rope_theta)
        for h in range(nq):
            o[j, h] = attend_one(qi[h], ks[:p + i + 1, h // group], vs[:p + i + 1, h // group])
    x = x + o.reshape(len(rows), nq * d) @ lw["wo"].T
    m = rmsnorm(x, lw["g2"], desc.rms_eps)
    x = x + (silu(m @ lw["wg"].T) * (m @ lw["wu"].T)) @ lw["wd"].T
    return x


class Oracle:
    """Holds weights (cast to `dtype`) and a paged KV cache; runs prefill chunks and decode steps."""

    def __init__(self, desc, weights, n_pages, dtype=np.float64):
        self.desc = desc
        self.dtype = dtype
        cast = lambda t: np.asarray(t, dtype=dtype)
        self.w = {"emb": cast(weights["emb"]), "lm": cast(weights["lm"]), "gf": cast(weights["gf"]),
                  "layers": [{k: cast(v) for k, v in lw.items()} for lw in weights["layers"]]}
        self.kv = PagedKV(len(self.w["layers"]), n_pages, desc.n_kv_heads, desc.page_tokens,
                          desc.head_dim, dtype)
        self._hidden: dict[int, np.ndarray] = {}     # seq -> [n_new, h] between layer slices
        self._next_layer: dict[int, int] = {}

    # -- prefill ---------------------------------------------------------------------------
    def prefill_append(self, seq, tokens, layer_begin=0, layer_end=None):
        """Append `tokens` after the sequence's cached context, running layers
        [layer_begin, layer_end). Layer slices must be issued in order. When the last
        layer has run, the sequence length grows by len(tokens) and the logits [vocab]
        of the last new token are returned; otherwise None."""
        n_layers = len(self.w["layers"])
        layer_end = n_layers if layer_end is None else layer_end
        p = self.kv.length[seq]
        if layer_begin == 0:
            self._hidden[seq] = self.w["emb"][np.asarray(tokens)].copy()
            self._next_layer[seq] = 0
        assert self._next_layer.get(seq) == layer_begin, "layer slices out of order"
        x = self._hidden[seq]
        for l in range(layer_begin, layer_end):
            lw = self.w["layers"][l]
            x = layer_chunk(self.desc, lw, l, self.kv, seq, p, x, self.dtype)
        self._hidden[seq] = x
        self._next_layer[seq] = layer_end
        if layer_end < n_layers:
            return None
        self.kv.length[seq] = p + len(tokens)
        del self._hidden[seq], self._next_layer[seq]
        self.last_hidden = x
        return self.logits(x[-1])

    # -- decode ----------------------------------------------------------------------------
    def decode_step(self, seqs, in_tokens):
        """One decode step: request r feeds `in_tokens[r]` at position length[r], attends
        to positions 0..length[r] and gets logits [vocab]. Returns [n, vocab]."""
        out = []
        for seq, tok in zip(seqs, in_tokens):
            pos = self.kv.length[seq]
            x = self.w["emb"][tok][None, :].copy()
            for l, lw in enumerate(self.w["layers"]):
                x = layer_chunk(self.desc, lw, l, self.kv, seq, pos, x, self.dtype)
            self.kv.length[seq] = pos + 1
            out.append(self.logits(x[0]))
        return np.stack(out)

    def logits(self, x):
        return self.w["lm"] @ rmsnorm(x, self.w["gf"], self.desc.rms_eps)


def greedy(logits):
    """argmax with the lowest index winning ties."""
    return int(np.argmax(logits))


# ---- single operations, for per-kernel parity (inputs are whatever the caller rounded) ----
def op_linear(x, w):
    """x [m, k] times w [n, k] transposed."""
    return x @ w.T


def op_causal_attention(q, k, v, prior):
    """q [t, nq, d]; k, v [prior + t, nkv, d]; query i sits at position prior + i."""
    t, nq, d = q.shape
    group = nq // k.shape[1]
    o = np.empty_like(q)
    for i in range(t):
        for h in range(nq):
            o[i, h] = attend_one(q[i, h], k[:prior + i + 1, h // group], v[:prior + i + 1, h // group])
    return o
