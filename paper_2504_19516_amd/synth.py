"""Seeded synthetic inputs: model shapes, weights, tokens, context lengths, page
permutations and arrival traces.

This module serves the CPU oracle's tests and the GPU path's tests alike. It holds
none of the serving method's arithmetic: no transformer math, no latency model, no
scheduling. It must import neither `oracle` nor the HIP binding.

Weight specification (both the numpy code here and the on-device generator in the
HIP library implement it, independently, and must agree bit for bit):

    mix(z):  z += 0x9E3779B97F4A7C15
             z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9
             z = (z ^ (z >> 27)) * 0x94D049BB133111EB
             z ^= z >> 31                                   (all mod 2^64)
    base(seed, tensor_id) = mix(seed ^ mix(tensor_id))
    r_j(i) = mix(base ^ (4*i + j)),  j = 0, 1, 2            (i = flat element index)
    S = sum of the twelve 16-bit fields of r_0, r_1, r_2    (0 .. 786420)
    w = float32(S - 393210) * float32(0.02) * 2^-16

S - 393210 has mean 0 and standard deviation sqrt(65536^2 - 1), so w is a
twelve-term Irwin-Hall approximation of N(0, 0.02) with tails cut at +-6 sigma;
every operation is an integer operation or a single fp32 multiply, which is what
makes the two implementations agree exactly. Element index i is the row-major
index in the logical [out_features, in_features] weight. When the model's dtype is
bf16 the value is then rounded to bf16 (round to nearest even).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, asdict

import numpy as np

U64 = np.uint64
_GOLD = U64(0x9E3779B97F4A7C15)
_M1 = U64(0xBF58476D1CE4E5B9)
_M2 = U64(0x94D049BB133111EB)

# tensor ids: globals, then (layer + 1) * 16 + slot
TID_EMB, TID_LM = 0, 1
SLOT = {"wq": 0, "wk": 1, "wv": 2, "wo": 3, "wg": 4, "wu": 5, "wd": 6}


def tensor_id(name: str, layer: int | None = None) -> int:
    if name == "emb":
        return TID_EMB
    if name == "lm":
        return TID_LM
    return (layer + 1) * 16 + SLOT[name]


@dataclass(frozen=True)
class ModelDesc:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    mlp: int
    vocab: int
    page_tokens: int = 16
    rope_theta: float = 1.0e4
    rms_eps: float = 1.0e-5
    dtype: str = "bf16"          # "fp32": weights kept as generated; "bf16": rounded to bf16

    def shape(self, name: str) -> tuple[int, int]:
        qd, kvd = self.n_q_heads * self.head_dim, self.n_kv_heads * self.head_dim
        return {"emb": (self.vocab, self.hidden), "lm": (self.vocab, self.hidden),
                "wq": (qd, self.hidden), "wk": (kvd, self.hidden), "wv": (kvd, self.hidden),
                "wo": (self.hidden, qd), "wg": (self.mlp, self.hidden),
                "wu": (self.mlp, self.hidden), "wd": (self.hidden, self.mlp)}[name]

    def as_dict(self) -> dict:
        return asdict(self)


def tiny_model(dtype: str = "fp32") -> ModelDesc:
    """The small parity configuration: 2 layers, hidden 256, 4 heads x 64, MLP 1024."""
    return ModelDesc(2, 256, 4, 4, 64, 1024, 1024, 16, 1.0e4, 1.0e-5, dtype)


def llama8b_model(n_layers: int = 32, vocab: int = 128256) -> ModelDesc:
    return ModelDesc(n_layers, 4096, 32, 8, 128, 14336, vocab, 16, 5.0e5, 1.0e-5, "bf16")


def llama70b_model(n_layers: int = 80, vocab: int = 128256) -> ModelDesc:
    return ModelDesc(n_layers, 8192, 64, 8, 128, 28672, vocab, 16, 5.0e5, 1.0e-5, "bf16")


# ----------------------------------------------------------------------------- weights
def _mix(z: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = z + _GOLD
        z = (z ^ (z >> U64(30))) * _M1
        z = (z ^ (z >> U64(27))) * _M2
        return z ^ (z >> U64(31))


def _mix_scalar(z: int) -> int:
    m = (1 << 64) - 1
    z = (z + 0x9E3779B97F4A7C15) & m
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & m
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & m
    return z ^ (z >> 31)


def to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + (np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """The 16-bit patterns of bf16-representable fp32 values."""
    return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bf16_from_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def weight_slice(seed: int, tid: int, start: int, count: int, bf16: bool) -> np.ndarray:
    """Elements [start, start+count) of tensor `tid` (flat row-major), as fp32."""
    base = _mix_scalar((seed ^ _mix_scalar(tid)) & ((1 << 64) - 1))
    out = np.empty(count, dtype=np.float32)
    step = 1 << 22
    scale = np.float32(0.02)
    for s in range(0, count, step):
        n = min(step, count - s)
        i4 = (np.arange(start + s, start + s + n, dtype=np.uint64) << U64(2))
        acc = np.zeros(n, dtype=np.int64)
        for j in range(3):
            r = _mix(U64(base) ^ (i4 + U64(j)))
            for sh in (0, 16, 32, 48):
                acc += ((r >> U64(sh)) & U64(0xFFFF)).astype(np.int64)
        v = (acc - 393210).astype(np.float32) * scale          # one fp32 rounding
        out[s:s + n] = v * np.float32(2.0 ** -16)               # exact
    return to_bf16(out) if bf16 else out


def make_weights(desc: ModelDesc, seed: int, layers: range | None = None) -> dict:
    """All weights of the model as fp32 arrays shaped [out_features, in_features]."""
    bf = desc.dtype == "bf16"
    w: dict = {}
    for name in ("emb", "lm"):
        r, c = desc.shape(name)
        w[name] = weight_slice(seed, tensor_id(name), 0, r * c, bf).reshape(r, c)
    w["gf"] = np.ones(desc.hidden, dtype=np.float32)
    w["layers"] = []
    for l in (layers if layers is not None else range(desc.n_layers)):
        lw = {}
        for name in SLOT:
            r, c = desc.shape(name)
            lw[name] = weight_slice(seed, tensor_id(name, l), 0, r * c, bf).reshape(r, c)
        lw["g1"] = np.ones(desc.hidden, dtype=np.float32)
        lw["g2"] = np.ones(desc.hidden, dtype=np.float32)
        w["layers"].append(lw)
    return w


def normal_weights(desc: ModelDesc, seed: int, emb_block_rows: int | None = None) -> dict:
    """Weights for tests that LOAD them into the library instead of having the device generate
    them: numpy's N(0, 0.02) deviates (much faster on the host than the counter-based recipe above),
    rounded to bf16 when the model says so. With emb_block_rows the embedding table repeats one
    random block of that many rows (token t reads block row t mod emb_block_rows): tests that look
    up a few tokens need not draw a whole vocabulary of rows."""
    bf = desc.dtype == "bf16"
    rng = np.random.default_rng([seed, 17])

    def draw(shape):
        x = rng.standard_normal(size=shape, dtype=np.float32)
        x *= np.float32(0.02)
        return to_bf16(x) if bf else x

    w: dict = {}
    if emb_block_rows:
        block = draw((emb_block_rows, desc.hidden))
        w["emb"] = np.tile(block, (-(-desc.vocab // emb_block_rows), 1))[:desc.vocab]
    else:
        w["emb"] = draw(desc.shape("emb"))
    w["lm"] = draw(desc.shape("lm"))
    w["gf"] = np.ones(desc.hidden, dtype=np.float32)
    w["layers"] = []
    for _ in range(desc.n_layers):
        lw = {name: draw(desc.shape(name)) for name in SLOT}
        lw["g1"] = np.ones(desc.hidden, dtype=np.float32)
        lw["g2"] = np.ones(desc.hidden, dtype=np.float32)
        w["layers"].append(lw)
    return w


# ------------------------------------------------------------------- request-level inputs
def tokens(seed: int, n: int, vocab: int) -> np.ndarray:
    return np.random.default_rng([seed, 11]).integers(0, vocab, size=n, dtype=np.int32)


def uniform_lengths(seed: int, n: int, lo: int, hi: int) -> np.ndarray:
    """n lengths uniform on {lo, ..., hi}."""
    return np.random.default_rng([seed, 12]).integers(lo, hi + 1, size=n, dtype=np.int32)


def lognormal_lengths(seed: int, n: int, median: float, sigma: float, cap: int, lo: int = 1) -> np.ndarray:
    """n lengths min(cap, floor(exp(N(ln median, sigma^2)))), at least `lo`."""
    z = np.random.default_rng([seed, 13]).normal(math.log(median), sigma, size=n)
    return np.clip(np.floor(np.exp(z)), lo, cap).astype(np.int32)


def page_permutation(seed: int, n_pages: int) -> np.ndarray:
    return np.random.default_rng([seed, 14]).permutation(n_pages).astype(np.int32)


def normal_bf16(seed: int, shape, std: float = 1.0) -> np.ndarray:
    """bf16-representable N(0, std) values as fp32 (used to fill KV pools and activations)."""
    x = np.random.default_rng([seed, 15]).standard_normal(size=shape, dtype=np.float32) * np.float32(std)
    return to_bf16(x)


def poisson_trace(seed: int, rate_per_s: float, window_s: float, in_dist: dict, out_dist: dict) -> np.ndarray:
    """Arrival trace: rows (arrival_ns, in_len, out_len), int64, sorted by arrival.

    `in_dist` / `out_dist`: {"kind": "lognormal", "median", "sigma", "cap"} or
    {"kind": "uniform", "lo", "hi"}.
    """
    rng = np.random.default_rng([seed, 16])
    t, arr = 0.0, []
    while True:
        t += rng.exponential(1.0 / rate_per_s)
        if t >= window_s:
            break
        arr.append(int(t * 1e9))
    n = len(arr)

    def draw(dist, sub):
        if dist["kind"] == "lognormal":
            return lognormal_lengths(seed * 7 + sub, n, dist["median"], dist["sigma"], dist["cap"])
        return uniform_lengths(seed * 7 + sub, n, dist["lo"], dist["hi"])

    out = np.empty((n, 3), dtype=np.int64)
    out[:, 0] = arr
    out[:, 1] = draw(in_dist, 1)
    out[:, 2] = draw(out_dist, 2)
    return out


def kv_values(seed: int, layer: int, which: str, pos0: int, n: int, n_kv: int, d: int) -> np.ndarray:
    """Synthetic cached K (which="k") or V ("v") of positions [pos0, pos0+n): unit-variance
    deviates of the same generator as the weights (stream id 0x4B000000 + 2*layer, +1 for V;
    element index (pos*n_kv + head)*d + dd; no 0.02 factor), rounded to bf16. [n, n_kv, d]."""
    tid = 0x4B000000 + 2 * layer + (1 if which == "v" else 0)
    base = _mix_scalar((seed ^ _mix_scalar(tid)) & ((1 << 64) - 1))
    per = n_kv * d
    i4 = (np.arange(pos0 * per, (pos0 + n) * per, dtype=np.uint64) << U64(2))
    acc = np.zeros(n * per, dtype=np.int64)
    for j in range(3):
        r = _mix(U64(base) ^ (i4 + U64(j)))
        for sh in (0, 16, 32, 48):
            acc += ((r >> U64(sh)) & U64(0xFFFF)).astype(np.int64)
    v = (acc - 393210).astype(np.float32) * np.float32(2.0 ** -16)
    return to_bf16(v).reshape(n, n_kv, d)
