"""ctypes binding of libsts.so: the same calls as include/sts.h, argument marshalling only.

Every step of the path runs in the library's HIP kernels; there is no Python or CPU fallback.
The library is loaded on first use and a missing library is an error (build it with
`python -m paper_2504_19516_amd.build` or `__graft_entry__.build()`).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsts.so")
_lib = None

OK, EINVAL, ENOMEM, ESTATE, EHIP, EIO = 0, -1, -2, -3, -4, -5
K_NAMES = ["embed", "norm", "qkv", "rope", "attn", "attn_merge", "o", "gateup", "swiglu", "down", "reduce", "head", "sample"]
GEMM_CFGS = {"128x128": 0, "64x256": 1, "64x128": 2, "256x256": 3, "128x256": 4,
             "64x256s": 5, "64x320s": 6, "64x384s": 7, "64x448s": 8, "64x512s": 9}
INF_NS = 1 << 60


class StsError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        hip = lib().sts_last_hip_error() if code == EHIP else 0
        msg = lib().sts_strerror(code).decode()
        super().__init__(f"{what}: {msg} (code {code}" + (f", hip error {hip})" if code == EHIP else ")"))


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "mlp", "vocab", "page_tokens")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float)]


class InitParams(C.Structure):
    _fields_ = [("weight_seed", C.c_uint64)] + [(n, C.c_int32) for n in (
        "init_weights", "kv_pool_pages", "max_prefill_tokens", "max_prefill_seqs", "max_decode_batch", "max_seqs", "max_pages_per_seq")]


class ExecState(C.Structure):
    _fields_ = [("n_prefill", C.c_int32), ("prefill_len", C.POINTER(C.c_int32)), ("prefill_ctx", C.POINTER(C.c_int32)),
                ("n_decode", C.c_int32), ("decode_ctx", C.POINTER(C.c_int32)),
                ("prefill_cus", C.c_int32), ("decode_cus", C.c_int32), ("layer_begin", C.c_int32), ("n_layers_step", C.c_int32)]


class SchedConfig(C.Structure):
    _fields_ = [("ttft_slo_ns", C.c_int64), ("tpot_slo_ns", C.c_int64)] + [(n, C.c_int32) for n in (
        "layers_per_step", "max_batch_tokens", "max_decode_batch", "kv_pool_pages", "mode", "fixed_prefill_cus", "decode_boost_cus", "min_batch_tokens")]


class SchedReq(C.Structure):
    _fields_ = [("id", C.c_int32), ("in_len", C.c_int32), ("out_len", C.c_int32), ("arrival_ns", C.c_int64)]


class SchedDec(C.Structure):
    _fields_ = [("in_len", C.c_int32), ("n_dec", C.c_int32), ("first_token_ns", C.c_int64)]


class SchedState(C.Structure):
    _fields_ = [("now_ns", C.c_int64), ("n_queue", C.c_int32), ("queue", C.POINTER(SchedReq)),
                ("n_inflight", C.c_int32), ("inflight", C.POINTER(SchedReq)), ("layers_done", C.c_int32),
                ("n_decode", C.c_int32), ("decode", C.POINTER(SchedDec)), ("pages_free", C.c_int32),
                ("cur_prefill_cus", C.c_int32), ("cur_decode_cus", C.c_int32)]


class SchedChoice(C.Structure):
    _fields_ = [("cap_tasks", C.c_int32), ("task_ids", C.POINTER(C.c_int32)), ("cap_queue", C.c_int32), ("queue_ids", C.POINTER(C.c_int32)),
                ("n_tasks", C.c_int32), ("n_queue", C.c_int32), ("admitted", C.c_int32), ("layer_begin", C.c_int32),
                ("layer_end", C.c_int32), ("prefill_cus", C.c_int32), ("decode_cus", C.c_int32), ("branch", C.c_int32),
                ("predicted_ns", C.c_int64)]


class Decision(C.Structure):
    _fields_ = [("t_ns", C.c_int64), ("n_tasks", C.c_int32), ("first_req", C.c_int32), ("tasks_hash", C.c_int64),
                ("layer_begin", C.c_int32), ("layer_end", C.c_int32), ("prefill_cus", C.c_int32), ("decode_cus", C.c_int32),
                ("branch", C.c_int32), ("decode_batch", C.c_int32), ("predicted_ns", C.c_int64)]


class ReplayStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("n_requests", "n_finished", "out_tokens", "makespan_ns", "ttft_sum_ns", "tpot_sum_ns",
                                          "n_tpot", "n_slo_ok", "n_decisions")]


EXPORTS = [
    "sts_strerror", "sts_last_hip_error", "sts_init", "sts_destroy", "sts_release_streams", "sts_load_weights", "sts_read_weights",
    "sts_seq_create", "sts_seq_free", "sts_seq_length", "sts_seq_truncate", "sts_seq_reserve", "sts_pages_free", "sts_seq_set_block_table",
    "sts_seq_get_block_table", "sts_kv_write", "sts_kv_read", "sts_kv_fill_random", "sts_prefill_batch",
    "sts_prefill_append", "sts_prefill_launch", "sts_decode_launch", "sts_phase_done", "sts_prefill_finish",
    "sts_decode_finish", "sts_prefill_abort", "sts_decode_step", "sts_step_concurrent", "sts_last_timing", "sts_read_hidden",
    "sts_set_partition", "sts_get_partition", "sts_kernel_timing", "sts_kernel_times", "sts_kernel_name",
    "sts_probe_copy", "sts_profile_observe", "sts_op_gemm", "sts_op_attn_prefill", "sts_op_attn_decode", "sts_wave_quant",
    "sts_profile_parse", "sts_profile_load", "sts_profile_dump", "sts_profile_free", "sts_latency_query",
    "sts_latency_roofline", "sts_sched_decide", "sts_sched_replay", "sts_max_pages_per_seq_limit", "sts_decode_chunk_plan", "sts_decode_gemm_plan", "sts_probe_read", "sts_set_stream_model", "sts_profile_stream_model", "sts_op_gemm_noalloc", "sts_weight_packed_index", "sts_probe_gemm", "sts_set_tile_model",
    "sts_profile_tile_model",
]


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build the HIP library first (python -m paper_2504_19516_amd.build)")
        _lib = C.CDLL(LIB_PATH)
        _lib.sts_strerror.restype = C.c_char_p
        _lib.sts_kernel_name.restype = C.c_char_p
    return _lib


def _ck(code, what):
    if code != OK:
        raise StsError(code, what)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _p(a, t=C.c_int32):
    return a.ctypes.data_as(C.POINTER(t)) if a is not None else None


def model_desc(d) -> ModelDesc:
    """From a synth.ModelDesc-like object."""
    return ModelDesc(d.n_layers, d.hidden, d.n_q_heads, d.n_kv_heads, d.head_dim, d.mlp, d.vocab, d.page_tokens,
                     d.rope_theta, d.rms_eps)


class Engine:
    """Owns one sts_ctx."""

    def __init__(self, desc, weight_seed=0, init_weights=True, kv_pool_pages=256, max_prefill_tokens=256,
                 max_prefill_seqs=8, max_decode_batch=16, max_seqs=64, max_pages_per_seq=64):
        self.desc = desc
        self._d = model_desc(desc)
        prm = InitParams(weight_seed, int(init_weights), kv_pool_pages, max_prefill_tokens, max_prefill_seqs,
                         max_decode_batch, max_seqs, max_pages_per_seq)
        self._ctx = C.c_void_p()
        _ck(lib().sts_init(C.byref(self._d), C.byref(prm), C.byref(self._ctx)), "sts_init")

    def close(self):
        if self._ctx:
            lib().sts_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # weights
    def load_weights(self, layer, name, arr):
        a = _f32(arr)
        _ck(lib().sts_load_weights(self._ctx, layer, name.encode(), _p(a, C.c_float), C.c_size_t(a.size)), f"sts_load_weights({name})")

    def read_weights(self, layer, name, shape):
        out = np.empty(shape, dtype=np.float32)
        _ck(lib().sts_read_weights(self._ctx, layer, name.encode(), _p(out, C.c_float), C.c_size_t(out.size)), f"sts_read_weights({name})")
        return out

    def load_all(self, weights):
        """weights: dict as produced by synth.make_weights."""
        self.load_weights(0, "emb", weights["emb"]); self.load_weights(0, "lm", weights["lm"]); self.load_weights(0, "gf", weights["gf"])
        for l, lw in enumerate(weights["layers"]):
            for k, v in lw.items():
                self.load_weights(l, k, v)

    # sequences
    def seq_create(self):
        s = C.c_int32()
        _ck(lib().sts_seq_create(self._ctx, C.byref(s)), "sts_seq_create")
        return s.value

    def seq_free(self, seq):
        _ck(lib().sts_seq_free(self._ctx, seq), "sts_seq_free")

    def seq_length(self, seq):
        n = C.c_int32()
        _ck(lib().sts_seq_length(self._ctx, seq, C.byref(n)), "sts_seq_length")
        return n.value

    def seq_truncate(self, seq, new_len):
        _ck(lib().sts_seq_truncate(self._ctx, seq, new_len), "sts_seq_truncate")

    def seq_reserve(self, seq, n_tokens):
        _ck(lib().sts_seq_reserve(self._ctx, seq, n_tokens), "sts_seq_reserve")

    def pages_free(self):
        n = C.c_int32()
        _ck(lib().sts_pages_free(self._ctx, C.byref(n)), "sts_pages_free")
        return n.value

    def seq_set_block_table(self, seq, pages):
        a = _i32(pages)
        _ck(lib().sts_seq_set_block_table(self._ctx, seq, _p(a), a.size), "sts_seq_set_block_table")

    def seq_get_block_table(self, seq, cap=4096):
        a = np.zeros(cap, dtype=np.int32); n = C.c_int32()
        _ck(lib().sts_seq_get_block_table(self._ctx, seq, _p(a), cap, C.byref(n)), "sts_seq_get_block_table")
        return a[:n.value].copy()

    def kv_write(self, layer, seq, pos0, k, v):
        k, v = _f32(k), _f32(v)
        _ck(lib().sts_kv_write(self._ctx, layer, seq, pos0, k.shape[0], _p(k, C.c_float), _p(v, C.c_float)), "sts_kv_write")

    def kv_read(self, layer, seq, pos0, n):
        shape = (n, self.desc.n_kv_heads, self.desc.head_dim)
        k, v = np.empty(shape, np.float32), np.empty(shape, np.float32)
        _ck(lib().sts_kv_read(self._ctx, layer, seq, pos0, n, _p(k, C.c_float), _p(v, C.c_float)), "sts_kv_read")
        return k, v

    def kv_fill_random(self, seq, n, seed):
        _ck(lib().sts_kv_fill_random(self._ctx, seq, n, C.c_uint64(seed)), "sts_kv_fill_random")

    # the step
    def prefill_batch(self, seqs, token_lists, layer_begin=0, layer_end=None, want_logits=True):
        layer_end = self.desc.n_layers if layer_end is None else layer_end
        seqs = _i32(seqs)
        lens = _i32([len(t) for t in token_lists])
        toks = _i32(np.concatenate([np.asarray(t, dtype=np.int32) for t in token_lists]))
        logits = np.empty((len(seqs), self.desc.vocab), np.float32) if (want_logits and layer_end == self.desc.n_layers) else None
        _ck(lib().sts_prefill_batch(self._ctx, len(seqs), _p(seqs), _p(lens), _p(toks), layer_begin, layer_end,
                                    _p(logits, C.c_float)), "sts_prefill_batch")
        return logits

    def prefill_append(self, seq, tokens, layer_begin=0, layer_end=None, want_logits=True):
        layer_end = self.desc.n_layers if layer_end is None else layer_end
        toks = _i32(tokens)
        logits = np.empty(self.desc.vocab, np.float32) if (want_logits and layer_end == self.desc.n_layers) else None
        _ck(lib().sts_prefill_append(self._ctx, seq, _p(toks), toks.size, layer_begin, layer_end, _p(logits, C.c_float)), "sts_prefill_append")
        return logits

    # launch / poll / finish
    def prefill_launch(self, seqs, token_lists, layer_begin, layer_end, want_logits=False):
        seqs = _i32(seqs)
        lens = _i32([len(t) for t in token_lists])
        toks = _i32(np.concatenate([np.asarray(t, dtype=np.int32) for t in token_lists])) if layer_begin == 0 else None
        _ck(lib().sts_prefill_launch(self._ctx, len(seqs), _p(seqs), _p(lens), _p(toks), layer_begin, layer_end, int(want_logits)),
            "sts_prefill_launch")

    def decode_launch(self, seqs, in_tokens, want_logits=False, want_next=True):
        seqs, toks = _i32(seqs), _i32(in_tokens)
        _ck(lib().sts_decode_launch(self._ctx, _p(seqs), _p(toks), len(seqs), int(want_logits), int(want_next)), "sts_decode_launch")

    def phase_done(self, phase):
        d = C.c_int32()
        _ck(lib().sts_phase_done(self._ctx, phase, C.byref(d)), "sts_phase_done")
        return bool(d.value)

    def prefill_finish(self, n_seqs=0, want_logits=False):
        logits = np.empty((n_seqs, self.desc.vocab), np.float32) if want_logits else None
        _ck(lib().sts_prefill_finish(self._ctx, _p(logits, C.c_float)), "sts_prefill_finish")
        return logits

    def decode_finish(self, n, want_logits=False, want_next=True):
        logits = np.empty((n, self.desc.vocab), np.float32) if want_logits else None
        nxt = np.empty(n, np.int32) if want_next else None
        _ck(lib().sts_decode_finish(self._ctx, _p(logits, C.c_float), _p(nxt)), "sts_decode_finish")
        return logits, nxt

    def prefill_abort(self):
        _ck(lib().sts_prefill_abort(self._ctx), "sts_prefill_abort")

    def decode_step(self, seqs, in_tokens, want_logits=True, want_next=True):
        seqs, toks = _i32(seqs), _i32(in_tokens)
        logits = np.empty((len(seqs), self.desc.vocab), np.float32) if want_logits else None
        nxt = np.empty(len(seqs), np.int32) if want_next else None
        _ck(lib().sts_decode_step(self._ctx, _p(seqs), _p(toks), len(seqs), _p(logits, C.c_float), _p(nxt)), "sts_decode_step")
        return logits, nxt

    def step_concurrent(self, pseqs, ptoken_lists, layer_begin, layer_end, dseqs, dtokens, want_plogits=True,
                        want_dlogits=True, want_dnext=True):
        pseqs = _i32(pseqs); dseqs = _i32(dseqs); dtok = _i32(dtokens)
        plens = _i32([len(t) for t in ptoken_lists])
        ptoks = _i32(np.concatenate([np.asarray(t, dtype=np.int32) for t in ptoken_lists])) if len(ptoken_lists) else _i32([])
        last = layer_end == self.desc.n_layers
        plog = np.empty((len(pseqs), self.desc.vocab), np.float32) if (want_plogits and last and len(pseqs)) else None
        dlog = np.empty((len(dseqs), self.desc.vocab), np.float32) if (want_dlogits and len(dseqs)) else None
        dnext = np.empty(len(dseqs), np.int32) if (want_dnext and len(dseqs)) else None
        _ck(lib().sts_step_concurrent(self._ctx, len(pseqs), _p(pseqs), _p(plens), _p(ptoks), layer_begin, layer_end,
                                      _p(plog, C.c_float), _p(dseqs), _p(dtok), len(dseqs), _p(dlog, C.c_float), _p(dnext)),
            "sts_step_concurrent")
        return plog, dlog, dnext

    def last_timing(self):
        a, b, w = C.c_int64(), C.c_int64(), C.c_int64()
        _ck(lib().sts_last_timing(self._ctx, C.byref(a), C.byref(b), C.byref(w)), "sts_last_timing")
        return a.value, b.value, w.value

    def read_hidden(self, phase, rows):
        out = np.empty((rows, self.desc.hidden), np.float32)
        _ck(lib().sts_read_hidden(self._ctx, phase, _p(out, C.c_float), rows), "sts_read_hidden")
        return out

    # partition and measurement
    def set_partition(self, prefill_cus, decode_cus):
        _ck(lib().sts_set_partition(self._ctx, prefill_cus, decode_cus), "sts_set_partition")

    def set_tile_model(self, gemm_rate_128, gemm_rate_256, gemm_rate_128x256, gemm_fixed_128x256, partial_bw_cu):
        """GFLOP/s per busy CU of the three prefill tile shapes, the fixed ns of a 128x256 tile and MB/s per CU for partial
        tiles (Profile.tile_model())."""
        _ck(lib().sts_set_tile_model(self._ctx, C.c_int64(int(gemm_rate_128)), C.c_int64(int(gemm_rate_256)), C.c_int64(int(gemm_rate_128x256)),
                                     C.c_int64(int(gemm_fixed_128x256)), C.c_int64(int(partial_bw_cu))), "sts_set_tile_model")

    def set_stream_model(self, stream_bw_cu, stream_bw_gpu):
        _ck(lib().sts_set_stream_model(self._ctx, C.c_int64(int(stream_bw_cu)), C.c_int64(int(stream_bw_gpu))), "sts_set_stream_model")

    def probe_gemm(self, cus, tile_cfg, m, n, iters=10, product="gateup"):
        ns = C.c_int64()
        _ck(lib().sts_probe_gemm(self._ctx, cus, GEMM_CFGS[tile_cfg], {"gateup": 0, "o": 1, "down": 2}[product], m, n, iters, C.byref(ns)),
            "sts_probe_gemm")
        return ns.value

    def get_partition(self):
        a, b, t = C.c_int32(), C.c_int32(), C.c_int32()
        _ck(lib().sts_get_partition(self._ctx, C.byref(a), C.byref(b), C.byref(t)), "sts_get_partition")
        return a.value, b.value, t.value

    def kernel_timing(self, on):
        _ck(lib().sts_kernel_timing(self._ctx, int(on)), "sts_kernel_timing")

    def kernel_times(self, phase, reset=False):
        ns = (C.c_int64 * len(K_NAMES))(); cnt = (C.c_int64 * len(K_NAMES))()
        _ck(lib().sts_kernel_times(self._ctx, phase, ns, cnt, int(reset)), "sts_kernel_times")
        return {K_NAMES[i]: (ns[i], cnt[i]) for i in range(len(K_NAMES)) if cnt[i]}

    def probe_copy(self, side, cus, nbytes, iters):
        ns = C.c_int64()
        _ck(lib().sts_probe_copy(self._ctx, side, cus, C.c_size_t(nbytes), iters, C.byref(ns)), "sts_probe_copy")
        return ns.value

    def probe_read(self, side, cus, nbytes, iters):
        ns = C.c_int64()
        _ck(lib().sts_probe_read(self._ctx, side, cus, C.c_size_t(nbytes), iters, C.byref(ns)), "sts_probe_read")
        return ns.value


# ---- single operations
def op_gemm(a, w, tile_cfg="128x128", epilogue=1, split_k=1, c_in=None, tail_slots=0):
    a, w = _f32(a), _f32(w)
    m, k = a.shape
    n = w.shape[0] // 2 if epilogue == 3 else w.shape[0]
    c = _f32(c_in).copy() if c_in is not None else np.zeros((m, n), np.float32)
    _ck(lib().sts_op_gemm(_p(a, C.c_float), _p(w, C.c_float), _p(c, C.c_float), m, n, k, GEMM_CFGS[tile_cfg], epilogue, split_k, tail_slots), "sts_op_gemm")
    return c


def op_gemm_noalloc(a_dev, w_dev, c_dev, m, n, k, tile_cfg="64x128", split_k=1, tail_slots=0, stream=None):
    """a_dev, w_dev (bf16) and c_dev (fp32) are device addresses (ints) of the caller's buffers; the
    kernels are queued on `stream` (a hipStream_t value, None = the null stream) and not waited for."""
    _ck(lib().sts_op_gemm_noalloc(C.c_void_p(a_dev), C.c_void_p(w_dev), C.c_void_p(c_dev), m, n, k, GEMM_CFGS[tile_cfg], split_k,
                                  tail_slots, C.c_void_p(stream)), "sts_op_gemm_noalloc")


def op_attn_prefill(q, k, v, prior, pages, n_pool_pages):
    q, k, v, pages = _f32(q), _f32(k), _f32(v), _i32(pages)
    t, n_q, d = q.shape
    out = np.empty_like(q)
    _ck(lib().sts_op_attn_prefill(_p(q, C.c_float), _p(k, C.c_float), _p(v, C.c_float), _p(out, C.c_float), t, prior,
                                  n_q, k.shape[1], d, _p(pages), n_pool_pages), "sts_op_attn_prefill")
    return out


def op_attn_decode(q, k, v, ctx, chunk_pages):
    q, k, v, ctx = _f32(q), _f32(k), _f32(v), _i32(ctx)
    n, n_q, d = q.shape
    out = np.empty_like(q)
    _ck(lib().sts_op_attn_decode(_p(q, C.c_float), _p(k, C.c_float), _p(v, C.c_float), _p(out, C.c_float), n, _p(ctx),
                                 n_q, k.shape[1], d, chunk_pages), "sts_op_attn_decode")
    return out


def release_streams():
    """Destroys the process-wide CU-masked streams (every Engine must be closed; no Engine can be created
    afterwards). The last library call of a program that runs under a profiler."""
    _ck(lib().sts_release_streams(), "sts_release_streams")


def max_pages_per_seq_limit(page_tokens=16):
    return lib().sts_max_pages_per_seq_limit(page_tokens)


def decode_chunk_plan(n_pages, n_kv_heads, cus, page_tokens, max_pages_per_seq):
    """(pages per chunk, chunks of the longest context, chunks per context the engine allocates for)."""
    a = _i32(n_pages)
    cp, mc, ac = C.c_int32(), C.c_int32(), C.c_int32()
    _ck(lib().sts_decode_chunk_plan(_p(a), a.size, n_kv_heads, cus, page_tokens, max_pages_per_seq, C.byref(cp), C.byref(mc), C.byref(ac)),
        "sts_decode_chunk_plan")
    return cp.value, mc.value, ac.value


def decode_gemm_plan(m, n, k, cus, may_split=True, partials=True, gemm_rate_256=4967, partial_bw_cu=22504, stream_bw_cu=59000,
                     stream_bw_gpu=6400000):
    """(tile configuration name, split along K, estimated ns) of a decode-side GEMM; host only."""
    cfg, sp, ns = C.c_int32(), C.c_int32(), C.c_int64()
    _ck(lib().sts_decode_gemm_plan(m, n, k, cus, int(may_split), int(partials), C.c_int64(int(gemm_rate_256)), C.c_int64(int(partial_bw_cu)),
                                   C.c_int64(int(stream_bw_cu)), C.c_int64(int(stream_bw_gpu)), C.byref(cfg), C.byref(sp), C.byref(ns)),
        "sts_decode_gemm_plan")
    name = {v: k_ for k_, v in GEMM_CFGS.items()}[cfg.value]
    return name, sp.value, ns.value


# ---- performance estimator and scheduler (host only)
def wave_quant(g, n, b=1):
    w, t, num, den = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
    _ck(lib().sts_wave_quant(C.c_int64(g), C.c_int64(n), C.c_int64(b), C.byref(w), C.byref(t), C.byref(num), C.byref(den)), "sts_wave_quant")
    return w.value, t.value, num.value, den.value


class Profile:
    def __init__(self, text=None, path=None):
        self._p = C.c_void_p()
        if text is not None:
            _ck(lib().sts_profile_parse(text.encode(), C.byref(self._p)), "sts_profile_parse")
        else:
            _ck(lib().sts_profile_load(path.encode(), C.byref(self._p)), "sts_profile_load")

    def __del__(self):
        if getattr(self, "_p", None):
            lib().sts_profile_free(self._p)
            self._p = C.c_void_p()

    def tile_model(self):
        v = [C.c_int64() for _ in range(5)]
        _ck(lib().sts_profile_tile_model(self._p, *[C.byref(x) for x in v]), "sts_profile_tile_model")
        return tuple(x.value for x in v)

    def stream_model(self):
        v = [C.c_int64() for _ in range(2)]
        _ck(lib().sts_profile_stream_model(self._p, *[C.byref(x) for x in v]), "sts_profile_stream_model")
        return tuple(x.value for x in v)

    def dump(self) -> str:
        need = C.c_size_t()
        _ck(lib().sts_profile_dump(self._p, None, C.c_size_t(0), C.byref(need)), "sts_profile_dump")
        buf = C.create_string_buffer(need.value)
        _ck(lib().sts_profile_dump(self._p, buf, C.c_size_t(need.value), None), "sts_profile_dump")
        return buf.value.decode()

    def _es(self, es):
        pl, pc, dc = _i32(es.get("prefill_len", [])), _i32(es.get("prefill_ctx", [])), _i32(es.get("decode_ctx", []))
        st = ExecState(pl.size, _p(pl), _p(pc), dc.size, _p(dc), es.get("prefill_cus", 0), es.get("decode_cus", 0),
                       es.get("layer_begin", 0), es.get("n_layers_step", 1))
        return st, (pl, pc, dc)

    def query(self, desc, es, roofline=False):
        st, keep = self._es(es)
        d = model_desc(desc)
        a, b = C.c_int64(), C.c_int64()
        fn = lib().sts_latency_roofline if roofline else lib().sts_latency_query
        _ck(fn(self._p, C.byref(d), C.byref(st), C.byref(a), C.byref(b)), "sts_latency_query")
        return a.value, b.value

    def observe(self, desc, es, measured_prefill_ns=0, measured_decode_ns=0, weight_ppm=100_000):
        """Online recalibration: blend one measured slice / step at execution state es into alpha."""
        st, keep = self._es(es)
        d = model_desc(desc)
        _ck(lib().sts_profile_observe(self._p, C.byref(d), C.byref(st), C.c_int64(int(measured_prefill_ns)),
                                      C.c_int64(int(measured_decode_ns)), C.c_int64(int(weight_ppm))), "sts_profile_observe")

    @staticmethod
    def _sched_config(cfg):
        return SchedConfig(cfg["ttft_slo_ns"], cfg["tpot_slo_ns"], cfg["layers_per_step"], cfg["max_batch_tokens"],
                           cfg["max_decode_batch"], cfg["kv_pool_pages"], cfg.get("mode", 0), cfg.get("fixed_prefill_cus", 0),
                           cfg.get("decode_boost_cus", 0), cfg.get("min_batch_tokens", 0))

    def decide(self, desc, cfg: dict, now_ns, queue, inflight, layers_done, decode, pages_free, cur_pm, cur_dm):
        """One cycle of Algorithm 1. queue / inflight: lists of (id, arrival_ns, in_len, out_len);
        decode: list of (first_token_ns, n_dec, in_len). Returns a dict."""
        q = (SchedReq * max(1, len(queue)))(*[SchedReq(i, il, ol, a) for i, a, il, ol in queue])
        p = (SchedReq * max(1, len(inflight)))(*[SchedReq(i, il, ol, a) for i, a, il, ol in inflight])
        d = (SchedDec * max(1, len(decode)))(*[SchedDec(il, nd, ft) for ft, nd, il in decode])
        st = SchedState(now_ns, len(queue), q, len(inflight), p, layers_done, len(decode), d, pages_free, cur_pm, cur_dm)
        cap = len(queue) + len(inflight) + 1
        tids, qids = (C.c_int32 * cap)(), (C.c_int32 * cap)()
        ch = SchedChoice(cap, tids, cap, qids)
        sc = self._sched_config(cfg)
        md = model_desc(desc)
        _ck(lib().sts_sched_decide(self._p, C.byref(md), C.byref(sc), C.byref(st), C.byref(ch)), "sts_sched_decide")
        return dict(tasks=list(tids[:ch.n_tasks]), queue=list(qids[:ch.n_queue]), admitted=bool(ch.admitted),
                    layer_begin=ch.layer_begin, layer_end=ch.layer_end, prefill_cus=ch.prefill_cus, decode_cus=ch.decode_cus,
                    branch=ch.branch, predicted_ns=ch.predicted_ns)

    def replay(self, desc, cfg: dict, trace, max_decisions=1 << 20):
        tr = np.ascontiguousarray(trace, dtype=np.int64)
        sc = self._sched_config(cfg)
        dec = (Decision * max_decisions)()
        stats = ReplayStats()
        d = model_desc(desc)
        _ck(lib().sts_sched_replay(self._p, C.byref(d), C.byref(sc), _p(tr, C.c_int64), C.c_int64(tr.shape[0]), dec,
                                   C.c_int64(max_decisions), C.byref(stats)), "sts_sched_replay")
        n = min(max_decisions, stats.n_decisions)
        fields = [f[0] for f in Decision._fields_]
        return [tuple(getattr(dec[i], f) for f in fields) for i in range(n)], {f[0]: getattr(stats, f[0]) for f in ReplayStats._fields_}
