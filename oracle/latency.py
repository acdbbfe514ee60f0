"""Oracle, part 2: the performance estimator.  TEST INFRASTRUCTURE.

Follows the paper's Section 2.2.1 (wave quantisation: waves, tail, idle ratio), Section
3.2.2 (SM-scaling roofline model, Eq. 1, and the calibration factor alpha, Eq. 2, with
linear inter/extrapolation between sampled execution states), Section 3.2.3 (decode
uses the bandwidth D_{p,sl} measured next to an sl-token prefill) — in the paper's
order and notation. "SM" in the paper is "CU" here.

All arithmetic on the decision path is integer (Python ints): nanoseconds, flop,
bytes, flop/ns, bytes/ns and alpha in parts per million, with floor division, so that
a second implementation can reproduce every number bit for bit.

Readings where the paper is silent (listed in the design document):
  * kernel flop/byte counts are closed forms of the layer shapes (the paper takes them
    from a model viewer); activations and weights count 2 bytes per element
  * wave quantisation enters as T'_k / (1 - idle_k) for prefill GEMM and attention
    kernels before alpha is applied; a switch in the profile turns it off
  * alpha is sampled on a rectilinear grid — prefill over (CUs, new tokens), decode over
    (CUs, batch size, mean context per request) — and interpolated multilinearly, extrapolated
    from the nearest segment outside the grid, clamped to half the smallest sample
  * a phase with zero CUs has latency INF_NS
"""
from __future__ import annotations

from dataclasses import dataclass, field
from fractions import Fraction

INF_NS = 1 << 60
PPM = 1_000_000


# ------------------------------------------------------------------ Section 2.2.1
def wave_quant(g: int, n: int, b: int = 1):
    """Waves w, active units in the last wave `tail`, and the idle ratio (exact Fraction)
    of a kernel with g workgroups on n units holding b workgroups each."""
    w = -(-g // (b * n))
    tail = -(-(g - b * n * (w - 1)) // b)          # ceil(g/b - n (w-1))
    return w, tail, Fraction(n - tail, n * w)


# ------------------------------------------------------------------ profile (hardware + samples)
@dataclass
class Grid:
    """Samples on a rectilinear grid: axes[i] ascending ints, values nested lists."""
    axes: list
    values: list

    def min_value(self):
        def walk(v):
            return min(walk(x) for x in v) if isinstance(v, list) else v
        return walk(self.values)


@dataclass
class Profile:
    n_cu: int = 256
    granule: int = 32
    c_peak: int = 2_500_000            # flop per ns at all CUs
    d_peak: int = 8_000                # bytes per ns
    n_d: int = 64                      # CUs at which memory bandwidth saturates
    tile_m: int = 256
    tile_n: int = 256
    tile_q: int = 128
    wgs_per_cu: int = 1                # b of Section 2.2.1: workgroups resident per CU
    use_waveq: int = 1
    tail_cut: int = 0                  # > 0: the GEMMs cut the tiles of a partly filled last wave along K, into at most this many pieces
    # measured rates the GPU library's tile choice reads from the same file; the estimator does not use them:
    # GFLOP/s per busy CU of the 128x128, 256x256 and 128x256 GEMM tiles, MB/s per CU for partial tiles written and read back
    gemm_rate_128: int = 3500
    gemm_rate_256: int = 4800
    gemm_rate_128x256: int = 5000
    gemm_fixed_128x256: int = 25000    # ns: start-up and epilogue of that tile, which runs one per CU
    partial_bw_cu: int = 20000
    # MB/s of a plain read-only stream, per CU of a 32-CU partition and of the whole GPU (the GPU library plans its decode GEMMs with them)
    stream_bw_cu: int = 59000
    stream_bw_gpu: int = 6400000
    bw: Grid | None = None             # D_{p,sl}: axes (decode CUs, co-running prefill tokens) -> bytes/ns
    # slowdown (ppm) of a prefill slice beside a decode step, over the decode CUs it shares the GPU
    # with; None = none. Section 3.2.3 measures this direction of the contention as small and
    # drops it; kept here as a measured table because it is not small on every part
    prefill_corun: Grid | None = None
    alpha_prefill: Grid = field(default_factory=lambda: Grid([[256], [2048]], [[PPM]]))
    alpha_decode: Grid = field(default_factory=lambda: Grid([[256], [64], [65536]], [[[PPM]]]))


@dataclass(frozen=True)
class Shape:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    mlp: int
    vocab: int


def floor_div(a: int, b: int) -> int:
    return a // b


def interp(grid_axes, values, x) -> int:
    """Multilinear interpolation on a rectilinear grid, first axis outermost; outside the
    grid the nearest segment is extended. Integer arithmetic, floor at every stage."""
    if not grid_axes:
        return values
    ax = grid_axes[0]
    if len(ax) == 1:
        return interp(grid_axes[1:], values[0], x[1:])
    i = 0
    while i + 2 < len(ax) and x[0] >= ax[i + 1]:
        i += 1
    v0 = interp(grid_axes[1:], values[i], x[1:])
    v1 = interp(grid_axes[1:], values[i + 1], x[1:])
    return v0 + floor_div((v1 - v0) * (x[0] - ax[i]), ax[i + 1] - ax[i])


def alpha_at(grid: Grid, x) -> int:
    return max(interp(grid.axes, grid.values, list(x)), grid.min_value() // 2, 1)


# ------------------------------------------------------------------ kernel work counts
def _cdiv(a, b):
    return -(-a // b)


def prefill_kernels(s: Shape, hw: Profile, reqs, with_head: bool, whole_tiles: bool | None = None):
    """One layer of prefill for requests [(sl_i, p_i)]: (name, flop, bytes, workgroups or 0).
    The head entry (final norm + LM head for one row per request) is appended when asked."""
    h, d = s.hidden, s.head_dim
    qd, kvd = s.n_q_heads * d, s.n_kv_heads * d
    qkvn = qd + 2 * kvd
    t = sum(sl for sl, _ in reqs)
    tm, tn = hw.tile_m, hw.tile_n
    rows = _cdiv(t, tm)
    # thread blocks compute whole tiles: with the tile-level (wave quantisation) model on, the GEMM
    # flop count pads the rows to the tile height; whole_tiles=False asks for the exact counts
    if whole_tiles is None:
        whole_tiles = bool(hw.use_waveq)
    tp = rows * tm if whole_tiles else t
    att_flop = sum(4 * qd * (sl * p + sl * (sl + 1) // 2) for sl, p in reqs)
    att_mem = sum(2 * (2 * sl * qd + 2 * (p + sl) * kvd) for sl, p in reqs)
    att_g = sum(_cdiv(sl, hw.tile_q) * s.n_q_heads for sl, _ in reqs)
    ks = [("norm1", 4 * t * h, 4 * t * h, 0),
          ("qkv", 2 * tp * h * qkvn, 2 * (h * qkvn + t * h + t * qkvn), rows * _cdiv(qkvn, tn)),
          ("rope", 4 * t * qkvn, 4 * t * qkvn, 0),
          ("attn", att_flop, att_mem, att_g),
          ("o", 2 * tp * qd * h, 2 * (qd * h + t * qd + 2 * t * h), rows * _cdiv(h, tn)),
          ("norm2", 4 * t * h, 4 * t * h, 0),
          ("gateup", 4 * tp * h * s.mlp, 2 * (2 * h * s.mlp + t * h + t * s.mlp), rows * _cdiv(2 * s.mlp, tn)),
          ("down", 2 * tp * s.mlp * h, 2 * (s.mlp * h + t * s.mlp + 2 * t * h), rows * _cdiv(h, tn))]
    head = []
    if with_head:
        b = len(reqs)
        head = [("head", 2 * b * h * s.vocab, 2 * (h * s.vocab + b * h + b * s.vocab), 0)]
    return ks, head


def decode_kernels(s: Shape, cls):
    """One layer of a decode step for contexts cl_i (the new token attends to cl_i + 1
    positions), and the head."""
    h, d = s.hidden, s.head_dim
    qd, kvd = s.n_q_heads * d, s.n_kv_heads * d
    qkvn = qd + 2 * kvd
    b = len(cls)
    ctx = sum(c + 1 for c in cls)
    ks = [("norm1", 4 * b * h, 4 * b * h, 0),
          ("qkv", 2 * b * h * qkvn, 2 * (h * qkvn + b * h + b * qkvn), 0),
          ("rope", 4 * b * qkvn, 4 * b * qkvn, 0),
          ("attn", 4 * qd * ctx, 2 * (2 * kvd * ctx + 2 * b * qd), 0),
          ("o", 2 * b * qd * h, 2 * (qd * h + b * qd + 2 * b * h), 0),
          ("norm2", 4 * b * h, 4 * b * h, 0),
          ("gateup", 4 * b * h * s.mlp, 2 * (2 * h * s.mlp + b * h + b * s.mlp), 0),
          ("down", 2 * b * s.mlp * h, 2 * (s.mlp * h + b * s.mlp + 2 * b * h), 0)]
    head = [("head", 2 * b * h * s.vocab, 2 * (h * s.vocab + b * h + b * s.vocab), 0)]
    return ks, head


# ------------------------------------------------------------------ Section 3.2.2, Eq. 1
def srm_ns(flop: int, mem: int, n_p: int, hw: Profile, d_override: int | None = None) -> int:
    """T'_k on n_p CUs: flop / min(flop/mem * D_p, C_p) == max(flop / C_p, mem / D_p), with
    C_p = C_peak n_p / N and D_p = D_peak min(1, n_p / N_d) (or a measured D)."""
    t_c = floor_div(flop * hw.n_cu, hw.c_peak * n_p)
    if d_override is not None:
        t_m = floor_div(mem, max(d_override, 1))
    else:
        t_m = floor_div(mem * hw.n_d, hw.d_peak * min(n_p, hw.n_d))
    return max(t_c, t_m)


def _waveq_adjust(t: int, g: int, n_p: int, b: int = 1) -> int:
    w, tail, _ = wave_quant(g, n_p, b)
    return floor_div(t * n_p * w, n_p * w - n_p + tail)


GEMM_KERNELS = ("qkv", "o", "gateup", "down")
PIECE_COST_PPM = 30_000      # start-up and partial-tile store of one K piece, as a share of a tile time


def tail_plan(g: int, slots: int, max_cut: int):
    """The GEMM kernels' remedy for wave quantisation (Section 2.2.1 states the problem): of g
    tiles on `slots` resident workgroups, full = g // slots waves run whole; the `rest` tiles of
    the last wave are cut along K into f pieces each, which then take ceil(rest f / slots) rounds
    of 1/f tile time (plus a fixed cost per piece). f is the cut in 2..max_cut with the smallest
    such time, used only when it saves at least a tenth of a tile time; otherwise f = 1.
    Returns (full, rest, f, rounds)."""
    full = g // slots
    rest = g - full * slots
    if rest == 0 or max_cut < 2:
        return full, rest, 1, 1 if rest else 0
    best, best_cost = 1, PPM
    for cut in range(2, max_cut + 1):
        rounds = _cdiv(rest * cut, slots)
        cost = rounds * (PPM // cut + PIECE_COST_PPM)
        if cost < best_cost:
            best, best_cost = cut, cost
    if best_cost > 900_000:
        return full, rest, 1, 1
    return full, rest, best, _cdiv(rest * best, slots)


def _waveq_tail_adjust(t: int, g: int, n_p: int, b: int, max_cut: int) -> int:
    """As _waveq_adjust, for a kernel that cuts its last wave: the busy-time share g / slots of a
    wave count becomes full + rounds (1/f + piece cost)."""
    slots = b * n_p
    full, rest, f, rounds = tail_plan(g, slots, max_cut)
    if f == 1:
        return _waveq_adjust(t, g, n_p, b)
    waves_ppm = full * PPM + rounds * (PPM // f + PIECE_COST_PPM)
    return floor_div(t * waves_ppm * slots, g * PPM)


def prefill_roofline_ns(s: Shape, hw: Profile, reqs, pm: int, layer_begin: int, n_layers_step: int) -> int:
    """T'_{p,ES}: the sum of T'_k over the kernels of `n_layers_step` layers (and the head
    if the slice ends at the last layer)."""
    with_head = layer_begin + n_layers_step >= s.n_layers
    ks, head = prefill_kernels(s, hw, reqs, with_head)
    per_layer = 0
    for name, flop, mem, g in ks:
        t = srm_ns(flop, mem, pm, hw)
        if hw.use_waveq and g > 0:
            if hw.tail_cut > 0 and name in GEMM_KERNELS:
                t = _waveq_tail_adjust(t, g, pm, hw.wgs_per_cu, hw.tail_cut)
            else:
                t = _waveq_adjust(t, g, pm, hw.wgs_per_cu)
        per_layer += t
    total = per_layer * n_layers_step
    for _, flop, mem, _ in head:
        total += srm_ns(flop, mem, pm, hw)
    return total


def decode_roofline_ns(s: Shape, hw: Profile, cls, dm: int, co_prefill_tokens: int) -> int:
    d_meas = None
    if hw.bw is not None:
        d_meas = max(interp(hw.bw.axes, hw.bw.values, [dm, co_prefill_tokens]), 1)
    ks, head = decode_kernels(s, cls)
    per_layer = sum(srm_ns(flop, mem, dm, hw, d_meas) for _, flop, mem, _ in ks)
    return per_layer * s.n_layers + sum(srm_ns(flop, mem, dm, hw, d_meas) for _, flop, mem, _ in head)


# ------------------------------------------------------------------ Eq. 2 and the prediction
def alpha_from_measurement(t_measured_ns: int, t_roofline_ns: int) -> int:
    """alpha = T_measured / T', in parts per million."""
    return floor_div(t_measured_ns * PPM, max(t_roofline_ns, 1))


def prefill_corun_ppm(hw: Profile, co_decode_cus: int) -> int:
    """Slowdown of a prefill slice that runs beside a decode step on co_decode_cus other CUs."""
    if co_decode_cus <= 0 or hw.prefill_corun is None:
        return PPM
    return alpha_at(hw.prefill_corun, [co_decode_cus])


def predict_prefill_ns(s: Shape, hw: Profile, reqs, pm: int, layer_begin: int, n_layers_step: int, co_decode_cus: int = 0) -> int:
    if pm <= 0 or not reqs:
        return INF_NS if reqs else 0
    t = prefill_roofline_ns(s, hw, reqs, pm, layer_begin, n_layers_step)
    a = alpha_at(hw.alpha_prefill, [pm, sum(sl for sl, _ in reqs)])
    alone = floor_div(t * a, PPM)
    return floor_div(alone * prefill_corun_ppm(hw, co_decode_cus), PPM)


def co_decode_cus(hw: Profile, es: dict) -> int:
    """The decode CUs a prefill slice of execution state es shares the GPU with: a decode batch on a
    disjoint CU set; 0 when nothing decodes or the two sets overlap."""
    dm = es["decode_cus"]
    return dm if (len(es["decode_ctx"]) > 0 and dm > 0 and es["prefill_cus"] + dm <= hw.n_cu) else 0


def predict_decode_ns(s: Shape, hw: Profile, cls, dm: int, co_prefill_tokens: int) -> int:
    if not cls:
        return 0
    if dm <= 0:
        return INF_NS
    t = decode_roofline_ns(s, hw, cls, dm, co_prefill_tokens)
    a = alpha_at(hw.alpha_decode, [dm, len(cls), sum(cls) // len(cls)])
    return floor_div(t * a, PPM)


def latency_query(s: Shape, hw: Profile, es: dict):
    """es: prefill_len[], prefill_ctx[], decode_ctx[], prefill_cus, decode_cus, layer_begin,
    n_layers_step. Returns (prefill_ns for the slice, decode_ns for one step)."""
    reqs = list(zip(es["prefill_len"], es["prefill_ctx"]))
    co = sum(es["prefill_len"]) if es["prefill_cus"] > 0 else 0
    return (predict_prefill_ns(s, hw, reqs, es["prefill_cus"], es["layer_begin"], es["n_layers_step"], co_decode_cus(hw, es)),
            predict_decode_ns(s, hw, list(es["decode_ctx"]), es["decode_cus"], co))


# ------------------------------------------------------------------ online recalibration (Section 3.2.4)
def _cell_corners(grid: Grid, x):
    """Index tuples of the samples the interpolation at x reads: per axis both ends of its segment
    (the single sample of a one-point axis)."""
    per_axis = []
    for ax, xv in zip(grid.axes, x):
        if len(ax) == 1:
            per_axis.append([0])
            continue
        i = 0
        while i + 2 < len(ax) and xv >= ax[i + 1]:
            i += 1
        per_axis.append([i, i + 1])
    corners = [[]]
    for choices in per_axis:
        corners = [c + [k] for c in corners for k in choices]
    return corners


def _blend(grid: Grid, x, t_measured: int, t_roofline: int, weight_ppm: int) -> None:
    """One observation: Eq. 2 gives alpha_obs = T_measured / T' at x. Every sample the interpolation
    at x reads moves by weight * (alpha_obs / alpha_predicted - 1) of its own value, so the
    prediction at x moves by that share toward the measurement; samples stay >= 1."""
    a_pred = alpha_at(grid, x)
    a_obs = alpha_from_measurement(t_measured, t_roofline)
    for idx in _cell_corners(grid, x):
        node = grid.values
        for i in idx[:-1]:
            node = node[i]
        old = node[idx[-1]]
        target = floor_div(old * a_obs, a_pred)
        node[idx[-1]] = max(1, old + floor_div((target - old) * weight_ppm, PPM))


def observe(s: Shape, hw: Profile, es: dict, measured_prefill_ns: int, measured_decode_ns: int, weight_ppm: int) -> None:
    """Recalibrate alpha from one measured slice and/or step at execution state es (a measurement
    <= 0 is skipped). Mutates hw."""
    reqs = list(zip(es["prefill_len"], es["prefill_ctx"]))
    if measured_prefill_ns > 0 and reqs and es["prefill_cus"] > 0:
        roof = prefill_roofline_ns(s, hw, reqs, es["prefill_cus"], es["layer_begin"], es["n_layers_step"])
        roof = floor_div(roof * prefill_corun_ppm(hw, co_decode_cus(hw, es)), PPM)      # alpha stays the stand-alone factor
        _blend(hw.alpha_prefill, [es["prefill_cus"], sum(sl for sl, _ in reqs)], measured_prefill_ns, roof, weight_ppm)
    cls = list(es["decode_ctx"])
    if measured_decode_ns > 0 and cls and es["decode_cus"] > 0:
        co = sum(es["prefill_len"]) if es["prefill_cus"] > 0 else 0
        roof = decode_roofline_ns(s, hw, cls, es["decode_cus"], co)
        _blend(hw.alpha_decode, [es["decode_cus"], len(cls), sum(cls) // len(cls)], measured_decode_ns, roof, weight_ppm)


# ------------------------------------------------------------------ profile file (text)
def _flatten(v):
    return [y for x in v for y in _flatten(x)] if isinstance(v, list) else [v]


def _nest(flat, dims):
    if len(dims) == 1:
        return list(flat)
    step = len(flat) // dims[0]
    return [_nest(flat[i * step:(i + 1) * step], dims[1:]) for i in range(dims[0])]


def dump_profile(hw: Profile) -> str:
    lines = ["sts-profile 1"]
    for k in ("n_cu", "granule", "c_peak", "d_peak", "n_d", "tile_m", "tile_n", "tile_q", "wgs_per_cu", "use_waveq", "tail_cut",
              "gemm_rate_128", "gemm_rate_256", "gemm_rate_128x256", "gemm_fixed_128x256", "partial_bw_cu", "stream_bw_cu", "stream_bw_gpu"):
        lines.append(f"{k} {getattr(hw, k)}")
    for name in ("bw", "prefill_corun", "alpha_prefill", "alpha_decode"):
        g = getattr(hw, name)
        if g is None:
            continue
        lines.append(f"grid {name} {len(g.axes)}")
        for ax in g.axes:
            lines.append("axis " + " ".join(str(a) for a in ax))
        lines.append("values " + " ".join(str(v) for v in _flatten(g.values)))
    return "\n".join(lines) + "\n"


def parse_profile(text: str) -> Profile:
    hw = Profile()
    lines = [l.split() for l in text.splitlines() if l.strip() and not l.startswith("#")]
    assert lines[0] == ["sts-profile", "1"]
    i = 1
    while i < len(lines):
        t = lines[i]
        if t[0] == "grid":
            name, nd = t[1], int(t[2])
            axes = [[int(x) for x in lines[i + 1 + j][1:]] for j in range(nd)]
            flat = [int(x) for x in lines[i + 1 + nd][1:]]
            setattr(hw, name, Grid(axes, _nest(flat, [len(a) for a in axes])))
            i += nd + 2
        else:
            setattr(hw, t[0], int(t[1]))
            i += 1
    return hw
