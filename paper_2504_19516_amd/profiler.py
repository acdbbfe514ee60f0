"""Offline profiling for the performance estimator (paper Section 3.2.4): one sweep of memory
and compute throughput over CU counts builds the SM-scaling roofline (D_peak, N_d, C_peak,
D_{p,sl}), then a sparse set of execution states calibrates alpha (Eq. 2). Writes the profile
text that `sts_profile_load` reads, and can score a profile on held-out execution states.

    python -m paper_2504_19516_amd.profiler --model 8b --layers 32 --out profiles/mi355x_llama8b.profile
"""
from __future__ import annotations

import argparse
import json
import threading
import time

import numpy as np

from . import sts, synth

PPM = 1_000_000


def profile_text(hw: dict, grids: dict) -> str:
    lines = ["sts-profile 1"]
    for k in ("n_cu", "granule", "c_peak", "d_peak", "n_d", "tile_m", "tile_n", "tile_q", "wgs_per_cu", "use_waveq", "tail_cut",
              "gemm_rate_128", "gemm_rate_256", "gemm_rate_128x256", "gemm_fixed_128x256", "partial_bw_cu", "stream_bw_cu", "stream_bw_gpu"):
        lines.append(f"{k} {int(hw[k])}")
    for name in ("bw", "prefill_corun", "alpha_prefill", "alpha_decode"):
        if name not in grids:
            continue
        axes, values = grids[name]
        lines.append(f"grid {name} {len(axes)}")
        for ax in axes:
            lines.append("axis " + " ".join(str(int(a)) for a in ax))
        lines.append("values " + " ".join(str(int(v)) for v in np.asarray(values).reshape(-1)))
    return "\n".join(lines) + "\n"


class Profiler:
    def __init__(self, desc, max_tokens=8192, max_batch=224, max_ctx=8192, granule=32):
        self.desc, self.granule = desc, granule
        # room for the largest decode samples: 64 requests at max_ctx, or max_batch requests at 2048 tokens
        pages = (max(64 * (max_ctx + 64), max_batch * (2048 + 64)) + 2 * max_tokens) // 16 + 64
        self.eng = sts.Engine(desc, weight_seed=1, init_weights=True, kv_pool_pages=pages, max_prefill_tokens=max_tokens,
                              max_prefill_seqs=4, max_decode_batch=max_batch, max_seqs=max_batch + 8,
                              max_pages_per_seq=(max_ctx + 128) // 16)
        self.n_cu = self.eng.get_partition()[2]
        self.hw = dict(n_cu=self.n_cu, granule=granule, c_peak=2_500_000, d_peak=8_000, n_d=self.n_cu, tile_m=128, tile_n=128,
                       tile_q=128, wgs_per_cu=2, use_waveq=1, tail_cut=16,
                       gemm_rate_128=3500, gemm_rate_256=4800, gemm_rate_128x256=5000, gemm_fixed_128x256=25000, partial_bw_cu=20000,
                       stream_bw_cu=59000, stream_bw_gpu=6400000)      # the library's defaults until measured
        self.max_tokens = max_tokens
        self.grids = {}

    def close(self):
        self.eng.close()

    # ---- raw measurements ------------------------------------------------------------------
    def copy_bw(self, cus, nbytes=1 << 28, iters=8):
        """bytes/ns moved (read + written) by the copy probe on `cus` CUs of the decode side."""
        ns = self.eng.probe_copy(1, cus, nbytes, iters)
        return 2 * nbytes * iters / ns

    def prefill_ns(self, pm, tokens, ctx=0, layers=4, reps=2):
        eng = self.eng
        eng.set_partition(pm, self.n_cu)
        layers = min(layers, self.desc.n_layers)
        toks = synth.tokens(3, tokens, self.desc.vocab)
        best = None
        for _ in range(reps + 1):
            s = eng.seq_create()
            if ctx:
                eng.kv_fill_random(s, ctx, 77)
            eng.prefill_append(s, toks, 0, layers, want_logits=False)
            t = eng.last_timing()[0]
            if layers < self.desc.n_layers:
                eng.prefill_abort()
            eng.seq_free(s)
            best = t if best is None else min(best, t)
        return best, layers

    def make_decode_batch(self, ctxs):
        seqs = []
        for i, c in enumerate(ctxs):
            s = self.eng.seq_create()
            self.eng.kv_fill_random(s, int(c), 500 + i)
            self.eng.seq_reserve(s, int(c) + 32)
            seqs.append(s)
        return seqs

    def decode_ns(self, dm, seqs, reps=3):
        eng = self.eng
        eng.set_partition(self.n_cu, dm)
        toks = synth.tokens(4, len(seqs), self.desc.vocab)
        best = None
        for _ in range(reps + 1):
            eng.decode_step(seqs, toks, want_logits=False, want_next=True)
            t = eng.last_timing()[1]
            best = t if best is None else min(best, t)
        return best

    def corun_copy_bw(self, dm, prefill_tokens):
        """Copy bandwidth on dm decode CUs while a prefill of `prefill_tokens` runs on the rest."""
        if prefill_tokens == 0:
            return self.copy_bw(dm)
        eng = self.eng
        pm = self.n_cu - dm
        eng.set_partition(pm, dm)
        toks = synth.tokens(3, prefill_tokens, self.desc.vocab)
        s = eng.seq_create()
        # size the prefill slice so it outlasts the probe
        layers = self.desc.n_layers
        th = threading.Thread(target=lambda: eng.prefill_append(s, toks, 0, layers, want_logits=False))
        th.start()
        time.sleep(0.004)
        bw = self.copy_bw(dm, nbytes=1 << 27, iters=6)
        th.join()
        eng.seq_free(s)
        return bw

    # ---- the sweep -----------------------------------------------------------------------
    def sweep_hardware(self, log=print):
        g, n = self.granule, self.n_cu
        cus = list(range(g, n + 1, g))
        bws = {c: self.copy_bw(c) for c in cus}
        d_peak = max(bws.values())
        n_d = next(c for c in cus if bws[c] >= 0.95 * d_peak)
        self.hw.update(d_peak=int(d_peak), n_d=n_d)
        log(f"copy bandwidth bytes/ns by CUs: { {c: round(b) for c, b in bws.items()} } -> D_peak {d_peak:.0f}, N_d {n_d}")
        self.measure_tile_model(bws, log)
        # compute peak: the largest prefill GEMM at full GPU
        self.eng.kernel_timing(True)
        self.eng.kernel_times(0, reset=True)
        t, layers = self.prefill_ns(n, 4096, layers=2, reps=1)
        kt = self.eng.kernel_times(0, reset=True)
        self.eng.kernel_timing(False)
        gu_ns, cnt = kt["gateup"]
        flop = 2 * 4096 * self.desc.hidden * 2 * self.desc.mlp
        c_peak = flop / (gu_ns / cnt)
        self.hw.update(c_peak=int(c_peak))
        log(f"gate/up GEMM at {n} CUs: {c_peak / 1e3:.0f} TFLOP/s -> C_peak {c_peak:.0f} flop/ns")
        return bws

    def measure_tile_model(self, bws, log=print):
        """What the engine's GEMM tile choice needs to know about the part: the rate of a busy CU with each
        prefill tile shape (the gate/up product on whole waves of tiles, on the partition prefill usually
        gets: all CUs but one granule) and the per-CU rate at which partial tiles are written and read
        back (the copy probe's). Stored in the profile and handed to the engine before alpha is calibrated."""
        cus = max(self.granule, self.n_cu - self.granule)
        m = min(2048, self.max_tokens) // 256 * 256
        d = self.desc
        if m:
            self.prefill_ns(cus, m, layers=1, reps=0)          # the probes run on what the workspace holds: real activations
        for key, name, tm, tn, per_cu in (("gemm_rate_128", "128x128", 128, 128, 2), ("gemm_rate_256", "256x256", 256, 256, 1)):
            slots, rows = per_cu * cus, m // tm if m else 0
            if not rows or slots % rows:
                continue
            per_wave = slots // rows * tn                      # weight rows that make one whole wave of tiles
            waves = min(4, 2 * d.mlp // per_wave)
            if waves < 1:
                continue                                       # a model too narrow to fill the partition: keep the default
            n = waves * per_wave
            ns = self.eng.probe_gemm(cus, name, m, n, iters=20) / 20
            rate = 2 * m * n * d.hidden / ns / cus             # GFLOP/s per busy CU
            self.hw[key] = int(rate)
            log(f"{name} tiles, {m} x {n} x {d.hidden} on {cus} CUs ({waves} whole waves): {ns / 1e3:.1f} us -> {rate / 1e3:.2f} TFLOP/s per busy CU")
        # 128x256 tiles run one per CU (the O and down projections: little more than one tile per CU), so a tile's start-up
        # and residual epilogue are exposed: time one wave of tiles of both projections and fit fixed + flops / rate
        rows = m // 128 if m else 0
        if rows and cus % rows == 0 and cus // rows * 256 <= d.hidden:
            n = cus // rows * 256
            qd = d.n_q_heads * d.head_dim
            t_o = self.eng.probe_gemm(cus, "128x256", m, n, iters=20, product="o") / 20
            t_d = self.eng.probe_gemm(cus, "128x256", m, n, iters=20, product="down") / 20
            if d.mlp > qd and t_d > t_o:
                rate = 2 * 128 * 256 * (d.mlp - qd) / (t_d - t_o)              # flop/ns = GFLOP/s of one CU
                fixed = max(0.0, t_o - 2 * 128 * 256 * qd / rate)
                self.hw["gemm_rate_128x256"], self.hw["gemm_fixed_128x256"] = int(rate), int(fixed)
                log(f"128x256 tiles, one per CU on {cus} CUs, {m} x {n}: K = {qd} {t_o / 1e3:.1f} us, K = {d.mlp} {t_d / 1e3:.1f} us -> "
                    f"{fixed / 1e3:.1f} us + flops at {rate / 1e3:.2f} TFLOP/s per CU")
        self.hw["partial_bw_cu"] = int(bws[cus] / cus * 1e3)
        log(f"partial tiles: {self.hw['partial_bw_cu'] / 1e3:.1f} GB/s per CU (copy probe on {cus} CUs)")
        self.eng.set_tile_model(self.hw["gemm_rate_128"], self.hw["gemm_rate_256"], self.hw["gemm_rate_128x256"], self.hw["gemm_fixed_128x256"],
                                self.hw["partial_bw_cu"])
        # what a read-only stream reaches on a small decode partition (per CU) and on the whole GPU: the decode GEMM planner's rates
        small = min(32, self.n_cu)
        nbytes, iters = 512 << 20, 5
        per_cu = nbytes * iters / self.eng.probe_read(1, small, nbytes, iters) / small * 1e3          # bytes/ns -> MB/s, per CU
        whole = nbytes * iters / self.eng.probe_read(1, self.n_cu, nbytes, iters) * 1e3
        self.hw["stream_bw_cu"], self.hw["stream_bw_gpu"] = int(per_cu), int(max(whole, per_cu))
        log(f"read-only stream: {per_cu / 1e3:.1f} GB/s per CU on {small} CUs, {whole / 1e6:.2f} TB/s on {self.n_cu} CUs")
        self.eng.set_stream_model(self.hw["stream_bw_cu"], self.hw["stream_bw_gpu"])

    def sweep_contention(self, dms=(32, 64, 128, 192), sls=(0, 2048, 8192), log=print):
        vals = [[int(self.corun_copy_bw(dm, sl)) for sl in sls] for dm in dms]
        # a full-GPU decode never co-runs: repeat the solo figure
        full = int(self.copy_bw(self.n_cu))
        dms = list(dms) + [self.n_cu]
        vals.append([full] * len(sls))
        self.grids["bw"] = ([dms, list(sls)], vals)
        log(f"D_p,sl bytes/ns (rows: decode CUs {dms}, cols: co-running prefill tokens {list(sls)}): {vals}")

    def prefill_host_ns(self, tokens, layers=4, reps=3):
        """Host-clock time of a prefill slice on the prefill CUs in force (usable while decode runs)."""
        eng = self.eng
        layers = min(layers, self.desc.n_layers)
        toks = synth.tokens(3, tokens, self.desc.vocab)
        best = None
        for _ in range(reps + 1):
            s = eng.seq_create()
            t0 = time.perf_counter_ns()
            eng.prefill_launch([s], [toks], 0, layers, want_logits=False)
            while not eng.phase_done(0):
                time.sleep(10e-6)
            eng.prefill_finish()
            t = time.perf_counter_ns() - t0
            if layers < self.desc.n_layers:
                eng.prefill_abort()
            eng.seq_free(s)
            best = t if best is None else min(best, t)
        return best

    def sweep_prefill_corun(self, dms=(32, 64, 128, 192), tokens=2048, batch=64, ctx=1024, log=print):
        """Slowdown of a prefill slice on n - dm CUs while decode steps of a resident batch run back to
        back on the other dm CUs, against the same slice alone (both on the host clock)."""
        eng, n = self.eng, self.n_cu
        vals = [PPM]
        for dm in dms:
            eng.set_partition(n - dm, dm)
            alone = self.prefill_host_ns(tokens)
            seqs = self.make_decode_batch([ctx] * batch)
            dtoks = synth.tokens(4, batch, self.desc.vocab)
            stop = [False]

            def decode_loop():
                while not stop[0]:
                    eng.decode_step(seqs, dtoks, want_logits=False, want_next=True)
            th = threading.Thread(target=decode_loop)
            th.start()
            time.sleep(0.03)
            beside = self.prefill_host_ns(tokens)
            stop[0] = True
            th.join()
            for s in seqs:
                eng.seq_free(s)
            vals.append(max(PPM, beside * PPM // max(alone, 1)))
            log(f"prefill slice ({tokens} tokens, 4 layers) on {n - dm} CUs: alone {alone / 1e6:.3f} ms, beside decode on {dm} CUs {beside / 1e6:.3f} ms "
                f"-> x{vals[-1] / PPM:.3f}")
        eng.set_partition(n, n)
        self.grids["prefill_corun"] = ([[0] + list(dms)], vals)

    def _roofline(self, es):
        text = profile_text(self.hw, {k: v for k, v in self.grids.items() if k == "bw"})
        return sts.Profile(text=text).query(self.desc, es, roofline=True)

    def calibrate_prefill(self, pms=(32, 64, 96, 128, 160, 192, 224, 256), tokens=(256, 512, 1024, 2048, 4096, 8192), log=print):
        vals = []
        for pm in pms:
            row = []
            for t in tokens:
                ns, layers = self.prefill_ns(pm, t)
                es = dict(prefill_len=[t], prefill_ctx=[0], prefill_cus=pm, decode_cus=0, layer_begin=0, n_layers_step=layers)
                if layers >= self.desc.n_layers:
                    es["n_layers_step"] = self.desc.n_layers
                roof = self._roofline(es)[0]
                # slices that stop before the last layer carry no LM head in the roofline either
                row.append(max(1, ns * PPM // max(roof, 1)))
            vals.append(row)
            log(f"alpha_prefill pm={pm}: {[round(v / PPM, 3) for v in row]}")
        self.grids["alpha_prefill"] = ([list(pms), list(tokens)], vals)

    def calibrate_decode(self, dms=(32, 64, 128, 256), batches=(8, 64, 224), mean_ctx=(256, 2048), log=print):
        vals = np.zeros((len(dms), len(batches), len(mean_ctx)), dtype=np.int64)
        ctx_axis = None
        for bi, b in enumerate(batches):
            for ci, mc in enumerate(mean_ctx):
                ctxs = [mc] * b
                seqs = self.make_decode_batch(ctxs)
                for di, dm in enumerate(dms):
                    ns = self.decode_ns(dm, seqs)
                    cur = [self.eng.seq_length(s) for s in seqs]
                    es = dict(decode_ctx=cur, decode_cus=dm, prefill_cus=0)
                    roof = self._roofline(es)[1]
                    vals[di, bi, ci] = max(1, ns * PPM // max(roof, 1))
                for s in seqs:
                    self.eng.seq_free(s)
        self.grids["alpha_decode"] = ([list(dms), list(batches), [int(mc) for mc in mean_ctx]], vals.tolist())
        for di, dm in enumerate(dms):
            log(f"alpha_decode dm={dm}: {np.round(vals[di] / PPM, 3).tolist()}")

    def text(self):
        return profile_text(self.hw, self.grids)


def measure_heldout(profiler: Profiler, n_prefill=24, n_decode=16, seed=11, step=None, log=print):
    """Measured latencies of seeded execution states that are not calibration samples: a list of
    (phase, execution state, measured ns). CU counts are multiples of `step` (default: the
    scheduler's granule, the only counts Algorithm 1 can choose)."""
    rng = np.random.default_rng(seed)
    desc, n = profiler.desc, profiler.n_cu
    step = step or profiler.granule
    out = []
    on_grid = step % profiler.granule == 0
    fixed_p = [(96, 700), (160, 1536), (224, 3000), (256, 6000), (64, 5000), (128, 384), (192, 1300)] if on_grid else []
    rand_p = [(int(rng.integers(32 // step, n // step + 1)) * step, int(rng.integers(200, 8000))) for _ in range(max(0, n_prefill - len(fixed_p)))]
    for pm, t in fixed_p + rand_p:
        ns, layers = profiler.prefill_ns(pm, t)
        es = dict(prefill_len=[t], prefill_ctx=[0], prefill_cus=pm, decode_cus=0, layer_begin=0, n_layers_step=layers)
        out.append(("prefill", es, ns))
        log(f"held-out prefill pm={pm} tokens={t}: measured {ns / 1e6:.3f} ms")
    fixed_d = [(96, 32, 1024), (160, 16, 512), (224, 48, 1500), (64, 64, 700), (256, 24, 3000), (32, 150, 900), (64, 200, 600),
               (128, 120, 1200)] if on_grid else []
    rand_d = [(int(rng.integers(32 // step, n // step + 1)) * step, int(rng.integers(4, 65)), int(rng.integers(200, 3000)))
              for _ in range(max(0, n_decode - len(fixed_d)))]
    for dm, b, mc in fixed_d + rand_d:
        r2 = np.random.default_rng(b)
        ctxs = np.clip(r2.normal(mc, mc / 4, b), 16, 8000).astype(int)
        seqs = profiler.make_decode_batch(ctxs)
        ns = profiler.decode_ns(dm, seqs)
        es = dict(decode_ctx=[profiler.eng.seq_length(s) for s in seqs], decode_cus=dm, prefill_cus=0)
        out.append(("decode", es, ns))
        log(f"held-out decode dm={dm} batch={b} mean ctx={mc}: measured {ns / 1e6:.3f} ms")
        for s in seqs:
            profiler.eng.seq_free(s)
    return out


def score(prof_text, desc, heldout, log=None):
    """MAPE of a profile's predictions on the held-out states: (prefill, decode)."""
    p = sts.Profile(text=prof_text)
    errs = {"prefill": [], "decode": []}
    for phase, es, ns in heldout:
        pred = p.query(desc, es)[0 if phase == "prefill" else 1]
        errs[phase].append(abs(pred - ns) / ns)
        if log:
            log(f"{phase} {({k: v for k, v in es.items() if k in ('prefill_len', 'prefill_cus', 'decode_cus')})}"
                f"{' batch ' + str(len(es['decode_ctx'])) if phase == 'decode' else ''}: measured {ns / 1e6:.3f} ms predicted {pred / 1e6:.3f} ms")
    return float(np.mean(errs["prefill"])) if errs["prefill"] else 0.0, float(np.mean(errs["decode"])) if errs["decode"] else 0.0


def subsample(grid, keep):
    """A calibration grid restricted to the axis positions in keep (one index list per axis)."""
    axes, values = grid
    v = np.asarray(values)
    for ax, idx in enumerate(keep):
        v = np.take(v, idx, axis=ax)
    return [[axes[a][i] for i in idx] for a, idx in enumerate(keep)], v.tolist()


def sample_count_study(profiler: Profiler, heldout, log=print):
    """Accuracy against the number of calibration samples (the experiment of Table 2): profiles built
    from subsets of the measured alpha grids, scored on the same held-out states; the small subsets
    leave the larger held-out states outside their range (extrapolation)."""
    gp, gd = profiler.grids["alpha_prefill"], profiler.grids["alpha_decode"]
    npm, nt = len(gp[0][0]), len(gp[0][1])
    ndm, nb, nc = len(gd[0][0]), len(gd[0][1]), len(gd[0][2])
    every = lambda n, k: sorted(set(list(range(0, n, k)) + [n - 1]))
    p_sets = [("ends of the CU axis, tokens <= %d" % gp[0][1][min(2, nt - 1)], [[0, npm - 1], list(range(min(3, nt)))]),
              ("every other CU count, tokens <= %d" % gp[0][1][min(3, nt - 1)], [every(npm, 2), list(range(min(4, nt)))]),
              ("full grid", [list(range(npm)), list(range(nt))])]
    d_sets = [("ends of the CU and batch axes", [[0, ndm - 1], sorted({0, nb - 1}), list(range(nc))]),
              ("full grid", [list(range(ndm)), list(range(nb)), list(range(nc))])]
    rows = []
    for name, keep in p_sets:
        grids = dict(profiler.grids, alpha_prefill=subsample(gp, keep))
        mp, _ = score(profile_text(profiler.hw, grids), profiler.desc, heldout)
        rows.append(("prefill", int(np.prod([len(k) for k in keep])), name, mp))
    for name, keep in d_sets:
        grids = dict(profiler.grids, alpha_decode=subsample(gd, keep))
        _, md = score(profile_text(profiler.hw, grids), profiler.desc, heldout)
        rows.append(("decode", int(np.prod([len(k) for k in keep])), name, md))
    for phase, cnt, name, m in rows:
        log(f"sample-count study: {phase} {cnt} samples ({name}): MAPE {100 * m:.1f} %")
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--model", default="8b", choices=["8b", "70b", "tiny"])
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--vocab", type=int, default=128256)
    ap.add_argument("--out", required=True)
    ap.add_argument("--report", default=None)
    args = ap.parse_args()
    desc = {"8b": synth.llama8b_model, "70b": synth.llama70b_model}.get(args.model, None)
    desc = desc(args.layers, args.vocab) if desc else synth.tiny_model()
    lines = []

    def log(msg):
        print(msg, flush=True)
        lines.append(msg)

    pr = Profiler(desc)
    pr.sweep_hardware(log)
    pr.sweep_contention(log=log)
    pr.sweep_prefill_corun(log=log)
    pr.calibrate_prefill(log=log)
    pr.calibrate_decode(log=log)
    text = pr.text()
    with open(args.out, "w") as f:
        f.write(text)
    heldout = measure_heldout(pr, log=log)
    mp, md = score(text, desc, heldout, log)
    log(f"MAPE on {len(heldout)} held-out execution states: prefill {100 * mp:.1f} %, decode {100 * md:.1f} %")
    sample_count_study(pr, heldout, log)
    # CU counts between the scheduler's grid points: the hardware deals workgroups to the shader engines of an
    # XCD, not to its enabled CUs, so a count that leaves the engines unequal runs the one-workgroup-per-CU
    # GEMMs in two rounds; Algorithm 1 never chooses such a count, the figure is reported for reference
    off = [h for h in measure_heldout(pr, n_prefill=10, n_decode=6, seed=12, step=8, log=log)
           if (h[1]["prefill_cus"] or h[1]["decode_cus"]) % pr.granule]
    mpo, mdo = score(text, desc, off, log)
    log(f"MAPE on {len(off)} execution states whose CU count is off the scheduler's grid: prefill {100 * mpo:.1f} %, decode {100 * mdo:.1f} %")
    if args.report:
        with open(args.report, "w") as f:
            f.write("\n".join(lines) + "\n")
    pr.close()


if __name__ == "__main__":
    main()
