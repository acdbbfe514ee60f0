"""Chunked prefill of one long prompt, chunk by chunk, on the whole GPU (paper Section 2.2.2).

A prompt of `--tokens` tokens is prefilled through all layers in chunks of cs tokens, each chunk
appended after the tokens already cached, so its attention re-reads them. Per chunk: device time,
the chunk's algorithmic flop (GEMMs 2*T*W per layer, attention 4*T*(p + (T+1)/2)*n_q*d per
layer) and the compute efficiency against the bf16 MFMA peak; per chunk size: last / first chunk
time, mean chunk time, total against the unchunked run. No decode requests are batched with the
chunks (the paper's figure makes the same simplification).

    python -m paper_2504_19516_amd.chunk_study --model 8b --tokens 16384 --chunks 512,1024,2048,4096 --out report.md
"""
from __future__ import annotations

import argparse

import numpy as np

from . import sts, synth

PEAK_FLOPS = 2.5e15          # MI355X dense bf16 MFMA


def chunk_flop(desc, t, p):
    qd, kvd = desc.n_q_heads * desc.head_dim, desc.n_kv_heads * desc.head_dim
    w = desc.hidden * (qd + 2 * kvd) + qd * desc.hidden + 3 * desc.hidden * desc.mlp
    return desc.n_layers * (2 * t * w + 4 * t * (p + (t + 1) / 2) * qd)


def run_chunks(eng, desc, tokens, cs, reps=2):
    """Per-chunk device times (ns, best of reps) of prefilling `tokens` in chunks of cs."""
    best = None
    for _ in range(reps):
        s = eng.seq_create()
        times = []
        for p in range(0, len(tokens), cs):
            eng.prefill_append(s, tokens[p:p + cs], 0, desc.n_layers, want_logits=False)
            times.append(eng.last_timing()[0])
        eng.seq_free(s)
        best = times if best is None else [min(a, b) for a, b in zip(best, times)]
    return best


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--model", default="8b", choices=["8b", "70b", "tiny"])
    ap.add_argument("--layers", type=int, default=0)
    ap.add_argument("--tokens", type=int, default=16384)
    ap.add_argument("--chunks", default="512,1024,2048,4096")
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
    make = {"8b": synth.llama8b_model, "70b": synth.llama70b_model}.get(args.model)
    desc = (make(args.layers) if args.layers else make()) if make else synth.tiny_model()
    n = args.tokens
    eng = sts.Engine(desc, weight_seed=1, init_weights=True, kv_pool_pages=2 * (n // 16) + 64, max_prefill_tokens=n, max_prefill_seqs=1,
                     max_decode_batch=8, max_seqs=8, max_pages_per_seq=n // 16 + 8)
    n_cu = eng.get_partition()[2]
    eng.set_partition(n_cu, n_cu)
    tokens = synth.tokens(5, n, desc.vocab)
    lines = [f"# Chunked prefill of one {n}-token prompt, {args.model} shape ({desc.n_layers} layers), whole GPU ({n_cu} CUs)", "",
             f"Command: `python -m paper_2504_19516_amd.chunk_study --model {args.model} --tokens {n} --chunks {args.chunks}`", "",
             "Efficiency = algorithmic flop of the chunk / device time / 2.5 PFLOP/s (dense bf16 MFMA peak).", ""]
    whole = run_chunks(eng, desc, tokens, n)[0]
    eff_whole = chunk_flop(desc, n, 0) / (whole * 1e-9) / PEAK_FLOPS
    lines += ["| chunk size | chunks | first chunk ms (eff.) | last chunk ms (eff.) | last / first | mean chunk ms | total ms | total / unchunked |",
              "|---|---|---|---|---|---|---|---|",
              f"| {n} (unchunked) | 1 | {whole / 1e6:.2f} ({100 * eff_whole:.1f} %) | | | {whole / 1e6:.2f} | {whole / 1e6:.2f} | 1.00 |"]
    curves = {}
    for cs in [int(x) for x in args.chunks.split(",")]:
        t = run_chunks(eng, desc, tokens, cs)
        eff = [chunk_flop(desc, min(cs, n - i * cs), i * cs) / (ns * 1e-9) / PEAK_FLOPS for i, ns in enumerate(t)]
        curves[cs] = (t, eff)
        lines.append(f"| {cs} | {len(t)} | {t[0] / 1e6:.2f} ({100 * eff[0]:.1f} %) | {t[-1] / 1e6:.2f} ({100 * eff[-1]:.1f} %) | {t[-1] / t[0]:.2f} | "
                     f"{np.mean(t) / 1e6:.2f} | {sum(t) / 1e6:.2f} | {sum(t) / whole:.3f} |")
    lines.append("")
    for cs, (t, eff) in curves.items():
        lines += [f"Chunk size {cs}: per-chunk ms " + " ".join(f"{x / 1e6:.2f}" for x in t),
                  f"Chunk size {cs}: per-chunk efficiency % " + " ".join(f"{100 * e:.1f}" for e in eff), ""]
    text = "\n".join(lines)
    print(text, flush=True)
    if args.out:
        with open(args.out, "w") as f:
            f.write(text + "\n")
    eng.close()


if __name__ == "__main__":
    main()
