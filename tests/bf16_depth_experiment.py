"""CPU-only experiment: how far do correct implementations of the same bfloat16-storage decoder drift apart?

Runs the verification forward of a model-scale configuration three times on the host, with no GPU code
involved: the float64 oracle (oracle/forward.py), a float32-accumulating implementation (tests/f32_forward.py)
and the same one with every projection summed in 8 K-chunks (another summation order).  All three round the
same tensors to bfloat16 at the same points.  After 1, 2, 4, ... layers the LM head is applied to each
residual stream and the largest |logit difference| / (largest |logit| of the row) is printed - the measure
the parity tests use ("2e-2 relative" read against the row scale).

    python -m tests.bf16_depth_experiment --config cfg3 --layers 32

The numbers decide which tolerance a free-running comparison of a deep bf16 stack can be held to.
"""
import argparse
import dataclasses
import json
import sys
import time

import numpy as np

from oracle import forward as fw
from paper_2512_09963_amd import synth
from tests import f32_forward as f32


def rel_to_row_scale(a, b):
    return float((np.abs(a - b) / np.abs(b).max(axis=1, keepdims=True)).max())


def rms_rel(a, b):
    return float(np.sqrt(np.mean((a - b) ** 2) / np.mean(b ** 2)))


def run(cfg_name="cfg3", n_layers=32, checkpoints=None, ms=None, log=print):
    make = {"cfg3": synth.config3, "cfg4": synth.config4, "cfg5": synth.config5}[cfg_name]
    base = ms or {"cfg3": synth.LLAMA3_8B, "cfg4": synth.LLAMA3_8B, "cfg5": synth.LLAMA3_70B}[cfg_name]
    ms = dataclasses.replace(base, n_layers=n_layers)
    cfg = make(ms=ms)
    b, seed = cfg.batch, cfg.seed
    checkpoints = checkpoints or sorted({d for d in (1, 2, 4, 8, 16, 32, 48, 64, 80) if d <= n_layers} | {n_layers})
    top = synth.top_weights(ms, seed)
    x64 = fw.embed_rows(top, cfg.tokens)
    xa = f32.embed(top, cfg.tokens)
    xb = xa.copy()
    args = (b.gamma, b.ctx_len, b.block_table, b.page_size)
    rows = []
    t0 = time.time()
    for l in range(n_layers):
        W = synth.layer_weights(ms, seed, l)
        kv = lambda which: synth.kv_layer_cache(ms, seed, l, which, b.n_pages, b.page_size)
        x64 = fw.layer_forward(ms, x64, W, kv("k").astype(np.float64), kv("v").astype(np.float64), *args)
        xa = f32.layer(ms, xa, W, kv("k"), kv("v"), *args)
        xb = f32.layer(ms, xb, W, kv("k"), kv("v"), *args, k_splits=8)
        del W
        if l + 1 in checkpoints:
            want = fw.lm_head(ms, x64, top)
            la, lb = f32.head(ms, xa, top), f32.head(ms, xb, top, k_splits=8)
            rec = {"layers": l + 1,
                   "f32_vs_f64": rel_to_row_scale(la, want), "f32split_vs_f64": rel_to_row_scale(lb, want),
                   "f32_vs_f32split": rel_to_row_scale(la, lb.astype(np.float64)),
                   "f32_vs_f64_rms": rms_rel(la, want)}
            rows.append(rec)
            log(json.dumps(rec) + f"  [{time.time() - t0:.0f} s]")
    return rows


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="cfg3", choices=["cfg3", "cfg4", "cfg5"])
    ap.add_argument("--layers", type=int, default=32)
    a = ap.parse_args()
    run(a.config, a.layers, log=lambda s: print(s, flush=True))
