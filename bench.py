#!/usr/bin/env python3
"""Benchmark of the verification step on one MI355X.

A step is one pass of the whole hot path on one batch of synthetic input:
gs_verify_batch (decoder forward over the ragged blocks + rejection-verification),
the copy of the 3N result scalars to the host, and gs_schedule_gamma.

Workload (default): Llama-3-8B-shaped random-init bf16 decoder, 8 draft servers with
gamma drawn uniformly from [3, 8], 2048 cached tokens per server in 16-token pages.
Prints one JSON line; `value` is verified draft tokens per second (sum(gamma) / step time).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0   # dense bf16

# HBM bytes per projection launch from the FETCH_SIZE / WRITE_SIZE counter runs summarised in
# profiles/hbm_traffic_counters.md (121.79 MB fetched + 5.34 MB written, scaled by the copy-kernel factors
# given there).  Valid only for the kernel source it was taken with: reported as null once gemm.hip changes.
GEMM_TRAFFIC = {"gemm_hip_sha256": "def0d05baaf8661cf2cf8a42697f8573210332859236e6e404e9fda1c04617e1",
                "bytes_per_launch": 127128302}


def measured_traffic():
    import hashlib
    src = os.path.join(ROOT, "paper_2512_09963_amd", "csrc", "gemm.hip")
    try:
        h = hashlib.sha256(open(src, "rb").read()).hexdigest()
    except OSError:
        return None
    return GEMM_TRAFFIC["bytes_per_launch"] if h == GEMM_TRAFFIC["gemm_hip_sha256"] else None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--layers", type=int, default=0, help="debug only: fewer layers (result is marked invalid)")
    ap.add_argument("--workload", choices=["cfg3", "cfg4", "cfg5", "cfg3w4", "cfg5w4", "rows1024"], default="cfg3",
                    help="cfg3 (default) is the configuration the metric is quoted on; cfg4 (32 ragged servers, "
                         "paged) and cfg5 (70B shape) are extra measurements")
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--skip-accept-leg", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three 256 MiB device-to-device copies (reference dispatches for HBM byte counters)")
    return ap.parse_args()


WORKLOADS = {
    "cfg3": "llama3-8b-shaped verify (32 layers, d 4096, 32q/8kv heads, ffn 14336, vocab 128256), "
            "8 draft servers, gamma U[3,8], ctx 2048, 16-token KV pages",
    "cfg4": "llama3-8b-shaped verify, 32 draft servers, gamma U[1,16], ctx log-uniform [512,8192], "
            "permuted 16-token KV pages",
    "cfg5": "llama3-70b-shaped verify (80 layers, d 8192, 64q/8kv heads, ffn 28672, vocab 128256), "
            "16 draft servers, gamma U[2,8], ctx 4096",
    "cfg3w4": "cfg3 with 4-bit projection weights (groups of 128, synthetic checkpoint of the same random model); "
              "not the configuration the metric is quoted on",
    "cfg5w4": "cfg5 (70B shape) with 4-bit projection weights, the format family of the paper's larger verifier",
    "rows1024": "llama3-8b-shaped verify at a compute-bound row count: 8 servers x 128-row blocks on an empty "
                "cache (1024 target rows); not the paper's operating point, shows the projection kernel "
                "against the MFMA peak",
}


def build_workload(ms, seed, name="cfg3"):
    import torch
    from paper_2512_09963_amd import synth, workload as wl
    cfg = {"cfg3": synth.config3, "cfg4": synth.config4, "cfg5": synth.config5, "cfg3w4": synth.config3, "cfg5w4": synth.config5,
           "rows1024": synth.config_rows1024}[name](seed, ms)
    t0 = time.time()
    ver, kv, db = wl.upload_config(cfg, progress=True)
    torch.cuda.synchronize()
    print(f"[bench] weights + KV generated and uploaded in {time.time() - t0:.1f} s", file=sys.stderr, flush=True)
    return dict(ver=ver, kv=kv, db=db, batch=cfg.batch, tokens=cfg.tokens, q=cfg.q_probs, ua=cfg.u_accept,
                ur=cfg.u_resample)


def projection_weight_bytes(ms):
    """Bytes of all projection matrices as stored: 2 per weight for bf16; for the 4-bit format half a byte per
    weight plus one 4-byte word of scale and zero point per output row and group of 128 inputs."""
    per_layer = ms.qkv_out * ms.d_model + ms.d_model * ms.n_heads * ms.head_dim + 3 * ms.d_ffn * ms.d_model
    n_weights = ms.n_layers * per_layer + ms.vocab * ms.d_model
    if ms.dtype == "w4":
        return n_weights // 2 + n_weights // 128 * 4
    return 2 * n_weights


def run_steps(w, n_steps, sched):
    """n_steps full steps; returns list of host results of the last step."""
    import torch
    from paper_2512_09963_amd import binding as gsb, workload as wl
    db, ver, kv = w["db"], w["ver"], w["kv"]
    last = None
    for _ in range(n_steps):
        wl.verify(ver, kv, db, workspace=w["ws"], want_logits=False, out=w["out"])
        torch.cuda.current_stream().synchronize()     # the 3N result scalars land in pinned host memory
        m = w["host"]["accepted_len"].numpy()
        st = w["host"]["accept_stat"].numpy()
        last = gsb.gs_schedule_gamma(m, st, db.gamma, sched["alpha"], sched["X"], sched["eta"], sched["beta"],
                                     sched["C"], 0, -1)
    return last


def accept_leg(seed, bf16=False):
    """gs_accept_reject alone: 64 servers x gamma 8 over vocab 151936, sigma = 1 (bf16: the same inputs rounded
    to bfloat16 through gs_accept_reject_bf16, half the bytes)."""
    import torch
    from paper_2512_09963_amd import binding as gsb, synth
    dev = torch.device("cuda:0")
    N, g, V = 64, 8, 151936
    gamma = np.full(N, g, np.int32)
    inp = synth.accept_inputs(seed, gamma, V, 1.0)
    R, G = N * (g + 1), N * g
    wide = torch.bfloat16 if bf16 else torch.float32
    tl0 = torch.from_numpy(inp.target_logits).to(dev).to(wide)
    q0 = torch.from_numpy(inp.q_probs).to(dev).to(wide)
    tok0 = torch.from_numpy(inp.draft_tokens).to(dev)
    ua = torch.from_numpy(inp.u_accept).to(dev)
    ur = torch.from_numpy(inp.u_resample).to(dev)
    sets = []
    for k in range(5):   # rotated copies: 5 x 0.66 GB so that no cache level serves a repeat
        sh = 1000 * k
        sets.append((torch.roll(tl0, sh, 1).contiguous(), torch.roll(q0, sh, 1).contiguous(),
                     ((tok0 + sh) % V).int()))
    cu = torch.from_numpy(synth.cu_rows_of(gamma)).to(dev)
    out = gsb.make_accept_out(N, G, dev, want_ratio=False)
    ws = torch.empty(gsb.gs_accept_workspace_bytes(N, R, V), dtype=torch.uint8, device=dev)

    entry = gsb.gs_accept_reject_bf16 if bf16 else gsb.gs_accept_reject

    def call(k):
        tl, q, tok = sets[k % len(sets)]
        entry(gamma, cu, V, tl, q, tok, ua, ur, out, ws)

    for k in range(10):
        call(k)
    torch.cuda.synchronize()
    iters, n_rej = 100, 0
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for k in range(iters):
        call(k)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / iters
    n_rej = int((out["accepted_len"] < g).sum().item())
    alg = (2.0 if bf16 else 4.0) * V * (R + n_rej)
    gbs = alg / us / 1e3
    return {"workload": f"accept/reject+resample, 64 servers x gamma 8, vocab 151936, {'bf16' if bf16 else 'fp32'} inputs, sigma 1.0",
            "us_per_call": round(us, 2), "algorithmic_bytes": alg, "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4), "rejecting_servers": n_rej}


def plain_read_leg():
    """The practical ceiling of a read stream on this machine: gs_probe_stream_read over four rotated 1 GiB
    buffers (together far beyond every cache), 40 timed launches."""
    import torch
    from paper_2512_09963_amd import binding as gsb
    dev = torch.device("cuda:0")
    bufs = [torch.full((1 << 30,), k + 1, dtype=torch.uint8, device=dev) for k in range(4)]
    sink = torch.zeros(1 << 16, dtype=torch.uint8, device=dev)
    for k in range(8):
        gsb.gs_probe_stream_read(bufs[k % 4], sink)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    iters = 40
    e0.record()
    for k in range(iters):
        gsb.gs_probe_stream_read(bufs[k % 4], sink)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / iters
    gbs = (1 << 30) / us / 1e3
    return {"kernel": "stream_read_kernel (1 GiB per launch, 16-byte non-temporal loads)", "us_per_launch": round(us, 2),
            "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4)}


def cpu_baseline(ms, w, seed):
    """The oracle as it stands on the host cores, timed in full on the same workload: embedding, every decoder
    layer, final norm + LM head, softmax + accept/reject + resample.  Weights and cache contents are generated
    layer by layer from the seed outside the timed sections (they are inputs, not part of the method)."""
    from oracle import accept_reject as ar, forward as fw
    from paper_2512_09963_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    batch = w["batch"]
    top = synth.top_weights(ms, seed)
    t_fwd = 0.0
    t0 = time.perf_counter()
    x = fw.embed_rows(top, w["tokens"])
    t_fwd += time.perf_counter() - t0
    for l in range(ms.n_layers):
        W = synth.layer_weights(ms, seed, l)
        k = synth.kv_layer_cache(ms, seed, l, "k", batch.n_pages, batch.page_size)
        v = synth.kv_layer_cache(ms, seed, l, "v", batch.n_pages, batch.page_size)
        t0 = time.perf_counter()
        x = fw.layer_forward(ms, x, W, k, v, batch.gamma, batch.ctx_len, batch.block_table, batch.page_size)
        t_fwd += time.perf_counter() - t0
        del W, k, v
        if (l + 1) % 8 == 0:
            print(f"[bench] cpu baseline: oracle layer {l + 1}/{ms.n_layers}", file=sys.stderr, flush=True)
    t0 = time.perf_counter()
    logits = fw.lm_head(ms, x, top)
    t_fwd += time.perf_counter() - t0
    cu = batch.cu_rows
    d_tok = np.concatenate([w["tokens"][cu[i] + 1:cu[i + 1]] for i in range(batch.n_servers)])
    t0 = time.perf_counter()
    ar.accept_reject(batch.gamma, logits.astype(np.float32), w["q"], d_tok, w["ua"], w["ur"])
    t_acc = time.perf_counter() - t0
    total = t_fwd + t_acc
    return {"value": round(batch.n_draft / total, 3), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"one whole step of the same workload, timed in full: forward oracle over all {ms.n_layers} "
                      f"layers + LM head {t_fwd:.1f} s, accept stage {t_acc:.2f} s (weights and cache contents "
                      f"regenerated from the seed outside the timed sections)"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (no collectives, no sharding)", file=sys.stderr)
        sys.exit(2)
    import dataclasses
    import torch
    from paper_2512_09963_amd import binding as gsb, synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    gsb.lib()
    seed = synth.MASTER_SEED
    ms = synth.LLAMA3_70B if args.workload in ("cfg5", "cfg5w4") else synth.LLAMA3_8B
    if args.workload in ("cfg3w4", "cfg5w4"):
        ms = dataclasses.replace(ms, dtype="w4")
    if args.layers:
        ms = dataclasses.replace(ms, n_layers=args.layers)
    w = build_workload(ms, seed, args.workload)
    db, ver = w["db"], w["ver"]
    dev = torch.device("cuda:0")
    w["ws"] = torch.empty(ver.gs_workspace_bytes(db.n_rows, db.n_servers, db.max_ctx), dtype=torch.uint8, device=dev)
    # the kernels store the 3N result scalars straight into pinned (device-mapped) host memory: the host
    # scheduler reads them after the stream synchronisation, no copy is enqueued
    w["host"] = {"accepted_len": torch.zeros(db.n_servers, dtype=torch.int32, pin_memory=True),
                 "next_token": torch.zeros(db.n_servers, dtype=torch.int32, pin_memory=True),
                 "accept_stat": torch.zeros(db.n_servers, dtype=torch.float32, pin_memory=True)}
    w["out"] = dict(w["host"], ratio=None)
    sched = dict(alpha=np.full(db.n_servers, 0.5), X=np.ones(db.n_servers), eta=0.2, beta=0.5, C=int(db.n_draft))

    # timed region: K full steps, no instrumentation
    run_steps(w, args.warmup, sched)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(w, args.steps, sched)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # the same K steps again with a pair of HIP events around every stage on the launch stream:
    # per-kernel durations for the roofline (the event records themselves slow the step down,
    # which is why this pass is not the one that is timed)
    ver.gs_profile_enable(True)
    run_steps(w, args.steps, sched)
    torch.cuda.synchronize()
    stages = ver.gs_profile_read()
    ver.gs_profile_enable(False)
    # what an event pair measures with nothing between its two records (the bracket's own cost)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(200)]
    for a, b in pairs:
        a.record()
        b.record()
    torch.cuda.synchronize()
    pair_us = sorted(a.elapsed_time(b) * 1e3 for a, b in pairs)[len(pairs) // 2]

    ms_step = dt * 1e3 / args.steps
    emitted = float(w["host"]["accepted_len"].sum().item() + db.n_servers)
    gemm_ms, gemm_launches = stages["gemm"]
    w_bytes = projection_weight_bytes(ms)
    gemm_us_raw = gemm_ms * 1e3 / gemm_launches
    # What a bracket adds to the launch it times: the brackets of a step tile its timeline, so their sum
    # exceeds the un-instrumented step time by (brackets per step) x (cost of one bracket).  Subtracting
    # that cost gives the launch's duration inside the running step (launch ramp and drain included),
    # which is also what a kernel trace of the same command reports per dispatch.  (An event pair with
    # nothing between its records costs more than that, pair_us: most of it overlaps the kernel's own ramp.)
    n_brackets = sum(v[1] for v in stages.values()) / args.steps
    bracket_us = max(0.0, (sum(v[0] for v in stages.values()) / args.steps - ms_step) * 1e3 / n_brackets)
    gemm_us = gemm_us_raw - bracket_us
    achieved = w_bytes / (gemm_launches / args.steps) / (gemm_us * 1e-6) / 1e9
    res = {
        "metric": "verified_tokens_per_s", "value": round(db.n_draft / (ms_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 (4-bit weights)" if ms.dtype == "w4" else "bf16", "data": "synthetic",
        "config": {"workload": WORKLOADS[args.workload],
                   "n_servers": db.n_servers, "draft_tokens": db.n_draft, "target_rows": db.n_rows,
                   "gamma": [int(g) for g in db.gamma]},
        "emitted_tokens_per_s": round(emitted / (ms_step * 1e-3), 1),
        "roofline": {"kernel": "gemm_bf16 (all projections of a step)", "bound": "hbm",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": measured_traffic() if args.workload == "cfg3" else None,
                     "bytes_per_launch": round(w_bytes / (gemm_launches / args.steps)),
                     "us_per_launch": round(gemm_us, 2), "us_per_launch_event_bracket": round(gemm_us_raw, 2),
                     "bracket_overhead_us": round(bracket_us, 2), "empty_event_pair_us": round(pair_us, 2)},
        "stage_ms_per_step": {k: round(v[0] / args.steps, 4) for k, v in stages.items()},
    }
    if args.workload == "rows1024":     # the projections are bound by the MFMA pipes at this row count
        flops = w_bytes * db.n_rows     # 2 flops per weight and row, 2 bytes per weight
        tflops = flops / (gemm_launches / args.steps) / (gemm_us * 1e-6) / 1e12
        res["roofline"].update({"bound": "mfma", "achieved": round(tflops, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                                "unit": "TFLOP/s", "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4)})
    if args.layers:
        res["invalid"] = "debug run with fewer layers"
    if args.calibrate_copy:
        src = torch.full((256 << 20,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    if not args.skip_accept_leg and args.workload == "cfg3":
        res["accept_kernel"] = accept_leg(seed)
        res["accept_kernel_bf16_inputs"] = accept_leg(seed, bf16=True)
        res["plain_read_ceiling"] = plain_read_leg()
    if not args.skip_cpu_baseline and args.workload == "cfg3":
        res["cpu_baseline"] = cpu_baseline(ms, w, seed)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
