"""Device-side assembly of synthetic workloads for the C-ABI entry points (torch for memory only).

Takes the numpy inputs made by `synth`, uploads them in the layouts the library
documents, and wraps the calls.  No arithmetic of the method happens here.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as gsb
from . import synth


def _dev():
    return torch.device("cuda:0")


def storage_dtype(ms: synth.ModelShape):
    """Storage type of activations, KV pages and the embedding table."""
    return torch.float32 if ms.dtype == "f32" else torch.bfloat16


def to_device(a, dtype):
    if isinstance(a, torch.Tensor):
        return a.to(_dev()).to(dtype)
    return torch.from_numpy(np.ascontiguousarray(a)).to(_dev()).to(dtype)


def _progress(msg, sink=True):
    """Progress line of a long upload: to `sink` if it is callable, else to stderr."""
    if callable(sink):
        sink(msg)
        return
    import sys
    print(msg, file=sys.stderr, flush=True)


def upload_model(ms: synth.ModelShape, top: dict, get_layer, progress=False):
    """Returns a binding.Verifier for weights given as float32 numpy arrays (for ms.dtype "w4" the projection
    matrices are given as (codes, scales, zeros) triples instead).  progress: False, True (lines to stderr) or a
    callable that takes the line."""
    dt = storage_dtype(ms)
    if ms.dtype == "w4":
        # a projection matrix arrives as a 4-bit checkpoint triple (codes, scales, zeros), see synth.quantize_w4
        def packed(t):
            codes, scales, zeros = t
            return gsb.gs_pack_weight_w4(to_device(codes, torch.uint8), to_device(scales, torch.bfloat16),
                                         to_device(zeros, torch.uint8))
    else:
        packed = lambda a: gsb.gs_pack_weight(to_device(a, dt))      # the row-major upload is dropped after the repack
    top_d = {"embed": to_device(top["embed"], dt), "lm_head": packed(top["lm_head"]),
             "final_norm": to_device(top["final_norm"], torch.float32)}
    layers = []
    for l in range(ms.n_layers):
        W = get_layer(l)
        layers.append({k: packed(W[k]) for k in ("wqkv", "wo", "wgu", "wd")} |
                      {k: to_device(W[k], torch.float32) for k in ("norm1", "norm2")})
        if progress and (l + 1) % 8 == 0:
            _progress(f"[workload] uploaded {l + 1}/{ms.n_layers} layers", progress)
    desc = dict(n_layers=ms.n_layers, d_model=ms.d_model, n_heads=ms.n_heads, n_kv_heads=ms.n_kv_heads,
                head_dim=ms.head_dim, d_ffn=ms.d_ffn, vocab=ms.vocab, rope_theta=ms.rope_theta, rms_eps=ms.rms_eps,
                dtype=ms.dtype)
    return gsb.Verifier(desc, top_d, layers)


class KVCache:
    """K pages [layers][pages][H_kv][slot][hd] and V pages [layers][pages][H_kv][hd][slot] on the device."""

    def __init__(self, ms: synth.ModelShape, n_pages, page_size, zero=True):
        dt = storage_dtype(ms)
        shape_k = (ms.n_layers, n_pages, ms.n_kv_heads, page_size, ms.head_dim)
        shape_v = (ms.n_layers, n_pages, ms.n_kv_heads, ms.head_dim, page_size)
        make = torch.zeros if zero else torch.empty
        self.k = make(shape_k, dtype=dt, device=_dev())
        self.v = make(shape_v, dtype=dt, device=_dev())
        self.page_size, self.n_pages = page_size, n_pages

    def set_layer(self, layer, k_np, v_np):
        """k_np, v_np: [pages][H_kv][slot][hd] float32 arrays (the slot-major layout on both)."""
        self.k[layer].copy_(torch.from_numpy(k_np).to(self.k.dtype))
        self.v[layer].copy_(torch.from_numpy(np.ascontiguousarray(v_np)).to(self.v.dtype).transpose(2, 3))

    def get_layer(self, layer):
        """Slot-major float32 numpy copies [pages][H_kv][slot][hd] of both caches."""
        return (self.k[layer].float().cpu().numpy(),
                self.v[layer].transpose(2, 3).float().cpu().numpy())


class DeviceBatch:
    """Device copies of one ragged batch descriptor plus its draft-side inputs."""

    def __init__(self, batch: synth.BatchShape, tokens, q_probs=None, u_accept=None, u_resample=None):
        d = _dev()
        self.gamma = np.ascontiguousarray(batch.gamma, dtype=np.int32)
        self.ctx_len_host = np.ascontiguousarray(batch.ctx_len, dtype=np.int32)
        self.cu_rows = torch.from_numpy(batch.cu_rows).to(d)
        self.ctx_len = torch.from_numpy(self.ctx_len_host).to(d)
        self.block_table = torch.from_numpy(np.ascontiguousarray(batch.block_table, dtype=np.int32)).to(d)
        self.tokens = torch.from_numpy(np.ascontiguousarray(tokens, dtype=np.int32)).to(d)
        f = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(d)
        self.q_probs, self.u_accept, self.u_resample = f(q_probs), f(u_accept), f(u_resample)
        self.n_rows, self.n_draft, self.n_servers = batch.n_rows, batch.n_draft, batch.n_servers
        self.max_ctx = int((batch.ctx_len + batch.gamma + 1).max())


def verify(ver: gsb.Verifier, kv: KVCache, db: DeviceBatch, workspace=None, want_logits=True, out=None, stream=None):
    """Calls gs_verify_batch; returns (out dict or None, logits tensor or None, workspace)."""
    V = ver.desc["vocab"]
    if workspace is None:
        workspace = torch.empty(ver.gs_workspace_bytes(db.n_rows, db.n_servers, db.max_ctx), dtype=torch.uint8,
                                device=_dev())
    logits = torch.empty(db.n_rows, V, dtype=torch.float32, device=_dev()) if want_logits else None
    if db.q_probs is not None and out is None:
        out = gsb.make_accept_out(db.n_servers, db.n_draft, _dev())
    ver.gs_verify_batch(kv.k, kv.v, kv.page_size, kv.n_pages, db.gamma, db.ctx_len_host, db.cu_rows, db.ctx_len,
                        db.tokens, db.block_table, db.q_probs, db.u_accept, db.u_resample, out, logits, workspace,
                        stream)
    return out, logits, workspace


def quantize_w4_device(w):
    """synth.quantize_w4 with torch ops on the device (same float32 arithmetic, so the same checkpoint):
    used for full-size synthetic models, where the host version takes minutes.  w: float32 numpy [N, K]."""
    g = synth.W4_GROUP
    t = torch.from_numpy(np.ascontiguousarray(w, dtype=np.float32)).to(_dev())
    n, k = t.shape
    tg = t.view(n, k // g, g)
    lo = torch.clamp(tg.amin(dim=2), max=0.0)
    hi = torch.clamp(tg.amax(dim=2), min=0.0)
    scale = ((hi - lo) / 15.0).to(torch.bfloat16).to(torch.float32)
    scale = torch.where(scale > 0, scale, torch.ones_like(scale))
    zero = torch.clamp(torch.round(-lo / scale), 0, 15)
    codes = torch.clamp(torch.round(tg / scale[:, :, None]) + zero[:, :, None], 0, 15)
    return codes.view(n, k).to(torch.uint8), scale, zero.to(torch.uint8)


def upload_config(cfg: synth.VerifyConfig, ver=None, progress=False):
    """Device side of a synth.VerifyConfig: model (random init from the seed), synthetic KV, batch.
    For ms.dtype "w4" the random bf16 matrices are turned into a synthetic 4-bit checkpoint first."""
    import dataclasses
    ms, seed, batch = cfg.ms, cfg.seed, cfg.batch
    gen = dataclasses.replace(ms, dtype="bf16") if ms.dtype == "w4" else ms      # what the generators see
    if ver is None:
        top = synth.top_weights(gen, seed)
        if ms.dtype == "w4":
            def quantized(W):
                return {k: (quantize_w4_device(v) if k in ("wqkv", "wo", "wgu", "wd", "lm_head") else v)
                        for k, v in W.items()}
            ver = upload_model(ms, quantized(top), lambda l: quantized(synth.layer_weights(gen, seed, l)), progress)
        else:
            ver = upload_model(ms, top, lambda l: synth.layer_weights(ms, seed, l), progress)
        del top
    kv = KVCache(ms, batch.n_pages, batch.page_size, zero=False)
    for l in range(ms.n_layers):
        kv.set_layer(l, synth.kv_layer_cache(gen, seed, l, "k", batch.n_pages, batch.page_size),
                     synth.kv_layer_cache(gen, seed, l, "v", batch.n_pages, batch.page_size))
        if progress and (l + 1) % 16 == 0:
            _progress(f"[workload] KV of {l + 1}/{ms.n_layers} layers in place", progress)
    db = DeviceBatch(batch, cfg.tokens, cfg.q_probs, cfg.u_accept, cfg.u_resample)
    return ver, kv, db
