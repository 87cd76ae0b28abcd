"""Parity of gs_verify_batch on models with 4-bit projection weights (GS_W4) against the oracle.

Both sides get the same synthetic 4-bit checkpoint (codes, scales, zeros per matrix).  The oracle dequantises
it by its own routine and runs the ordinary bf16 forward with the resulting weights; the GPU packs it with
gs_pack_weight_w4 and dequantises inside the projection kernel.  Same bars as the bf16 models: logits and
K/V rows within 2e-2 of the row scale, decisions teacher-forced on the GPU's logits.
"""
import dataclasses

import numpy as np
import pytest

from oracle import forward as fw
from oracle import quant
from paper_2512_09963_amd import synth
from tests.parity import check_accept_outputs
from tests.test_verify_gpu import TOL, _check_kv_rows, _oracle_cache, assert_logits_close

pytestmark = pytest.mark.gpu

MATS = ("wqkv", "wo", "wgu", "wd")


def _checkpoint(ms, seed, std):
    """(GPU side: triples, oracle side: dequantised float64) for the top and every layer."""
    top = synth.top_weights(ms, seed, std)
    lm = synth.quantize_w4(top["lm_head"])
    top_gpu = dict(top, lm_head=lm)
    top_ora = dict(top, lm_head=quant.dequant_w4(*lm))
    lay_gpu, lay_ora = [], []
    for l in range(ms.n_layers):
        W = synth.layer_weights(ms, seed, l, std)
        trip = {k: synth.quantize_w4(W[k]) for k in MATS}
        lay_gpu.append(dict(W, **trip))
        lay_ora.append(dict(W, **{k: quant.dequant_w4(*trip[k]) for k in MATS}))
    return top_gpu, lay_gpu, top_ora, lay_ora


def _run(ms, seed, gamma, ctx, std=0.08):
    import torch
    from paper_2512_09963_amd import workload as wl
    tol = TOL["bf16"]
    top_gpu, lay_gpu, top_ora, lay_ora = _checkpoint(ms, seed, std)
    batch = synth.make_batch(seed, gamma, ctx, 16, permute_pages=True)
    tokens, q, ua, ur = synth.verify_side_inputs(seed, ms.vocab, batch.gamma, sigma=0.5)
    cache = _oracle_cache(ms, seed, batch.n_pages, 16, True)
    ms_gpu = dataclasses.replace(ms, dtype="w4")
    ver = wl.upload_model(ms_gpu, top_gpu, lambda l: lay_gpu[l])
    kv = wl.KVCache(ms_gpu, batch.n_pages, 16)
    for l in range(ms.n_layers):
        kv.set_layer(l, cache[l][0], cache[l][1])
    db = wl.DeviceBatch(batch, tokens, q, ua, ur)
    out, logits, _ = wl.verify(ver, kv, db)
    torch.cuda.synchronize()
    got_logits = logits.cpu().numpy()
    want = fw.verify_forward(ms, tokens, batch.gamma, batch.ctx_len, batch.block_table, 16, top_ora,
                             lambda l: lay_ora[l], lambda l: cache[l])
    worst = assert_logits_close(got_logits, want, tol)
    _check_kv_rows(ms, kv, cache, batch, tol)
    got = {k: v.cpu().numpy() for k, v in out.items()}
    cu = batch.cu_rows
    d_tok = np.concatenate([tokens[cu[i] + 1:cu[i + 1]] for i in range(batch.n_servers)])
    bands = check_accept_outputs(batch.gamma, got_logits, q, d_tok, ua, ur, got)
    print("w4 worst logits error / scale:", worst, bands)


@pytest.mark.parametrize("gamma,ctx", [
    ([3, 1, 5], [20, 100, 7]),                            # 12 rows: one row tile
    ([8, 6, 5, 4, 4, 3, 5, 7], [300, 64, 0, 129, 31, 500, 17, 250]),    # 50 rows: the headline row count
    ([16, 12, 9, 15, 11, 14, 13, 10, 16, 12], [40, 0, 200, 90, 33, 150, 5, 260, 70, 128]),   # 138 rows: chunks of 64
])
def test_w4_model_matches_oracle(gamma, ctx):
    ms = synth.ModelShape(2, 256, 4, 2, 64, 384, 1024, 10000.0, dtype="bf16")
    _run(ms, 95, np.array(gamma, np.int32), np.array(ctx, np.int32))


def test_w4_wide_matrices_use_eight_waves():
    # N / 128 >= 192 for gate/up (2F = 24576) and the LM head: the 8-wave launch shape
    ms = synth.ModelShape(1, 128, 2, 1, 64, 12288, 24576, 10000.0, dtype="bf16")
    _run(ms, 96, np.array([4, 2], np.int32), np.array([10, 40], np.int32), std=0.05)


def test_w4_wide_matrices_with_more_than_64_rows():
    # 68 rows and N / 512 >= 96 for gate/up (2F = 49152) and the LM head: 8 waves with two column tiles each
    ms = synth.ModelShape(1, 128, 2, 1, 64, 24576, 49152, 10000.0, dtype="bf16")
    _run(ms, 97, np.array([16, 16, 16, 16], np.int32), np.array([10, 40, 0, 77], np.int32), std=0.05)


def test_w4_real_8b_widths():
    """The widths bench.py times with 4-bit weights: d 4096, QKV 6144, FFN 14336, vocab 128256, K up to 14336
    with its K splits; two layers, the 50 rows and 2048-token contexts of the headline configuration."""
    ms = dataclasses.replace(synth.LLAMA3_8B, n_layers=2)
    gamma = synth.uniform_int(synth.MASTER_SEED, ("cfg3", "gamma"), 3, 8, 8)
    _run(ms, 98, gamma, np.full(8, 2048, np.int32), std=0.02)


def test_w4_real_70b_widths():
    """d 8192, QKV 10240, FFN 28672 (K up to 28672), vocab 128256; one layer, 98 rows (the kernel shape with two
    column tiles per wave), 4096-token contexts."""
    ms = dataclasses.replace(synth.LLAMA3_70B, n_layers=1)
    gamma = synth.uniform_int(synth.MASTER_SEED, ("cfg5", "gamma"), 2, 8, 16)
    _run(ms, 99, gamma, np.full(16, 4096, np.int32), std=0.02)


def test_w4_shapes_are_validated():
    import torch
    from paper_2512_09963_amd import binding as gsb
    dev = torch.device("cuda:0")
    codes = torch.zeros(64, 192, dtype=torch.uint8, device=dev)
    with pytest.raises(gsb.GsError):
        gsb.gs_pack_weight_w4(codes, torch.zeros(64, 1, dtype=torch.bfloat16, device=dev),
                              torch.zeros(64, 1, dtype=torch.uint8, device=dev))
