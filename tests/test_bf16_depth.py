"""CPU only: the float32-accumulating forward of tests/f32_forward.py is the same function as the oracle's,
and under bfloat16 storage the two drift apart with depth (the evidence behind the depth-dependent bound of
the free-running comparison in tests/test_configs_gpu.py; the model-scale numbers come from
`python -m tests.bf16_depth_experiment`)."""
import dataclasses

import numpy as np

from oracle import forward as fw
from paper_2512_09963_amd import synth
from tests import f32_forward as f32

SHAPE = synth.ModelShape(8, 512, 8, 2, 64, 1536, 4096, 500000.0, dtype="bf16")


def _both(ms, seed=21):
    gamma, ctx = np.array([3, 0, 6, 2], np.int32), np.array([40, 7, 130, 64], np.int32)
    batch = synth.make_batch(seed, gamma, ctx, 16, permute_pages=True)
    tokens, _, _, _ = synth.verify_side_inputs(seed, ms.vocab, gamma)
    top = synth.top_weights(ms, seed, 0.04)
    args = (batch.gamma, batch.ctx_len, batch.block_table, batch.page_size)
    x64, x32 = fw.embed_rows(top, tokens), f32.embed(top, tokens)
    errs = []
    for l in range(ms.n_layers):
        W = synth.layer_weights(ms, seed, l, 0.04)
        kv = lambda which: synth.kv_layer_cache(ms, seed, l, which, batch.n_pages, 16)
        x64 = fw.layer_forward(ms, x64, W, kv("k").astype(np.float64), kv("v").astype(np.float64), *args)
        x32 = f32.layer(ms, x32, W, kv("k"), kv("v"), *args, k_splits=1 + l % 3)
        want, got = fw.lm_head(ms, x64, top), f32.head(ms, x32, top)
        errs.append(float((np.abs(got - want) / np.abs(want).max(axis=1, keepdims=True)).max()))
    return errs


def test_float32_forward_is_the_same_function_as_the_oracle():
    errs = _both(dataclasses.replace(SHAPE, n_layers=3, dtype="f32"))
    assert max(errs) < 2e-5, errs          # float32 sums against float64 sums, nothing else differs


def test_bf16_storage_makes_two_correct_forwards_drift_apart_with_depth():
    errs = _both(SHAPE)
    # one layer: already a sizeable fraction of a bfloat16 step (2^-8 = 3.9e-3) of the row scale, a hundred
    # times the float32 difference above; eight layers: clearly more, yet within the 2e-2 of a shallow stack
    assert 5e-4 < errs[0] < 8e-3, errs
    assert errs[7] > 1.5 * errs[0] and max(errs) < 2e-2, errs
