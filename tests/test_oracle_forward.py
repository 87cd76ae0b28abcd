"""Pins of the forward oracle: library special cases, closed forms and invariants."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import forward as fw
from paper_2512_09963_amd import synth


def _small_model(dtype="f32", n_kv=2):
    return synth.ModelShape(2, 64, 4, n_kv, 16, 96, 50, rope_theta=10000.0, dtype=dtype)


def _weights(ms, seed=5):
    top = synth.top_weights(ms, seed)
    layers = [synth.layer_weights(ms, seed, l) for l in range(ms.n_layers)]
    rng = np.random.default_rng(seed)
    for W in layers:                      # non-trivial norm weights so a dropped weight shows
        W["norm1"] = rng.uniform(0.5, 1.5, ms.d_model).astype(np.float32)
        W["norm2"] = rng.uniform(0.5, 1.5, ms.d_model).astype(np.float32)
        for k in ("wqkv", "wo", "wgu", "wd"):
            W[k] = (W[k] * 8).astype(np.float32)   # larger weights: attention far from uniform
    top["final_norm"] = rng.uniform(0.5, 1.5, ms.d_model).astype(np.float32)
    return top, layers


def _empty_cache(ms, n_pages, page):
    return [(np.zeros((n_pages, ms.n_kv_heads, page, ms.head_dim)),
             np.zeros((n_pages, ms.n_kv_heads, page, ms.head_dim))) for _ in range(ms.n_layers)]


def _run(ms, top, layers, tokens, gamma, ctx, bt, page, cache):
    return fw.verify_forward(ms, tokens, gamma, ctx, bt, page, top, lambda l: layers[l], lambda l: cache[l])


def _torch_dense_logits(ms, top, layers, seq):
    """Whole-sequence dense causal decoder from torch library ops (float64)."""
    t = lambda a: torch.tensor(np.asarray(a), dtype=torch.float64)
    H, Hk, hd = ms.n_heads, ms.n_kv_heads, ms.head_dim
    x = t(top["embed"])[torch.tensor(seq)]
    n = len(seq)
    pos = torch.arange(n, dtype=torch.float64)
    inv = 1.0 / (ms.rope_theta ** (torch.arange(0, hd, 2, dtype=torch.float64) / hd))
    z = torch.polar(torch.ones(n, hd // 2, dtype=torch.float64), pos[:, None] * inv[None, :])   # e^{i pos w}

    def rot(v):                                # complex multiplication of the (i, i + hd/2) pairs
        c = torch.complex(v[..., : hd // 2], v[..., hd // 2:]) * z[:, None, :]
        return torch.cat([c.real, c.imag], dim=-1)

    for W in layers:
        h = F.rms_norm(x, (ms.d_model,), t(W["norm1"]), ms.rms_eps)
        qkv = F.linear(h, t(W["wqkv"]))
        q = rot(qkv[:, : H * hd].view(n, H, hd))
        k = rot(qkv[:, H * hd:(H + Hk) * hd].view(n, Hk, hd))
        v = qkv[:, (H + Hk) * hd:].view(n, Hk, hd)
        k = k.repeat_interleave(H // Hk, dim=1)
        v = v.repeat_interleave(H // Hk, dim=1)
        o = F.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1), v.transpose(0, 1), is_causal=True)
        x = x + F.linear(o.transpose(0, 1).reshape(n, H * hd), t(W["wo"]))
        h = F.rms_norm(x, (ms.d_model,), t(W["norm2"]), ms.rms_eps)
        gu = F.linear(h, t(W["wgu"]))
        x = x + F.linear(F.silu(gu[:, : ms.d_ffn]) * gu[:, ms.d_ffn:], t(W["wd"]))
    h = F.rms_norm(x, (ms.d_model,), t(top["final_norm"]), ms.rms_eps)
    return F.linear(h, t(top["lm_head"])).numpy()


@pytest.mark.parametrize("n_kv", [4, 2, 1])
def test_paged_incremental_forward_equals_dense_library_decoder(n_kv):
    """Prefill 13 tokens into pages, then a 5-row block: the block's logits equal the
    last rows of a dense whole-sequence pass built from torch library routines."""
    ms = _small_model(n_kv=n_kv)
    top, layers = _weights(ms)
    rng = np.random.default_rng(0)
    seq = rng.integers(0, ms.vocab, 18).tolist()
    page = 4
    bt = np.array([[3, 0, 4, 1, 2]], dtype=np.int32)       # scrambled physical pages
    cache = _empty_cache(ms, 5, page)
    pre = _run(ms, top, layers, seq[:13], [12], [0], bt, page, cache)
    blk = _run(ms, top, layers, seq[13:], [4], [13], bt, page, cache)
    dense = _torch_dense_logits(ms, top, layers, seq)
    np.testing.assert_allclose(pre, dense[:13], rtol=1e-9, atol=1e-9)
    np.testing.assert_allclose(blk, dense[13:], rtol=1e-9, atol=1e-9)


def test_block_equals_sequential_single_token_steps_and_servers_are_independent():
    ms = _small_model()
    top, layers = _weights(ms, 9)
    rng = np.random.default_rng(1)
    page = 4
    gamma = np.array([3, 0, 2])
    ctx = np.array([5, 2, 7])
    batch = synth.make_batch(3, gamma, ctx, page, permute_pages=True)
    toks_ctx = [rng.integers(0, ms.vocab, c).tolist() for c in ctx]
    toks_blk = [rng.integers(0, ms.vocab, g + 1).tolist() for g in gamma]

    def prefilled():
        cache = _empty_cache(ms, batch.n_pages, page)
        for i in range(3):
            _run(ms, top, layers, toks_ctx[i], [ctx[i] - 1], [0], batch.block_table[i:i + 1], page, cache)
        return cache

    cache = prefilled()
    flat = sum(toks_blk, [])
    full = _run(ms, top, layers, flat, gamma, ctx, batch.block_table, page, cache)
    cu = synth.cu_rows_of(gamma)
    for i in range(3):
        c2 = prefilled()
        alone = _run(ms, top, layers, toks_blk[i], [gamma[i]], [ctx[i]], batch.block_table[i:i + 1], page, c2)
        np.testing.assert_allclose(full[cu[i]:cu[i + 1]], alone, rtol=1e-10, atol=1e-10)
        c3 = prefilled()
        for j, tok in enumerate(toks_blk[i]):
            one = _run(ms, top, layers, [tok], [0], [ctx[i] + j], batch.block_table[i:i + 1], page, c3)
            np.testing.assert_allclose(full[cu[i] + j], one[0], rtol=1e-10, atol=1e-10)


def test_rope_is_a_plane_rotation_and_scores_depend_on_relative_position():
    v = np.array([1.0, 0.0])                                       # hd = 2: a single pair, frequency 1
    np.testing.assert_allclose(fw.rope(v, 0.5, 10000.0), [np.cos(0.5), np.sin(0.5)], atol=1e-15)
    np.testing.assert_allclose(fw.rope(np.array([0.0, 1.0]), 0.5, 10000.0), [-np.sin(0.5), np.cos(0.5)], atol=1e-15)
    w = np.arange(8.0)                                             # hd = 8: pair i turns by pos * theta^(-2i/8)
    out = fw.rope(w, 3, 100.0)
    for i in range(4):
        ang = 3 * 100.0 ** (-2 * i / 8)
        np.testing.assert_allclose([out[i], out[i + 4]],
                                   [w[i] * np.cos(ang) - w[i + 4] * np.sin(ang), w[i + 4] * np.cos(ang) + w[i] * np.sin(ang)])
    rng = np.random.default_rng(2)
    a, b = rng.normal(size=16), rng.normal(size=16)
    s1 = fw.rope(a, 7, 500000.0) @ fw.rope(b, 3, 500000.0)
    s2 = fw.rope(a, 107, 500000.0) @ fw.rope(b, 103, 500000.0)
    assert s1 == pytest.approx(s2, abs=1e-10)
    assert np.linalg.norm(fw.rope(a, 11, 10000.0)) == pytest.approx(np.linalg.norm(a))


def test_rmsnorm_and_attention_closed_forms():
    rng = np.random.default_rng(3)
    x = rng.normal(size=(5, 32)) * 4
    y = fw.rmsnorm(x, np.ones(32), 0.0)
    np.testing.assert_allclose(np.sqrt((y * y).mean(-1)), 1.0)
    np.testing.assert_allclose(fw.rmsnorm(x, 2 * np.ones(32), 0.0), 2 * y)
    assert fw.silu(0.0) == 0.0 and fw.silu(20.0) == pytest.approx(20.0, rel=1e-8)
    assert fw.silu(1.0) == pytest.approx(1.0 / (1.0 + np.exp(-1.0)))
    # one cached key: the output is that key's value; identical keys: the mean of the visible values
    q = rng.normal(size=(2, 2, 8))
    k = np.tile(rng.normal(size=(1, 1, 8)), (1, 3, 1))
    v = rng.normal(size=(1, 3, 8))
    o = fw.attention_server(q, k, v, 1, 2, 1)
    np.testing.assert_allclose(o[0, 0], v[0, :2].mean(0)); np.testing.assert_allclose(o[1, 1], v[0, :3].mean(0))
    o1 = fw.attention_server(q[:1], k[:, :1], v[:, :1], 0, 2, 1)
    np.testing.assert_allclose(o1[0, 0], v[0, 0])
    # GQA: query head h reads KV head h // group
    k2 = rng.normal(size=(2, 1, 8)); v2 = rng.normal(size=(2, 1, 8))
    o2 = fw.attention_server(rng.normal(size=(1, 4, 8)), k2, v2, 0, 4, 2)
    np.testing.assert_allclose(o2[0, 1], v2[0, 0]); np.testing.assert_allclose(o2[0, 2], v2[1, 0])


def test_bf16_rounding_is_nearest_even():
    one = 1.0
    ulp = 2.0 ** -7
    vals = np.array([one + ulp / 2, one + 3 * ulp / 2, one + ulp / 2 + 2.0 ** -20, -(one + ulp / 2), 3.0e-5])
    got = fw.round_bf16(vals)
    np.testing.assert_array_equal(got[:4], [1.0, 1.0 + 2 * ulp, 1.0 + ulp, -1.0])
    assert got[4] == float(torch.tensor(3.0e-5, dtype=torch.float32).to(torch.bfloat16).float())
    x = np.random.default_rng(4).normal(size=1000).astype(np.float32)
    np.testing.assert_array_equal(fw.round_bf16(x), torch.from_numpy(x).to(torch.bfloat16).float().numpy().astype(np.float64))


def test_bf16_mode_rounds_only_storage_and_stays_close_to_f32_mode():
    ms32, ms16 = _small_model("f32"), _small_model("bf16")
    top, layers = _weights(ms16, 13)
    toks = list(range(6))
    bt = np.array([[0, 1]], dtype=np.int32)
    a = _run(ms32, top, layers, toks, [5], [0], bt, 4, _empty_cache(ms32, 2, 4))
    b = _run(ms16, top, layers, toks, [5], [0], bt, 4, _empty_cache(ms16, 2, 4))
    scale = np.abs(a).max()
    assert 0 < np.abs(a - b).max() < 3e-2 * scale
