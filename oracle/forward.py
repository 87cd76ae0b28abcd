"""Oracle: target-decoder forward over the ragged speculative blocks of N servers.

Test infrastructure only.  Float64 numpy; matrix products through numpy's matmul.

The paper (Section II-A) fixes only that the target model is a Transformer
decoder whose next-token distribution is softmax(W h) and that it scores all
drafted positions of a block in parallel against the server's prefix.  The
decoder itself is the Llama-style stack the benchmark configurations name:
pre-norm RMSNorm, rotary position embedding (rotate-half pairing
(i, i + hd/2), inverse frequency theta^(-2i/hd)), grouped-query causal
attention with scale 1/sqrt(hd) where query head h reads KV head h // (H/H_kv),
SwiGLU feed-forward, no biases, untied embedding and LM head.

Row layout: server i contributes T_i = gamma_i + 1 rows, the pending token (the
previous round's correction/bonus token, not yet in the cache) followed by its
gamma_i drafts, at positions L_i .. L_i + gamma_i where L_i is the cached
context length.  Row j of a server yields the logits of p_{j+1}, the
distribution of the token that follows row j's token.

Storage rounding: with dtype "bf16" the tensors that the data layout stores in
bfloat16 (normalised activations fed to a projection, rotated Q and K, V,
attention output, SwiGLU output) are rounded to nearest-even bfloat16 at the
point of storage, and every sum is float64.  With dtype "f32" nothing is rounded.
"""
import numpy as np


def round_bf16(x):
    """Nearest-even rounding of float64/float32 values to bfloat16, returned as float64."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    b = f.view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(np.float64)


def _store(x, dtype):
    return round_bf16(x) if dtype == "bf16" else np.asarray(x, dtype=np.float64)


def rmsnorm(x, w, eps):
    """x * w / sqrt(mean(x^2) + eps), row-wise."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * w


def rope(v, pos, theta):
    """Rotate vectors v[..., hd] by position pos with rotate-half pairing."""
    hd = v.shape[-1]
    half = hd // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = float(pos) * inv_freq
    c, s = np.cos(ang), np.sin(ang)
    a, b = v[..., :half], v[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def gather_kv(pages, block_row, n_tokens, page_size):
    """pages [n_pages, H_kv, page, hd] -> [H_kv, n_tokens, hd] following one server's block table."""
    n_blk = (n_tokens + page_size - 1) // page_size
    blocks = [pages[int(block_row[b])] for b in range(n_blk)]
    if not blocks:
        return np.zeros((pages.shape[1], 0, pages.shape[3]), dtype=np.float64)
    cat = np.concatenate(blocks, axis=1)
    return np.asarray(cat[:, :n_tokens, :], dtype=np.float64)


def attention_server(q, k_all, v_all, ctx_len, n_heads, n_kv_heads):
    """Causal GQA attention for one server's block.

    q [T, H, hd]; k_all, v_all [H_kv, ctx_len + T, hd] (cache followed by the block's
    own rows).  Row j attends to keys 0 .. ctx_len + j.  Returns [T, H, hd].
    """
    T, H, hd = q.shape
    group = n_heads // n_kv_heads
    out = np.zeros_like(q)
    scale = 1.0 / np.sqrt(hd)
    for j in range(T):
        n_keys = ctx_len + j + 1
        for h in range(H):
            kv = h // group
            s = (k_all[kv, :n_keys] @ q[j, h]) * scale
            e = np.exp(s - s.max())
            p = e / e.sum()
            out[j, h] = p @ v_all[kv, :n_keys]
    return out


def _row_offsets(gamma):
    gamma = np.asarray(gamma, dtype=np.int64)
    cu = np.zeros(gamma.size + 1, dtype=np.int64)
    cu[1:] = np.cumsum(gamma + 1)
    return gamma, cu


def embed_rows(top, tokens):
    """Residual stream entering the first layer: the embedding rows of the block tokens."""
    return np.asarray(top["embed"], dtype=np.float32)[np.asarray(tokens, dtype=np.int64)].astype(np.float64)


def layer_forward(ms, x, W, k_pages, v_pages, gamma, ctx_len, block_table, page_size):
    """One decoder layer on the residual stream x [R, d]; appends the block's K/V to the pages in place.

    W: dict(wqkv [(H+2H_kv)hd, d], wo [d, H hd], wgu [2F, d], wd [d, F], norm1, norm2);
    k_pages, v_pages [n_pages, H_kv, page, hd], written at positions ctx_len_i .. ctx_len_i + gamma_i.
    """
    gamma, cu = _row_offsets(gamma)
    n = gamma.size
    H, Hk, hd, F = ms.n_heads, ms.n_kv_heads, ms.head_dim, ms.d_ffn
    R = int(cu[-1])
    h = _store(rmsnorm(x, np.asarray(W["norm1"], dtype=np.float64), ms.rms_eps), ms.dtype)
    qkv = h @ np.asarray(W["wqkv"], dtype=np.float64).T
    attn = np.zeros((R, H * hd), dtype=np.float64)
    for i in range(n):
        T = int(gamma[i]) + 1
        L = int(ctx_len[i])
        rows = qkv[cu[i]:cu[i + 1]]
        q = rows[:, : H * hd].reshape(T, H, hd).copy()
        k = rows[:, H * hd:(H + Hk) * hd].reshape(T, Hk, hd).copy()
        v = rows[:, (H + Hk) * hd:].reshape(T, Hk, hd)
        for j in range(T):
            q[j] = rope(q[j], L + j, ms.rope_theta)
            k[j] = rope(k[j], L + j, ms.rope_theta)
        q = _store(q, ms.dtype)
        k = _store(k, ms.dtype)
        v = _store(v, ms.dtype)
        for j in range(T):
            pos = L + j
            pg = int(block_table[i][pos // page_size])
            k_pages[pg, :, pos % page_size, :] = k[j]
            v_pages[pg, :, pos % page_size, :] = v[j]
        k_all = gather_kv(k_pages, block_table[i], L + T, page_size)
        v_all = gather_kv(v_pages, block_table[i], L + T, page_size)
        o = attention_server(q, k_all, v_all, L, H, Hk)
        attn[cu[i]:cu[i + 1]] = o.reshape(T, H * hd)
    attn = _store(attn, ms.dtype)
    x = x + attn @ np.asarray(W["wo"], dtype=np.float64).T
    h = _store(rmsnorm(x, np.asarray(W["norm2"], dtype=np.float64), ms.rms_eps), ms.dtype)
    gu = h @ np.asarray(W["wgu"], dtype=np.float64).T
    act = _store(silu(gu[:, :F]) * gu[:, F:], ms.dtype)
    return x + act @ np.asarray(W["wd"], dtype=np.float64).T


def lm_head(ms, x, top):
    """Logits of the final residual stream: final RMSNorm, then the LM-head projection."""
    h = _store(rmsnorm(x, np.asarray(top["final_norm"], dtype=np.float64), ms.rms_eps), ms.dtype)
    return h @ np.asarray(top["lm_head"], dtype=np.float64).T


def verify_forward(ms, tokens, gamma, ctx_len, block_table, page_size, top, get_layer, get_kv):
    """Logits [R, V] of every row of the ragged batch; appends the block's K/V to the cache.

    ms: object with n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab,
        rope_theta, rms_eps, dtype.
    top: dict(embed [V, d], lm_head [V, d], final_norm [d]).
    get_layer(l): the layer's weight dict (see layer_forward).
    get_kv(l): (k_pages, v_pages) arrays [n_pages, H_kv, page, hd], written in place at
        positions ctx_len_i .. ctx_len_i + gamma_i of each server.
    """
    _, cu = _row_offsets(gamma)
    x = embed_rows(top, tokens[: int(cu[-1])])
    for l in range(ms.n_layers):
        k_pages, v_pages = get_kv(l)
        x = layer_forward(ms, x, get_layer(l), k_pages, v_pages, gamma, ctx_len, block_table, page_size)
    return lm_head(ms, x, top)
