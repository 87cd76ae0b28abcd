"""A second CPU decoder forward that accumulates in float32 (test helper, not the oracle, not the product).

Purpose: to show on the CPU alone how far two correct implementations of the same bfloat16-storage decoder
drift apart with depth.  It follows the same model definition and rounds the same tensors to bfloat16 at the
same points as oracle/forward.py (normalised activations, rotated Q and K, V, attention output, SwiGLU
output), and keeps the residual stream in float32, but every sum is a float32 sum in whatever order the BLAS
library and numpy's pairwise reductions choose.  The only differences from the oracle are therefore the
precision and the order of the additions - exactly what separates a GPU kernel from the float64 oracle.
Written independently of oracle/forward.py (batched einsum attention instead of per-row loops); shares no
code with it or with the HIP path.
"""
import numpy as np

F = np.float32


def to_bf16(x):
    """float32 values rounded to the nearest bfloat16 (ties to even), kept as float32."""
    bits = np.ascontiguousarray(x, dtype=F).view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    return ((bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)).view(F)


def _keep(x, dtype):
    return to_bf16(x) if dtype == "bf16" else np.asarray(x, dtype=F)


def _rms(x, w, eps):
    x = np.asarray(x, dtype=F)
    inv = F(1.0) / np.sqrt(np.mean(x * x, axis=-1, keepdims=True, dtype=F) + F(eps))
    return x * inv * np.asarray(w, dtype=F)


def _rotate(v, positions, theta):
    """v [T, heads, hd] rotated at the given positions (pairs (i, i + hd/2)); angles formed in double, then
    applied in float32."""
    hd = v.shape[-1]
    half = hd // 2
    freq = np.power(float(theta), -2.0 * np.arange(half) / hd)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * freq[None, :]
    c, s = np.cos(ang).astype(F)[:, None, :], np.sin(ang).astype(F)[:, None, :]
    lo, hi = v[..., :half], v[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def _mm(a, w, k_splits):
    """a [R, K] times w [N, K] transposed, float32; with k_splits > 1 the sum over K is formed as that many
    partial products added one after the other (a different summation order, like a split-K kernel's)."""
    w = np.asarray(w, dtype=F)
    if k_splits <= 1:
        return a @ w.T
    K = a.shape[1]
    edges = np.linspace(0, K, k_splits + 1).astype(int)
    out = np.zeros((a.shape[0], w.shape[0]), dtype=F)
    for lo, hi in zip(edges[:-1], edges[1:]):
        out += a[:, lo:hi] @ w[:, lo:hi].T
    return out


def embed(top, tokens):
    return np.asarray(top["embed"], dtype=F)[np.asarray(tokens, dtype=np.int64)]


def layer(ms, x, W, k_pages, v_pages, gamma, ctx_len, block_table, page_size, k_splits=1):
    """One decoder layer on the float32 residual stream x [R, d]; writes the block's K/V into the pages
    ([n_pages, H_kv, page, hd] float32 arrays) like the oracle's layer does."""
    gamma = np.asarray(gamma, dtype=np.int64)
    starts = np.concatenate([[0], np.cumsum(gamma + 1)])
    H, Hk, hd, Fd = ms.n_heads, ms.n_kv_heads, ms.head_dim, ms.d_ffn
    grp = H // Hk
    h = _keep(_rms(x, W["norm1"], ms.rms_eps), ms.dtype)
    qkv = _mm(h, W["wqkv"], k_splits)
    attn = np.empty((x.shape[0], H * hd), dtype=F)
    scale = F(1.0 / np.sqrt(hd))
    for i, g in enumerate(gamma):
        T, L = int(g) + 1, int(ctx_len[i])
        blk = qkv[starts[i]:starts[i + 1]]
        pos = np.arange(L, L + T)
        q = _keep(_rotate(blk[:, :H * hd].reshape(T, H, hd), pos, ms.rope_theta), ms.dtype)
        k = _keep(_rotate(blk[:, H * hd:(H + Hk) * hd].reshape(T, Hk, hd), pos, ms.rope_theta), ms.dtype)
        v = _keep(blk[:, (H + Hk) * hd:].reshape(T, Hk, hd), ms.dtype)
        pages = np.asarray(block_table[i], dtype=np.int64)
        k_pages[pages[pos // page_size], :, pos % page_size, :] = k
        v_pages[pages[pos // page_size], :, pos % page_size, :] = v
        n_blk = (L + T + page_size - 1) // page_size
        # [H_kv, keys, hd] of the server: its pages in logical order
        kk = k_pages[pages[:n_blk]].transpose(1, 0, 2, 3).reshape(Hk, n_blk * page_size, hd)[:, :L + T]
        vv = v_pages[pages[:n_blk]].transpose(1, 0, 2, 3).reshape(Hk, n_blk * page_size, hd)[:, :L + T]
        qg = q.reshape(T, Hk, grp, hd)
        s = np.einsum("tkgd,knd->tkgn", qg, kk.astype(F), optimize=True) * scale
        mask = np.arange(L + T)[None, :] > pos[:, None]          # key n visible to row t iff n <= L + t
        s = np.where(mask[:, None, None, :], F(-np.inf), s)
        e = np.exp(s - s.max(axis=-1, keepdims=True))
        p = e / e.sum(axis=-1, keepdims=True, dtype=F)
        o = np.einsum("tkgn,knd->tkgd", p.astype(F), vv.astype(F), optimize=True)
        attn[starts[i]:starts[i + 1]] = o.reshape(T, H * hd)
    x = x + _mm(_keep(attn, ms.dtype), W["wo"], k_splits)
    h = _keep(_rms(x, W["norm2"], ms.rms_eps), ms.dtype)
    gu = _mm(h, W["wgu"], k_splits)
    gate, up = gu[:, :Fd], gu[:, Fd:]
    act = _keep(gate / (F(1.0) + np.exp(-gate)) * up, ms.dtype)
    return x + _mm(act, W["wd"], k_splits)


def head(ms, x, top, k_splits=1):
    h = _keep(_rms(x, top["final_norm"], ms.rms_eps), ms.dtype)
    return _mm(h, top["lm_head"], k_splits)
