"""Seeded synthetic inputs for the verification step (numpy only).

Everything here is *input construction*: random tensors, the draft servers'
distributions q and their sampled draft tokens, model weights, cached K/V
contents, block tables.  Nothing in this module belongs to the verification
method itself (no target softmax, no accept test, no scheduler), so the CPU
oracle and the HIP path can both be fed from it without sharing arithmetic.

The paper evaluates on public prompt datasets and trained models (Section IV-A,
Testbed / Datasets).  What those contribute to the verification step is only
(i) how well each draft distribution matches the target and (ii) the spread of
context lengths; both are reproduced here by distribution.

Random streams: SFC64 bit generators keyed by SeedSequence([seed, *tags, chunk]).
A tensor is the concatenation of fixed-size chunks, each with its own stream, so
its values do not depend on how many threads generate it.
"""
from __future__ import annotations

import os
import zlib
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

MASTER_SEED = 20251209
_CHUNK = 1 << 22


def _tag_ints(tags):
    out = []
    for t in tags:
        if isinstance(t, str):
            out.append(zlib.crc32(t.encode()))
        else:
            out.append(int(t) & 0xFFFFFFFF)
    return out


def stream(seed, *tags):
    """Independent generator for (seed, tags)."""
    return np.random.Generator(np.random.SFC64(np.random.SeedSequence([int(seed)] + _tag_ints(tags))))


def _n_threads():
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        n = os.cpu_count() or 1
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        n = min(n, int(env)) if int(env) > 0 else n
    return max(1, min(n, 32))


def normal_f32(seed, tags, n, scale=1.0, out=None):
    """n standard normals (times scale) as float32, chunked and threaded."""
    n = int(n)
    if out is None:
        out = np.empty(n, dtype=np.float32)
    flat = out.reshape(-1)
    assert flat.size == n and flat.dtype == np.float32
    n_chunks = (n + _CHUNK - 1) // _CHUNK

    def fill(c):
        lo = c * _CHUNK
        hi = min(n, lo + _CHUNK)
        g = stream(seed, *tags, c)
        g.standard_normal(hi - lo, dtype=np.float32, out=flat[lo:hi])
        if scale != 1.0:
            flat[lo:hi] *= np.float32(scale)

    if n_chunks <= 1:
        for c in range(n_chunks):
            fill(c)
    else:
        with ThreadPoolExecutor(_n_threads()) as ex:
            list(ex.map(fill, range(n_chunks)))
    return out


def uniform01_f32(seed, tags, n):
    """n uniforms in [0, 1) on the 2^-24 grid, as float32."""
    bits = stream(seed, *tags).integers(0, 1 << 32, size=int(n), dtype=np.uint64)
    return ((bits >> 8).astype(np.float64) * 2.0 ** -24).astype(np.float32)


def round_to_bf16(x):
    """Round float32 values to the nearest bfloat16 (ties to even); returns float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    b = x.view(np.uint32)
    rounded = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x):
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


# ----------------------------------------------------------------------------
# Draft-side quantities (what a draft server would send)
# ----------------------------------------------------------------------------

def draft_probs_from_logits(draft_logits):
    """Row softmax of draft logits in float64, returned as float32 probabilities."""
    z = np.asarray(draft_logits, dtype=np.float64)
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return (e / e.sum(axis=-1, keepdims=True)).astype(np.float32)


def sample_tokens(q_probs, u):
    """Draw one token per row of q_probs by inverse CDF with the given uniforms.

    A token with q == 0 is never returned (searchsorted on the strict side,
    then clamp to the last token with positive mass).
    """
    q = np.asarray(q_probs, dtype=np.float64)
    out = np.empty(q.shape[0], dtype=np.int32)
    for r in range(q.shape[0]):
        c = np.cumsum(q[r])
        k = int(np.searchsorted(c, float(u[r]) * c[-1], side="right"))
        if k >= q.shape[1]:
            k = int(np.nonzero(q[r] > 0)[0][-1])
        out[r] = k
    return out


def cu_rows_of(gamma):
    """Prefix offsets of the per-server target rows T_i = gamma_i + 1."""
    g = np.asarray(gamma, dtype=np.int64)
    cu = np.zeros(g.size + 1, dtype=np.int32)
    cu[1:] = np.cumsum(g + 1)
    return cu


def cu_draft_of(gamma):
    """Prefix offsets of the per-server draft rows (gamma_i each)."""
    g = np.asarray(gamma, dtype=np.int64)
    cu = np.zeros(g.size + 1, dtype=np.int32)
    cu[1:] = np.cumsum(g)
    return cu


@dataclass
class AcceptInputs:
    """Inputs of the standalone accept/reject + resample stage."""
    gamma: np.ndarray          # [N] int32
    target_logits: np.ndarray  # [R, V] float32, R = sum(gamma + 1)
    q_probs: np.ndarray        # [Gamma, V] float32
    draft_tokens: np.ndarray   # [Gamma] int32
    u_accept: np.ndarray       # [Gamma] float32
    u_resample: np.ndarray     # [N] float32

    @property
    def vocab(self):
        return self.target_logits.shape[1]


def accept_inputs(seed, gamma, vocab, sigma, logit_scale=3.0, tag="accept"):
    """Standalone accept/reject workload.

    Target logits are logit_scale * N(0,1).  The draft logits of a server's
    j-th draft are the target logits of that server's row j-1 (the row whose
    softmax is p_j) plus sigma * N(0,1); q is their softmax; draft tokens are
    sampled from q.
    """
    gamma = np.asarray(gamma, dtype=np.int32)
    n = gamma.size
    cu_r = cu_rows_of(gamma)
    cu_d = cu_draft_of(gamma)
    R, G = int(cu_r[-1]), int(cu_d[-1])
    tl = normal_f32(seed, (tag, "target", float_tag(sigma)), R * vocab, scale=logit_scale).reshape(R, vocab)
    noise = normal_f32(seed, (tag, "noise", float_tag(sigma)), G * vocab, scale=sigma).reshape(G, vocab)
    q = np.empty((G, vocab), dtype=np.float32)
    for i in range(n):
        for j in range(int(gamma[i])):
            q[cu_d[i] + j] = draft_probs_from_logits(tl[cu_r[i] + j].astype(np.float64) + noise[cu_d[i] + j])
    del noise
    u_tok = uniform01_f32(seed, (tag, "u_tok", float_tag(sigma)), G)
    toks = sample_tokens(q, u_tok)
    return AcceptInputs(gamma, tl, q, toks,
                        uniform01_f32(seed, (tag, "u_acc", float_tag(sigma)), G),
                        uniform01_f32(seed, (tag, "u_res", float_tag(sigma)), n))


def loop_round_inputs(seed, round_idx, gamma, vocab, sigmas, logit_scale=3.0, tag="loop"):
    """One round of the closed loop: like accept_inputs, but draft server i perturbs the target logits with
    its own noise level sigmas[i] (heterogeneous acceptance rates), and every tensor is keyed by the round."""
    gamma = np.asarray(gamma, dtype=np.int32)
    sigmas = np.asarray(sigmas, dtype=np.float64)
    n = gamma.size
    cu_r = cu_rows_of(gamma)
    cu_d = cu_draft_of(gamma)
    R, G = int(cu_r[-1]), int(cu_d[-1])
    key = (tag, int(round_idx))
    tl = normal_f32(seed, key + ("target",), R * vocab, scale=logit_scale).reshape(R, vocab)
    noise = normal_f32(seed, key + ("noise",), max(G, 1) * vocab).reshape(max(G, 1), vocab)
    q = np.empty((G, vocab), dtype=np.float32)
    for i in range(n):
        for j in range(int(gamma[i])):
            q[cu_d[i] + j] = draft_probs_from_logits(tl[cu_r[i] + j].astype(np.float64)
                                                     + sigmas[i] * noise[cu_d[i] + j].astype(np.float64))
    toks = sample_tokens(q, uniform01_f32(seed, key + ("u_tok",), G)) if G else np.zeros(0, np.int32)
    return AcceptInputs(gamma, tl, q, toks, uniform01_f32(seed, key + ("u_acc",), G),
                        uniform01_f32(seed, key + ("u_res",), n))


def loop_policy_uniforms(seed, round_idx, count, tag="loop"):
    """Uniforms in [0, 1) that the random allocation policy of a round consumes."""
    return uniform01_f32(seed, (tag, int(round_idx), "policy"), count)


def float_tag(x):
    return int(round(float(x) * 1000))


# ----------------------------------------------------------------------------
# Target-model shapes, weights, KV cache contents
# ----------------------------------------------------------------------------

@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_theta: float = 10000.0
    rms_eps: float = 1e-5
    dtype: str = "bf16"  # storage type of weights, activations fed to GEMMs and KV: "f32" | "bf16"

    @property
    def qkv_out(self):
        return (self.n_heads + 2 * self.n_kv_heads) * self.head_dim

    def n_params(self):
        per_layer = (self.qkv_out * self.d_model + self.d_model * self.n_heads * self.head_dim
                     + 3 * self.d_ffn * self.d_model + 2 * self.d_model)
        return self.n_layers * per_layer + 2 * self.vocab * self.d_model + self.d_model


TINY = ModelShape(2, 256, 4, 4, 64, 1024, 1024, rope_theta=10000.0, dtype="f32")
LLAMA3_8B = ModelShape(32, 4096, 32, 8, 128, 14336, 128256, rope_theta=500000.0, dtype="bf16")
LLAMA3_70B = ModelShape(80, 8192, 64, 8, 128, 28672, 128256, rope_theta=500000.0, dtype="bf16")

# names and shapes of one layer's matrices, all stored [out_features, in_features]
def layer_matrix_shapes(ms: ModelShape):
    return {
        "wqkv": (ms.qkv_out, ms.d_model),          # rows: all Q heads, then K heads, then V heads
        "wo": (ms.d_model, ms.n_heads * ms.head_dim),
        "wgu": (2 * ms.d_ffn, ms.d_model),         # rows: gate [0, F), up [F, 2F)
        "wd": (ms.d_model, ms.d_ffn),
    }


def matrix(ms: ModelShape, seed, name, layer, shape, std=0.02):
    """One weight matrix N(0, std^2), rounded to the model's storage type; float32 array."""
    w = normal_f32(seed, ("w", name, layer), shape[0] * shape[1], scale=std).reshape(shape)
    if ms.dtype == "bf16":
        w = round_to_bf16(w)
    return w


def layer_weights(ms: ModelShape, seed, layer, std=0.02):
    """Dict of one layer's tensors (float32 arrays holding storage-type values)."""
    out = {k: matrix(ms, seed, k, layer, s, std) for k, s in layer_matrix_shapes(ms).items()}
    out["norm1"] = np.ones(ms.d_model, dtype=np.float32)
    out["norm2"] = np.ones(ms.d_model, dtype=np.float32)
    return out


W4_GROUP = 128


def quantize_w4(w, group=W4_GROUP):
    """Synthetic 4-bit checkpoint of a float matrix [N, K]: per row and group of `group` inputs an asymmetric
    min/max grid that contains zero.  Returns (codes uint8 [N, K] in 0..15, scales float32 [N, K/group]
    holding bf16 values, zeros uint8 [N, K/group] in 0..15).  This only manufactures inputs; what the
    verifier computes from them is defined on the two sides separately."""
    w = np.asarray(w, dtype=np.float32)
    n, k = w.shape
    assert k % group == 0
    g = w.reshape(n, k // group, group)
    lo = np.minimum(g.min(axis=2), 0.0)
    hi = np.maximum(g.max(axis=2), 0.0)
    scale = round_to_bf16(((hi - lo) / 15.0).astype(np.float32))
    scale = np.where(scale > 0, scale, np.float32(1.0)).astype(np.float32)
    zero = np.clip(np.rint(-lo / scale), 0, 15).astype(np.uint8)
    codes = np.clip(np.rint(g / scale[:, :, None]) + zero[:, :, None], 0, 15).astype(np.uint8)
    return codes.reshape(n, k), scale, zero


def top_weights(ms: ModelShape, seed, std=0.02):
    return {
        "embed": matrix(ms, seed, "embed", 0, (ms.vocab, ms.d_model), std),
        "lm_head": matrix(ms, seed, "lm_head", 0, (ms.vocab, ms.d_model), std),
        "final_norm": np.ones(ms.d_model, dtype=np.float32),
    }


@dataclass
class BatchShape:
    """Ragged batch geometry: per-server draft lengths, cached context lengths, page tables."""
    gamma: np.ndarray        # [N] int32
    ctx_len: np.ndarray      # [N] int32  tokens already cached
    page_size: int
    block_table: np.ndarray  # [N, max_blocks] int32 physical page ids (-1 = unused)
    n_pages: int

    @property
    def n_servers(self):
        return int(self.gamma.size)

    @property
    def cu_rows(self):
        return cu_rows_of(self.gamma)

    @property
    def n_rows(self):
        return int(self.cu_rows[-1])

    @property
    def n_draft(self):
        return int(np.sum(self.gamma))


def make_batch(seed, gamma, ctx_len, page_size=16, headroom=0, permute_pages=False, tag="batch"):
    """Block tables with room for ctx_len + gamma + 1 + headroom tokens per server."""
    gamma = np.asarray(gamma, dtype=np.int32)
    ctx_len = np.asarray(ctx_len, dtype=np.int32)
    need = (ctx_len.astype(np.int64) + gamma + 1 + headroom + page_size - 1) // page_size
    max_blocks = int(need.max())
    n_pages = int(need.sum())
    ids = np.arange(n_pages, dtype=np.int32)
    if permute_pages:
        ids = stream(seed, tag, "pages").permutation(n_pages).astype(np.int32)
    bt = np.full((gamma.size, max_blocks), -1, dtype=np.int32)
    o = 0
    for i in range(gamma.size):
        bt[i, : need[i]] = ids[o : o + need[i]]
        o += int(need[i])
    return BatchShape(gamma, ctx_len, page_size, bt, n_pages)


def kv_layer_cache(ms: ModelShape, seed, layer, which, n_pages, page_size):
    """Synthetic cached K (already rotated) or V of one layer: N(0,1) in storage type.

    Layout [n_pages, n_kv_heads, page_size, head_dim], float32 array of storage-type values.
    """
    shape = (n_pages, ms.n_kv_heads, page_size, ms.head_dim)
    x = normal_f32(seed, ("kv", which, layer), int(np.prod(shape))).reshape(shape)
    if ms.dtype == "bf16":
        x = round_to_bf16(x)
    return x


def uniform_int(seed, tags, lo, hi, n):
    """n integers uniform in [lo, hi]."""
    return stream(seed, *tags).integers(lo, hi + 1, size=int(n)).astype(np.int32)


def log_uniform_int(seed, tags, lo, hi, n):
    """n integers whose logarithm is uniform on [log lo, log hi]."""
    u = stream(seed, *tags).random(int(n))
    return np.clip(np.round(np.exp(np.log(lo) + u * (np.log(hi) - np.log(lo)))), lo, hi).astype(np.int32)


def verify_side_inputs(seed, ms_vocab, gamma, sigma=0.5, logit_scale=1.0, tag="vin"):
    """Draft-side inputs of a full verify step: pending+draft token ids, q, uniforms.

    Draft logits = logit_scale * (z + sigma * eps) with z, eps standard normal per row,
    independent of the target model.  The draft tokens are sampled from q; the pending
    token of each server is uniform over the vocabulary.
    Returns (tokens[R], q_probs[Gamma, V], u_accept[Gamma], u_resample[N]).
    """
    gamma = np.asarray(gamma, dtype=np.int32)
    n = gamma.size
    G = int(gamma.sum())
    cu_r = cu_rows_of(gamma)
    cu_d = cu_draft_of(gamma)
    V = int(ms_vocab)
    z = normal_f32(seed, (tag, "z"), G * V).reshape(G, V)
    if sigma != 0.0:
        eps = normal_f32(seed, (tag, "eps"), G * V, scale=sigma).reshape(G, V)
        z += eps
        del eps
    if logit_scale != 1.0:
        z *= np.float32(logit_scale)
    q = np.empty((G, V), dtype=np.float32)
    for r in range(G):
        q[r] = draft_probs_from_logits(z[r])
    del z
    d_tok = sample_tokens(q, uniform01_f32(seed, (tag, "u_tok"), G))
    pending = uniform_int(seed, (tag, "pending"), 0, V - 1, n)
    tokens = np.empty(int(cu_r[-1]), dtype=np.int32)
    for i in range(n):
        tokens[cu_r[i]] = pending[i]
        tokens[cu_r[i] + 1 : cu_r[i + 1]] = d_tok[cu_d[i] : cu_d[i + 1]]
    return tokens, q, uniform01_f32(seed, (tag, "u_acc"), G), uniform01_f32(seed, (tag, "u_res"), n)


# ----------------------------------------------------------------------------
# The named verify configurations (shapes and distributions only)
# ----------------------------------------------------------------------------

@dataclass
class VerifyConfig:
    name: str
    ms: ModelShape
    batch: BatchShape
    tokens: np.ndarray
    q_probs: np.ndarray
    u_accept: np.ndarray
    u_resample: np.ndarray
    seed: int


def _verify_config(name, ms, seed, gamma, ctx, permute, sigma, logit_scale):
    batch = make_batch(seed, gamma, ctx, 16, headroom=0, permute_pages=permute, tag=name)
    tokens, q, ua, ur = verify_side_inputs(seed, ms.vocab, gamma, sigma=sigma, logit_scale=logit_scale, tag=name)
    return VerifyConfig(name, ms, batch, tokens, q, ua, ur, seed)


def config3(seed=MASTER_SEED, ms=LLAMA3_8B):
    """8B-shaped verify: 8 servers, gamma uniform in [3, 8], 2048 cached tokens each, contiguous 16-token pages."""
    gamma = uniform_int(seed, ("cfg3", "gamma"), 3, 8, 8)
    return _verify_config("cfg3", ms, seed, gamma, np.full(8, 2048, np.int32), False, 0.5, 1.0)


def config4(seed=MASTER_SEED, ms=LLAMA3_8B, headroom=64):
    """8B-shaped ragged verify: 32 servers, gamma uniform in [1, 16], context log-uniform in [512, 8192],
    permuted 16-token pages with room for `headroom` more tokens per server (later rounds)."""
    gamma = uniform_int(seed, ("cfg4", "gamma"), 1, 16, 32)
    ctx = log_uniform_int(seed, ("cfg4", "ctx"), 512, 8192, 32)
    batch = make_batch(seed, np.full(32, 16, np.int32), ctx, 16, headroom=headroom, permute_pages=True, tag="cfg4")
    batch = BatchShape(gamma, ctx, 16, batch.block_table, batch.n_pages)
    tokens, q, ua, ur = verify_side_inputs(seed, ms.vocab, gamma, sigma=0.5, tag="cfg4")
    return VerifyConfig("cfg4", ms, batch, tokens, q, ua, ur, seed)


def config5(seed=MASTER_SEED, ms=LLAMA3_70B):
    """70B-shaped verify: 16 servers, gamma uniform in [2, 8], 4096 cached tokens each; draft logits are
    2 * N(0,1), independent of the target."""
    gamma = uniform_int(seed, ("cfg5", "gamma"), 2, 8, 16)
    return _verify_config("cfg5", ms, seed, gamma, np.full(16, 4096, np.int32), False, 0.0, 2.0)


def config_rows1024(seed=MASTER_SEED, ms=LLAMA3_8B):
    """Compute-bound row count for the projection kernels: 8 servers with blocks of 128 rows (the pending
    token and 127 drafts) on an empty cache, i.e. 1024 target rows through the same verify call."""
    gamma = np.full(8, 127, np.int32)
    return _verify_config("rows1024", ms, seed, gamma, np.zeros(8, np.int32), False, 0.5, 1.0)


def draft_tokens_of(cfg_tokens, gamma):
    """The draft tokens (without the pending tokens) in draft-row order."""
    cu = cu_rows_of(gamma)
    parts = [cfg_tokens[cu[i] + 1:cu[i + 1]] for i in range(len(gamma))]
    return np.concatenate(parts) if parts else np.zeros(0, np.int32)
