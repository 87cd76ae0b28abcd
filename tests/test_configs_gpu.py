"""Parity on the model-scale configurations, in the launch configuration bench.py times.

Default run: config 3 at full depth (32 layers); config 4 at full depth for one round plus its three-round
scheduler loop at 4 layers; config 5 (70B shape) at its real width, row count and context with 36 of its 80
layers, which puts the last layers' K/V pages beyond 4 GiB from the start of the cache (64-bit offsets).
GS_FULL_CONFIGS=1 runs the three-round loop at 32 layers and config 5 at 80 (minutes of host time for the
oracle, 141 GB of weights).

Three bars per step (see _verify_and_compare): every layer teacher-forced within 2e-2 of the row scale (the
binding one), the free-running logits within free_running_bound(depth), and the decisions of the oracle's
accept stage on the device's logits bit-exact outside the rounding bands.  Beside the float64 oracle the
free-running check of config 3 (of all three with GS_FULL_CONFIGS=1) also runs a float32-accumulating CPU
forward (tests/f32_forward.py): the device may not be further from the oracle than 1.5 times what that
second CPU implementation already is.
"""
import dataclasses
import os

import numpy as np
import pytest

from oracle import accept_reject as ar
from oracle import forward as fw
from oracle import schedule as sch
from paper_2512_09963_amd import synth
from tests import f32_forward as f32
from tests.conftest import progress
from tests.parity import check_accept_outputs
from tests.test_verify_gpu import assert_logits_close

pytestmark = pytest.mark.gpu
FULL = os.environ.get("GS_FULL_CONFIGS", "0") == "1"


def free_running_bound(n_layers):
    """Allowed |logit error| / row scale of a free-running bf16 forward of this depth: 2e-2 up to 11 layers,
    6e-3 * sqrt(depth) beyond.  The growth is a property of bfloat16 storage, not of a kernel: two CPU
    implementations that round the same tensors to bfloat16 and differ only in summing in float32 instead of
    float64 (tests/bf16_depth_experiment.py, no GPU code involved) part by 3.1e-3, 4.7e-3, 7.0e-3, 1.0e-2,
    1.6e-2 and 2.3e-2 of the row scale after 1, 2, 4, 8, 16 and 32 layers of this 8B shape - a rounding that
    flips in one of them is a full bfloat16 step (2^-8) in the other, and each layer adds its own flips."""
    return max(2e-2, 6e-3 * np.sqrt(n_layers))


def probability_band(logits, tol):
    """What a logit tolerance means for p = softmax(logits): if every logit of a row moves by at most
    delta = tol * max|logit|, each probability moves by a factor within exp(+-2 delta) (its own exponential by
    exp(+-delta), the normaliser by exp(-+delta)).  Returns exp(2 delta) - 1 per row: |p' - p| <= that * p."""
    delta = tol * np.abs(logits).max(axis=1)
    return np.expm1(2.0 * delta)


def softmax_rows(logits):
    return np.stack([ar.softmax(r) for r in logits])


def assert_probabilities_close(got_logits, want_logits, tol, what):
    """softmax of the device's logits against softmax of the oracle's, within the band the logit tolerance
    implies; returns the worst |dp| / p."""
    p_got, p_want = softmax_rows(got_logits), softmax_rows(want_logits)
    band = probability_band(want_logits, tol)[:, None]
    rel = np.abs(p_got - p_want) / np.maximum(p_want, 1e-300)
    assert np.all(np.abs(p_got - p_want) <= band * p_want + 1e-300), \
        f"{what}: probabilities outside exp(2 delta) - 1 (worst |dp|/p = {rel.max():.3g})"
    return float(rel.max())


class OracleState:
    """K/V rows appended by earlier rounds, which must be re-applied to the regenerated synthetic cache:
    one record for the teacher-forced oracle, one for the free-running one."""

    def __init__(self):
        self.tf, self.free, self.f32 = {}, {}, {}


def _with_rows(ms, seed, l, batch, rows):
    k = synth.kv_layer_cache(ms, seed, l, "k", batch.n_pages, batch.page_size)
    v = synth.kv_layer_cache(ms, seed, l, "v", batch.n_pages, batch.page_size)
    for (ll, pg, sl), (kr, vr) in rows.items():
        if ll == l:
            k[pg, :, sl, :], v[pg, :, sl, :] = kr, vr
    return k, v


def _record_rows(l, batch, k, v, rows):
    for i in range(batch.n_servers):
        for pos in range(int(batch.ctx_len[i]), int(batch.ctx_len[i] + batch.gamma[i] + 1)):
            pg, sl = int(batch.block_table[i, pos // batch.page_size]), pos % batch.page_size
            rows[(l, pg, sl)] = (k[pg, :, sl, :].copy(), v[pg, :, sl, :].copy())


def _rel_to_row_scale(got, want):
    return float((np.abs(got - want) / np.maximum(np.abs(want).max(axis=1, keepdims=True), 1e-30)).max())


def _verify_and_compare(cfg, ver, kv, db, state=None, with_f32=True):
    """One verification step on the device, checked three ways:
    (i) layer by layer, teacher-forced: the oracle's layer applied to the residual stream the device fed
        to that layer must reproduce the device's next residual stream, its appended K/V rows, and (from the
        final stream) its logits, within 2e-2 of the row scale;
    (ii) free-running: the oracle's own forward from the embeddings, within free_running_bound(depth);
    (iii) decisions: the oracle's accept stage on the device's logits must give the device's accepted
        lengths and tokens (outside the rounding bands)."""
    import torch
    from oracle import accept_reject as ar
    from paper_2512_09963_amd import workload as wl
    ms, b, seed = cfg.ms, cfg.batch, cfg.seed
    state = state or OracleState()
    trace = torch.empty(ms.n_layers + 1, b.n_rows, ms.d_model, dtype=torch.float32, device="cuda:0")
    ver.gs_trace_residual(trace)
    out, logits, _ = wl.verify(ver, kv, db)
    torch.cuda.synchronize()
    ver.gs_trace_residual(None)
    tr = trace.cpu().numpy().astype(np.float64)
    got_logits = logits.cpu().numpy()
    top = synth.top_weights(ms, seed)
    x_free = fw.embed_rows(top, cfg.tokens)
    np.testing.assert_array_equal(tr[0], x_free)               # the gather is exact
    x_f32 = f32.embed(top, cfg.tokens) if with_f32 else None   # second CPU implementation, float32 sums
    worst_layer = worst_kv = 0.0
    args = (b.gamma, b.ctx_len, b.block_table, b.page_size)
    for l in range(ms.n_layers):
        W = synth.layer_weights(ms, seed, l)
        k_tf, v_tf = _with_rows(ms, seed, l, b, state.tf)
        x_tf = fw.layer_forward(ms, tr[l], W, k_tf, v_tf, *args)
        worst_layer = max(worst_layer, _rel_to_row_scale(tr[l + 1], x_tf))
        k_g, v_g = kv.get_layer(l)
        for i in range(b.n_servers):
            for pos in range(int(b.ctx_len[i]), int(b.ctx_len[i] + b.gamma[i] + 1)):
                pg, sl = int(b.block_table[i, pos // b.page_size]), pos % b.page_size
                for got, want in ((k_g, k_tf), (v_g, v_tf)):
                    w_ = want[pg, :, sl, :].astype(np.float64)
                    worst_kv = max(worst_kv, np.abs(got[pg, :, sl, :] - w_).max() / max(np.abs(w_).max(), 1e-6))
        _record_rows(l, b, k_tf, v_tf, state.tf)
        k_fr, v_fr = _with_rows(ms, seed, l, b, state.free)
        x_free = fw.layer_forward(ms, x_free, W, k_fr, v_fr, *args)
        _record_rows(l, b, k_fr, v_fr, state.free)
        if with_f32:
            k_32, v_32 = _with_rows(ms, seed, l, b, state.f32)
            x_f32 = f32.layer(ms, x_f32, W, k_32, v_32, *args)
            _record_rows(l, b, k_32, v_32, state.f32)
            del k_32, v_32
        del W, k_tf, v_tf, k_fr, v_fr
        if (l + 1) % 4 == 0:
            progress(f"{cfg.name}: layer {l + 1}/{ms.n_layers} checked against the oracle")
    assert worst_layer <= 2e-2, f"teacher-forced layer output error / row scale = {worst_layer:.3g}"
    assert worst_kv <= 2e-2, f"appended K/V rows: {worst_kv:.3g}"
    head_err = assert_logits_close(got_logits, fw.lm_head(ms, tr[ms.n_layers], top), 2e-2, "teacher-forced logits")
    want_tf = fw.lm_head(ms, tr[ms.n_layers], top)
    p_tf = assert_probabilities_close(got_logits, want_tf, 2e-2, "teacher-forced")
    want_free = fw.lm_head(ms, x_free, top)
    bound = free_running_bound(ms.n_layers)
    free_err = assert_logits_close(got_logits, want_free, bound, "free-running logits")
    p_free = assert_probabilities_close(got_logits, want_free, bound, "free-running")
    cpu_err = None
    if with_f32:     # the device is not further from the oracle than a float32 CPU implementation is
        cpu_err = assert_logits_close(f32.head(ms, x_f32, top), want_free, bound, "float32 CPU forward against the oracle")
        assert free_err <= 1.5 * cpu_err + 1e-3, \
            f"free-running: device {free_err:.3g} of the row scale from the oracle, float32 CPU forward only {cpu_err:.3g}"
    got = {k: v.cpu().numpy() for k, v in out.items()}
    d_tok = synth.draft_tokens_of(cfg.tokens, b.gamma)
    bands = check_accept_outputs(b.gamma, got_logits, cfg.q_probs, d_tok, cfg.u_accept, cfg.u_resample, got)
    # the device's own probabilities p_j(s_j) = ratio_j * q_j(s_j) against the oracle's free-running ones
    cu_r, cu_d = synth.cu_rows_of(b.gamma), synth.cu_draft_of(b.gamma)
    rows_of_draft = np.concatenate([np.arange(cu_r[i], cu_r[i + 1] - 1) for i in range(b.n_servers)]).astype(int)
    if d_tok.size:
        q_tok = cfg.q_probs[np.arange(d_tok.size), d_tok].astype(np.float64)
        ok = q_tok > 0
        p_dev = got["ratio"].astype(np.float64)[ok] * q_tok[ok]
        p_own = softmax_rows(want_free[rows_of_draft])[np.arange(d_tok.size), d_tok][ok]
        band = probability_band(want_free[rows_of_draft], bound)[ok]
        assert np.all(np.abs(p_dev - p_own) <= band * p_own + 1e-6 * p_dev + 1e-300), "p_j(s_j) of the device outside the band"
    # Decisions against the oracle's own logits: a server's accepted length may differ only where the first
    # differing test has u within the band that the logit tolerance puts around the oracle's ratio.
    own = ar.accept_reject(b.gamma, want_free.astype(np.float32), cfg.q_probs, d_tok, cfg.u_accept, cfg.u_resample)
    flips = 0
    for i in range(b.n_servers):
        m_o, m_g = int(own["accepted_len"][i]), int(got["accepted_len"][i])
        if m_o == m_g:
            continue
        flips += 1
        j = int(cu_d[i]) + min(m_o, m_g)
        r_o = own["ratio"][j]
        width = probability_band(want_free[rows_of_draft[j]][None, :], bound)[0] * r_o
        assert abs(float(cfg.u_accept[j]) - r_o) <= width + 1e-5, \
            f"server {i}: accepted {m_g}, oracle with its own logits {m_o}; u = {cfg.u_accept[j]:.6f}, ratio = {r_o:.6f}"
    progress(f"{cfg.name}: layers {ms.n_layers}, rows {b.n_rows}: teacher-forced layer err {worst_layer:.2e}, K/V rows "
          f"{worst_kv:.2e}, head {head_err:.2e}, |dp|/p {p_tf:.2e}; free-running logits err/scale {free_err:.2e} "
          f"(bound {bound:.2e}; float32 CPU forward {cpu_err if cpu_err is None else round(cpu_err, 5)}), |dp|/p {p_free:.2e}; "
          f"bands {bands}; accepted {got['accepted_len'].tolist()}; "
          f"servers whose m differs with the oracle's own logits: {flips}")
    return got, state


def test_config3_llama8b_shape_full_size():
    from paper_2512_09963_amd import workload as wl
    cfg = synth.config3()
    ver, kv, db = wl.upload_config(cfg, progress=progress)
    _verify_and_compare(cfg, ver, kv, db)


def test_config4_ragged_paged_full_depth():
    """32 servers, ragged gamma and context, permuted pages, all 32 layers: one verification step."""
    from paper_2512_09963_amd import workload as wl
    cfg = synth.config4()
    ver, kv, db = wl.upload_config(cfg, progress=progress)
    _verify_and_compare(cfg, ver, kv, db, with_f32=FULL)       # (measured once with it: device 2.64e-2, CPU 2.37e-2)


def test_config4_ragged_paged_with_scheduler_in_the_loop():
    """32 servers, ragged gamma and context, permuted pages; three rounds in which the library's scheduler
    picks the next gamma from the accepted lengths and each round is checked against the oracle."""
    from paper_2512_09963_amd import binding as gsb, workload as wl
    ms = synth.LLAMA3_8B if FULL else dataclasses.replace(synth.LLAMA3_8B, n_layers=4)
    cfg = synth.config4(ms=ms)
    ver, kv, db = wl.upload_config(cfg, progress=progress)
    n, C = cfg.batch.n_servers, 272
    alpha, X = np.full(n, 0.5), np.ones(n)
    alpha_o, X_o = alpha.copy(), X.copy()
    state = None
    for rnd in range(3):
        got, state = _verify_and_compare(cfg, ver, kv, db, state, with_f32=False)
        m, stat, g_prev = got["accepted_len"], got["accept_stat"], cfg.batch.gamma
        g_next = gsb.gs_schedule_gamma(m, stat, g_prev, alpha, X, 0.2, 0.5, C, 1, 16)
        alpha_o, X_o, g_want = sch.schedule_round(m, stat, g_prev, alpha_o, X_o, 0.2, 0.5, C, 1, 16)
        np.testing.assert_array_equal(g_next, g_want)
        np.testing.assert_allclose(alpha, alpha_o, rtol=1e-14); np.testing.assert_allclose(X, X_o, rtol=1e-14)
        assert g_next.sum() == C and g_next.min() >= 1 and g_next.max() <= 16
        # next round: contexts advance by m + 1, the emitted token becomes the pending token
        ctx = cfg.batch.ctx_len + m + 1
        batch = synth.BatchShape(g_next, ctx.astype(np.int32), 16, cfg.batch.block_table, cfg.batch.n_pages)
        tokens, q, ua, ur = synth.verify_side_inputs(cfg.seed, ms.vocab, g_next, sigma=0.5, tag=f"cfg4r{rnd + 1}")
        cu = batch.cu_rows
        tokens[cu[:-1]] = got["next_token"]
        cfg = synth.VerifyConfig("cfg4", ms, batch, tokens, q, ua, ur, cfg.seed)
        db = wl.DeviceBatch(batch, tokens, q, ua, ur)
        # rows beyond the new context are dead and will be overwritten: drop them from the oracle's records
        page_owner = {int(pg): (i, blk) for i in range(n) for blk, pg in enumerate(batch.block_table[i]) if pg >= 0}
        for rows in (state.tf, state.free, state.f32):
            for key in [k for k in rows if page_owner[k[1]][1] * 16 + k[2] >= ctx[page_owner[k[1]][0]]]:
                del rows[key]


def test_config5_llama70b_shape():
    """70B shape; with 36 layers the K pages alone span 4.85 GB, so the last three layers lie beyond 2^32 bytes."""
    from paper_2512_09963_amd import workload as wl
    ms = synth.LLAMA3_70B if FULL else dataclasses.replace(synth.LLAMA3_70B, n_layers=36)
    cfg = synth.config5(ms=ms)
    ver, kv, db = wl.upload_config(cfg, progress=progress)
    assert kv.k[ms.n_layers - 1].data_ptr() - kv.k.data_ptr() > 1 << 32
    _verify_and_compare(cfg, ver, kv, db, with_f32=FULL)       # (the float32 CPU forward costs a minute here)
