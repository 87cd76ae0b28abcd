"""Parity on the model-scale configurations, in the launch configuration bench.py times.

The full-depth runs of the two largest configurations take minutes of host time for the oracle
(and, for the 70B shape, 141 GB of weights); by default they run at their real width, row count,
context lengths and paging but with 4 decoder layers.  GS_FULL_CONFIGS=1 runs them at full depth.
"""
import dataclasses
import os

import numpy as np
import pytest

from oracle import forward as fw
from oracle import schedule as sch
from paper_2512_09963_amd import synth
from tests.parity import check_accept_outputs
from tests.test_verify_gpu import assert_logits_close

pytestmark = pytest.mark.gpu
FULL = os.environ.get("GS_FULL_CONFIGS", "0") == "1"


def free_running_bound(n_layers):
    """Allowed |logit error| / row scale of a free-running bf16 forward of this depth.  Each bf16 storage
    point turns a relative discrepancy e between the fp32 and the float64 arithmetic into rounding flips
    worth sqrt(e * ulp), and later layers decorrelate further, so the end-to-end error of a random-init
    stack grows like sqrt(depth): 2e-2 up to 11 layers, 6e-3 * sqrt(depth) beyond."""
    return max(2e-2, 6e-3 * np.sqrt(n_layers))


class OracleState:
    """K/V rows appended by earlier rounds, which must be re-applied to the regenerated synthetic cache:
    one record for the teacher-forced oracle, one for the free-running one."""

    def __init__(self):
        self.tf, self.free = {}, {}


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


def _verify_and_compare(cfg, ver, kv, db, state=None):
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
        del W, k_tf, v_tf, k_fr, v_fr
        if (l + 1) % 8 == 0:
            print(f"[oracle] {cfg.name}: layer {l + 1}/{ms.n_layers} checked", flush=True)
    assert worst_layer <= 2e-2, f"teacher-forced layer output error / row scale = {worst_layer:.3g}"
    assert worst_kv <= 2e-2, f"appended K/V rows: {worst_kv:.3g}"
    head_err = assert_logits_close(got_logits, fw.lm_head(ms, tr[ms.n_layers], top), 2e-2, "teacher-forced logits")
    want_free = fw.lm_head(ms, x_free, top)
    free_err = assert_logits_close(got_logits, want_free, free_running_bound(ms.n_layers), "free-running logits")
    got = {k: v.cpu().numpy() for k, v in out.items()}
    d_tok = synth.draft_tokens_of(cfg.tokens, b.gamma)
    bands = check_accept_outputs(b.gamma, got_logits, cfg.q_probs, d_tok, cfg.u_accept, cfg.u_resample, got)
    # how many servers change their accepted length when the oracle uses its own logits (reported, not gated)
    own = ar.accept_reject(b.gamma, want_free.astype(np.float32), cfg.q_probs, d_tok, cfg.u_accept, cfg.u_resample)
    flips = int((own["accepted_len"] != got["accepted_len"]).sum())
    print(f"{cfg.name}: layers {ms.n_layers}, rows {b.n_rows}: teacher-forced layer err {worst_layer:.2e}, K/V rows "
          f"{worst_kv:.2e}, head {head_err:.2e}; free-running logits err/scale {free_err:.2e} "
          f"(bound {free_running_bound(ms.n_layers):.2e}); bands {bands}; accepted {got['accepted_len'].tolist()}; "
          f"servers whose m differs with the oracle's own logits: {flips}")
    return got, state


def test_config3_llama8b_shape_full_size():
    from paper_2512_09963_amd import workload as wl
    cfg = synth.config3()
    ver, kv, db = wl.upload_config(cfg, progress=True)
    _verify_and_compare(cfg, ver, kv, db)


def test_config4_ragged_paged_with_scheduler_in_the_loop():
    """32 servers, ragged gamma and context, permuted pages; three rounds in which the library's scheduler
    picks the next gamma from the accepted lengths and each round is checked against the oracle."""
    from paper_2512_09963_amd import binding as gsb, workload as wl
    ms = synth.LLAMA3_8B if FULL else dataclasses.replace(synth.LLAMA3_8B, n_layers=4)
    cfg = synth.config4(ms=ms)
    ver, kv, db = wl.upload_config(cfg, progress=True)
    n, C = cfg.batch.n_servers, 272
    alpha, X = np.full(n, 0.5), np.ones(n)
    alpha_o, X_o = alpha.copy(), X.copy()
    state = None
    for rnd in range(3):
        got, state = _verify_and_compare(cfg, ver, kv, db, state)
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
        for rows in (state.tf, state.free):
            for key in [k for k in rows if page_owner[k[1]][1] * 16 + k[2] >= ctx[page_owner[k[1]][0]]]:
                del rows[key]


def test_config5_llama70b_shape():
    from paper_2512_09963_amd import workload as wl
    ms = synth.LLAMA3_70B if FULL else dataclasses.replace(synth.LLAMA3_70B, n_layers=4)
    cfg = synth.config5(ms=ms)
    ver, kv, db = wl.upload_config(cfg, progress=True)
    _verify_and_compare(cfg, ver, kv, db)
