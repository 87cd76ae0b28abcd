"""Parity of gs_verify_batch (HIP, through the C ABI) with the forward + accept oracle.

Tolerances (relative to the row scale max|logit|, see tests/parity.py for the decisions):
fp32 models 1e-4, bf16 models 2e-2.
"""
import numpy as np
import pytest

from oracle import accept_reject as ar
from oracle import forward as fw
from paper_2512_09963_amd import synth
from tests.parity import check_accept_outputs

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def assert_logits_close(got, want, tol, what="logits"):
    scale = np.abs(want).max(axis=1, keepdims=True)
    err = np.abs(got.astype(np.float64) - want) / scale
    worst = err.max()
    assert worst <= tol, f"{what}: max |diff| / row scale = {worst:.3g} > {tol:g} (row {int(err.max(axis=1).argmax())})"
    return worst


def _model(ms, seed, std):
    top = synth.top_weights(ms, seed, std)
    layers = [synth.layer_weights(ms, seed, l, std) for l in range(ms.n_layers)]
    return top, layers


def _oracle_cache(ms, seed, n_pages, page, synthetic):
    out = []
    for l in range(ms.n_layers):
        if synthetic:
            out.append((synth.kv_layer_cache(ms, seed, l, "k", n_pages, page),
                        synth.kv_layer_cache(ms, seed, l, "v", n_pages, page)))
        else:
            shape = (n_pages, ms.n_kv_heads, page, ms.head_dim)
            out.append((np.zeros(shape, np.float32), np.zeros(shape, np.float32)))
    return out


def _check_kv_rows(ms, kv_dev, cache, batch, tol):
    """The block's appended K/V rows agree with the oracle's."""
    for l in range(ms.n_layers):
        k_g, v_g = kv_dev.get_layer(l)
        for i in range(batch.n_servers):
            for pos in range(int(batch.ctx_len[i]), int(batch.ctx_len[i] + batch.gamma[i] + 1)):
                pg, sl = int(batch.block_table[i, pos // batch.page_size]), pos % batch.page_size
                for got, want, name in ((k_g, cache[l][0], "K"), (v_g, cache[l][1], "V")):
                    w = want[pg, :, sl, :].astype(np.float64)
                    g = got[pg, :, sl, :].astype(np.float64)
                    assert np.abs(g - w).max() <= tol * max(np.abs(w).max(), 1e-6) + 1e-7, \
                        f"{name} layer {l} server {i} pos {pos}"


def _run_case(ms, seed, gamma, ctx_len, page, std, synthetic_kv=True, permute=True, sigma=0.5):
    import torch
    from paper_2512_09963_amd import workload as wl
    tol = TOL[ms.dtype]
    top, layers = _model(ms, seed, std)
    batch = synth.make_batch(seed, gamma, ctx_len, page, permute_pages=permute)
    tokens, q, ua, ur = synth.verify_side_inputs(seed, ms.vocab, batch.gamma, sigma=sigma)
    cache = _oracle_cache(ms, seed, batch.n_pages, page, synthetic_kv)
    ver = wl.upload_model(ms, top, lambda l: layers[l])
    kv = wl.KVCache(ms, batch.n_pages, page)
    for l in range(ms.n_layers):
        kv.set_layer(l, cache[l][0], cache[l][1])
    db = wl.DeviceBatch(batch, tokens, q, ua, ur)
    out, logits, _ = wl.verify(ver, kv, db)
    torch.cuda.synchronize()
    got_logits = logits.cpu().numpy()
    want_logits = fw.verify_forward(ms, tokens, batch.gamma, batch.ctx_len, batch.block_table, page, top,
                                    lambda l: layers[l], lambda l: cache[l])
    worst = assert_logits_close(got_logits, want_logits, tol)
    _check_kv_rows(ms, kv, cache, batch, tol)
    got = {k: v.cpu().numpy() for k, v in out.items()}
    cu = batch.cu_rows
    d_tok = np.concatenate([tokens[cu[i] + 1:cu[i + 1]] for i in range(batch.n_servers)]) if batch.n_draft else np.zeros(0, np.int32)
    # teacher-forced: the oracle's accept stage on the GPU's own logits must agree outside the bands
    bands = check_accept_outputs(batch.gamma, got_logits, q, d_tok, ua, ur, got)
    return dict(worst=worst, bands=bands, got=got, want_logits=want_logits, q=q, d_tok=d_tok, ua=ua, ur=ur,
                batch=batch)


def test_config1_tiny_fp32_with_real_prefill():
    """2 layers, d 256, 4 heads of 64, FFN 1024, vocab 1024; 4 servers, gamma [2,3,4,5], 64-token prefixes
    that both sides prefill themselves (the GPU through gs_verify_batch with 64-row blocks)."""
    import torch
    from paper_2512_09963_amd import workload as wl
    ms, seed, page = synth.TINY, synth.MASTER_SEED, 16
    top, layers = _model(ms, seed, 0.02)
    gamma, ctx = np.array([2, 3, 4, 5], np.int32), np.full(4, 64, np.int32)
    batch = synth.make_batch(seed, gamma, ctx, page, permute_pages=True)
    prefix = synth.uniform_int(seed, ("prefix",), 0, ms.vocab - 1, 4 * 64)
    pre_batch = synth.BatchShape(np.full(4, 63, np.int32), np.zeros(4, np.int32), page, batch.block_table, batch.n_pages)
    cache = _oracle_cache(ms, seed, batch.n_pages, page, synthetic=False)
    want_pre = fw.verify_forward(ms, prefix, pre_batch.gamma, pre_batch.ctx_len, batch.block_table, page, top,
                                 lambda l: layers[l], lambda l: cache[l])
    ver = wl.upload_model(ms, top, lambda l: layers[l])
    kv = wl.KVCache(ms, batch.n_pages, page)
    _, logits_pre, _ = wl.verify(ver, kv, wl.DeviceBatch(pre_batch, prefix))
    torch.cuda.synchronize()
    assert_logits_close(logits_pre.cpu().numpy(), want_pre, 1e-4, "prefill logits")

    tokens, q, ua, ur = synth.verify_side_inputs(seed, ms.vocab, gamma, sigma=0.5)
    out, logits, _ = wl.verify(ver, kv, wl.DeviceBatch(batch, tokens, q, ua, ur))
    torch.cuda.synchronize()
    want = fw.verify_forward(ms, tokens, gamma, ctx, batch.block_table, page, top, lambda l: layers[l], lambda l: cache[l])
    got_logits = logits.cpu().numpy()
    assert_logits_close(got_logits, want, 1e-4)
    _check_kv_rows(ms, kv, cache, batch, 1e-4)
    p_got = np.stack([ar.softmax(r) for r in got_logits]); p_want = np.stack([ar.softmax(r) for r in want])
    assert np.all(np.abs(p_got - p_want) <= 1e-4 * np.maximum(p_want, 1.0 / ms.vocab))
    got = {k: v.cpu().numpy() for k, v in out.items()}
    cu = batch.cu_rows
    d_tok = np.concatenate([tokens[cu[i] + 1:cu[i + 1]] for i in range(4)])
    check_accept_outputs(gamma, got_logits, q, d_tok, ua, ur, got)            # teacher-forced
    check_accept_outputs(gamma, want.astype(np.float32), q, d_tok, ua, ur, got)  # fully independent end to end


@pytest.mark.parametrize("name,ms", [
    ("g4_hd128", synth.ModelShape(2, 256, 4, 1, 128, 512, 1024, 500000.0, dtype="bf16")),
    ("g2_hd64", synth.ModelShape(2, 256, 8, 4, 64, 512, 1024, 10000.0, dtype="bf16")),
    ("g8_hd128", synth.ModelShape(1, 256, 8, 1, 128, 384, 2048, 500000.0, dtype="bf16")),
    ("g1_hd128", synth.ModelShape(1, 128, 2, 2, 128, 256, 1024, 500000.0, dtype="bf16")),
])
def test_small_bf16_models_ragged_paged(name, ms):
    gamma = np.array([0, 16, 3, 7, 1, 5], np.int32)
    ctx = np.array([5, 40, 300, 1000, 17, 0], np.int32)
    r = _run_case(ms, 77, gamma, ctx, 16, std=0.08)
    print(name, "worst logits error / scale:", r["worst"], r["bands"])


def test_small_f32_model_with_gqa_and_page_32():
    ms = synth.ModelShape(2, 128, 4, 2, 64, 256, 500, 10000.0, dtype="f32")
    r = _run_case(ms, 78, np.array([3, 0, 6], np.int32), np.array([33, 2, 130], np.int32), 32, std=0.08)
    print("worst", r["worst"])


@pytest.mark.parametrize("gamma", [[3, 1, 5], [16, 12, 9, 15, 11, 14]])
def test_bf16_wide_vocabulary_statistics_from_the_lm_head_epilogue(gamma):
    # V / 128 >= 192: the LM head takes the 8-wave kernel (12 rows) or the tall one (83 rows) as one launch, whose
    # epilogue leaves the softmax statistics per column block; the accept stage merges them instead of
    # reading the logits again.  The decisions below are therefore checked against the oracle on that path.
    ms = synth.ModelShape(1, 128, 2, 1, 64, 256, 24576, 10000.0, dtype="bf16")
    _run_case(ms, 86, np.array(gamma, np.int32), np.array([30, 0, 77, 5, 100, 64][:len(gamma)], np.int32), 16, std=0.08)


def test_bf16_page_size_64_and_single_server():
    ms = synth.ModelShape(1, 256, 4, 1, 128, 512, 1024, 500000.0, dtype="bf16")
    _run_case(ms, 79, np.array([8], np.int32), np.array([700], np.int32), 64, std=0.08)


@pytest.mark.parametrize("n_servers,gmax", [(10, 8), (24, 16)])
def test_bf16_many_rows_use_the_tall_projection_kernel(n_servers, gmax):
    # 60..250 target rows: more than one 64-row tile set, with and without row chunks
    ms = synth.ModelShape(2, 256, 4, 2, 128, 512, 1024, 500000.0, dtype="bf16")
    rng = np.random.default_rng(81 + n_servers)
    gamma = rng.integers(gmax // 2, gmax + 1, n_servers).astype(np.int32)
    ctx = rng.integers(0, 200, n_servers).astype(np.int32)
    assert int(gamma.sum()) + n_servers > 64
    _run_case(ms, 81, gamma, ctx, 16, std=0.08)


def test_bf16_many_rows_with_widths_that_are_not_multiples_of_128():
    # d = 192, the QKV width 192 and V = 960 are multiples of 64 only: these projections take the 64-column
    # kernel with row chunks (column blocks padded to a multiple of 8 in the grid), gate/up the 128-column one
    ms = synth.ModelShape(1, 192, 1, 1, 64, 320, 960, 10000.0, dtype="bf16")
    rng = np.random.default_rng(83)
    gamma = rng.integers(6, 13, 16).astype(np.int32)
    ctx = rng.integers(0, 120, 16).astype(np.int32)
    assert int(gamma.sum()) + 16 > 128
    _run_case(ms, 83, gamma, ctx, 16, std=0.08)


def test_bf16_block_of_hundreds_of_rows_on_an_empty_cache():
    # 6 x 112 = 672 rows: the projection shape for row counts where the MFMA pipes are the bound, and
    # attention with 28 query tiles per KV head (several passes of 8 waves) over keys of the block itself
    ms = synth.ModelShape(1, 256, 4, 1, 128, 512, 1024, 500000.0, dtype="bf16")
    _run_case(ms, 82, np.full(6, 111, np.int32), np.zeros(6, np.int32), 16, std=0.08)


@pytest.mark.parametrize("group,gamma,ctx", [
    # rows per KV head T*G around the 32-row wave tile; keys around the 32-key step and the 16-key page
    (4, [7, 8, 15, 16], [0, 1, 15, 16]),
    (4, [7, 8, 15, 16], [17, 24, 31, 32]),
    (8, [3, 4, 7, 8], [33, 63, 64, 65]),
    (1, [31, 32, 63, 0], [95, 96, 97, 191]),
    # contexts around multiples of the steps-per-workgroup choices (6 steps = 192 keys, and larger)
    (4, [2, 2, 2, 2, 2, 2], [190, 191, 192, 193, 383, 385]),
    (2, [5, 1, 9, 3], [1023, 1024, 2047, 2049]),
])
def test_bf16_attention_tile_and_split_boundaries(group, gamma, ctx):
    ms = synth.ModelShape(1, 128, 2 * group, 2, 64, 128, 512, 10000.0, dtype="bf16")
    _run_case(ms, 84, np.array(gamma, np.int32), np.array(ctx, np.int32), 16, std=0.08)


def test_bf16_more_servers_than_one_round_of_the_attention_work_list():
    # 300 servers (the work list is built 256 servers at a time), most with a single short split, a few long
    # enough for several; gamma 0..2, so that the row count stays small for the oracle
    ms = synth.ModelShape(1, 128, 4, 2, 64, 128, 512, 10000.0, dtype="bf16")
    rng = np.random.default_rng(85)
    gamma = rng.integers(0, 3, 300).astype(np.int32)
    ctx = rng.integers(0, 40, 300).astype(np.int32)
    ctx[[3, 130, 255, 256, 299]] = [900, 1500, 700, 2100, 1200]
    _run_case(ms, 85, gamma, ctx, 16, std=0.08)


def test_bf16_more_server_head_pairs_than_resident_workgroups():
    # 200 servers x 8 KV heads = 1600 (server, head) pairs, more than the attention launch keeps resident at once:
    # the planner's several-rounds branch, with a few contexts long enough for many uneven splits
    ms = synth.ModelShape(1, 128, 8, 8, 64, 128, 512, 10000.0, dtype="bf16")
    rng = np.random.default_rng(86)
    gamma = rng.integers(0, 3, 200).astype(np.int32)
    ctx = rng.integers(0, 60, 200).astype(np.int32)
    ctx[[0, 77, 199]] = [1300, 2500, 845]
    _run_case(ms, 86, gamma, ctx, 16, std=0.08)


@pytest.mark.parametrize("seed", range(8))
def test_bf16_seeded_random_shapes(seed):
    # model widths, head layout, page size, server count, draft lengths and contexts drawn from the seed: walks the
    # launch planners (row-tile variants of the projections, waves per attention workgroup, split counts)
    rng = np.random.default_rng(9000 + seed)
    hd = int(rng.choice([64, 128]))
    n_kv = int(rng.choice([1, 2, 4]))
    group = int(rng.choice([1, 2, 4, 8]))
    d = 64 * int(rng.integers(2, 6))
    F = 64 * int(rng.integers(2, 9))
    V = 64 * int(rng.integers(8, 24))
    ms = synth.ModelShape(int(rng.integers(1, 3)), d, n_kv * group, n_kv, hd, F, V, 10000.0, dtype="bf16")
    n = int(rng.integers(1, 12))
    gamma = rng.integers(0, int(rng.choice([3, 9, 17])), n).astype(np.int32)
    ctx = rng.integers(0, int(rng.choice([40, 400, 1500])), n).astype(np.int32)
    page = int(rng.choice([16, 32, 48, 64]))
    r = _run_case(ms, 9000 + seed, gamma, ctx, page, std=0.08)
    print(seed, ms, "servers", n, "rows", int(gamma.sum()) + n, "page", page, "worst", r["worst"], r["bands"])


def test_bf16_page_size_48_not_a_power_of_two():
    ms = synth.ModelShape(1, 256, 8, 2, 128, 512, 1024, 500000.0, dtype="bf16")
    _run_case(ms, 80, np.array([5, 2, 9], np.int32), np.array([100, 47, 530], np.int32), 48, std=0.08)


def test_verify_batch_rejects_bad_descriptors():
    import torch
    from paper_2512_09963_amd import binding as gsb, workload as wl
    ms = synth.ModelShape(1, 128, 2, 2, 64, 256, 512, 10000.0, dtype="f32")
    top, layers = _model(ms, 3, 0.02)
    ver = wl.upload_model(ms, top, lambda l: layers[l])
    batch = synth.make_batch(3, np.array([2, 2], np.int32), np.array([10, 10], np.int32), 16)
    tokens, q, ua, ur = synth.verify_side_inputs(3, ms.vocab, batch.gamma)
    kv = wl.KVCache(ms, batch.n_pages, 16)
    db = wl.DeviceBatch(batch, tokens, q, ua, ur)
    small = torch.empty(64, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(gsb.GsError) as e:
        wl.verify(ver, kv, db, workspace=small)
    assert e.value.code == -3
    db.ctx_len_host = np.array([10, 1000], np.int32)          # needs more blocks than the table has
    with pytest.raises(gsb.GsError) as e:
        wl.verify(ver, kv, db)
    assert e.value.code == -3 and "KV blocks" in str(e.value)
    with pytest.raises(gsb.GsError) as e:
        gsb.Verifier(dict(n_layers=1, d_model=100, n_heads=3, n_kv_heads=2, head_dim=64, d_ffn=256, vocab=512,
                          rope_theta=1e4, rms_eps=1e-5, dtype="f32"), ver._keep[0], ver._keep[1])
    assert e.value.code == -2


def test_check_batch_names_the_first_violation_and_bad_token_ids_are_never_used_as_indices():
    """gs_check_batch (debug aid) against deliberately inconsistent device-side descriptors, each of which
    the kernels' own guards keep in bounds; and the documented behaviour of gs_verify_batch without the check:
    a draft token id outside the vocabulary gives accepted_len = -1 for that server only."""
    import torch
    from paper_2512_09963_amd import binding as gsb, workload as wl
    ms = synth.ModelShape(1, 128, 2, 2, 64, 256, 512, 10000.0, dtype="bf16")
    top, layers = _model(ms, 5, 0.08)
    ver = wl.upload_model(ms, top, lambda l: layers[l])
    batch = synth.make_batch(5, np.array([2, 3, 1], np.int32), np.array([10, 40, 3], np.int32), 16)
    tokens, q, ua, ur = synth.verify_side_inputs(5, ms.vocab, batch.gamma)
    kv = wl.KVCache(ms, batch.n_pages, 16)
    db = wl.DeviceBatch(batch, tokens, q, ua, ur)
    ws = torch.empty(1024, dtype=torch.uint8, device="cuda:0")

    def check(d):
        ver.gs_check_batch(kv.k, kv.v, kv.page_size, kv.n_pages, d.gamma, d.ctx_len_host, d.cu_rows, d.ctx_len,
                           d.tokens, d.block_table, ws)

    check(db)                                            # consistent: passes
    good_out, good_logits, _ = wl.verify(ver, kv, db)
    torch.cuda.synchronize()
    good_m = good_out["accepted_len"].cpu().numpy().copy()

    bad = wl.DeviceBatch(batch, tokens, q, ua, ur)
    bad.tokens[4] = ms.vocab + 5                         # server 1's first draft token
    with pytest.raises(gsb.GsError) as e:
        check(bad)
    assert e.value.code == -1 and "tokens[4]" in str(e.value) and "vocabulary" in str(e.value)
    out, _, _ = wl.verify(ver, kv, bad)                  # without the check: flagged, nothing read out of range
    torch.cuda.synchronize()
    m = out["accepted_len"].cpu().numpy()
    assert m[1] == -1 and m[0] == good_m[0]

    bad = wl.DeviceBatch(batch, tokens, q, ua, ur)
    bad.cu_rows[2] += 1
    with pytest.raises(gsb.GsError) as e:
        check(bad)
    assert "cu_rows[2]" in str(e.value)
    bad = wl.DeviceBatch(batch, tokens, q, ua, ur)
    bad.ctx_len[0] = 11
    with pytest.raises(gsb.GsError) as e:
        check(bad)
    assert "ctx_len[0]" in str(e.value)
    bad = wl.DeviceBatch(batch, tokens, q, ua, ur)
    bad.block_table[1, 0] = batch.n_pages
    with pytest.raises(gsb.GsError) as e:
        check(bad)
    assert "block_table[1][0]" in str(e.value)


def test_stream_read_probe_runs_and_validates_its_arguments():
    """Measurement aid of bench.py: enqueues, leaves the source untouched, rejects a misaligned source."""
    import torch
    from paper_2512_09963_amd import binding as gsb
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda:0")
    sink = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda:0")
    gsb.gs_probe_stream_read(src, sink)
    gsb.gs_probe_stream_read(src[:1001], sink)              # ragged size
    torch.cuda.synchronize()
    assert int(src[-1]) == (1 << 20) - 1
    with pytest.raises(gsb.GsError):
        gsb.gs_probe_stream_read(src[1:], sink)
