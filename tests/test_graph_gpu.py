"""gs_verify_batch under HIP graph capture: the call allocates nothing, never synchronises and records no
memset, so a caller may capture it once and replay it.  The step is captured on a small bf16 model (whose
logits the ordinary parity test already holds to the oracle) and replayed several times with eager calls and
synchronisations in between; every replay must reproduce the eager result bit for bit, including after the
inputs in the (fixed) device buffers have been changed between replays.
"""
import numpy as np
import pytest

from paper_2512_09963_amd import synth

pytestmark = pytest.mark.gpu


def test_captured_step_replays_bit_exactly():
    import torch
    from paper_2512_09963_amd import binding as gsb, workload as wl
    ms = synth.ModelShape(2, 256, 4, 1, 128, 512, 1024, 500000.0, dtype="bf16")
    seed = 91
    top = synth.top_weights(ms, seed, std=0.08)
    layers = [synth.layer_weights(ms, seed, l, std=0.08) for l in range(ms.n_layers)]
    gamma = np.array([4, 0, 9, 2, 6], np.int32)
    ctx = np.array([37, 5, 260, 0, 129], np.int32)
    batch = synth.make_batch(seed, gamma, ctx, 16, permute_pages=True)
    tokens, q, ua, ur = synth.verify_side_inputs(seed, ms.vocab, batch.gamma, sigma=0.5)
    ver = wl.upload_model(ms, top, lambda l: layers[l])
    kv = wl.KVCache(ms, batch.n_pages, 16)
    for l in range(ms.n_layers):
        kv.set_layer(l, synth.kv_layer_cache(ms, seed, l, "k", batch.n_pages, 16),
                     synth.kv_layer_cache(ms, seed, l, "v", batch.n_pages, 16))
    db = wl.DeviceBatch(batch, tokens, q, ua, ur)
    dev = torch.device("cuda:0")
    ws = torch.empty(ver.gs_workspace_bytes(db.n_rows, db.n_servers, db.max_ctx), dtype=torch.uint8, device=dev)

    def eager():
        out, logits, _ = wl.verify(ver, kv, db, workspace=ws)
        torch.cuda.synchronize()
        return logits.clone(), {k: v.clone() for k, v in out.items() if v is not None}

    ref_logits, ref_out = eager()

    # capture: fixed output buffers, the library enqueues on the capturing stream
    g_out = gsb.make_accept_out(db.n_servers, db.n_draft, dev)
    g_logits = torch.empty(db.n_rows, ms.vocab, dtype=torch.float32, device=dev)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ver.gs_verify_batch(kv.k, kv.v, kv.page_size, kv.n_pages, db.gamma, db.ctx_len_host, db.cu_rows, db.ctx_len,
                            db.tokens, db.block_table, db.q_probs, db.u_accept, db.u_resample, g_out, g_logits, ws,
                            None)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ver.gs_verify_batch(kv.k, kv.v, kv.page_size, kv.n_pages, db.gamma, db.ctx_len_host, db.cu_rows, db.ctx_len,
                            db.tokens, db.block_table, db.q_probs, db.u_accept, db.u_resample, g_out, g_logits, ws,
                            None)

    def check(tag, want_logits, want_out):
        torch.cuda.synchronize()
        assert torch.equal(g_logits, want_logits), f"{tag}: logits differ from the eager call"
        for k, v in want_out.items():
            assert torch.equal(g_out[k], v), f"{tag}: {k} differs from the eager call"

    for rep in range(3):
        g_logits.zero_()
        for v in g_out.values():
            if v is not None:
                v.zero_()
        graph.replay()
        check(f"replay {rep}", ref_logits, ref_out)
        eager()                      # the program's own eager work between replays

    # same graph, other inputs in the same device buffers (token ids and uniforms)
    new_tokens = (db.tokens + 17) % ms.vocab
    db.tokens.copy_(new_tokens)
    db.u_resample.copy_(1.0 - db.u_resample.clamp(min=1e-3))
    ref2_logits, ref2_out = eager()
    assert not torch.equal(ref2_logits, ref_logits)
    graph.replay()
    check("replay with new inputs", ref2_logits, ref2_out)
