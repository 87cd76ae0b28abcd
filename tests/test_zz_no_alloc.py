"""gs_accept_reject_static (the entry point that allocates nothing) gives what gs_accept_reject gives.

Two calls in a row on the library's static scratch array, the second with a smaller batch, each compared
bit for bit with gs_accept_reject on a caller workspace and, to the parity bar, with the oracle.  Collected
last (file name), so that a failure here cannot hide another test behind `pytest -x`.
"""
import numpy as np
import pytest

from paper_2512_09963_amd import synth
from tests.parity import check_accept_outputs

pytestmark = pytest.mark.gpu


def _upload(inp):
    import torch
    dev = torch.device("cuda:0")
    t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a)).to(dt).to(dev)
    G = inp.q_probs.shape[0]
    return dict(tl=t(inp.target_logits, torch.float32), q=t(inp.q_probs, torch.float32) if G else None,
                tok=t(inp.draft_tokens, torch.int32) if G else None, ua=t(inp.u_accept, torch.float32) if G else None,
                ur=t(inp.u_resample, torch.float32), cu=torch.from_numpy(synth.cu_rows_of(inp.gamma)).to(dev))


def _both(inp):
    import torch
    from paper_2512_09963_amd import binding as gsb
    dev = torch.device("cuda:0")
    d = _upload(inp)
    n, G, V, R = inp.gamma.size, inp.q_probs.shape[0], inp.vocab, inp.target_logits.shape[0]
    ref, got = gsb.make_accept_out(n, G, dev), gsb.make_accept_out(n, G, dev)
    for o in (ref, got):
        o["accepted_len"].fill_(-7)
        o["next_token"].fill_(-7)
    ws = torch.empty(gsb.gs_accept_workspace_bytes(n, R, V), dtype=torch.uint8, device=dev)
    gsb.gs_accept_reject(inp.gamma, d["cu"], V, d["tl"], d["q"], d["tok"], d["ua"], d["ur"], ref, ws)
    gsb.gs_accept_reject_static(inp.gamma, d["cu"], V, d["tl"], d["q"], d["tok"], d["ua"], d["ur"], got)
    torch.cuda.synchronize()
    to_np = lambda o: {k: (v.cpu().numpy() if v is not None else None) for k, v in o.items()}
    return to_np(ref), to_np(got)


def test_static_scratch_entry_point_twice_the_second_call_smaller():
    big = synth.accept_inputs(41, np.array([5, 0, 8, 3, 1, 7, 2, 6, 4, 8, 0, 3], np.int32), 40000, 1.0)
    small = synth.accept_inputs(42, np.array([2, 4, 0], np.int32), 6152, 1.5)
    for inp in (big, small):
        ref, got = _both(inp)
        for k in ("accepted_len", "next_token", "accept_stat", "ratio"):
            np.testing.assert_array_equal(got[k], ref[k], err_msg=k)          # same kernels: bit-identical
        bands = check_accept_outputs(inp.gamma, inp.target_logits, inp.q_probs, inp.draft_tokens, inp.u_accept,
                                     inp.u_resample, got)
        assert bands["n_band_m"] + bands["n_band_tok"] <= 1


def test_static_scratch_rejects_batches_beyond_its_size():
    import torch
    from paper_2512_09963_amd import binding as gsb
    dev = torch.device("cuda:0")
    n, g, V = 4200, 1, 262144                       # 4200 servers x 128 tile sums of 8 bytes exceed the array
    gamma = np.full(n, g, np.int32)
    assert gsb.gs_accept_workspace_bytes(n, n * (g + 1), V) > (4 << 20)
    one = torch.zeros(1, dtype=torch.float32, device=dev)
    out = gsb.make_accept_out(n, n * g, dev)
    with pytest.raises(gsb.GsError) as e:           # rejected on the host before anything is read or launched
        gsb.gs_accept_reject_static(gamma, one, V, one, one, one, one, one, out)
    assert e.value.code == -3 and "static array" in str(e.value)
