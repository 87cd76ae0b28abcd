"""Parity of gs_accept_reject (HIP, through the C ABI) with the oracle on the same seeded inputs."""
import numpy as np
import pytest

from oracle import accept_reject as ar
from paper_2512_09963_amd import synth
from tests.parity import check_accept_outputs

pytestmark = pytest.mark.gpu


def _as_bf16(inp: synth.AcceptInputs):
    """The same inputs with target logits and q rounded to bfloat16 (held in float32 arrays): what a caller of the
    bfloat16 entry point hands over, and what the oracle is given."""
    import dataclasses
    return dataclasses.replace(inp, target_logits=synth.round_to_bf16(inp.target_logits),
                               q_probs=synth.round_to_bf16(inp.q_probs))


def _run_gpu(inp: synth.AcceptInputs, want_ratio=True, offset_elems=0, pinned_out=False, bf16=False):
    import torch
    from paper_2512_09963_amd import binding as gsb
    dev = torch.device("cuda:0")
    wide = torch.bfloat16 if bf16 else torch.float32
    n = inp.gamma.size
    R, G, V = inp.target_logits.shape[0], inp.q_probs.shape[0], inp.vocab

    def up(a, dtype):
        t = torch.from_numpy(np.ascontiguousarray(a)).to(dtype)
        if offset_elems:           # misaligned base: exercises the scalar-load path
            buf = torch.empty(t.numel() + offset_elems, dtype=dtype, device=dev)
            view = buf[offset_elems:].view(t.shape)
            view.copy_(t)
            return view
        return t.to(dev)

    tl, q = up(inp.target_logits, wide), up(inp.q_probs, wide) if G else None
    toks = up(inp.draft_tokens, torch.int32) if G else None
    ua = up(inp.u_accept, torch.float32) if G else None
    ur = up(inp.u_resample, torch.float32)
    cu = torch.from_numpy(synth.cu_rows_of(inp.gamma)).to(dev)
    out = gsb.make_accept_out(n, G, dev, want_ratio)
    if pinned_out:     # results stored by the kernels straight into device-mapped host memory
        out = {k: (torch.empty(v.shape, dtype=v.dtype, pin_memory=True) if v is not None else None)
               for k, v in out.items()}
    for k in ("accepted_len", "next_token"):
        out[k].fill_(-7)
    ws = torch.empty(gsb.gs_accept_workspace_bytes(n, R, V), dtype=torch.uint8, device=dev)
    (gsb.gs_accept_reject_bf16 if bf16 else gsb.gs_accept_reject)(inp.gamma, cu, V, tl, q, toks, ua, ur, out, ws)
    torch.cuda.synchronize()
    return {k: (v.cpu().numpy() if v is not None else None) for k, v in out.items()}


def _check(inp, got):
    return check_accept_outputs(inp.gamma, inp.target_logits, inp.q_probs, inp.draft_tokens, inp.u_accept,
                                inp.u_resample, got)


@pytest.mark.parametrize("vocab,offset", [(1024, 0), (6152, 0), (5003, 0), (6152, 1), (40000, 0)])
@pytest.mark.parametrize("sigma", [0.3, 1.5])
def test_small_ragged_batches(vocab, offset, sigma):
    gamma = np.array([2, 0, 5, 1, 8, 3, 0, 4], dtype=np.int32)
    inp = synth.accept_inputs(100 + vocab, gamma, vocab, sigma)
    got = _run_gpu(inp, offset_elems=offset)
    bands = _check(inp, got)
    assert bands["n_band_m"] + bands["n_band_tok"] <= 1


def test_outputs_in_pinned_host_memory():
    inp = synth.accept_inputs(synth.MASTER_SEED + 5, np.array([3, 0, 7, 2], np.int32), 1500, 1.0)
    got = _run_gpu(inp, pinned_out=True)
    check_accept_outputs(inp.gamma, inp.target_logits, inp.q_probs, inp.draft_tokens, inp.u_accept, inp.u_resample, got)


def test_more_drafts_than_lanes_and_single_server():
    inp = synth.accept_inputs(7, np.array([70], dtype=np.int32), 2048, 0.1)
    got = _run_gpu(inp)
    _check(inp, got)
    inp = synth.accept_inputs(8, np.array([0], dtype=np.int32), 4096, 1.0)
    got = _run_gpu(inp, want_ratio=False)
    _check(inp, got)


def test_all_gamma_zero():
    inp = synth.accept_inputs(9, np.zeros(5, dtype=np.int32), 3000, 1.0)
    got = _run_gpu(inp)
    _check(inp, got)
    assert np.all(got["accepted_len"] == 0)


def test_q_equal_p_accepts_everything_and_draws_the_bonus_from_p():
    gamma = np.array([3, 6], dtype=np.int32)
    inp = synth.accept_inputs(10, gamma, 4096, 0.0)          # sigma = 0: draft logits are the target logits
    inp.u_accept[:] = 0.9999                                # ratio is 1 up to fp32 rounding of q
    got = _run_gpu(inp)
    np.testing.assert_array_equal(got["accepted_len"], gamma)
    _check(inp, got)


def test_degenerate_distributions():
    """q = 0 at the draft token (ratio +inf: accept); disjoint supports (always reject, draw from p);
    residual without mass (q >= p everywhere on the support is impossible, so force it with q = p
    and a rejecting... ratio exactly 1 never rejects; instead: q one-hot on the target's argmax)."""
    V = 4096
    gamma = np.array([1, 1, 1], dtype=np.int32)
    inp = synth.accept_inputs(11, gamma, V, 1.0)
    # server 0: q puts zero mass on its draft token
    t0 = int(inp.draft_tokens[0])
    inp.q_probs[0, t0] = 0.0
    inp.u_accept[0] = 0.999
    # server 1: disjoint supports - target lives on tokens < V/2, draft on tokens >= V/2
    inp.target_logits[2, V // 2:] = -np.inf
    inp.q_probs[1, : V // 2] = 0.0
    inp.q_probs[1] /= inp.q_probs[1].sum()
    inp.draft_tokens[1] = V // 2 + 5
    inp.q_probs[1, V // 2 + 5] = max(inp.q_probs[1, V // 2 + 5], 1e-6)
    inp.u_accept[1] = 2.0 ** -24
    # server 2: one-hot q on the draft token, rejected -> residual is p with that token removed
    t2 = int(inp.draft_tokens[2])
    inp.q_probs[2] = 0.0
    inp.q_probs[2, t2] = 1.0
    inp.u_accept[2] = 0.99
    got = _run_gpu(inp)
    _check(inp, got)
    assert got["accepted_len"][0] == 1 and np.isinf(got["ratio"][0])
    assert got["accepted_len"][1] == 0 and got["next_token"][1] < V // 2
    assert got["accepted_len"][2] == 0 and got["next_token"][2] != t2


def test_residual_without_mass_falls_back_to_p():
    """Point-mass target and draft on the same token with a forced rejection (u > 1 cannot happen
    for real uniforms; the kernel must still follow the rule): max(0, p - q) is all zero."""
    V = 2048
    gamma = np.array([1], dtype=np.int32)
    inp = synth.accept_inputs(12, gamma, V, 1.0)
    inp.target_logits[0] = -np.inf
    inp.target_logits[0, 77] = 0.0
    inp.q_probs[0] = 0.0
    inp.q_probs[0, 77] = 1.0
    inp.draft_tokens[0] = 77
    inp.u_accept[0] = 1.5
    got = _run_gpu(inp)
    assert got["accepted_len"][0] == 0 and got["next_token"][0] == 77
    _check(inp, got)


@pytest.mark.parametrize("sigma", [0.3, 1.0, 3.0])
def test_config2_full_size(sigma):
    """64 servers x gamma 8 over vocab 151936 (576 target rows, 512 draft rows)."""
    gamma = np.full(64, 8, dtype=np.int32)
    inp = synth.accept_inputs(synth.MASTER_SEED, gamma, 151936, sigma)
    got = _run_gpu(inp)
    bands = _check(inp, got)
    rate = got["accepted_len"].mean() / 8
    print(f"sigma={sigma}: mean accepted/gamma = {rate:.3f}, bands = {bands}")
    assert bands["n_band_m"] + bands["n_band_tok"] <= 2


@pytest.mark.parametrize("vocab,offset", [(1024, 0), (6152, 0), (5003, 0), (6152, 1), (6152, 8), (40000, 0)])
@pytest.mark.parametrize("sigma", [0.3, 1.5])
def test_bf16_inputs_small_ragged_batches(vocab, offset, sigma):
    """gs_accept_reject_bf16: the oracle gets the same bfloat16 numbers (widened), so the bar is unchanged."""
    gamma = np.array([2, 0, 5, 1, 8, 3, 0, 4], dtype=np.int32)
    inp = _as_bf16(synth.accept_inputs(300 + vocab, gamma, vocab, sigma))
    got = _run_gpu(inp, offset_elems=offset, bf16=True)
    bands = _check(inp, got)
    assert bands["n_band_m"] + bands["n_band_tok"] <= 1


def test_bf16_inputs_degenerate_rows():
    """q = 0 at the draft token, a one-hot q that is rejected, all gamma zero: the special cases of the rule."""
    V = 4096
    inp = _as_bf16(synth.accept_inputs(13, np.array([1, 1, 0], dtype=np.int32), V, 1.0))
    inp.q_probs[0, int(inp.draft_tokens[0])] = 0.0
    inp.u_accept[0] = 0.999
    t1 = int(inp.draft_tokens[1])
    inp.q_probs[1] = 0.0
    inp.q_probs[1, t1] = 1.0
    inp.u_accept[1] = 0.99
    got = _run_gpu(inp, bf16=True)
    _check(inp, got)
    assert got["accepted_len"][0] == 1 and np.isinf(got["ratio"][0])
    assert got["accepted_len"][1] == 0 and got["next_token"][1] != t1


@pytest.mark.parametrize("sigma", [0.3, 1.0, 3.0])
def test_bf16_inputs_config2_full_size(sigma):
    gamma = np.full(64, 8, dtype=np.int32)
    inp = _as_bf16(synth.accept_inputs(synth.MASTER_SEED, gamma, 151936, sigma))
    got = _run_gpu(inp, bf16=True)
    bands = _check(inp, got)
    print(f"bf16 inputs, sigma={sigma}: mean accepted/gamma = {got['accepted_len'].mean() / 8:.3f}, bands = {bands}")
    assert bands["n_band_m"] + bands["n_band_tok"] <= 2
