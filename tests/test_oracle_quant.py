"""Pins of the 4-bit weight dequantisation of the oracle (format of Section IV-A's larger verifier).

What fixes it from outside: the definition worked by hand on small integers and halves (exact in every
format involved); the bf16 rounding checked against the generators' own, separately written rounding routine
on products that are exact in float32; the group structure (a scale or zero point acts on its 128 inputs
only); and, for the synthetic checkpoints the tests feed it, the bound every min/max grid gives: inside the
grid a dequantised weight is within half a step of the original (plus the bf16 rounding of the result), and
a weight of zero is reproduced exactly.
"""
import numpy as np

from oracle import quant
from paper_2512_09963_amd import synth


def test_dequant_by_hand():
    codes = np.zeros((1, 128), np.uint8)
    codes[0, :6] = [0, 15, 7, 8, 3, 12]
    out = quant.dequant_w4(codes, np.array([[0.5]]), np.array([[7]]))
    assert out.shape == (1, 128)
    assert out[0, :6].tolist() == [-3.5, 4.0, 0.0, 0.5, -2.0, 2.5]
    assert np.all(out[0, 6:] == -3.5)


def test_groups_are_independent():
    rng = np.random.default_rng(1)
    codes = rng.integers(0, 16, (3, 384)).astype(np.uint8)
    scales = np.array([[0.25, 0.5, 1.0]] * 3)
    zeros = rng.integers(0, 16, (3, 3)).astype(np.uint8)
    base = quant.dequant_w4(codes, scales, zeros)
    s2 = scales.copy()
    s2[1, 2] = 2.0
    z2 = zeros.copy()
    z2[0, 0] = (z2[0, 0] + 1) % 16
    out = quant.dequant_w4(codes, s2, z2)
    changed = out != base
    assert not changed[2].any()
    assert not changed[1, :256].any() and not changed[0, 128:].any()
    assert np.array_equal(out[1, 256:], 2.0 * base[1, 256:])
    assert changed[0, :128].all()


def test_result_is_rounded_to_bf16_as_torch_rounds():
    """The dequantised weight is (code - zero) * scale rounded once to bfloat16, ties to even: checked against
    torch's own float32 -> bfloat16 conversion (a library routine, not this repository's rounding expression)
    and on hand-made values that sit exactly on a tie."""
    import torch
    rng = np.random.default_rng(2)
    codes = rng.integers(0, 16, (8, 256)).astype(np.uint8)
    zeros = rng.integers(0, 16, (8, 2)).astype(np.uint8)
    scales = torch.from_numpy(rng.uniform(0.001, 0.02, (8, 2)).astype(np.float32)).to(torch.bfloat16).float().numpy()
    out = quant.dequant_w4(codes, scales, zeros)
    # (code - zero) * scale has at most 5 + 8 significant bits: exact in float32, then rounded once
    exact32 = (codes.astype(np.float32) - np.repeat(zeros, 128, axis=1).astype(np.float32)) * np.repeat(scales, 128, axis=1)
    want = torch.from_numpy(exact32).to(torch.bfloat16).float().numpy().astype(np.float64)
    assert np.array_equal(out, want)
    # by hand: scale 1 + 2^-7 (a bf16 value).  Code 3: 3.0234375 lies exactly halfway between the bf16 neighbours
    # 3.015625 and 3.03125 (step 2^-6); the tie goes to the even mantissa, 3.03125.  Code 5: 5.0390625 is a
    # quarter step (step 2^-5) above 5.03125 and rounds down to it.
    c = np.zeros((1, 128), np.uint8); c[0, 0], c[0, 1] = 3, 5
    got = quant.dequant_w4(c, np.array([[1.0 + 2.0 ** -7]], np.float32), np.zeros((1, 1), np.uint8))
    assert got[0, 0] == 3.03125 and got[0, 1] == 5.03125 and got[0, 2] == 0.0


def test_synthetic_checkpoint_is_within_half_a_step():
    rng = np.random.default_rng(3)
    w = synth.round_to_bf16((0.02 * rng.standard_normal((16, 512))).astype(np.float32))
    w[3, 100:140] = 0.0
    codes, scales, zeros = synth.quantize_w4(w)
    assert codes.dtype == np.uint8 and codes.max() <= 15 and zeros.max() <= 15
    assert np.array_equal(synth.round_to_bf16(scales), scales) and np.all(scales > 0)
    deq = quant.dequant_w4(codes, scales, zeros)
    step = np.repeat(scales, 128, axis=1).astype(np.float64)
    # half a step, plus the rounding of the scale (the grid end may fall short by 15 * 2^-9 of a step),
    # plus the bf16 rounding of the result
    bound = step * (0.5 + 15 * 2.0 ** -9) + np.abs(w) * 2.0 ** -8
    assert np.all(np.abs(deq - w) <= bound)
    assert np.all(deq[3, 100:140] == 0.0)
