"""Pins of the closed-loop oracle (Algorithm 1 with simulated draft servers; baselines of Section IV-A).

What fixes it from outside: the allocation constraint (every round's draft lengths sum to C), the baselines'
definitions on hand-worked inputs, the paper's qualitative result (Section IV-B: on heterogeneous draft
servers the gradient allocation reaches a higher log utility than the even split and the random split),
the symmetric special case (identical servers: the gradient allocation stays within one slot of the even
split), and the estimator property the paper plots (the smoothed goodput tracks the realised one).
"""
import numpy as np

from oracle import closed_loop as ol
from paper_2512_09963_amd import synth

SEED = 20251209


def _inputs(vocab, sigmas, seed=SEED):
    return lambda t, g: synth.loop_round_inputs(seed, t, g, vocab, sigmas)


def test_fixed_allocation_by_hand():
    assert ol.fixed_allocation(24, 6).tolist() == [4] * 6
    assert ol.fixed_allocation(10, 4).tolist() == [3, 3, 2, 2]
    assert ol.fixed_allocation(2, 4).tolist() == [1, 1, 0, 0]


def test_random_allocation_by_hand():
    u = np.array([0.0, 0.24, 0.25, 0.5, 0.99, 0.75, 0.1], dtype=np.float32)
    # floor(u * 4) = 0, 0, 1, 2, 3, 3 for the first six slots; the seventh uniform is not consumed
    assert ol.random_allocation(6, 4, u).tolist() == [2, 1, 1, 2]


def test_every_round_uses_the_whole_capacity():
    sig = np.array([0.3, 0.8, 1.5, 2.5])
    for policy in ("goodspeed", "fixed", "random"):
        h = ol.run(policy, 4, 14, 25, _inputs(256, sig), lambda t: synth.loop_policy_uniforms(SEED, t, 14))
        assert all(int(np.sum(g)) == 14 for g in h["gamma"]), policy
        for g, m in zip(h["gamma"], h["accepted_len"]):
            assert np.all(m >= 0) and np.all(m <= g)


def test_gradient_allocation_beats_the_baselines_on_heterogeneous_servers():
    sig = np.array([0.2, 0.4, 0.7, 1.0, 1.5, 2.5])
    runs = {p: ol.run(p, 6, 24, 150, _inputs(512, sig), lambda t: synth.loop_policy_uniforms(SEED, t, 24))
            for p in ("goodspeed", "fixed", "random")}
    u = {p: ol.utility(h) for p, h in runs.items()}
    assert u["goodspeed"] > u["fixed"] + 0.05 > u["random"] + 0.05, u
    # it does so by giving the well-aligned drafters longer blocks
    g_mean = np.mean(runs["goodspeed"]["gamma"][50:], axis=0)
    assert g_mean[0] > g_mean[-1] + 2
    # and its acceptance-rate estimates are ordered like the servers' noise levels
    a = runs["goodspeed"]["alpha_hat"]
    assert a[0] > a[2] > a[5]


def test_identical_servers_get_the_even_split():
    sig = np.full(4, 0.7)
    h = ol.run("goodspeed", 4, 16, 120, _inputs(256, sig))
    g_mean = np.mean(h["gamma"][20:], axis=0)
    assert np.all(np.abs(g_mean - 4.0) < 1.0), g_mean
    f = ol.run("fixed", 4, 16, 120, _inputs(256, sig))
    assert abs(ol.utility(h) - ol.utility(f)) < 0.15


def test_smoothed_goodput_tracks_the_realised_goodput():
    sig = np.array([0.3, 1.0, 2.0])
    h = ol.run("goodspeed", 3, 12, 200, _inputs(256, sig), beta=0.1)
    realised = (np.asarray(h["accepted_len"][100:], dtype=np.float64) + 1.0).mean(axis=0)
    assert np.all(np.abs(h["X"] - realised) / realised < 0.35), (h["X"], realised)
