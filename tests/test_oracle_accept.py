"""Pins of the accept/reject + resample oracle against what the paper and the
mathematics fix (Section II-A-2; the acceptance probability alpha of the same
section; the capped-geometric goodput of Section III-B)."""
import itertools

import numpy as np
import pytest

from oracle import accept_reject as ar
from oracle import schedule as sch


def _logits_of(p):
    return np.log(np.asarray(p, dtype=np.float64))


def _rand_dist(rng, V, zeros=0):
    w = rng.random(V) + 0.05
    if zeros:
        w[rng.choice(V, zeros, replace=False)] = 0.0
    return w / w.sum()


# ---------------------------------------------------------------- accept rule

def test_accepted_length_never_exceeds_gamma():
    rng = np.random.default_rng(1)
    for _ in range(50):
        V, S = 7, int(rng.integers(0, 6))
        tl = rng.normal(size=(S + 1, V))
        q = np.stack([_rand_dist(rng, V) for _ in range(S)]) if S else np.zeros((0, V))
        toks = rng.integers(0, V, S)
        m, sp, stat, ra = ar.verify_server(tl, q, toks, rng.random(S), rng.random())
        assert 0 <= m <= S and 0 <= sp < V and 0.0 <= stat <= 1.0


def test_q_equal_p_accepts_everything_for_any_uniform():
    rng = np.random.default_rng(2)
    V, S = 9, 5
    tl = rng.normal(size=(S + 1, V)) * 2
    q = np.stack([ar.softmax(tl[j]) for j in range(S)])  # float64: ratio is exactly 1
    toks = rng.integers(0, V, S)
    u_max = np.full(S, 1.0 - 2.0 ** -24)
    m, sp, stat, ra = ar.verify_server(tl, q, toks, u_max, 0.3)
    assert m == S and stat == 1.0 and np.all(ra == 1.0)
    # bonus token comes from p_{S+1}: inverse CDF of that row
    p_last = ar.softmax(tl[S])
    assert sp == int(np.searchsorted(np.cumsum(p_last), 0.3, side="right"))


def test_zero_uniforms_accept_everything():
    rng = np.random.default_rng(3)
    V, S = 6, 4
    tl = rng.normal(size=(S + 1, V))
    q = np.stack([_rand_dist(rng, V) for _ in range(S)])
    m, *_ = ar.verify_server(tl, q, rng.integers(0, V, S), np.zeros(S), 0.5)
    assert m == S


@pytest.mark.parametrize("a", [0.125, 0.5, 0.75])
def test_one_hot_draft_accepts_iff_u_le_target_prob(a):
    V, s = 4, 2
    p = np.full(V, (1 - a) / (V - 1)); p[s] = a
    tl = np.stack([_logits_of(p), _logits_of(p)])
    q = np.zeros((1, V)); q[0, s] = 1.0
    for u, want in [(a - 1e-9, 1), (a + 1e-9, 0), (0.0, 1), (0.999, 0)]:
        m, *_ = ar.verify_server(tl, q, [s], [u], 0.1)
        assert m == want
    # equality accepts (the paper rejects only when r > p/q); dyadic values make p/q exact
    tle = np.zeros((2, 4))
    qe = np.array([[0.0, 0.0, 0.5, 0.5]])
    m, *_ = ar.verify_server(tle, qe, [2], [0.5], 0.1)   # ratio = 0.25/0.5 = 0.5 exactly
    assert m == 1
    m, *_ = ar.verify_server(tle, qe, [2], [np.nextafter(0.5, 1)], 0.1)
    assert m == 0


def test_first_rejection_stops_the_count_but_not_the_statistic():
    V = 4
    tl = np.zeros((4, V))                       # p uniform = 1/4
    q = np.array([[0.5, 0.5, 0, 0], [0.5, 0.5, 0, 0], [0.125, 0.125, 0.25, 0.5]])
    toks = [0, 1, 0]                             # ratios 0.5, 0.5, 2.0
    m, sp, stat, ra = ar.verify_server(tl, q, toks, [0.4, 0.6, 0.0], 0.0)
    assert m == 1
    np.testing.assert_allclose(ra, [0.5, 0.5, 2.0])
    assert stat == pytest.approx((0.5 + 0.5 + 1.0) / 3)   # all S positions, capped at 1
    # residual at position 2: max(0, 1/4 - q) = (0, 0, 1/4, 1/4) -> u = 0 picks token 2
    assert sp == 2


def test_zero_draft_probability_accepts():
    tl = np.zeros((2, 4))
    q = np.array([[0.0, 1.0, 0.0, 0.0]])
    m, sp, stat, ra = ar.verify_server(tl, q, [0], [0.99], 0.2)
    assert m == 1 and np.isinf(ra[0]) and stat == 1.0


def test_gamma_zero_emits_bonus_from_p1():
    p = np.array([0.1, 0.2, 0.3, 0.4])
    m, sp, stat, ra = ar.verify_server(_logits_of(p)[None], np.zeros((0, 4)), [], [], 0.35)
    assert m == 0 and sp == 2 and stat == 0.0 and ra.size == 0


# ---------------------------------------------------------------- inverse CDF

def test_inverse_cdf_matches_linear_scan_and_skips_zero_mass():
    rng = np.random.default_rng(5)
    for _ in range(200):
        V = int(rng.integers(2, 12))
        w = _rand_dist(rng, V, zeros=int(rng.integers(0, V - 1)))
        u = rng.random()
        run, want = 0.0, None
        for s in range(V):                      # brute force: first s whose running sum exceeds u*total
            run += w[s]
            if run > u * w.sum():
                want = s
                break
        got = ar.inverse_cdf(w, u)
        if want is not None:
            assert got == want
        assert w[got] > 0
    assert ar.inverse_cdf(np.array([0.0, 0.0, 0.5, 0.5]), 0.0) == 2
    assert ar.inverse_cdf(np.array([0.5, 0.5, 0.0, 0.0]), 1.0 - 2 ** -24) == 1


def test_residual_special_cases():
    p = np.array([0.1, 0.2, 0.3, 0.4])
    np.testing.assert_allclose(ar.residual_weights(p, np.zeros(4)), p)          # q = 0 -> residual is p
    np.testing.assert_allclose(ar.residual_weights(p, p), p)                    # no mass -> fall back to p
    np.testing.assert_allclose(ar.residual_weights(p, np.array([0.4, 0.3, 0.2, 0.1])), [0, 0, 0.1, 0.3])


# ---------------------------------------------------------------- output law = target

@pytest.mark.parametrize("V", [3, 4, 5, 8])
def test_output_law_equals_target_by_enumeration(V):
    """min(p,q)(s) + (1 - sum min(p,q)) * res(s) = p(s), via the oracle's own ratio/residual routines."""
    rng = np.random.default_rng(100 + V)
    for trial in range(20):
        p = _rand_dist(rng, V, zeros=trial % 2)
        q = _rand_dist(rng, V, zeros=(trial // 2) % 2)
        acc = np.zeros(V)
        for s in range(V):
            if q[s] > 0:
                acc[s] = q[s] * min(1.0, ar.acceptance_ratio(p[s], q[s]))
        w = ar.residual_weights(p, q)
        law = acc + (1.0 - acc.sum()) * w / w.sum()
        np.testing.assert_allclose(law, p, atol=1e-12)
        assert acc.sum() == pytest.approx(np.minimum(p, q).sum(), abs=1e-12)   # alpha = sum min(p, q)


def test_output_law_through_entry_point_on_exact_grid():
    """Dyadic p, q put every decision threshold on a grid edge, so a midpoint grid of
    (u_accept, u_resample) integrates the emitted-token law exactly: it must equal p."""
    p = np.array([4, 2, 1, 1]) / 8.0
    q = np.array([1, 1, 2, 4]) / 8.0
    K = 8
    mid = (np.arange(K) + 0.5) / K
    tl = np.stack([_logits_of(p), _logits_of(p)])
    law = np.zeros(4)
    for s in range(4):
        for ua in mid:
            for ur in mid:
                m, sp, _, _ = ar.verify_server(tl, q[None], [s], [ua], ur)
                first = s if m == 1 else sp
                law[first] += q[s] / (K * K)
    np.testing.assert_allclose(law, p, atol=1e-12)


def test_disjoint_supports_always_reject_and_resample_from_p():
    p = np.array([0.5, 0.5, 0.0, 0.0])
    q = np.array([0.0, 0.0, 0.25, 0.75])
    with np.errstate(divide="ignore"):
        tl = np.stack([_logits_of(p), _logits_of(p)])
    K = 16
    mid = (np.arange(K) + 0.5) / K
    counts = np.zeros(4)
    for s in (2, 3):
        for ur in mid:
            m, sp, stat, _ = ar.verify_server(tl, q[None], [s], [2.0 ** -24], ur)
            assert m == 0 and stat == 0.0
            counts[sp] += 1
    np.testing.assert_allclose(counts / counts.sum(), p)


def _markov_setup(seed, V):
    rng = np.random.default_rng(seed)
    P = np.stack([_rand_dist(rng, V) for _ in range(V + 1)])   # row V: distribution after the prefix
    Q = np.stack([_rand_dist(rng, V) for _ in range(V + 1)])
    return P, Q


def test_two_token_joint_law_chi_square():
    """Chained rounds with a Markov target: the joint law of the first two emitted tokens is
    p(s1) p(s2 | s1).  Seeded, so the verdict is deterministic."""
    V, S, n_draws = 4, 2, 60000
    P, Q = _markov_setup(11, V)
    rng = np.random.default_rng(12)
    counts = np.zeros((V, V))
    for _ in range(n_draws):
        out, last = [], V
        while len(out) < 2:
            toks, qrows, prev = [], [], last
            for j in range(S):
                s = int(rng.choice(V, p=Q[prev]))
                toks.append(s); qrows.append(Q[prev]); prev = s
            ctx = [last] + toks
            tl = np.stack([_logits_of(P[c]) for c in ctx])
            m, sp, _, _ = ar.verify_server(tl, np.stack(qrows), toks, rng.random(S), rng.random())
            out += toks[:m] + [sp]
            last = out[-1]
        counts[out[0], out[1]] += 1
    expect = n_draws * P[V][:, None] * P[:V]
    chi2 = ((counts - expect) ** 2 / expect).sum()
    # 15 degrees of freedom: the 99.9 % point is 37.7
    assert chi2 < 37.7, chi2


# ---------------------------------------------------------------- alpha and the goodput closed form

def test_expected_tokens_closed_form_equals_capped_geometric_pmf():
    for alpha in (0.05, 0.5, 0.8, 0.97):
        for S in range(0, 12):
            pmf = [alpha ** k * (1 - alpha) for k in range(S)] + [alpha ** S]
            assert sum(pmf) == pytest.approx(1.0, abs=1e-12)
            mean = sum((k + 1) * pk for k, pk in enumerate(pmf))
            assert sch.expected_tokens(alpha, S) == pytest.approx(mean, abs=1e-12)


def test_monte_carlo_accepted_count_and_statistic_match_alpha():
    rng = np.random.default_rng(21)
    V, S, n = 6, 4, 20000
    p, q = _rand_dist(rng, V), _rand_dist(rng, V)
    alpha = np.minimum(p, q).sum()
    tl = np.tile(_logits_of(p), (S + 1, 1))
    qs = np.tile(q, (S, 1))
    emitted, stats = np.empty(n), np.empty(n)
    for t in range(n):
        toks = rng.choice(V, size=S, p=q)
        m, _, stat, _ = ar.verify_server(tl, qs, toks, rng.random(S), rng.random())
        emitted[t], stats[t] = m + 1, stat
    for sample, want in ((emitted, sch.expected_tokens(alpha, S)), (stats, alpha)):
        sigma = sample.std(ddof=1) / np.sqrt(n)
        assert abs(sample.mean() - want) < 4 * sigma


def test_batch_entry_point_is_the_per_server_routine_on_slices():
    rng = np.random.default_rng(31)
    V, gamma = 11, np.array([2, 0, 3, 1])
    R, G = int((gamma + 1).sum()), int(gamma.sum())
    tl = rng.normal(size=(R, V)).astype(np.float32)
    q = np.stack([_rand_dist(rng, V) for _ in range(G)]).astype(np.float32)
    toks = rng.integers(0, V, G)
    ua, ur = rng.random(G).astype(np.float32), rng.random(4).astype(np.float32)
    out = ar.accept_reject(gamma, tl, q, toks, ua, ur)
    r0 = d0 = 0
    for i, S in enumerate(gamma):
        m, sp, st, ra = ar.verify_server(tl[r0:r0 + S + 1], q[d0:d0 + S], toks[d0:d0 + S], ua[d0:d0 + S], ur[i])
        assert (out["accepted_len"][i], out["next_token"][i]) == (m, sp)
        r0 += S + 1; d0 += S


def test_resample_band_contains_the_oracle_token():
    rng = np.random.default_rng(41)
    V = 50
    for _ in range(50):
        tl = rng.normal(size=V) * 3
        q = _rand_dist(rng, V)
        u = rng.random()
        tok = ar.inverse_cdf(ar.residual_weights(ar.softmax(tl), q), u)
        lo, hi = ar.resample_band(tl, q, u)
        assert lo <= tok <= hi and hi - lo <= 1


def test_resample_band_is_no_wider_than_the_rounding_it_excuses():
    """Hand-built CDF with edges at 1/4 and 1/2 (p = [1/4, 1/4, 1/2], bonus draw): away from an edge the band is
    the oracle's token alone; within 1e-5 of an edge it is exactly the two tokens that meet there; just
    outside 1e-5 it is one token again.  A band that is too generous anywhere fails here."""
    tl = np.log(np.array([0.25, 0.25, 0.5]))
    band = lambda u: ar.resample_band(tl, None, u, 1e-5)
    for u, tok in ((0.0, 0), (0.1, 0), (0.2499, 0), (0.2501, 1), (0.3, 1), (0.4999, 1), (0.5001, 2), (0.99, 2)):
        assert band(u) == (tok, tok), u
        assert ar.inverse_cdf(ar.softmax(tl), u) == tok
    for u in (0.25, 0.25 - 0.9e-5, 0.25 + 0.9e-5):
        assert band(u) == (0, 1), u
    for u in (0.5, 0.5 - 0.9e-5, 0.5 + 0.9e-5):
        assert band(u) == (1, 2), u
    assert band(0.25 - 1.1e-5) == (0, 0) and band(0.25 + 1.1e-5) == (1, 1)
    assert band(0.5 - 1.1e-5) == (1, 1) and band(0.5 + 1.1e-5) == (2, 2)
    # the band scales with the total mass: residual max(0, p - q) with q = [1/4, 0, 1/4] is [0, 1/4, 1/4], total 1/2
    q = np.array([0.25, 0.0, 0.25])
    band_r = lambda u: ar.resample_band(tl, q, u, 1e-5)
    assert band_r(0.3) == (1, 1) and band_r(0.7) == (2, 2)
    assert band_r(0.5 + 0.9e-5) == (1, 2) and band_r(0.5 + 1.1e-5) == (2, 2) and band_r(0.5 - 1.1e-5) == (1, 1)
    # a token without weight between two edges widens the index range but is never a valid answer:
    # the comparison helper rejects it through its w > 0 test
    tl0 = np.log(np.array([0.5, 1e-300, 0.5]))
    tl0[1] = -np.inf
    assert ar.resample_band(tl0, None, 0.5, 1e-5) == (0, 2) and ar.softmax(tl0)[1] == 0.0


def test_output_law_when_the_verifier_sees_q_rounded_to_bfloat16():
    """Reading behind gs_accept_reject_bf16: the draft token is sampled from q, the verifier applies the rule
    with q~ = bfloat16(q).  The rule stays well defined (q~ need not sum to one) and the law of the emitted
    token, enumerated exactly with the oracle's own ratio and residual routines, stays within 2^-8 of p in
    total variation (q~/q is within 1 +- 2^-9); with the unrounded q it is p itself."""
    from oracle.forward import round_bf16
    rng = np.random.default_rng(61)
    worst = 0.0
    for _ in range(300):
        V = int(rng.integers(3, 9))
        p, q = _rand_dist(rng, V), _rand_dist(rng, V)
        for q_seen, exact in ((q, True), (round_bf16(q), False)):
            accept = np.array([min(1.0, ar.acceptance_ratio(p[s], q_seen[s])) for s in range(V)])
            w = ar.residual_weights(p, q_seen)
            law = q * accept + (1.0 - (q * accept).sum()) * w / w.sum()
            tv = 0.5 * np.abs(law - p).sum()
            if exact:
                assert tv < 1e-12
            else:
                worst = max(worst, tv)
                assert tv < 2.0 ** -8
    assert worst > 1e-5          # the rounding does change the law: the bound is not vacuous
