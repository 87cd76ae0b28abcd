"""Oracle: rejection-verification of one round of speculative decoding.

Test infrastructure only (see the package docstring).  Float64 throughout; the
inputs are the float32 arrays the HIP path receives, widened on entry.

Follows the paper's Section II-A-2 (Speculative Decoding): accept draft token
s_j iff r_j <= p_j(s_j)/q_j(s_j); the accepted count m is the index of the first
rejection minus one, or S if none; the extra token s' is drawn from the
normalised max(0, p_{m+1} - q_{m+1}) when m < S and from p_{S+1} otherwise.
The target distribution is the softmax of the logits (Section II-A-1).
The per-server statistic is the empirical mean of min(1, p/q) over all S drafted
positions, the quantity that enters the acceptance-rate update (Section III-C,
the update equation of alpha-hat).

Readings where the paper is silent:
  * q_j(s_j) == 0: the ratio is +inf, the token is accepted, min(1, ratio) = 1.
  * residual mass sum(max(0, p - q)) == 0 (rounding only): draw from p_{m+1}.
  * inverse CDF: token = smallest s with cumsum(w)[s] > u * sum(w), vocabulary in
    index order, so a token of zero weight is never returned; if rounding leaves
    no such s, the last token with w > 0.
  * S == 0: nothing to accept, m = 0, s' ~ p_1, statistic undefined (returned as 0).
"""
import numpy as np


def softmax(logits_row):
    """p = softmax(logits) (Section II-A-1), float64."""
    l = np.asarray(logits_row, dtype=np.float64)
    e = np.exp(l - l.max())
    return e / e.sum()


def acceptance_ratio(p_tok, q_tok):
    """p_j(s_j) / q_j(s_j), +inf when q_j(s_j) == 0."""
    if q_tok == 0.0:
        return np.inf
    return p_tok / q_tok


def residual_weights(p, q):
    """Unnormalised max(0, p - q); falls back to p when it has no mass."""
    w = np.maximum(0.0, p - q)
    if not w.sum() > 0.0:
        return p.copy()
    return w


def inverse_cdf(w, u):
    """Smallest index s with w[0] + ... + w[s] > u * sum(w) (sequential float64 sums)."""
    c = np.cumsum(np.asarray(w, dtype=np.float64))
    hit = np.nonzero(c > float(u) * c[-1])[0]
    if hit.size:
        return int(hit[0])
    return int(np.nonzero(w > 0)[0][-1])


def verify_server(target_logits, q_probs, draft_tokens, u_accept, u_resample):
    """One server's block.

    target_logits [S+1, V]: row j (0-based) holds the logits of p_{j+1}.
    q_probs [S, V], draft_tokens [S], u_accept [S], u_resample scalar.
    Returns (m, s_prime, stat, ratios[S]).
    """
    S = len(draft_tokens)
    ratios = np.empty(S, dtype=np.float64)
    for j in range(S):
        p = softmax(target_logits[j])
        s = int(draft_tokens[j])
        ratios[j] = acceptance_ratio(p[s], float(q_probs[j][s]))
    m = S
    for j in range(S):
        if float(u_accept[j]) > ratios[j]:
            m = j
            break
    p_next = softmax(target_logits[m])
    if m < S:
        w = residual_weights(p_next, np.asarray(q_probs[m], dtype=np.float64))
    else:
        w = p_next
    s_prime = inverse_cdf(w, u_resample)
    stat = float(np.minimum(1.0, ratios).mean()) if S > 0 else 0.0
    return m, s_prime, stat, ratios


def accept_reject(gamma, target_logits, q_probs, draft_tokens, u_accept, u_resample):
    """All servers of a ragged batch.

    gamma[N]; target_logits [sum(gamma+1), V] with each server's rows contiguous;
    q_probs [sum(gamma), V]; draft_tokens, u_accept [sum(gamma)]; u_resample [N].
    Returns dict(accepted_len[N] int32, next_token[N] int32, accept_stat[N] f64, ratio[sum(gamma)] f64).
    """
    gamma = np.asarray(gamma, dtype=np.int64)
    n = gamma.size
    m_out = np.zeros(n, dtype=np.int32)
    tok_out = np.zeros(n, dtype=np.int32)
    stat_out = np.zeros(n, dtype=np.float64)
    ratio_out = np.zeros(int(gamma.sum()), dtype=np.float64)
    r0 = 0
    d0 = 0
    for i in range(n):
        S = int(gamma[i])
        m, sp, st, ra = verify_server(target_logits[r0:r0 + S + 1], q_probs[d0:d0 + S],
                                      draft_tokens[d0:d0 + S], u_accept[d0:d0 + S], u_resample[i])
        m_out[i], tok_out[i], stat_out[i] = m, sp, st
        ratio_out[d0:d0 + S] = ra
        r0 += S + 1
        d0 += S
    return {"accepted_len": m_out, "next_token": tok_out, "accept_stat": stat_out, "ratio": ratio_out}


def resample_band(target_logits_row, q_row, u_resample, rel=1e-5):
    """Tokens a float32 prefix sum may legitimately return instead of the oracle's.

    Returns (lo_token, hi_token): every token g with w(g) > 0 whose float64 CDF
    interval [CDF(g-1), CDF(g)] comes within rel * sum(w) of u * sum(w) lies in
    [lo_token, hi_token].  q_row is None for the bonus draw from p.
    """
    p = softmax(target_logits_row)
    w = p if q_row is None else residual_weights(p, np.asarray(q_row, dtype=np.float64))
    c = np.cumsum(w)
    t = float(u_resample) * c[-1]
    eps = rel * c[-1]
    lo = int(np.searchsorted(c, t - eps, side="left"))
    hi = int(np.searchsorted(c, t + eps, side="right"))
    V = w.size
    return min(lo, V - 1), min(hi, V - 1)
