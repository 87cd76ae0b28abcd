"""Comparison of the HIP path's verification outputs with the oracle's (test helper).

Bar: accepted lengths and tokens are bit-exact, except that
  * a server whose accept decision at some draft j has |u_j - ratio_j| < 1e-5 may
    differ in m (and then in everything that depends on m);
  * the drawn token g may differ from the oracle's when u * total falls within
    1e-5 * total of an edge of g's float64 CDF interval and g has positive weight.
Ratios and the statistic are fp32 quantities: relative 1e-4 (fp32 tolerance).
"""
import numpy as np

from oracle import accept_reject as ar

BAND = 1e-5


def check_accept_outputs(gamma, target_logits, q_probs, draft_tokens, u_accept, u_resample, got, oracle_out=None,
                         ratio_rtol=1e-4):
    """got: dict of numpy arrays accepted_len, next_token, accept_stat, ratio (ratio optional).
    Returns dict(n_band_m, n_band_tok) - how many servers needed a band."""
    gamma = np.asarray(gamma)
    want = oracle_out or ar.accept_reject(gamma, target_logits, q_probs, draft_tokens, u_accept, u_resample)
    n = gamma.size
    cu_r = np.concatenate([[0], np.cumsum(gamma + 1)])
    cu_d = np.concatenate([[0], np.cumsum(gamma)])
    n_band_m = n_band_tok = 0
    if got.get("ratio") is not None and cu_d[-1] > 0:
        r_w, r_g = want["ratio"], np.asarray(got["ratio"], dtype=np.float64)
        fin = np.isfinite(r_w)
        assert np.array_equal(np.isinf(r_w), np.isinf(r_g)), "ratio: +inf (q = 0) positions differ"
        np.testing.assert_allclose(r_g[fin], r_w[fin], rtol=ratio_rtol, atol=1e-30, err_msg="ratio")
    for i in range(n):
        S = int(gamma[i])
        d0, r0 = int(cu_d[i]), int(cu_r[i])
        m_w, m_g = int(want["accepted_len"][i]), int(got["accepted_len"][i])
        assert 0 <= m_g <= S, f"server {i}: accepted_len {m_g} outside [0, {S}]"
        if m_g != m_w:
            j = min(m_g, m_w)          # first decision on which the two sides differ
            gap = abs(float(u_accept[d0 + j]) - want["ratio"][d0 + j])
            assert gap < BAND, f"server {i}: accepted_len {m_g} != oracle {m_w}, |u - ratio| = {gap:g} at draft {j}"
            n_band_m += 1
            continue
        if S > 0:
            np.testing.assert_allclose(got["accept_stat"][i], want["accept_stat"][i], rtol=ratio_rtol, atol=1e-6,
                                       err_msg=f"accept_stat[{i}]")
        else:
            assert got["accept_stat"][i] == 0.0
        t_w, t_g = int(want["next_token"][i]), int(got["next_token"][i])
        if t_g != t_w:
            q_row = q_probs[d0 + m_w] if m_w < S else None
            lo, hi = ar.resample_band(target_logits[r0 + m_w], q_row, u_resample[i], BAND)
            p = ar.softmax(target_logits[r0 + m_w])
            w = p if q_row is None else ar.residual_weights(p, np.asarray(q_row, dtype=np.float64))
            assert lo <= t_g <= hi and w[t_g] > 0, \
                f"server {i}: next_token {t_g} != oracle {t_w} and outside the rounding band [{lo}, {hi}]"
            n_band_tok += 1
    return {"n_band_m": n_band_m, "n_band_tok": n_band_tok}
