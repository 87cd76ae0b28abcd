"""Oracle of the closed loop (test infrastructure, never imported by the product path).

Algorithm 1 with simulated draft servers: verification by oracle.accept_reject (Section II-A-2),
estimator updates and the gradient allocation by oracle.schedule (Section III-C), against the two
baselines of Section IV-A (an even fixed split, a uniformly random split per round).  Inputs of a round
are handed in by the caller (a function round -> inputs for given draft lengths), so this module holds no
generator and shares nothing with the GPU path.
"""
import numpy as np

from . import accept_reject as ar
from . import schedule as sch


def fixed_allocation(capacity, n):
    """C / N drafts each; the remainder goes to the lowest indices."""
    g = np.full(n, capacity // n, dtype=np.int64)
    g[: capacity % n] += 1
    return g


def random_allocation(capacity, n, uniforms):
    """Each of the C draft slots goes to server floor(u * N)."""
    idx = np.minimum(n - 1, np.floor(np.asarray(uniforms[:capacity], dtype=np.float64) * n).astype(np.int64))
    return np.bincount(idx, minlength=n).astype(np.int64)


def run(policy, n, capacity, n_rounds, round_inputs, policy_uniforms=None, eta=0.2, beta=0.5, alpha0=0.5,
        x0=1.0):
    """Returns dict of per-round lists gamma, accepted_len, next_token, accept_stat, and the final
    estimator state.  round_inputs(t, gamma) -> object with target_logits, q_probs, draft_tokens, u_accept,
    u_resample; policy_uniforms(t) -> uniforms for the random policy."""
    gamma = fixed_allocation(capacity, n)
    alpha = np.full(n, float(alpha0))
    X = np.full(n, float(x0))
    hist = {"gamma": [], "accepted_len": [], "next_token": [], "accept_stat": []}
    for t in range(n_rounds):
        inp = round_inputs(t, gamma)
        out = ar.accept_reject(gamma, inp.target_logits, inp.q_probs, inp.draft_tokens, inp.u_accept,
                               inp.u_resample)
        hist["gamma"].append(np.asarray(gamma).copy())
        hist["accepted_len"].append(out["accepted_len"].copy())
        hist["next_token"].append(out["next_token"].copy())
        hist["accept_stat"].append(out["accept_stat"].copy())
        if policy == "goodspeed":
            alpha, X, gamma = sch.schedule_round(out["accepted_len"], out["accept_stat"], gamma, alpha, X, eta,
                                                 beta, capacity)
        elif policy == "random":
            gamma = random_allocation(capacity, n, policy_uniforms(t))
        elif policy != "fixed":
            raise ValueError(policy)
    hist["alpha_hat"], hist["X"] = alpha, X
    return hist


def mean_goodput(hist):
    return (np.asarray(hist["accepted_len"], dtype=np.float64) + 1.0).mean(axis=0)


def utility(hist):
    """Sum over servers of the log of the time-averaged goodput (objective of Section III-A)."""
    return float(np.log(mean_goodput(hist)).sum())
