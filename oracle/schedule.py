"""Oracle: estimator updates and the per-round gradient scheduling problem.

Test infrastructure only.  Follows Section III-C of the paper:
  * acceptance-rate smoothing  a_i(t) = (1-eta) a_i(t-1) + eta * stat_i(t),
    stat_i = mean over the S_i drafted positions of min(1, p/q);
  * goodput smoothing          X_i(t) = (1-beta) X_i(t-1) + beta * x_i(t),
    x_i(t) = accepted tokens + 1 (the correction / bonus token);
  * the scheduling problem     max_S sum_i U_i'(X_i(t)) * xhat_i(S_i)
    subject to sum_i S_i <= C, S_i a non-negative integer, with
    xhat_i(S) = (1 - a_i^(S+1)) / (1 - a_i) and U_i = log, so U_i'(X) = 1/X.
Both estimators are updated before the problem is solved (Algorithm 1 orders the
update step before the solve step, and the problem is stated in terms of X(t)
and alpha-hat(t)).

Two solvers: exhaustive enumeration of the feasible set (the definition; tiny
N and C only) and the slot-by-slot marginal allocation that the separable
concave objective admits (each extra slot of server i adds U_i' * a_i^(S_i+1)).

Readings where the paper is silent: alpha-hat is clamped to [1e-6, 1 - 1e-6]
inside the solvers (the analysis assumes alpha-hat <= alpha_max < 1); box
bounds gamma_min <= S_i <= gamma_max are optional extras; ties go to the lowest
server index; a server with S_i(t) = 0 keeps its alpha-hat.
"""
import itertools

import numpy as np

ALPHA_LO = 1e-6
ALPHA_HI = 1.0 - 1e-6


def expected_tokens(alpha, S):
    """xhat = (1 - alpha^(S+1)) / (1 - alpha): mean of a geometric count capped at S+1."""
    return (1.0 - alpha ** (S + 1)) / (1.0 - alpha)


def update_alpha_hat(alpha_prev, stat, gamma_prev, eta):
    """Acceptance-rate smoothing; servers that drafted nothing keep their estimate."""
    a = np.array(alpha_prev, dtype=np.float64)
    for i in range(a.size):
        if gamma_prev[i] > 0:
            a[i] = (1.0 - eta) * a[i] + eta * float(stat[i])
    return a


def update_goodput(x_prev, accepted_len, beta):
    """Goodput smoothing with realised goodput x_i = accepted + 1."""
    X = np.array(x_prev, dtype=np.float64)
    for i in range(X.size):
        X[i] = (1.0 - beta) * X[i] + beta * (float(accepted_len[i]) + 1.0)
    return X


def objective(alpha_hat, X, S):
    """sum_i (1/X_i) * xhat_i(S_i)."""
    total = 0.0
    for a, x, s in zip(alpha_hat, X, S):
        a = min(max(float(a), ALPHA_LO), ALPHA_HI)
        total += (1.0 / float(x)) * expected_tokens(a, int(s))
    return total


def schedule_exhaustive(alpha_hat, X, C, gamma_min=0, gamma_max=None):
    """Best objective over every feasible S; returns (best_value, one maximiser)."""
    n = len(alpha_hat)
    hi = C if gamma_max is None else min(C, gamma_max)
    best_v, best_s = -np.inf, None
    for S in itertools.product(range(gamma_min, hi + 1), repeat=n):
        if sum(S) > C:
            continue
        v = objective(alpha_hat, X, S)
        if v > best_v:
            best_v, best_s = v, S
    return best_v, (None if best_s is None else np.array(best_s, dtype=np.int32))


def schedule_greedy(alpha_hat, X, C, gamma_min=0, gamma_max=None):
    """Slot-by-slot marginal allocation, O(C*N): every slot goes to argmax_i (1/X_i) a_i^(S_i+1)."""
    n = len(alpha_hat)
    a = [min(max(float(v), ALPHA_LO), ALPHA_HI) for v in alpha_hat]
    r = [1.0 / float(x) for x in X]
    S = [int(gamma_min)] * n
    gain = [r[i] * a[i] ** (S[i] + 1) for i in range(n)]
    left = int(C) - sum(S)
    while left > 0:
        best = -1
        for i in range(n):
            if gamma_max is not None and S[i] >= gamma_max:
                continue
            if best < 0 or gain[i] > gain[best]:
                best = i
        if best < 0:
            break
        S[best] += 1
        gain[best] = r[best] * a[best] ** (S[best] + 1)
        left -= 1
    return np.array(S, dtype=np.int32)


def schedule_round(accepted_len, accept_stat, gamma_prev, alpha_hat, X, eta, beta, C,
                   gamma_min=0, gamma_max=None):
    """Estimator updates followed by the solve: returns (alpha_hat', X', gamma_next)."""
    a = update_alpha_hat(alpha_hat, accept_stat, gamma_prev, eta)
    Xn = update_goodput(X, accepted_len, beta)
    return a, Xn, schedule_greedy(a, Xn, C, gamma_min, gamma_max)
