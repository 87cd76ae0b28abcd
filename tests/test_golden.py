"""The oracle against the hand-worked fixtures under tests/golden/ (each file cites the passage it is worked from)."""
import json
import os

import numpy as np
import pytest

from oracle import accept_reject as ar
from oracle import schedule as sch

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _lines(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [l.strip() for l in f if l.strip() and not l.startswith("#")]


def test_expected_tokens_fixture():
    rows = _lines("expected_tokens.txt")
    assert len(rows) == 6
    for row in rows:
        alpha, S, value = row.split()
        assert sch.expected_tokens(float(alpha), int(S)) == pytest.approx(float(value), rel=1e-12)


def test_scheduler_fixture():
    cases = [json.loads(l) for l in _lines("scheduler_worked_examples.txt")]
    assert len(cases) == 4
    for c in cases:
        a, X = np.array(c["alpha"]), np.array(c["X"])
        np.testing.assert_array_equal(sch.schedule_greedy(a, X, c["C"]), c["S"])
        best_value, _ = sch.schedule_exhaustive(a, X, c["C"])        # ties: compare the objective
        assert best_value == pytest.approx(sch.objective(a, X, c["S"]), rel=1e-14)


def test_estimator_fixture():
    cases = [json.loads(l) for l in _lines("estimator_updates.txt")]
    assert len(cases) == 6
    for c in cases:
        if c["kind"] == "alpha":
            got = sch.update_alpha_hat([c["prev"]], [c["stat"]], [1], c["eta"])[0]
        else:
            got = sch.update_goodput([c["prev"]], [c["accepted"]], c["beta"])[0]
        assert got == pytest.approx(c["next"], rel=1e-12)


def test_accept_rule_fixture():
    cases = [json.loads(l) for l in _lines("accept_rule.txt")]
    assert len(cases) == 4
    for c in cases:
        p, q = np.array(c["p"]), np.array(c["q"])
        logits = np.log(p)[None, :].repeat(2, axis=0)       # rows for the draft position and the bonus position
        for u_res in (0.0, 0.37, 0.99):
            m, tok, _, _ = _verify(logits, q[None, :], c["token"], c["u"], u_res)
            assert (m == 1) == c["accepted"]
            if not c["accepted"]:
                np.testing.assert_allclose(ar.residual_weights(ar.softmax(logits[0]), q), c["residual"], atol=1e-12)
                assert tok == c["replacement"]


def _verify(logits, q, token, u, u_res):
    return ar.verify_server(logits, q, np.array([token]), np.array([u]), u_res)
