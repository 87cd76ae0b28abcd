"""Closed loop on the GPU against the oracle loop, round by round (Algorithm 1; baselines of Section IV-A).

Both sides get the same seeded inputs.  Every round the GPU's verification outputs are held to the
accept/reject parity bar against the oracle run on that round's inputs, and the allocation that the
library's scheduler derives from them must equal the oracle scheduler's on the same outputs (teacher-forced:
the oracle's estimator state follows the GPU's outputs, which differ from its own only inside the bands).
"""
import numpy as np
import pytest

from oracle import closed_loop as ol
from oracle import schedule as sch
from paper_2512_09963_amd import closed_loop as cl
from paper_2512_09963_amd import synth
from tests.parity import check_accept_outputs

pytestmark = pytest.mark.gpu
SEED = 20251209


@pytest.mark.parametrize("policy", ["goodspeed", "fixed", "random"])
def test_loop_matches_oracle_round_by_round(policy):
    sig = np.array([0.2, 0.5, 0.9, 1.4, 2.0, 0.0])      # the last server drafts from the target itself
    n, C, V, T = sig.size, 22, 1000, 40
    state = {"alpha": np.full(n, 0.5), "X": np.ones(n), "bands": 0, "gamma_next": ol.fixed_allocation(C, n)}

    def on_round(t, inp, gamma, m, tok, st):
        assert np.array_equal(gamma, state["gamma_next"]), f"round {t}: allocation differs from the oracle's"
        assert int(gamma.sum()) == C
        b = check_accept_outputs(gamma, inp.target_logits, inp.q_probs, inp.draft_tokens, inp.u_accept,
                                 inp.u_resample, {"accepted_len": m, "next_token": tok, "accept_stat": st})
        state["bands"] += b["n_band_m"] + b["n_band_tok"]
        if policy == "goodspeed":
            state["alpha"], state["X"], g = sch.schedule_round(m, st.astype(np.float64), gamma, state["alpha"],
                                                               state["X"], 0.2, 0.5, C)
            state["gamma_next"] = np.asarray(g)
        elif policy == "random":
            state["gamma_next"] = ol.random_allocation(C, n, synth.loop_policy_uniforms(SEED, t, C))

    res = cl.run(policy, sig, C, V, T, seed=SEED, on_round=on_round)
    assert len(res.accepted_len) == T
    # whole-run figures against the free-running oracle loop (identical unless a band was hit)
    h = ol.run(policy, n, C, T, lambda t, g: synth.loop_round_inputs(SEED, t, g, V, sig),
               lambda t: synth.loop_policy_uniforms(SEED, t, C))
    if state["bands"] == 0:
        assert np.array_equal(np.asarray(res.accepted_len), np.asarray(h["accepted_len"]))
        assert np.array_equal(np.asarray(res.next_token), np.asarray(h["next_token"]))
        assert abs(res.utility() - ol.utility(h)) < 1e-12
    print(policy, "utility", res.utility(), "bands", state["bands"])
