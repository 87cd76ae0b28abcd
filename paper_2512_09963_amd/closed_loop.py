"""Closed loop of the verification server against simulated draft servers (Algorithm 1, Section IV).

Every round the draft servers hand over their blocks, gs_accept_reject verifies them on the GPU and the
allocation policy fixes the draft lengths of the next round.  The target forward is not part of this loop:
target logits and draft distributions come from the seeded generators (server i drafts from the target
logits perturbed with its own noise level, so acceptance rates differ across servers), which is what
the loop needs to compare allocation policies:

  goodspeed  gs_schedule_gamma: smoothed acceptance rates and goodputs, then the gradient allocation
             (Section III-C)
  fixed      gs_allocate_fixed: the capacity split evenly and never changed (Fixed-S of Section IV-A)
  random     gs_allocate_random: the capacity dealt to servers uniformly at random every round (Random-S)

Runs on the HIP library only; there is no CPU path here.
"""
import time
from dataclasses import dataclass, field

import numpy as np
import torch

from . import binding as gsb
from . import synth

POLICIES = ("goodspeed", "fixed", "random")


@dataclass
class LoopResult:
    gamma: list = field(default_factory=list)          # per round: draft lengths used [N]
    accepted_len: list = field(default_factory=list)   # per round: m_i [N]
    next_token: list = field(default_factory=list)
    accept_stat: list = field(default_factory=list)
    x_smooth: list = field(default_factory=list)       # per round: smoothed goodput X_i after the update (goodspeed)
    alpha_hat: list = field(default_factory=list)      # per round: estimated acceptance rates (goodspeed)
    verify_ms: float = 0.0       # GPU time of the gs_accept_reject calls (HIP events), all rounds
    schedule_ms: float = 0.0     # host time of the allocation policy, all rounds

    def goodput(self):
        """Realised goodput x_i(t) = m_i(t) + 1, as an array [rounds, N]."""
        return np.asarray(self.accepted_len, dtype=np.float64) + 1.0

    def mean_goodput(self):
        return self.goodput().mean(axis=0)

    def utility(self, n_rounds=None):
        """Sum of log average goodputs (the objective of Section III-A evaluated on the first n_rounds of the run)."""
        g = self.goodput() if n_rounds is None else self.goodput()[:n_rounds]
        return float(np.log(g.mean(axis=0)).sum())


def even_split(capacity, n):
    """Fixed-S (library call)."""
    return gsb.gs_allocate_fixed(n, capacity)


def random_split(capacity, n, uniforms):
    """Random-S (library call)."""
    return gsb.gs_allocate_random(n, capacity, uniforms)


def run(policy, sigmas, capacity, vocab, n_rounds, seed=synth.MASTER_SEED, eta=0.2, beta=0.5, alpha0=0.5, x0=1.0,
        device="cuda:0", on_round=None):
    """n_rounds of the loop on the GPU.  sigmas[i] is draft server i's noise level.  Returns a LoopResult."""
    if policy not in POLICIES:
        raise ValueError(f"policy must be one of {POLICIES}")
    gsb.lib()
    dev = torch.device(device)
    n = len(sigmas)
    gamma = even_split(capacity, n)
    alpha = np.full(n, float(alpha0))
    X = np.full(n, float(x0))
    res = LoopResult()
    max_rows = capacity + n
    ws = torch.empty(gsb.gs_accept_workspace_bytes(n, max_rows, vocab), dtype=torch.uint8, device=dev)
    for t in range(n_rounds):
        inp = synth.loop_round_inputs(seed, t, gamma, vocab, sigmas)
        G = int(gamma.sum())
        out = gsb.make_accept_out(n, G, dev, want_ratio=False)
        cu = torch.from_numpy(synth.cu_rows_of(gamma)).to(dev)
        dev_in = [torch.from_numpy(inp.target_logits).to(dev),
                  torch.from_numpy(inp.q_probs).to(dev) if G else None,
                  torch.from_numpy(inp.draft_tokens).to(dev) if G else None,
                  torch.from_numpy(inp.u_accept).to(dev) if G else None,
                  torch.from_numpy(inp.u_resample).to(dev)]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        gsb.gs_accept_reject(gamma, cu, vocab, *dev_in, out, ws)
        e1.record()
        torch.cuda.current_stream().synchronize()
        res.verify_ms += e0.elapsed_time(e1)
        m = out["accepted_len"].cpu().numpy()
        st = out["accept_stat"].cpu().numpy()
        tok = out["next_token"].cpu().numpy()
        res.gamma.append(gamma.copy())
        res.accepted_len.append(m)
        res.next_token.append(tok)
        res.accept_stat.append(st)
        if on_round is not None:
            on_round(t, inp, gamma, m, tok, st)
        t0 = time.perf_counter()
        if policy == "goodspeed":
            gamma = gsb.gs_schedule_gamma(m, st, gamma, alpha, X, eta, beta, capacity, 0, -1)
            res.x_smooth.append(X.copy())
            res.alpha_hat.append(alpha.copy())
        elif policy == "random":
            gamma = random_split(capacity, n, synth.loop_policy_uniforms(seed, t, capacity))
        # fixed: unchanged
        res.schedule_ms += (time.perf_counter() - t0) * 1e3
    return res


def main(argv=None):
    """Runs the three policies on the same simulated servers and prints one JSON line per policy: log utility
    of the average goodput after 50, 100, 200, ... rounds (the quantity of Fig. 4), average goodput and draft
    length per server, and for GoodSpeed the smoothed goodput next to the realised one (Fig. 2)."""
    import argparse
    import json
    ap = argparse.ArgumentParser(description=main.__doc__)
    ap.add_argument("--rounds", type=int, default=600)
    ap.add_argument("--capacity", type=int, default=44)
    ap.add_argument("--vocab", type=int, default=32000)
    ap.add_argument("--sigmas", type=float, nargs="+", default=[0.2, 0.4, 0.6, 0.8, 1.0, 1.4, 1.9, 2.5])
    ap.add_argument("--eta", type=float, default=0.2)
    ap.add_argument("--beta", type=float, default=0.5)
    ap.add_argument("--seed", type=int, default=synth.MASTER_SEED)
    a = ap.parse_args(argv)
    sig = np.asarray(a.sigmas, dtype=np.float64)
    marks = [t for t in (50, 100, 200, 300, 400, 600, 1000) if t <= a.rounds]
    if not marks or marks[-1] != a.rounds:
        marks.append(a.rounds)
    for policy in POLICIES:
        t0 = time.perf_counter()
        r = run(policy, sig, a.capacity, a.vocab, a.rounds, seed=a.seed, eta=a.eta, beta=a.beta)
        line = {"policy": policy, "servers": len(sig), "capacity": a.capacity, "vocab": a.vocab, "rounds": a.rounds,
                "log_utility_after": {str(t): round(r.utility(t), 4) for t in marks},
                "mean_goodput": [round(float(v), 3) for v in r.mean_goodput()],
                "mean_draft_length": [round(float(v), 2) for v in np.asarray(r.gamma, dtype=np.float64).mean(axis=0)],
                "verify_ms_per_round": round(r.verify_ms / a.rounds, 4),
                "schedule_ms_per_round": round(r.schedule_ms / a.rounds, 4),
                "wall_s": round(time.perf_counter() - t0, 1)}
        if policy == "goodspeed":
            tail = max(1, a.rounds // 6)
            line["smoothed_goodput_last"] = [round(float(v), 3) for v in np.asarray(r.x_smooth[-tail:]).mean(axis=0)]
            line["realised_goodput_last"] = [round(float(v), 3) for v in r.goodput()[-tail:].mean(axis=0)]
            line["alpha_hat_last"] = [round(float(v), 3) for v in np.asarray(r.alpha_hat[-tail:]).mean(axis=0)]
        print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
