"""Closed loop of the verification server against simulated draft servers (Algorithm 1, Section IV).

Every round the draft servers hand over their blocks, gs_accept_reject verifies them on the GPU and the
allocation policy fixes the draft lengths of the next round.  The target forward is not part of this loop:
target logits and draft distributions come from the seeded generators (server i drafts from the target
logits perturbed with its own noise level, so acceptance rates differ across servers), which is what
the loop needs to compare allocation policies:

  goodspeed  gs_schedule_gamma: smoothed acceptance rates and goodputs, then the gradient allocation
             (Section III-C)
  fixed      the capacity split evenly and never changed (Fixed-S of Section IV-A)
  random     the capacity dealt to servers uniformly at random every round (Random-S of Section IV-A)

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
    verify_ms: float = 0.0       # GPU time of the gs_accept_reject calls (HIP events), all rounds
    schedule_ms: float = 0.0     # host time of the allocation policy, all rounds

    def goodput(self):
        """Realised goodput x_i(t) = m_i(t) + 1, as an array [rounds, N]."""
        return np.asarray(self.accepted_len, dtype=np.float64) + 1.0

    def mean_goodput(self):
        return self.goodput().mean(axis=0)

    def utility(self):
        """Sum of log average goodputs (the objective of Section III-A evaluated on the run)."""
        return float(np.log(self.mean_goodput()).sum())


def even_split(capacity, n):
    base, extra = divmod(int(capacity), n)
    return np.array([base + (1 if i < extra else 0) for i in range(n)], dtype=np.int32)


def random_split(capacity, n, uniforms):
    g = np.zeros(n, dtype=np.int32)
    for u in uniforms[:capacity]:
        g[min(n - 1, int(float(u) * n))] += 1
    return g


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
        elif policy == "random":
            gamma = random_split(capacity, n, synth.loop_policy_uniforms(seed, t, capacity))
        # fixed: unchanged
        res.schedule_ms += (time.perf_counter() - t0) * 1e3
    return res
