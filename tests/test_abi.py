"""The C-ABI library loads and exports every symbol the header declares; host-only entry points
(the scheduler, argument validation) are exercised against the oracle.  No GPU needed."""
import os
import re

import numpy as np
import pytest

from oracle import schedule as sch
from paper_2512_09963_amd import binding as gsb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "goodspeed.h")).read()
    declared = set(re.findall(r"\b(gs_[a-z0-9_]+)\s*\(", header))
    assert declared == set(gsb.EXPORTS)
    L = gsb.lib()
    for name in declared:
        assert hasattr(L, name), name


@pytest.mark.parametrize("seed", range(20))
def test_schedule_gamma_equals_oracle(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 40))
    gmin = int(rng.integers(0, 2))
    gmax = int(rng.choice([-1, 6, 16]))
    C = int(rng.integers(n * gmin, 12 * n + 1))
    g_prev = rng.integers(0, 9, n)
    m = np.array([rng.integers(0, g + 1) for g in g_prev])
    stat = rng.random(n).astype(np.float32)
    a0 = rng.uniform(0.05, 0.99, n)
    X0 = rng.uniform(0.3, 8.0, n)
    eta, beta = float(rng.uniform(0.05, 0.9)), float(rng.uniform(0.05, 0.9))
    a_w, X_w, g_w = sch.schedule_round(m, stat, g_prev, a0, X0, eta, beta, C, gmin, None if gmax < 0 else gmax)
    a, X = a0.copy(), X0.copy()
    g = gsb.gs_schedule_gamma(m, stat, g_prev, a, X, eta, beta, C, gmin, gmax)
    np.testing.assert_allclose(a, a_w, rtol=1e-15)
    np.testing.assert_allclose(X, X_w, rtol=1e-15)
    if not np.array_equal(g, g_w):       # several maximisers exist only on exact ties: compare what is unique
        hi = None if gmax < 0 else gmax
        assert sch.objective(a_w, X_w, g) == pytest.approx(sch.objective(a_w, X_w, g_w), rel=1e-13)
        assert g.sum() == g_w.sum() and g.min() >= gmin and (hi is None or g.max() <= hi)
    else:
        assert g.sum() == (C if gmax < 0 else min(C, n * gmax))


def test_schedule_gamma_hand_cases_and_ties():
    a, X = np.array([0.5, 0.8]), np.array([1.0, 1.0])
    # eta = beta = 0 leaves the state as given: gains 0.8, 0.64, 0.512 beat 0.5
    g = gsb.gs_schedule_gamma([0, 0], [0, 0], [1, 1], a, X, 0.0, 0.0, 3)
    np.testing.assert_array_equal(g, [0, 3])
    a, X = np.array([0.7] * 3), np.array([2.0] * 3)
    np.testing.assert_array_equal(gsb.gs_schedule_gamma([0] * 3, [0] * 3, [1] * 3, a, X, 0.0, 0.0, 4), [2, 1, 1])
    a, X = np.array([0.5, 0.5]), np.array([1.0, 1.0])
    g = gsb.gs_schedule_gamma([3, 0], [1.0, 0.0], [3, 3], a, X, 0.2, 0.5, 4)
    np.testing.assert_allclose(a, [0.6, 0.4]); np.testing.assert_allclose(X, [2.5, 1.0])
    np.testing.assert_array_equal(g, [2, 2])


def test_schedule_gamma_rejects_bad_arguments():
    a, X = np.array([0.5]), np.array([1.0])
    with pytest.raises(gsb.GsError) as e:
        gsb.gs_schedule_gamma([2], [0.5], [1], a, X, 0.2, 0.5, 4)
    assert e.value.code == -1 and "accepted_len" in str(e.value)
    with pytest.raises(gsb.GsError):
        gsb.gs_schedule_gamma([0], [0.5], [1], a, X, 1.5, 0.5, 4)
    with pytest.raises(gsb.GsError):
        gsb.gs_schedule_gamma([0], [0.5], [1], a, X, 0.2, 0.5, 0, gamma_min=1)
    np.testing.assert_array_equal(a, [0.5])          # a failed call changed nothing


def test_accept_reject_validates_on_the_host_before_any_launch():
    L = gsb.lib()
    assert L.gs_accept_workspace_bytes(64, 576, 151936) > 0
    assert L.gs_accept_workspace_bytes(0, 576, 151936) == 0
    g = np.array([1, -2], dtype=np.int32)
    rc = L.gs_accept_reject(2, g.ctypes.data, 8, 16, 8, 8, 8, 8, 8, None, 8, 0, None)
    assert rc == -1
    out = gsb.gs_accept_out(8, 8, 8, None)
    import ctypes as C
    rc = L.gs_accept_reject(2, g.ctypes.data, 8, 16, 8, 8, 8, 8, 8, C.byref(out), 8, 0, None)
    assert rc == -1 and b"gamma[1]" in L.gs_last_error()
    g[1] = 2
    rc = L.gs_accept_reject(2, g.ctypes.data, 8, 16, 8, 8, 8, 8, 8, C.byref(out), 8, 16, None)
    assert rc == -3


def test_static_scratch_entry_point_rejects_oversized_batches_on_the_host():
    """gs_accept_reject_static: sizes beyond its array fail with GS_ECAPACITY before any HIP call."""
    import ctypes as C
    L = gsb.lib()
    n = 4200
    g = np.ones(n, dtype=np.int32)
    assert L.gs_accept_workspace_bytes(n, 2 * n, 262144) > (4 << 20)
    out = gsb.gs_accept_out(8, 8, 8, None)
    rc = L.gs_accept_reject_static(n, g.ctypes.data, 8, 262144, 8, 8, 8, 8, 8, C.byref(out), None)
    assert rc == -3 and b"static array" in L.gs_last_error()
    g[7] = -1
    assert L.gs_accept_reject_static(n, g.ctypes.data, 8, 262144, 8, 8, 8, 8, 8, C.byref(out), None) == -1


def test_accept_reject_rejects_more_rows_than_a_grid_holds():
    import ctypes as C
    L = gsb.lib()
    n = 3000
    g = np.full(n, 2000, dtype=np.int32)             # 6 million rows
    out = gsb.gs_accept_out(8, 8, 8, None)
    rc = L.gs_accept_reject(n, g.ctypes.data, 8, 1024, 8, 8, 8, 8, 8, C.byref(out), 8, 1 << 40, None)
    assert rc == -1 and b"too many rows" in L.gs_last_error()


def test_baseline_allocation_policies_of_the_loop_equal_the_oracle():
    """Host logic of the closed loop: the even and the random split (no GPU involved)."""
    from oracle import closed_loop as ol
    from paper_2512_09963_amd import closed_loop as cl
    rng = np.random.default_rng(5)
    for _ in range(50):
        n = int(rng.integers(1, 12))
        C = int(rng.integers(0, 60))
        np.testing.assert_array_equal(cl.even_split(C, n), ol.fixed_allocation(C, n))
        u = rng.random(C + 3).astype(np.float32)
        got = cl.random_split(C, n, u)
        np.testing.assert_array_equal(got, ol.random_allocation(C, n, u))
        assert got.sum() == C


def _serpentine_busiest(steps, t, n_kv):
    """Brute force of what the planner models: split lengths sorted longest first, dealt to 256 compute units in
    rounds that alternate direction counted from the last (forward) round."""
    lens = []
    for st in steps:
        n = -(-st // t)
        base, rem = divmod(st, n)
        lens += [base + 1] * (rem * n_kv) + [base] * ((n - rem) * n_kv)
    lens.sort(reverse=True)
    rounds = -(-len(lens) // 256)
    load = [0] * 256
    for p, l in enumerate(lens):
        r, c = divmod(p, 256)
        load[255 - c if (rounds - 1 - r) & 1 else c] += l
    return len(lens), max(load)


@pytest.mark.parametrize("seed", range(30))
def test_attention_plan_invariants_on_random_batches(seed):
    rng = np.random.default_rng(7000 + seed)
    n = int(rng.choice([1, 3, 8, 32, 200, 900]))
    n_kv = int(rng.choice([1, 2, 8]))
    group = int(rng.choice([1, 4, 8]))
    gamma = rng.integers(0, int(rng.choice([2, 9, 17])), n)
    ctx = rng.integers(0, int(rng.choice([50, 3000, 40000])), n)
    sps, items, busiest = gsb.gs_plan_attention(n_kv, group, gamma, ctx)
    steps = ((ctx + gamma + 1 + 31) // 32).tolist()
    assert 1 <= sps <= max(steps)
    assert sps >= min(6, max(steps))                      # floor on the split length
    assert max(-(-s // sps) for s in steps) <= 32         # at most 32 splits per server
    want_items, want_busiest = _serpentine_busiest(steps, sps, n_kv)
    assert items == want_items == sum(-(-s // sps) for s in steps) * n_kv
    assert busiest == want_busiest
    assert busiest >= -(-sum(steps) * n_kv // 256)        # no compute unit below the mean is the busiest


def test_attention_plan_of_the_measured_workloads():
    # uniform contexts: 8 servers at 2048 tokens keep the shortest splits (6 steps, 704 workgroups); 16 servers at
    # 4096 tokens with 8 KV heads take 6 splits of 22 steps (3 per compute unit) instead of 7 of 19
    assert gsb.gs_plan_attention(8, 4, np.full(8, 6), np.full(8, 2048)) == (6, 704, 18)
    sps, items, busiest = gsb.gs_plan_attention(8, 8, np.full(16, 8), np.full(16, 4096))   # 72 query rows: 3 waves
    assert (sps, items) == (22, 768) and busiest <= 66
    # one server: all of the chip's workgroups come from its own splits
    sps, items, _ = gsb.gs_plan_attention(8, 4, [4], [131072])
    assert items == 8 * -(-4097 // sps) and items <= 32 * 8
    with pytest.raises(gsb.GsError):
        gsb.gs_plan_attention(8, 4, [-1], [10])
