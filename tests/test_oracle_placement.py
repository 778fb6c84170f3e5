"""Pins of the oracle's placement functions (Sec. IV-B), CPU only."""
import itertools
import math

import numpy as np

from oracle import placement as pl


def test_cost_models_closed_forms():
    assert pl.t_comp(0, 2.5, 0.01) == 2.5                        # alpha_inv is the value at d = 0
    assert math.isclose(pl.t_comp(100, 2.0, 0.01) / pl.t_comp(0, 2.0, 0.01), math.e)
    assert pl.t_comm(64, 3.0, 0.5) == 3.0 + 0.5 * 2080           # 2080 packed elements for d = 64 (Sec. IV-A)


def test_constructed_two_worker_example_reproduces_the_stated_savings():
    """The paper's figure of four tensors on two workers is not available; this is an example built
    to have the properties its text states: balancing saves one time slot over the sequential
    placement, and letting the small tensor be computed everywhere saves another half slot."""
    slot = 1.0
    comp = {40: 1.5 * slot, 30: 1.5 * slot, 20: 0.5 * slot, 10: 0.5 * slot}   # keyed by dimension
    comm = {d: 1.0 * slot for d in comp}
    dims = [40, 20, 30, 10]
    seq = pl.seq_dist(4, 2)                                                   # worker 0: 40, 30; worker 1: 20, 10
    t_seq = pl.overall_time(seq, dims, 2, comp.get, comm.get)
    assert t_seq == 5.0 * slot
    never = lambda d: 0.0                                                     # placement that ignores communication
    bal = pl.lbp(dims, 2, comp.get, never, weight_power=1)
    assert bal == [0, 1, 1, 0]                                                # 40 + 10 against 30 + 20
    t_bal = pl.overall_time(bal, dims, 2, comp.get, comm.get)
    assert t_seq - t_bal == 1.0 * slot
    full = pl.lbp(dims, 2, comp.get, comm.get, weight_power=1)
    assert full == [0, -1, 1, -1]                                             # the two small ones are cheaper to compute than to receive
    t_full = pl.overall_time(full, dims, 2, comp.get, comm.get)
    assert t_bal - t_full == 0.5 * slot


def test_every_tensor_is_placed_once_or_everywhere():
    rng = np.random.default_rng(0)
    for _ in range(50):
        N, P = int(rng.integers(1, 30)), int(rng.integers(1, 9))
        dims = [int(d) for d in rng.integers(1, 5000, N)]
        owner = pl.lbp(dims, P, lambda d: 1e-6 * d ** 2, lambda d: 3.0 + 1e-7 * d * (d + 1) / 2)
        assert len(owner) == N and all(-1 <= o < P for o in owner)
        # the rule for non-communicated tensors depends on the tensor alone
        for d, o in zip(dims, owner):
            assert (o == -1) == (1e-6 * d ** 2 < 3.0 + 1e-7 * d * (d + 1) / 2)


def test_greedy_is_within_grahams_bound_of_the_optimum():
    """With no communication and bucket weight = cost, Algorithm 1 is largest-first list scheduling,
    whose makespan is at most (4/3 - 1/(3P)) times the optimum (brute force on small instances)."""
    rng = np.random.default_rng(1)
    for _ in range(40):
        N, P = int(rng.integers(2, 8)), int(rng.integers(2, 4))
        dims = [int(d) for d in rng.integers(1, 100, N)]
        cost = lambda d: float(d)
        owner = pl.lbp(dims, P, cost, lambda d: 0.0, weight_power=1)
        t = pl.overall_time(owner, dims, P, cost, lambda d: 0.0)
        best = min(max(sum(dims[i] for i in range(N) if a[i] == p) for p in range(P))
                   for a in itertools.product(range(P), repeat=N))
        assert best <= t <= (4.0 / 3.0 - 1.0 / (3 * P)) * best + 1e-9


def test_sequential_placement_is_round_robin():
    assert pl.seq_dist(5, 2) == [0, 1, 0, 1, 0]
    dims = [4, 3, 2, 1]
    assert pl.overall_time(pl.seq_dist(4, 2), dims, 2, float, lambda d: 0.0) == 6.0
