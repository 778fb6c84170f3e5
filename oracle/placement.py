"""Load-balancing placement of the inversions on P workers (TEST INFRASTRUCTURE).

Plain Python statement of what Sec. IV-B defines: the two cost models (Eq. inverting-model,
Eq. broadcast-model), the load-balancing placement (Algorithm 1) with its rule for communicated /
non-communicated tensors, the sequential placement it is compared with, and the objective (overall
time) of the problem statement.  Shares no code with the library's kfac_place_inversions and is
imported only by tests.

`lbp` is written from the definition, not from the printed listing: a tensor whose inverse is
cheaper to compute than to receive is computed by everybody, which loads every worker alike and so
never changes which worker is the lightest; the placement is therefore decided by the communicated
tensors alone, largest first, each to the worker that carries the least so far.

Readings of garbled places: Algorithm 1 adds d_i to a worker's load while the text balances d_i^2;
`weight_power` selects d_i ** weight_power (1 = as the listing prints, 2 = as the text says).  The
sequential placement is printed as "i % p = 0"; it is taken as round-robin, tensor i on worker
i mod P.
"""
from __future__ import annotations

import math
from typing import Callable, List, Sequence


def t_comp(d: int, alpha_inv: float, beta_inv: float) -> float:
    """Eq. inverting-model: time of inverting a d x d matrix."""
    return alpha_inv * math.exp(beta_inv * d)


def t_comm(d: int, alpha_bcast: float, beta_bcast: float) -> float:
    """Eq. broadcast-model: time of broadcasting the d(d+1)/2 packed elements of an inverse."""
    return alpha_bcast + beta_bcast * (d * (d + 1) / 2)


def lbp(dims: Sequence[int], P: int, est_comp: Callable[[int], float], est_comm: Callable[[int], float],
        weight_power: int = 1) -> List[int]:
    """Load-balancing placement (Sec. IV-B, Algorithm 1).  Returns owner[i]: the worker that inverts
    tensor i, or -1 when every worker does (a non-communicated tensor: its inverse is cheaper to
    compute than to receive)."""
    everybody = {i for i, d in enumerate(dims) if est_comp(d) < est_comm(d)}
    owner = [-1] * len(dims)
    carried = [0.0] * P          # load from communicated tensors only; the replicated ones add the same to all
    communicated = [i for i in range(len(dims)) if i not in everybody]
    communicated.sort(key=lambda i: dims[i], reverse=True)     # stable: equal sizes keep their input order
    for i in communicated:
        lightest = carried.index(min(carried))                  # lowest index among equally light workers
        owner[i] = lightest
        carried[lightest] += float(dims[i]) ** weight_power
    return owner


def seq_dist(N: int, P: int) -> List[int]:
    """The sequential placement of earlier work: every tensor is communicated, tensor i on worker i mod P."""
    return [i % P for i in range(N)]


def overall_time(owner: Sequence[int], dims: Sequence[int], P: int, est_comp: Callable[[int], float],
                 est_comm: Callable[[int], float]) -> float:
    """Objective of the problem statement: max over workers of the computation time of the tensors
    placed on it plus the communication time of those among them that are communicated."""
    t = [0.0] * P
    for i, o in enumerate(owner):
        if o < 0:
            for p in range(P):
                t[p] += est_comp(dims[i])
        else:
            t[o] += est_comp(dims[i]) + est_comm(dims[i])
    return max(t) if P > 0 else 0.0
