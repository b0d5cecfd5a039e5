"""Hand-built fleets for the tests (plain namespaces with the array attributes of
workloads.Fleet): inputs only, none of the path's arithmetic."""
from types import SimpleNamespace

import numpy as np

CLASSES = [(2e-5, 0.012, 2e-4, 2e-8), (5e-5, 0.025, 4e-4, 5e-8), (1.2e-4, 0.05, 8e-4, 1e-7)]


def fleet(inst_class, actives, queued, incoming, budgets, act_budget=None, refreshed=None,
          classes=CLASSES, max_len=4096):
    """actives: per instance arrays (prompt, gen, rem) as [n,3]; queued: [n,2]; incoming: [R,2]."""
    i32 = lambda a: np.ascontiguousarray(a, dtype=np.int32)
    A = [np.asarray(a, dtype=np.int64).reshape(-1, 3) for a in actives]
    Q = [np.asarray(q, dtype=np.int64).reshape(-1, 2) for q in queued]
    a = np.concatenate(A) if A else np.zeros((0, 3), np.int64)
    q = np.concatenate(Q) if Q else np.zeros((0, 2), np.int64)
    inc = np.asarray(incoming, dtype=np.int64).reshape(-1, 2)
    names = ("delta", "alpha", "beta", "gamma")
    na = len(a)
    return SimpleNamespace(
        coef={k: np.array([c[i] for c in classes], dtype=np.float64) for i, k in enumerate(names)},
        inst_class=i32(inst_class), max_len=max_len,
        act_off=i32(np.cumsum([0] + [len(x) for x in A])),
        act_prompt=i32(a[:, 0]), act_gen=i32(a[:, 1]), act_rem=i32(a[:, 2]),
        act_rem_refreshed=i32(a[:, 2] if refreshed is None else refreshed),
        act_budget=np.ascontiguousarray(np.full(na, 1e9) if act_budget is None else act_budget,
                                        dtype=np.float32),
        q_off=i32(np.cumsum([0] + [len(x) for x in Q])),
        q_prompt=i32(q[:, 0]), q_len=i32(q[:, 1]),
        in_prompt=i32(inc[:, 0]), in_len=i32(inc[:, 1]),
        in_budget=np.ascontiguousarray(budgets, dtype=np.float32))


def rand_entries(rng, n, max_len=4096):
    return np.stack([rng.integers(128, 2049, n), rng.integers(0, 201, n),
                     np.clip(np.rint(rng.lognormal(5, 1, n)), 1, max_len)], axis=1)


def solo(P, L, c=CLASSES[0]):
    return c[0] * P + L * (c[1] + c[2]) + c[3] * (P * L + L * (L - 1) / 2)


def two_equal_minima_in_one_lane(n_between: int = 63):
    """A fleet in which two different instances give some requests the same latency bit for
    bit (fp64 and fp32 alike: every term is a small multiple of a power of two), sit
    ``n_between + 1`` positions apart in capability order, and beat everybody else:

      * instance 0          class B (alpha 1/4), one queued request of 2 048 prompt tokens: q = 2
      * instances 1..n      class C (alpha 3/8), a long queue: q = 20
      * instance n + 1      class A (alpha 1/2), idle

    with delta = 2^-10 and beta = gamma = 0 everywhere.  T_A = c0/1024 + L/2 and
    T_B = 2 + c0/1024 + L/4 meet at L = 8; A is first in capability order (largest d_g), B has
    the lower index.  Requests of length 8 with a deadline nobody meets must go to instance 0
    (smallest T, ties to the lowest index); shorter ones go to A, longer ones to B.
    Half of the requests have deadlines everybody meets (just-enough: the first in
    capability order, instance n + 1)."""
    classes = [(2.0 ** -10, 0.5, 0.0, 0.0), (2.0 ** -10, 0.25, 0.0, 0.0), (2.0 ** -10, 0.375, 0.0, 0.0)]
    M = n_between + 2
    inst_class = [1] + [2] * n_between + [0]
    queued = [[(2048, 1)]] + [[(2048, 3)] * 10 for _ in range(n_between)] + [[]]
    rng = np.random.default_rng(7)
    n = 96
    L = np.tile(np.array([8, 8, 4, 16, 8, 7, 9, 8]), n // 8)
    c0 = rng.integers(1, 2049, n)
    budgets = np.where(np.arange(n) % 2 == 0, 0.25, 1e6)
    fl = fleet(inst_class, [[] for _ in range(M)], queued, np.stack([c0, L], 1), budgets, classes=classes,
               max_len=64)
    return fl
