"""CPU reference, second part (test infrastructure only): the EMA-smoothed
black-box instance status of Sec. 3.3 / Alg. 1, Eq. 2 formed from it, and its
blend with the white-box estimate of ``goodroute_oracle.c``.

Plain numpy in fp64, one formula per function:

  * Alg. 1 updates ``q_g <- a*w_g + (1-a)*q_g`` from the observed waiting time
    before it forms T(r,g); Sec. 3.3 smooths p_g and d_g the same way.
  * Eq. 2 with that status: ``T = q_g + p_g*(L_in - H) + d_g*L_out``.
  * The blend is a straight line between the two estimates, weight ``lam`` on
    the black-box one (``lam = 0``: the white-box model alone; ``lam = 1``: the
    paper's estimator alone).  The same weight blends the instance's decode
    speed d_g that Alg. 1's argmax ranks by, and the expected finish of the
    requests an instance already holds (black-box: d_g per remaining token for
    a running request; q_g + p_g*prompt + d_g*length for a queued one).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np


def ema_step(prev: Optional[np.ndarray], sample, weight: float) -> np.ndarray:
    """One exponential-moving-average step, Alg. 1's ``q <- a*w + (1-a)*q``.
    Without an earlier estimate the sample is the estimate."""
    sample = np.asarray(sample, dtype=np.float64)
    if prev is None:
        return sample.copy()
    return weight * sample + (1.0 - weight) * np.asarray(prev, dtype=np.float64)


@dataclass
class SmoothedStatus:
    """Per-instance smoothed observations: queuing delay, prefill seconds per
    token, decode seconds per token (Eq. 2's q_g, p_g, d_g)."""
    q: Optional[np.ndarray] = None
    p: Optional[np.ndarray] = None
    d: Optional[np.ndarray] = None

    def observe(self, weight: float, wait=None, prefill=None, decode=None) -> None:
        if wait is not None:
            self.q = ema_step(self.q, wait, weight)
        if prefill is not None:
            self.p = ema_step(self.p, prefill, weight)
        if decode is not None:
            self.d = ema_step(self.d, decode, weight)


def eq2_latency(st: SmoothedStatus, c0, length, H=None) -> np.ndarray:
    """Eq. 2 for every pair: [n, M].  H: [n, M] cached prefix lengths or None."""
    c0 = np.asarray(c0, dtype=np.float64)[:, None]
    L = np.asarray(length, dtype=np.float64)[:, None]
    h = 0.0 if H is None else np.asarray(H, dtype=np.float64)
    return st.q[None, :] + st.p[None, :] * (c0 - h) + st.d[None, :] * L


def blend(model, blackbox, lam: float):
    return (1.0 - lam) * np.asarray(model, dtype=np.float64) + lam * np.asarray(blackbox, dtype=np.float64)


def dense_hits(hits, n_req: int, n_inst: int, c0) -> np.ndarray:
    """[n, M] matrix of cached prefix lengths from the CSR lists (longest entry per pair, cut to c0)."""
    H = np.zeros((n_req, n_inst), dtype=np.int64)
    if hits is None:
        return H
    off, inst, ln = (np.asarray(x) for x in hits)
    for r in range(n_req):
        for k in range(off[r], off[r + 1]):
            g = int(inst[k])
            if 0 <= g < n_inst:
                H[r, g] = max(H[r, g], int(ln[k]))
    return np.minimum(H, np.asarray(c0, dtype=np.int64)[:, None])


def select(T: np.ndarray, d: np.ndarray, deadline, exclude=None):
    """Alg. 1 for every row of T: feasible set {g: T <= D}; the feasible
    instance of largest d_g (ties: lowest index); none feasible: smallest T
    (ties: lowest index).  numpy's argmax/argmin return the first, i.e. lowest,
    index among equals.  Returns (inst, slack, fallback, T_chosen)."""
    T = np.array(T, dtype=np.float64)
    n, M = T.shape
    D = np.asarray(deadline, dtype=np.float64)
    allowed = np.ones((n, M), dtype=bool)
    if exclude is not None:
        ex = np.asarray(exclude)
        rows = np.flatnonzero((ex >= 0) & (ex < M))
        allowed[rows, ex[rows]] = False
    feasible = allowed & (T <= D[:, None])
    by_speed = np.where(feasible, np.asarray(d, dtype=np.float64)[None, :], -np.inf)
    pick_feasible = np.argmax(by_speed, axis=1)
    pick_least = np.argmin(np.where(allowed, T, np.inf), axis=1)
    any_feasible = feasible.any(axis=1)
    inst = np.where(any_feasible, pick_feasible, pick_least).astype(np.int32)
    inst[~allowed.any(axis=1)] = -1
    ok = inst >= 0
    Tc = np.zeros(n)
    Tc[ok] = T[np.flatnonzero(ok), inst[ok]]
    slack = np.where(ok, D - Tc, 0.0)
    return inst, slack, (~any_feasible).astype(np.uint8), Tc


class BlendedFleet:
    """A simulated fleet seen through the blend: same attributes and methods
    as ``oracle.SimulatedFleet`` (what the parity checks use)."""

    def __init__(self, sim, fleet, status: SmoothedStatus, lam: float, act_rem=None):
        from . import Routing
        self._Routing = Routing
        self.sim, self.status, self.lam = sim, status, float(lam)
        self.n_inst = sim.n_inst
        self.q, self.smax = sim.q, sim.smax
        self.d = blend(sim.d, status.d, lam)
        rem = np.asarray(fleet.act_rem if act_rem is None else act_rem, dtype=np.float64)
        inst_a = np.repeat(np.arange(self.n_inst), np.diff(np.asarray(fleet.act_off)))
        inst_q = np.repeat(np.arange(self.n_inst), np.diff(np.asarray(fleet.q_off)))
        self.act_finish = blend(sim.act_finish, status.d[inst_a] * rem, lam)
        self.q_finish = blend(sim.q_finish,
                              status.q[inst_q] + status.p[inst_q] * np.asarray(fleet.q_prompt, dtype=np.float64)
                              + status.d[inst_q] * np.asarray(fleet.q_len, dtype=np.float64), lam)
        self.act_off = sim.act_off

    @property
    def rank(self) -> np.ndarray:
        order = np.lexsort((np.arange(self.n_inst), -self.d))
        rank = np.empty(self.n_inst, dtype=np.int32)
        rank[order] = np.arange(self.n_inst, dtype=np.int32)
        return rank

    def pair_T(self, c0, length, hits=None) -> np.ndarray:
        H = dense_hits(hits, len(c0), self.n_inst, c0)
        return blend(self.sim.pair_T(c0, length, hits=hits), eq2_latency(self.status, c0, length, H), self.lam)

    def route(self, c0, length, deadline, exclude=None, hits=None):
        T = self.pair_T(c0, length, hits=hits)
        inst, slack, fb, Tc = select(T, self.d, deadline, exclude)
        return self._Routing(inst, slack, fb, Tc)
