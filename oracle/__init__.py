"""Python face of the CPU reference (test infrastructure only).

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It wraps ``goodroute_oracle.c`` (plain C, fp64, compiled with
gcc) with numpy arrays and composes the periodic risk re-check of Sec. 3.4 out
of the two primitives the C file provides: simulate every instance, and run
Alg. 1 by exhaustive scan.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "goodroute_oracle.c")
_SO = os.path.join(_HERE, "libgoodroute_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C reference with gcc.  -ffp-contract=off keeps every
    multiply-add exactly as written; the only fused operations are the explicit
    fma() calls."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        p = C.c_void_p
        lib.gro_simulate.restype = p
        lib.gro_simulate.argtypes = [C.c_int32, C.c_int32] + [p] * 15
        lib.gro_free.argtypes = [p]
        lib.gro_status.argtypes = [p, p, p, p]
        lib.gro_step_table.argtypes = [p, C.c_int32, p]
        lib.gro_pair_T.argtypes = [p, C.c_int64] + [p] * 6
        lib.gro_route.argtypes = [p, C.c_int64] + [p] * 11
        lib.gro_band.argtypes = [p, C.c_int64] + [p] * 8 + [C.c_double] + [p] * 7
        lib.gro_threads.restype = C.c_int32
        _lib = lib
    return _lib


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def threads() -> int:
    return int(_load().gro_threads())


@dataclass
class Routing:
    inst: np.ndarray        # int32, chosen instance (-1: none allowed)
    slack: np.ndarray       # float64, D - T(r, chosen)
    fallback: np.ndarray    # uint8, 1 when no instance was feasible
    T: np.ndarray           # float64, T(r, chosen)


@dataclass
class Band:
    """Per request, what decides whether Alg. 1's answer survives a relative error eps
    on every latency (see gro_band in the C file); ranks are positions in capability order."""
    sure: np.ndarray        # int32, first surely feasible rank, n_inst if none
    maybe: np.ndarray       # int32, first possibly feasible rank, n_inst if none
    tmin: np.ndarray        # float64, least latency over the allowed instances
    near: np.ndarray        # int32, instances within 2 eps of the least latency
    equal: np.ndarray       # int32, instances whose latency equals the least one bit for bit
    picked_T: np.ndarray    # float64, latency of the pair (request, picked instance)


class SimulatedFleet:
    """Result of simulating every instance of a fleet step by step."""

    def __init__(self, coef, inst_class, act_off, act_prompt, act_gen, act_rem,
                 q_off, q_prompt, q_len, cap=None):
        lib = _load()
        self.n_inst = int(len(inst_class))
        self._keep = [_f64(coef[k]) for k in ("delta", "alpha", "beta", "gamma")]
        args = [_i32(inst_class), _i32(act_off), _i32(act_prompt), _i32(act_gen), _i32(act_rem),
                _i32(q_off), _i32(q_prompt), _i32(q_len)]
        self.act_finish = np.zeros(len(args[2]), dtype=np.float64)
        self.q_finish = np.zeros(len(args[6]), dtype=np.float64)
        self._cap = None if cap is None else _i32(cap)      # concurrent requests per instance (Sec. 3.1)
        self._h = lib.gro_simulate(self.n_inst, len(self._keep[0]),
                                   *[_ptr(a) for a in self._keep], *[_ptr(a) for a in args],
                                   _ptr(self._cap), _ptr(self.act_finish), _ptr(self.q_finish))
        if not self._h:
            raise MemoryError("gro_simulate failed")
        self.q = np.zeros(self.n_inst, dtype=np.float64)
        self.d = np.zeros(self.n_inst, dtype=np.float64)
        self.smax = np.zeros(self.n_inst, dtype=np.int32)
        lib.gro_status(self._h, _ptr(self.q), _ptr(self.d), _ptr(self.smax))
        self.act_off = args[1]

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:
            _lib.gro_free(self._h)
            self._h = None

    @property
    def rank(self) -> np.ndarray:
        """Position of each instance in capability order: slowest current
        decode step first (largest d_g), equal d_g by index (Alg. 1's argmax)."""
        order = np.lexsort((np.arange(self.n_inst), -self.d))
        rank = np.empty(self.n_inst, dtype=np.int32)
        rank[order] = np.arange(self.n_inst, dtype=np.int32)
        return rank

    def step_table(self, g: int) -> np.ndarray:
        w = np.zeros(int(self.smax[g]) + 1, dtype=np.float64)
        _load().gro_step_table(self._h, int(g), _ptr(w))
        return w

    @staticmethod
    def _hits(hits):
        """hits: None or (hit_off[n+1], hit_inst, hit_len): cached prefixes by request (Eq. 2's H)."""
        if hits is None:
            return None, None, None
        return tuple(_i32(a) for a in hits)

    def pair_T(self, c0, length, hits=None) -> np.ndarray:
        c0, length = _i32(c0), _i32(length)
        ho, hi, hl = self._hits(hits)
        out = np.zeros((len(c0), self.n_inst), dtype=np.float64)
        _load().gro_pair_T(self._h, len(c0), _ptr(c0), _ptr(length), _ptr(ho), _ptr(hi), _ptr(hl), _ptr(out))
        return out

    def route(self, c0, length, deadline, exclude=None, hits=None) -> Routing:
        c0, length, deadline = _i32(c0), _i32(length), _f64(deadline)
        n = len(c0)
        ex = None if exclude is None else _i32(exclude)
        ho, hi, hl = self._hits(hits)
        r = Routing(np.zeros(n, np.int32), np.zeros(n, np.float64),
                    np.zeros(n, np.uint8), np.zeros(n, np.float64))
        _load().gro_route(self._h, n, _ptr(c0), _ptr(length), _ptr(deadline), _ptr(ex),
                          _ptr(ho), _ptr(hi), _ptr(hl),
                          _ptr(r.inst), _ptr(r.slack), _ptr(r.fallback), _ptr(r.T))
        return r

    def band(self, c0, length, deadline, picked, eps: float, exclude=None, hits=None) -> Band:
        c0, length, deadline, picked = _i32(c0), _i32(length), _f64(deadline), _i32(picked)
        n = len(c0)
        ex = None if exclude is None else _i32(exclude)
        ho, hi, hl = self._hits(hits)
        rank = _i32(self.rank)
        b = Band(np.zeros(n, np.int32), np.zeros(n, np.int32), np.zeros(n, np.float64),
                 np.zeros(n, np.int32), np.zeros(n, np.int32), np.zeros(n, np.float64))
        _load().gro_band(self._h, n, _ptr(c0), _ptr(length), _ptr(deadline), _ptr(ex),
                         _ptr(ho), _ptr(hi), _ptr(hl), _ptr(rank), float(eps), _ptr(picked),
                         _ptr(b.sure), _ptr(b.maybe), _ptr(b.tmin), _ptr(b.near), _ptr(b.equal),
                         _ptr(b.picked_T))
        return b


def simulate(fleet, act_rem=None) -> SimulatedFleet:
    """fleet: any object with the array attributes of workloads.Fleet; an
    optional attribute ``batch_cap`` (int per instance) bounds each batch."""
    return SimulatedFleet(fleet.coef, fleet.inst_class, fleet.act_off, fleet.act_prompt,
                          fleet.act_gen, fleet.act_rem if act_rem is None else act_rem,
                          fleet.q_off, fleet.q_prompt, fleet.q_len, cap=getattr(fleet, "batch_cap", None))


@dataclass
class RiskScan:
    sim: SimulatedFleet
    finish: np.ndarray      # float64 per active request
    flag: np.ndarray        # uint8, 1 when the expected finish exceeds the deadline left
    target: np.ndarray      # int32, migration target of flagged requests, -1 otherwise
    target_slack: np.ndarray


def risk_scan(fleet, act_rem_refreshed, act_budget, only: Optional[np.ndarray] = None,
              view=None) -> RiskScan:
    """Sec. 3.4's periodic re-check against one snapshot of the fleet: simulate
    with the refreshed lengths; a request whose finish exceeds its budget is
    flagged and re-routed by Alg. 1 among the other instances, where it
    prefills prompt + generated tokens again and still has its refreshed
    length to decode.  ``only`` restricts target selection to a subset of
    active-request indices (large fleets).  ``view`` maps the simulated fleet
    to the object whose estimates are used (default: the simulation itself)."""
    sim = simulate(fleet, act_rem_refreshed)
    if view is not None:        # e.g. the blend with the black-box status: same interface, other numbers
        sim = view(sim)
    budget = np.asarray(act_budget, dtype=np.float64)
    flag = (sim.act_finish > budget).astype(np.uint8)
    n = len(flag)
    target = np.full(n, -1, dtype=np.int32)
    tslack = np.zeros(n, dtype=np.float64)
    idx = np.flatnonzero(flag)
    if only is not None:
        idx = np.intersect1d(idx, np.asarray(only))
    if len(idx):
        inst_of = (np.searchsorted(np.asarray(fleet.act_off), idx, side="right") - 1).astype(np.int32)
        c0 = np.asarray(fleet.act_prompt)[idx].astype(np.int64) + np.asarray(fleet.act_gen)[idx]
        r = sim.route(c0, np.asarray(act_rem_refreshed)[idx], budget[idx], exclude=inst_of)
        target[idx] = r.inst
        tslack[idx] = r.slack
    return RiskScan(sim, sim.act_finish, flag, target, tslack)


class _Extended:
    """A fleet with more queued requests appended per instance (plain arrays, as workloads.Fleet)."""

    def __init__(self, fleet, extra):
        M = len(fleet.inst_class)
        self.coef, self.inst_class = fleet.coef, fleet.inst_class
        if getattr(fleet, "batch_cap", None) is not None:
            self.batch_cap = fleet.batch_cap
        self.act_off, self.act_prompt = fleet.act_off, fleet.act_prompt
        self.act_gen, self.act_rem = fleet.act_gen, fleet.act_rem
        qp, ql, off = [], [], [0]
        for g in range(M):
            a, b = int(fleet.q_off[g]), int(fleet.q_off[g + 1])
            qp += list(fleet.q_prompt[a:b]) + [e[0] for e in extra[g]]
            ql += list(fleet.q_len[a:b]) + [e[1] for e in extra[g]]
            off.append(len(qp))
        self.q_off = np.array(off, dtype=np.int32)
        self.q_prompt = np.array(qp, dtype=np.int32)
        self.q_len = np.array(ql, dtype=np.int32)


def route_with_feedback(fleet, c0, length, deadline, chunk: int, exclude=None, follow=None):
    """Alg. 1 with the fleet's status kept up to date between decisions, the way
    the paper's proxy routes (one request after the other, each seeing the
    requests routed before it): the batch is taken ``chunk`` requests at a time
    in arrival order; a chunk is decided against one snapshot, then each of its
    requests joins the queue of the instance it was sent to (prompt = its
    tokens to prefill, length = its predicted decode length), and the next
    chunk sees the fleet simulated anew.  ``chunk = 1`` is request by request.

    ``follow``: instance per request to commit instead of this function's own
    choice (to check another implementation step by step from the states it
    really went through).  Returns (Routing, list of per-chunk (rows, T, rank)
    with T the [chunk, M] latencies and rank the capability order the chunk saw)."""
    c0, length = _i32(c0), _i32(length)
    deadline = _f64(deadline)
    n, M = len(c0), len(fleet.inst_class)
    extra = [[] for _ in range(M)]
    out = Routing(np.zeros(n, np.int32), np.zeros(n, np.float64), np.zeros(n, np.uint8), np.zeros(n, np.float64))
    seen = []
    for s in range(0, n, chunk):
        rows = np.arange(s, min(s + chunk, n))
        sim = simulate(_Extended(fleet, extra))
        ex = None if exclude is None else _i32(exclude)[rows]
        r = sim.route(c0[rows], length[rows], deadline[rows], exclude=ex)
        out.inst[rows], out.slack[rows], out.fallback[rows], out.T[rows] = r.inst, r.slack, r.fallback, r.T
        seen.append((rows, sim.pair_T(c0[rows], length[rows]), sim.rank))
        commit = r.inst if follow is None else np.asarray(follow)[rows]
        for i, g in zip(rows, commit):
            if g >= 0:
                extra[int(g)].append((int(c0[i]), int(length[i])))
    return out, seen


from .blackbox import BlendedFleet, SmoothedStatus  # noqa: E402,F401
