"""Seeded synthetic fleets: the inputs of the routing path, nothing else.

The paper replays prompts of three agentic benchmarks on a production arrival
trace (Sec. 4.1, "Workloads"); only token counts and deadlines ever reach the
routing math (Eq. 2, Alg. 1), so a fleet here is a set of integer length
arrays plus float deadlines drawn from stated distributions.  The deadline
recipe follows the paper's own (Sec. 4.1: solo latency on a reference GPU
times a relaxation factor).

This module holds no routing arithmetic.  It is imported by the tests, by the
benchmark and by the smoke check; neither the CPU checker nor the GPU library
imports it.  All draws come from ``numpy.random.Generator(PCG64(seed))`` in a
fixed order: active (prompt, generated, remaining), queued (prompt, length),
incoming (prompt, length, SLO factor), active SLO factors, drift factors,
per-instance occupancy jitter.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Tuple

import numpy as np

# Per-class coefficients of the linear step-time model: prefill costs delta
# seconds per prompt token; one decode step of a batch costs
# alpha + beta * batch + gamma * (sum of context lengths) seconds.
_CLASS0 = dict(delta=2e-5, alpha=0.012, beta=2e-4, gamma=2e-8)
_CLASS1 = dict(delta=5e-5, alpha=0.025, beta=4e-4, gamma=5e-8)
_CLASS2 = dict(delta=1.2e-4, alpha=0.05, beta=8e-4, gamma=1e-7)
_COEF_NAMES = ("delta", "alpha", "beta", "gamma")


def _coef_table(classes) -> Dict[str, np.ndarray]:
    return {k: np.array([c[k] for c in classes], dtype=np.float64) for k in _COEF_NAMES}


def _geometric_classes(n: int) -> Dict[str, np.ndarray]:
    """n classes, each coefficient spaced geometrically from class 0's value to
    three times class 2's value."""
    out = {}
    for k in _COEF_NAMES:
        lo, hi = _CLASS0[k], 3.0 * _CLASS2[k]
        out[k] = lo * (hi / lo) ** (np.arange(n, dtype=np.float64) / (n - 1))
    return out


@dataclass(frozen=True)
class FleetSpec:
    name: str
    n_inst: int
    class_pattern: Tuple[int, ...]          # class of instance g = pattern[g % len]
    coef: Dict[str, np.ndarray] = field(hash=False, compare=False, default=None)
    n_active: int = 64                      # active requests per instance (before jitter)
    n_queued: int = 0                       # queued requests per instance
    n_incoming: int = 16
    len_dist: str = "lognormal"             # decode lengths: "lognormal" | "pareto"
    max_len: int = 4096                     # clip of decode lengths
    prompt_dist: str = "uniform"            # "uniform" [128, 2048] | "lognormal" (7, 1)
    max_prompt: int = 2048
    slo_lo: float = 1.5
    slo_hi: float = 4.0
    slo_scale: float = 1.0                  # multiplies every SLO factor (decision-mix variants)
    drift_sigma: float = 0.0                # refreshed length = original * lognormal(0, sigma)
    occupancy_jitter: bool = False          # per-instance active count in [0.25, 1] * n_active
    seed: int = 0

    @property
    def n_class(self) -> int:
        return len(self.coef["delta"])

    @property
    def max_entries(self) -> int:
        return self.n_active + self.n_queued


def spec(name: str, **overrides) -> FleetSpec:
    """The five benchmark fleets ("tiny", "mid", "large", "migrate", "heavy")."""
    base = {
        "tiny": FleetSpec("tiny", 4, (0, 1), _coef_table([_CLASS0, _CLASS1]),
                          n_active=64, n_queued=8, n_incoming=16),
        "mid": FleetSpec("mid", 32, (0, 1, 2), _coef_table([_CLASS0, _CLASS1, _CLASS2]),
                         n_active=256, n_queued=32, n_incoming=4096),
        "large": FleetSpec("large", 256, (0, 1, 1, 2), _coef_table([_CLASS0, _CLASS1, _CLASS2]),
                           n_active=512, n_queued=0, n_incoming=65536),
        "migrate": FleetSpec("migrate", 1024, (0, 1, 1, 2),
                             _coef_table([_CLASS0, _CLASS1, _CLASS2]),
                             n_active=1000, n_queued=0, n_incoming=0, drift_sigma=0.5),
        "heavy": FleetSpec("heavy", 4096, (0, 1, 2, 3, 4, 5), _geometric_classes(6),
                           n_active=512, n_queued=0, n_incoming=262144,
                           len_dist="pareto", max_len=16384,
                           prompt_dist="lognormal", max_prompt=32768, drift_sigma=0.5),
    }[name]
    return replace(base, **overrides) if overrides else base


SPEC_NAMES = ("tiny", "mid", "large", "migrate", "heavy")


@dataclass
class Fleet:
    spec: FleetSpec
    coef: Dict[str, np.ndarray]             # float64 [n_class] each
    inst_class: np.ndarray                  # int32 [M]
    act_off: np.ndarray                     # int32 [M+1]
    act_prompt: np.ndarray                  # int32 [sum A]
    act_gen: np.ndarray                     # int32
    act_rem: np.ndarray                     # int32, predicted remaining decode length
    act_rem_refreshed: np.ndarray           # int32, re-predicted at scan time
    act_budget: np.ndarray                  # float32, arrival + SLO - now
    q_off: np.ndarray                       # int32 [M+1]
    q_prompt: np.ndarray                    # int32 [sum Q]
    q_len: np.ndarray                       # int32
    in_prompt: np.ndarray                   # int32 [R]
    in_len: np.ndarray                      # int32
    in_budget: np.ndarray                   # float32, E2E-SLO of each incoming request

    @property
    def n_inst(self) -> int:
        return int(self.inst_class.shape[0])


def _decode_lengths(rng, spec: FleetSpec, n: int) -> np.ndarray:
    if spec.len_dist == "lognormal":
        x = rng.lognormal(5.0, 1.0, n)
    elif spec.len_dist == "pareto":
        x = 32.0 * (1.0 + rng.pareto(1.3, n))       # classical Pareto, x_m = 32
    else:
        raise ValueError(spec.len_dist)
    return np.clip(np.rint(x), 1, spec.max_len).astype(np.int32)


def _prompts(rng, spec: FleetSpec, n: int) -> np.ndarray:
    if spec.prompt_dist == "uniform":
        return rng.integers(128, 2049, n).astype(np.int32)
    if spec.prompt_dist == "lognormal":
        return np.clip(np.rint(rng.lognormal(7.0, 1.0, n)), 1, spec.max_prompt).astype(np.int32)
    raise ValueError(spec.prompt_dist)


def _solo_latency_class0(coef, prompt, length) -> np.ndarray:
    """Latency of a request served alone on an idle class-0 instance: the
    reference the SLO factor multiplies (Sec. 4.1 sets SLOs the same way on
    its reference GPU)."""
    p = prompt.astype(np.float64)
    l = length.astype(np.float64)
    d, a, b, g = (coef[k][0] for k in _COEF_NAMES)
    return d * p + l * (a + b) + g * (p * l + l * (l - 1.0) * 0.5)


def make_fleet(spec: FleetSpec) -> Fleet:
    rng = np.random.Generator(np.random.PCG64(spec.seed))
    M, A, Q, R = spec.n_inst, spec.n_active, spec.n_queued, spec.n_incoming
    coef = {k: np.asarray(v, dtype=np.float64).copy() for k, v in spec.coef.items()}
    pat = np.asarray(spec.class_pattern, dtype=np.int32)
    inst_class = pat[np.arange(M) % len(pat)].astype(np.int32)

    a_prompt = _prompts(rng, spec, M * A)
    a_gen = rng.integers(0, 201, M * A).astype(np.int32)
    a_rem = _decode_lengths(rng, spec, M * A)
    qp = _prompts(rng, spec, M * Q)
    ql = _decode_lengths(rng, spec, M * Q)
    in_prompt = _prompts(rng, spec, R)
    in_len = _decode_lengths(rng, spec, R)
    in_u = rng.uniform(spec.slo_lo, spec.slo_hi, R) * spec.slo_scale
    a_u = rng.uniform(spec.slo_lo, spec.slo_hi, M * A) * spec.slo_scale
    drift = rng.lognormal(0.0, spec.drift_sigma, M * A) if spec.drift_sigma > 0 else None
    if spec.occupancy_jitter:
        keep_n = np.maximum(0, np.rint(rng.uniform(0.25, 1.0, M) * A)).astype(np.int64)
        keep_n[rng.integers(0, M)] = 0              # one idle instance
    else:
        keep_n = np.full(M, A, dtype=np.int64)

    keep = (np.arange(A)[None, :] < keep_n[:, None]).reshape(-1)
    act_off = np.zeros(M + 1, dtype=np.int32)
    act_off[1:] = np.cumsum(keep_n)
    q_off = (np.arange(M + 1, dtype=np.int64) * Q).astype(np.int32)

    a_rem_new = a_rem if drift is None else np.clip(
        np.rint(a_rem.astype(np.float64) * drift), 1, spec.max_len).astype(np.int32)

    # Deadline left for each active request: SLO of the whole request minus the
    # time it has already spent, the latter taken as its prefill plus its
    # generated tokens at the instance's current step time.
    inst_of = np.repeat(np.arange(M), A)
    cls_of = inst_class[inst_of]
    ctx = (a_prompt.astype(np.int64) + a_gen)
    n_g = keep_n.astype(np.float64) + Q
    ctx_sum = np.bincount(inst_of[keep], weights=ctx[keep].astype(np.float64), minlength=M)
    if Q:
        ctx_sum = ctx_sum + qp.reshape(M, Q).sum(axis=1, dtype=np.float64)
    step_now = coef["alpha"][inst_class] + coef["beta"][inst_class] * n_g \
        + coef["gamma"][inst_class] * ctx_sum
    slo = a_u * _solo_latency_class0(coef, a_prompt, a_gen.astype(np.int64) + a_rem)
    elapsed = coef["delta"][cls_of] * a_prompt + a_gen * step_now[inst_of]
    act_budget = (slo - elapsed).astype(np.float32)

    in_budget = (in_u * _solo_latency_class0(coef, in_prompt, in_len)).astype(np.float32)

    return Fleet(
        spec=spec, coef=coef, inst_class=inst_class,
        act_off=act_off, act_prompt=a_prompt[keep], act_gen=a_gen[keep], act_rem=a_rem[keep],
        act_rem_refreshed=a_rem_new[keep], act_budget=act_budget[keep],
        q_off=q_off, q_prompt=qp, q_len=ql,
        in_prompt=in_prompt, in_len=in_len, in_budget=in_budget,
    )


def cached_prefixes(fl: Fleet, mean_hits: float = 2.0, seed: int = 0):
    """Cached prompt prefixes of the incoming requests, as Eq. 2's H_{r,g}: a
    CSR (hit_off[R+1], hit_inst, hit_len).  Each request has a prefix on a
    Poisson(mean_hits) number of distinct instances (agentic sessions return
    to instances that served their earlier turns), of a length uniform in
    [1, prompt].  Draw order: counts, instances, lengths."""
    rng = np.random.Generator(np.random.PCG64(seed))
    R, M = len(fl.in_prompt), fl.n_inst
    cnt = np.minimum(rng.poisson(mean_hits, R), M).astype(np.int64)
    off = np.zeros(R + 1, dtype=np.int32)
    off[1:] = np.cumsum(cnt)
    n = int(off[-1])
    owner = np.repeat(np.arange(R), cnt)
    # distinct instances per request: a random start and a stride coprime to M walk M distinct values
    start = rng.integers(0, M, R)
    stride = 2 * rng.integers(0, max(M // 2, 1), R) + 1 if M % 2 == 0 else np.ones(R, dtype=np.int64)
    k = np.arange(n) - off[owner]
    inst = ((start[owner] + k * stride[owner]) % M).astype(np.int32)
    frac = rng.uniform(0.0, 1.0, n)
    ln = np.maximum(1, np.ceil(frac * fl.in_prompt[owner])).astype(np.int32)
    return off, inst, ln


def observed_status(fl: Fleet, rounds: int = 3, seed: int = 0):
    """Black-box observations of every instance, as Sec. 3.3 collects them: per
    round the average waiting time (seconds), the prefill seconds per token and
    the decode seconds per token (TPOT) of each instance, float32.  Values are
    the instance class's nominal figures at its current load times lognormal
    jitter (sigma 0.3), waiting times uniform in [0, 2] s.  Returns a list of
    (ema_weight, wait, prefill, decode) with weight 0.3; draw order per round:
    wait, prefill, decode."""
    rng = np.random.Generator(np.random.PCG64(seed))
    M = fl.n_inst
    n_g = (np.diff(fl.act_off) + np.diff(fl.q_off)).astype(np.float64)
    c = fl.inst_class
    out = []
    for _ in range(rounds):
        wait = rng.uniform(0.0, 2.0, M).astype(np.float32)
        prefill = (fl.coef["delta"][c] * rng.lognormal(0.0, 0.3, M)).astype(np.float32)
        decode = ((fl.coef["alpha"][c] + fl.coef["beta"][c] * n_g) * rng.lognormal(0.0, 0.3, M)).astype(np.float32)
        out.append((0.3, wait, prefill, decode))
    return out


def batch_caps(fl: Fleet, lo: float = 0.5, hi: float = 1.2, seed: int = 0) -> np.ndarray:
    """A cap on the requests each instance may decode together (the paper's memory
    constraint, Sec. 3.1, for which it gives no figures): the instance's current number
    of requests (running + queued) times a factor uniform in [lo, hi], at least 1.
    Factors below 1 make the queue wait; above 1 the cap does not bind."""
    rng = np.random.Generator(np.random.PCG64(seed))
    n_g = (np.diff(fl.act_off) + np.diff(fl.q_off)).astype(np.float64)
    return np.maximum(1, np.rint(n_g * rng.uniform(lo, hi, fl.n_inst))).astype(np.int32)
