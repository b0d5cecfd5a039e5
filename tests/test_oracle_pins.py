"""Pins of the CPU reference (oracle/) against things other than itself:
hand-worked values, a pure-Python brute force, closed forms of special cases
and invariants of the model.  No GPU, no GPU library."""
import json
import os
from types import SimpleNamespace

import numpy as np
import pytest

import oracle
from paper_2605_16867_amd import workloads
from tests import brute

HERE = os.path.dirname(os.path.abspath(__file__))


def make(coefs, inst_class, actives, queued):
    """actives / queued: per instance lists of tuples."""
    names = ("delta", "alpha", "beta", "gamma")
    coef = {k: np.array([c[i] for c in coefs], dtype=np.float64) for i, k in enumerate(names)}
    a_off = np.cumsum([0] + [len(a) for a in actives]).astype(np.int32)
    q_off = np.cumsum([0] + [len(q) for q in queued]).astype(np.int32)
    flat_a = [x for a in actives for x in a]
    flat_q = [x for q in queued for x in q]
    col = lambda rows, i: np.array([r[i] for r in rows], dtype=np.int32)
    return SimpleNamespace(
        coef=coef, inst_class=np.array(inst_class, dtype=np.int32),
        act_off=a_off, act_prompt=col(flat_a, 0), act_gen=col(flat_a, 1), act_rem=col(flat_a, 2),
        q_off=q_off, q_prompt=col(flat_q, 0), q_len=col(flat_q, 1))


def random_tiny(rng, n_inst=3, n_class=2, max_n=8, max_len=20):
    coefs = [(rng.uniform(1e-3, 1e-2), rng.uniform(0.1, 1.0), rng.uniform(0.01, 0.1),
              rng.uniform(1e-4, 1e-3)) for _ in range(n_class)]
    inst_class = [int(rng.integers(0, n_class)) for _ in range(n_inst)]
    actives = [[(int(rng.integers(1, 50)), int(rng.integers(0, 10)), int(rng.integers(1, max_len + 1)))
                for _ in range(int(rng.integers(0, max_n + 1)))] for _ in range(n_inst)]
    queued = [[(int(rng.integers(1, 50)), int(rng.integers(1, max_len + 1)))
               for _ in range(int(rng.integers(0, 4)))] for _ in range(n_inst)]
    return coefs, inst_class, actives, queued


# --------------------------------------------------------------------------- hand-worked
def test_hand_worked_example():
    """One instance, delta=0.01 alpha=1 beta=0.1 gamma=0.001.
    actives (prompt, gen, rem) = (10,0,2), (20,5,1); queued (prompt, len) = (5,3).
      q = 0.01*5 = 0.05;  contexts 10, 25, 5.
      step 1: B=3, C=40 -> 1+0.3+0.040 = 1.340 ; second active done at 0.05+1.34 = 1.39
      step 2: B=2, C=11+6=17 -> 1+0.2+0.017 = 1.217 ; first active done at 2.607
      step 3: B=1, C=7 -> 1.107 ; queued done at 3.714
    incoming c0=8, len=4: waits 0.05, prefills 0.08, then
      step 1: B=4, C=48 -> 1.448 ; step 2: B=3, C=11+6+9=26 -> 1.326
      step 3: B=2, C=7+10=17 -> 1.217 ; step 4: B=1, C=11 -> 1.111 ; T = 0.13+5.102 = 5.232
    """
    ex = json.load(open(os.path.join(HERE, "golden", "hand_example.json")))
    c = ex["class"]
    f = make([(c["delta"], c["alpha"], c["beta"], c["gamma"])], [0],
             [[(a["prompt"], a["gen"], a["rem"]) for a in ex["active"]]],
             [[(q["prompt"], q["len"]) for q in ex["queued"]]])
    sim = oracle.simulate(f)
    assert sim.q[0] == pytest.approx(ex["q"], rel=1e-12)
    assert sim.d[0] == pytest.approx(ex["d"], rel=1e-12)
    np.testing.assert_allclose(sim.act_finish, ex["active_finish"], rtol=1e-12)
    np.testing.assert_allclose(sim.q_finish, ex["queued_finish"], rtol=1e-12)
    np.testing.assert_allclose(np.diff(sim.step_table(0)), ex["steps"], rtol=1e-12)
    inc = ex["incoming"]
    assert sum(inc["steps_with_it"]) + ex["q"] + c["delta"] * inc["c0"] == pytest.approx(inc["T"], rel=1e-12)
    T = sim.pair_T([inc["c0"]], [inc["len"]])
    assert T[0, 0] == pytest.approx(inc["T"], rel=1e-12)


# --------------------------------------------------------------------------- brute force
@pytest.mark.parametrize("seed", range(8))
def test_matches_brute_force_replay(seed):
    rng = np.random.default_rng(100 + seed)
    coefs, inst_class, actives, queued = random_tiny(rng, n_inst=4)
    f = make(coefs, inst_class, actives, queued)
    sim = oracle.simulate(f)
    reqs = [(int(rng.integers(1, 60)), int(rng.integers(1, 31))) for _ in range(12)]
    # lengths beyond, equal to and below the instance's own lengths all occur (max_len 20 vs 30)
    T = sim.pair_T([r[0] for r in reqs], [r[1] for r in reqs])
    for g in range(4):
        q, first, fin = brute.replay(coefs[inst_class[g]], actives[g], queued[g])
        assert sim.q[g] == pytest.approx(q, rel=1e-12, abs=1e-15)
        assert sim.d[g] == pytest.approx(first, rel=1e-12)
        got = np.concatenate([sim.act_finish[f.act_off[g]:f.act_off[g + 1]],
                              sim.q_finish[f.q_off[g]:f.q_off[g + 1]]])
        np.testing.assert_allclose(got, np.array(fin, dtype=np.float64), rtol=1e-12)
        for r, (c0, ln) in enumerate(reqs):
            want = brute.latency_if_routed(coefs[inst_class[g]], actives[g], queued[g], c0, ln)
            assert T[r, g] == pytest.approx(want, rel=1e-11)


@pytest.mark.parametrize("seed", range(6))
def test_selection_matches_brute_force(seed):
    rng = np.random.default_rng(200 + seed)
    coefs, inst_class, actives, queued = random_tiny(rng, n_inst=4)
    f = make(coefs, inst_class, actives, queued)
    sim = oracle.simulate(f)
    n = 40
    c0 = rng.integers(1, 60, n)
    ln = rng.integers(1, 31, n)
    T = np.array([[brute.latency_if_routed(coefs[inst_class[g]], actives[g], queued[g],
                                           int(c0[r]), int(ln[r])) for g in range(4)]
                  for r in range(n)])
    d = [brute.replay(coefs[inst_class[g]], actives[g], queued[g])[1] for g in range(4)]
    # deadlines spread so that 0, some and all instances are feasible
    D = T.min(axis=1) * rng.uniform(0.5, 2.5, n)
    ex = rng.integers(-1, 4, n).astype(np.int32)
    for exclude in (None, ex):
        got = sim.route(c0, ln, D, exclude=exclude)
        for r in range(n):
            pick, fb = brute.select(list(T[r]), d, D[r], -1 if exclude is None else int(ex[r]))
            assert got.inst[r] == pick
            assert bool(got.fallback[r]) == fb
            assert got.slack[r] == pytest.approx(D[r] - T[r, pick], rel=1e-9, abs=1e-12)
    assert 0 < got.fallback.sum() < n      # both branches were taken


def test_risk_scan_matches_brute_force():
    rng = np.random.default_rng(7)
    coefs, inst_class, actives, queued = random_tiny(rng, n_inst=4, max_n=6)
    f = make(coefs, inst_class, actives, queued)
    new_rem = np.maximum(1, f.act_rem + rng.integers(-3, 4, len(f.act_rem))).astype(np.int32)
    act2 = [[(p, g, int(new_rem[f.act_off[i] + k])) for k, (p, g, _) in enumerate(a)]
            for i, a in enumerate(actives)]
    fin, d = [], []
    for g in range(4):
        _, first, fg = brute.replay(coefs[inst_class[g]], act2[g], queued[g])
        fin += fg[:len(act2[g])]
        d.append(first)
    fin = np.array(fin)
    budget = fin * rng.uniform(0.6, 1.4, len(fin))
    rs = oracle.risk_scan(f, new_rem, budget)
    np.testing.assert_allclose(rs.finish, fin, rtol=1e-12)
    np.testing.assert_array_equal(rs.flag, (fin > budget).astype(np.uint8))
    assert 0 < rs.flag.sum() < len(fin)
    i = 0
    for g in range(4):
        for (p, gen, rem) in act2[g]:
            if rs.flag[i]:
                T = [brute.latency_if_routed(coefs[inst_class[h]], act2[h], queued[h], p + gen, rem)
                     for h in range(4)]
                pick, _ = brute.select(T, d, budget[i], exclude=g)
                assert rs.target[i] == pick and pick != g
                assert rs.target_slack[i] == pytest.approx(budget[i] - T[pick], rel=1e-9, abs=1e-12)
            else:
                assert rs.target[i] == -1
            i += 1


# --------------------------------------------------------------------------- cached prefixes (Eq. 2's H)
def random_hits(rng, n_req, n_inst, c0, density=0.5):
    """CSR (hit_off, hit_inst, hit_len): each request has a cached prefix on a random subset of instances."""
    off, inst, ln = [0], [], []
    for r in range(n_req):
        gs = [g for g in range(n_inst) if rng.random() < density]
        for g in gs:
            inst.append(g)
            ln.append(int(rng.integers(1, int(c0[r]) + 1)))
        off.append(len(inst))
    return (np.array(off, np.int32), np.array(inst, np.int32), np.array(ln, np.int32))


@pytest.mark.parametrize("seed", range(5))
def test_cached_prefix_matches_brute_force_replay(seed):
    """Eq. 2: the cached part of the prompt is not prefilled.  The brute force
    replays the instance with the request appended, charging prefill for the
    uncached tokens only and carrying all tokens as context."""
    rng = np.random.default_rng(300 + seed)
    coefs, inst_class, actives, queued = random_tiny(rng, n_inst=4)
    f = make(coefs, inst_class, actives, queued)
    sim = oracle.simulate(f)
    n = 30
    c0 = rng.integers(1, 60, n)
    ln = rng.integers(1, 31, n)
    hits = random_hits(rng, n, 4, c0)
    T = sim.pair_T(c0, ln, hits=hits)
    T0 = sim.pair_T(c0, ln)
    H = np.zeros((n, 4), dtype=np.int64)
    for r in range(n):
        for k in range(hits[0][r], hits[0][r + 1]):
            H[r, hits[1][k]] = hits[2][k]
    want = np.array([[brute.latency_if_routed(coefs[inst_class[g]], actives[g], queued[g],
                                              int(c0[r]), int(ln[r]), int(H[r, g])) for g in range(4)]
                     for r in range(n)])
    np.testing.assert_allclose(T, want, rtol=1e-11)
    # closed form of the difference: exactly the prefill of the cached tokens
    delta = np.array([coefs[c][0] for c in inst_class])
    np.testing.assert_allclose(T0 - T, H * delta[None, :], rtol=1e-9, atol=1e-12)
    assert (H > 0).any() and (H == 0).any()
    # selection with hits against the brute force's Alg. 1
    d = [brute.replay(coefs[inst_class[g]], actives[g], queued[g])[1] for g in range(4)]
    D = want.min(axis=1) * rng.uniform(0.5, 2.5, n)
    ex = rng.integers(-1, 4, n).astype(np.int32)
    got = sim.route(c0, ln, D, exclude=ex, hits=hits)
    for r in range(n):
        pick, fb = brute.select(list(want[r]), d, D[r], int(ex[r]))
        assert got.inst[r] == pick and bool(got.fallback[r]) == fb
        assert got.slack[r] == pytest.approx(D[r] - want[r, pick], rel=1e-9, abs=1e-12)


def test_cached_prefix_special_cases():
    rng = np.random.default_rng(7)
    coefs, inst_class, actives, queued = random_tiny(rng, n_inst=3)
    f = make(coefs, inst_class, actives, queued)
    sim = oracle.simulate(f)
    c0, ln = np.array([40, 40, 40]), np.array([5, 5, 5])
    base = sim.pair_T(c0, ln)
    # no entries, zero-length entries: nothing changes
    empty = (np.zeros(4, np.int32), np.zeros(0, np.int32), np.zeros(0, np.int32))
    assert np.array_equal(sim.pair_T(c0, ln, hits=empty), base)
    zero = (np.array([0, 1, 2, 3], np.int32), np.array([0, 1, 2], np.int32), np.zeros(3, np.int32))
    assert np.array_equal(sim.pair_T(c0, ln, hits=zero), base)
    # a prefix longer than the request is cut to the request; the whole prompt cached = no prefill at all
    full = (np.array([0, 1, 2, 3], np.int32), np.array([0, 1, 2], np.int32), np.array([40, 1000, 39], np.int32))
    T = sim.pair_T(c0, ln, hits=full)
    delta = np.array([coefs[c][0] for c in inst_class])
    assert T[0, 0] == pytest.approx(base[0, 0] - 40 * delta[0], rel=1e-12)
    assert T[1, 1] == pytest.approx(base[1, 1] - 40 * delta[1], rel=1e-12)
    assert T[2, 2] == pytest.approx(base[2, 2] - 39 * delta[2], rel=1e-12)
    # an instance named twice: the longer prefix counts
    twice = (np.array([0, 2, 2, 2], np.int32), np.array([1, 1], np.int32), np.array([7, 30], np.int32))
    assert sim.pair_T(c0, ln, hits=twice)[0, 1] == pytest.approx(base[0, 1] - 30 * delta[1], rel=1e-12)
    # a hit can only help: it never raises a latency, and a hit on a feasible choice leaves it feasible
    hits = random_hits(rng, 3, 3, c0, density=1.0)
    assert np.all(sim.pair_T(c0, ln, hits=hits) <= base)


# --------------------------------------------------------------------------- closed forms
def tri(x):
    return x * (x - 1) / 2


def test_isolated_request_closed_form():
    """Idle instance: T = delta*P + L*(alpha+beta) + gamma*(P*L + L(L-1)/2)."""
    coefs = [(2e-5, 0.012, 2e-4, 2e-8), (5e-5, 0.025, 4e-4, 5e-8)]
    f = make(coefs, [0, 1], [[], []], [[], []])
    sim = oracle.simulate(f)
    P = np.array([1, 128, 2048, 777]); L = np.array([1, 2, 4096, 313])
    T = sim.pair_T(P, L)
    for g, (d, a, b, gm) in enumerate(coefs):
        want = d * P + L * (a + b) + gm * (P * L + tri(L))
        np.testing.assert_allclose(T[:, g], want, rtol=1e-12)
    np.testing.assert_array_equal(sim.d, [0.012, 0.025])


def test_reduces_to_linear_model_of_eq2():
    """beta = gamma = 0: every step costs alpha, so T = q_g + p_g*L_in + d_g*L_out
    with p_g = delta, d_g = alpha (Eq. 2), whatever else runs on the instance."""
    rng = np.random.default_rng(3)
    coefs = [(3e-5, 0.02, 0.0, 0.0), (7e-5, 0.05, 0.0, 0.0)]
    _, inst_class, actives, queued = random_tiny(rng, n_inst=4)
    f = make(coefs, inst_class, actives, queued)
    sim = oracle.simulate(f)
    P = rng.integers(1, 3000, 20); L = rng.integers(1, 60, 20)
    T = sim.pair_T(P, L)
    for g in range(4):
        d, a, _, _ = coefs[inst_class[g]]
        q = d * sum(p for p, _ in queued[g])
        np.testing.assert_allclose(T[:, g], q + d * P + a * L, rtol=1e-12)
        np.testing.assert_allclose(sim.act_finish[f.act_off[g]:f.act_off[g + 1]],
                                   q + a * np.array([r for _, _, r in actives[g]], dtype=float),
                                   rtol=1e-12)
        assert sim.d[g] == a
    # just-enough on a linear fleet = slowest class that still fits
    picks = sim.route(P, L, np.full(20, np.inf)).inst
    slowest = max(coefs[c][1] for c in inst_class)
    first_slowest = min(g for g in range(4) if coefs[inst_class[g]][1] == slowest)
    np.testing.assert_array_equal(picks, np.full(20, first_slowest))


def test_equal_lengths_single_segment():
    """All N requests have R steps left: the batch never changes, so every
    finish = q + R*(alpha + beta*N + gamma*S) + gamma*N*R(R-1)/2."""
    coef = (2e-5, 0.012, 2e-4, 2e-8)
    ctxs = [(100, 7), (2000, 0), (333, 150), (128, 200), (1500, 99)]
    R = 57
    f = make([coef], [0], [[(p, g, R) for p, g in ctxs]], [[(640, R)]])
    sim = oracle.simulate(f)
    N = 6
    S = sum(p + g for p, g in ctxs) + 640
    want = coef[0] * 640 + R * (coef[1] + coef[2] * N + coef[3] * S) + coef[3] * N * tri(R)
    np.testing.assert_allclose(sim.act_finish, want, rtol=1e-12)
    np.testing.assert_allclose(sim.q_finish, want, rtol=1e-12)


def test_two_segment_closed_form():
    """Two groups of lengths R1 < R2: sum of two arithmetic series."""
    a, b, g = 0.03, 5e-4, 3e-8
    R1, R2 = 10, 25
    grp1 = [(200, 5), (300, 0), (90, 44)]
    grp2 = [(1000, 1), (50, 50)]
    f = make([(1e-5, a, b, g)], [0],
             [[(p, gen, R1) for p, gen in grp1] + [(p, gen, R2) for p, gen in grp2]], [[]])
    sim = oracle.simulate(f)
    S1 = sum(p + gen for p, gen in grp1 + grp2)
    S2 = sum(p + gen for p, gen in grp2)
    F1 = R1 * (a + b * 5 + g * S1) + g * 5 * tri(R1)
    F2 = F1 + (R2 - R1) * (a + b * 2 + g * S2) + g * 2 * (tri(R2) - tri(R1))
    np.testing.assert_allclose(sim.act_finish, [F1] * 3 + [F2] * 2, rtol=1e-12)


# --------------------------------------------------------------------------- invariants
@pytest.fixture(scope="module")
def tiny():
    fl = workloads.make_fleet(workloads.spec("tiny"))
    return fl, oracle.simulate(fl)


def test_step_table_increasing_and_consistent(tiny):
    fl, sim = tiny
    for g in range(fl.n_inst):
        w = sim.step_table(g)
        assert w[0] == 0.0 and np.all(np.diff(w) > 0)
        # steps shorten only when requests leave: step time right after a departure is smaller
        a0, a1 = fl.act_off[g], fl.act_off[g + 1]
        rem = np.concatenate([fl.act_rem[a0:a1], fl.q_len[fl.q_off[g]:fl.q_off[g + 1]]])
        assert sim.smax[g] == rem.max()
        fin = np.concatenate([sim.act_finish[a0:a1], sim.q_finish[fl.q_off[g]:fl.q_off[g + 1]]])
        np.testing.assert_allclose(fin, sim.q[g] + w[rem], rtol=1e-13)
        assert np.diff(w)[0] == sim.d[g]


def test_added_load_never_helps(tiny):
    """Adding a request to an instance delays nobody less: finish times on it
    and every T(., g) are non-decreasing (all coefficients are >= 0)."""
    fl, sim = tiny
    P, L = fl.in_prompt, fl.in_len
    T0 = sim.pair_T(P, L)
    for extra_rem in (1, 50, 5000):
        g = 1
        pos = fl.act_off[g + 1]
        more = SimpleNamespace(**vars(fl))
        more.act_prompt = np.insert(fl.act_prompt, pos, 900)
        more.act_gen = np.insert(fl.act_gen, pos, 10)
        more.act_rem = np.insert(fl.act_rem, pos, extra_rem)
        more.act_off = fl.act_off.copy(); more.act_off[g + 1:] += 1
        sim1 = oracle.simulate(more)
        T1 = sim1.pair_T(P, L)
        assert np.all(T1[:, g] > T0[:, g])
        np.testing.assert_array_equal(np.delete(T1, g, axis=1), np.delete(T0, g, axis=1))
        old = np.delete(sim1.act_finish, pos)
        assert np.all(old >= sim.act_finish)
        sl = slice(fl.act_off[g], fl.act_off[g + 1])
        assert np.all(old[sl] > sim.act_finish[sl])


def test_choice_rules(tiny):
    fl, sim = tiny
    P, L = fl.in_prompt, fl.in_len
    T = sim.pair_T(P, L)
    rng = np.random.default_rng(0)
    D = T.min(axis=1) * rng.uniform(0.7, 3.0, len(P))
    got = sim.route(P, L, D)
    for r in range(len(P)):
        feas = np.flatnonzero(T[r] <= D[r])
        g = got.inst[r]
        if len(feas):
            assert g in feas and not got.fallback[r]
            assert sim.d[g] == sim.d[feas].max()
            assert g == feas[sim.d[feas] == sim.d[g]].min()
        else:
            assert got.fallback[r] and g == np.argmin(T[r])
        assert got.slack[r] == D[r] - T[r, g]
    # no deadline pressure: the instance with the slowest current step; hopeless: least-late
    np.testing.assert_array_equal(sim.route(P, L, np.full(len(P), np.inf)).inst,
                                  np.full(len(P), np.flatnonzero(sim.rank == 0)[0]))
    z = sim.route(P, L, np.zeros(len(P)))
    np.testing.assert_array_equal(z.inst, T.argmin(axis=1))
    assert z.fallback.all()
    # boundary: T == D is feasible (Alg. 1 uses <=)
    g_slow = int(np.flatnonzero(sim.rank == 0)[0])
    edge = sim.route(P, L, T[:, g_slow])
    np.testing.assert_array_equal(edge.inst, np.full(len(P), g_slow))
    assert not edge.fallback.any()
    below = sim.route(P, L, np.nextafter(T[:, g_slow], -np.inf))
    assert np.all(below.inst != g_slow)


def test_equal_d_ties_go_to_lowest_index():
    coef = (2e-5, 0.012, 2e-4, 2e-8)
    same = [(500, 10, 40), (600, 0, 80)]
    f = make([coef], [0, 0, 0], [same, same, [(100, 0, 5)]], [[], [], []])
    sim = oracle.simulate(f)
    assert sim.d[0] == sim.d[1] > sim.d[2]
    np.testing.assert_array_equal(sim.rank, [0, 1, 2])
    r = sim.route([300], [20], [1e9])
    assert r.inst[0] == 0
    r = sim.route([300], [20], [1e9], exclude=[0])
    assert r.inst[0] == 1
    r = sim.route([300], [20], [0.0])            # fallback: instance 2 is least loaded
    assert r.inst[0] == 2 and r.fallback[0]
    T = sim.pair_T([300], [20])
    assert T[0, 0] == T[0, 1]
    r = sim.route([300], [20], [0.0], exclude=[2])
    assert r.inst[0] == 0                        # equal T: lowest index


def test_order_within_instance_and_relabelling(tiny):
    fl, sim = tiny
    rng = np.random.default_rng(5)
    sh = SimpleNamespace(**vars(fl))
    perm = np.arange(len(fl.act_rem))
    for g in range(fl.n_inst):
        sl = slice(fl.act_off[g], fl.act_off[g + 1])
        perm[sl] = rng.permutation(perm[sl])
    for k in ("act_prompt", "act_gen", "act_rem"):
        setattr(sh, k, getattr(fl, k)[perm])
    sim2 = oracle.simulate(sh)
    np.testing.assert_allclose(sim2.act_finish, sim.act_finish[perm], rtol=1e-13)
    np.testing.assert_allclose(sim2.pair_T(fl.in_prompt, fl.in_len),
                               sim.pair_T(fl.in_prompt, fl.in_len), rtol=1e-13)
    # relabel instances: reverse their order
    M = fl.n_inst
    rev = SimpleNamespace(**vars(fl))
    rev.inst_class = fl.inst_class[::-1].copy()
    blocks = lambda arr, off: np.concatenate([arr[off[g]:off[g + 1]] for g in range(M - 1, -1, -1)])
    for k in ("act_prompt", "act_gen", "act_rem"):
        setattr(rev, k, blocks(getattr(fl, k), fl.act_off))
    for k in ("q_prompt", "q_len"):
        setattr(rev, k, blocks(getattr(fl, k), fl.q_off))
    rev.act_off = np.concatenate([[0], np.cumsum(np.diff(fl.act_off)[::-1])]).astype(np.int32)
    rev.q_off = np.concatenate([[0], np.cumsum(np.diff(fl.q_off)[::-1])]).astype(np.int32)
    sim3 = oracle.simulate(rev)
    D = fl.in_budget.astype(np.float64)
    a = sim.route(fl.in_prompt, fl.in_len, D)
    b = sim3.route(fl.in_prompt, fl.in_len, D)
    np.testing.assert_array_equal(b.inst, M - 1 - a.inst)
    np.testing.assert_allclose(b.slack, a.slack, rtol=1e-12)


def test_empty_fleet_pieces():
    coef = (2e-5, 0.012, 2e-4, 2e-8)
    f = make([coef], [0, 0], [[], [(100, 0, 3)]], [[], []])
    sim = oracle.simulate(f)
    assert sim.smax[0] == 0 and sim.q[0] == 0 and sim.d[0] == 0.012
    r = sim.route(np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(0))
    assert len(r.inst) == 0
    one = make([coef], [0], [[(10, 0, 2)]], [[]])
    r = oracle.simulate(one).route([5], [5], [1.0], exclude=[0])
    assert r.inst[0] == -1


# --------------------------------------------------------------------------- EMA-smoothed black-box status (Sec. 3.3, Alg. 1)
def test_ema_closed_form_and_limits():
    """q_n = (1-a)^n w_0 + a * sum_k (1-a)^(n-k) w_k for the update q <- a*w + (1-a)*q of Alg. 1."""
    from oracle import blackbox
    rng = np.random.default_rng(0)
    w = rng.uniform(0.1, 5.0, (7, 3))
    for a in (0.0, 0.2, 0.5, 0.9, 1.0):
        st = blackbox.SmoothedStatus()
        for k in range(7):
            st.observe(a, wait=w[k], decode=2 * w[k])
        n = 6
        want = (1 - a) ** n * w[0] + a * sum((1 - a) ** (n - k) * w[k] for k in range(1, 7))
        np.testing.assert_allclose(st.q, want, rtol=1e-13)
        np.testing.assert_allclose(st.d, 2 * want, rtol=1e-13)
        assert st.p is None                       # never observed
    st = blackbox.SmoothedStatus()
    for k in range(5):
        st.observe(1.0, wait=w[k])
    assert np.array_equal(st.q, w[4])             # weight 1: the latest sample
    st = blackbox.SmoothedStatus()
    for k in range(5):
        st.observe(0.3, wait=np.full(3, 2.5))
    np.testing.assert_allclose(st.q, 2.5, rtol=1e-15)   # a constant signal is its own average


def test_eq2_with_smoothed_status_by_hand():
    from oracle import blackbox
    st = blackbox.SmoothedStatus(q=np.array([1.0, 0.0]), p=np.array([0.01, 0.02]), d=np.array([0.1, 0.05]))
    T = blackbox.eq2_latency(st, [100], [50], H=np.array([[20, 0]]))
    # 1 + 0.01*80 + 0.1*50 = 6.8 ;  0 + 0.02*100 + 0.05*50 = 4.5
    np.testing.assert_allclose(T, [[6.8, 4.5]], rtol=1e-14)


@pytest.mark.parametrize("seed", range(4))
def test_numpy_selection_matches_brute_force(seed):
    from oracle import blackbox
    rng = np.random.default_rng(400 + seed)
    n, M = 60, 7
    T = rng.uniform(1, 10, (n, M))
    T[:, 3] = T[:, 1]                              # exact ties in T
    d = rng.uniform(0.1, 1.0, M)
    d[5] = d[2]                                    # and in d
    D = rng.uniform(0.5, 12, n)
    ex = rng.integers(-1, M, n)
    for exclude in (None, ex):
        inst, slack, fb, Tc = blackbox.select(T, d, D, exclude)
        for r in range(n):
            pick, fall = brute.select(list(T[r]), list(d), D[r], -1 if exclude is None else int(ex[r]))
            assert inst[r] == pick and bool(fb[r]) == fall
            assert slack[r] == pytest.approx(D[r] - T[r, pick])
    inst, _, _, _ = blackbox.select(T[:, :1], d[:1], D, np.zeros(n, dtype=np.int64))
    assert np.all(inst == -1)                      # the only instance is barred


def test_blend_end_points_and_midpoint(tiny):
    from oracle import blackbox
    fl, sim = tiny
    M = fl.n_inst
    rng = np.random.default_rng(5)
    st = blackbox.SmoothedStatus(q=rng.uniform(0, 2, M), p=rng.uniform(1e-5, 1e-3, M), d=rng.uniform(0.01, 0.2, M))
    c0, ln = fl.in_prompt, fl.in_len
    hits = random_hits(rng, len(c0), M, c0)
    D = fl.in_budget.astype(np.float64)
    zero = blackbox.BlendedFleet(sim, fl, st, 0.0)
    np.testing.assert_array_equal(zero.pair_T(c0, ln, hits=hits), sim.pair_T(c0, ln, hits=hits))
    np.testing.assert_array_equal(zero.d, sim.d)
    np.testing.assert_array_equal(zero.act_finish, sim.act_finish)
    assert np.array_equal(zero.route(c0, ln, D, hits=hits).inst, sim.route(c0, ln, D, hits=hits).inst)
    one = blackbox.BlendedFleet(sim, fl, st, 1.0)
    H = blackbox.dense_hits(hits, len(c0), M, c0)
    np.testing.assert_allclose(one.pair_T(c0, ln, hits=hits), blackbox.eq2_latency(st, c0, ln, H), rtol=1e-15)
    assert np.array_equal(np.argsort(one.rank), np.lexsort((np.arange(M), -st.d)))
    inst_a = np.repeat(np.arange(M), np.diff(fl.act_off))
    np.testing.assert_allclose(one.act_finish, st.d[inst_a] * fl.act_rem, rtol=1e-15)
    half = blackbox.BlendedFleet(sim, fl, st, 0.5)
    np.testing.assert_allclose(half.pair_T(c0, ln), 0.5 * (sim.pair_T(c0, ln) + one.pair_T(c0, ln)), rtol=1e-14)
    np.testing.assert_allclose(half.q_finish, 0.5 * (sim.q_finish + one.q_finish), rtol=1e-14)


# --------------------------------------------------------------------------- routing with status feedback (Alg. 1, request after request)
@pytest.mark.parametrize("seed", range(4))
def test_feedback_routing_matches_brute_force_sequence(seed):
    """chunk = 1 against a pure-Python proxy: every request is scored by replaying each instance
    with it appended, Alg. 1 picks, and the request is really appended to the instance it got."""
    rng = np.random.default_rng(500 + seed)
    coefs, inst_class, actives, queued = random_tiny(rng, n_inst=4)
    f = make(coefs, inst_class, actives, queued)
    n = 25
    c0 = rng.integers(1, 60, n)
    ln = rng.integers(1, 31, n)
    solo = np.array([brute.latency_if_routed(coefs[0], [], [], int(c0[r]), int(ln[r])) for r in range(n)])
    D = solo * rng.uniform(1.0, 12.0, n)
    ex = rng.integers(-1, 4, n).astype(np.int32)
    got, _ = oracle.route_with_feedback(f, c0, ln, D, chunk=1, exclude=ex)
    queues = [list(q) for q in queued]
    for r in range(n):
        T = [brute.latency_if_routed(coefs[inst_class[g]], actives[g], queues[g], int(c0[r]), int(ln[r]))
             for g in range(4)]
        d = [brute.replay(coefs[inst_class[g]], actives[g], queues[g])[1] for g in range(4)]
        pick, fb = brute.select(T, d, D[r], int(ex[r]))
        assert got.inst[r] == pick and bool(got.fallback[r]) == fb
        assert got.slack[r] == pytest.approx(D[r] - T[pick], rel=1e-9, abs=1e-12)
        queues[pick].append((int(c0[r]), int(ln[r])))
    snap = oracle.simulate(f).route(c0, ln, D, exclude=ex)
    assert not np.allclose(snap.slack, got.slack)  # later requests do see the earlier ones


def test_feedback_routing_limits(tiny):
    fl, sim = tiny
    D = fl.in_budget.astype(np.float64) * 3
    n = len(fl.in_prompt)
    # one chunk holding the whole batch is the snapshot decision
    whole, seen = oracle.route_with_feedback(fl, fl.in_prompt, fl.in_len, D, chunk=n)
    snap = sim.route(fl.in_prompt, fl.in_len, D)
    assert np.array_equal(whole.inst, snap.inst) and np.array_equal(whole.slack, snap.slack) and len(seen) == 1
    # what one routed request adds to its instance: its prefill to q_g, beta + gamma*prompt to d_g
    one, seen = oracle.route_with_feedback(fl, fl.in_prompt[:2], fl.in_len[:2], D[:2], chunk=1)
    g = int(one.inst[0])
    c = int(fl.inst_class[g])
    extended = oracle.simulate(oracle._Extended(fl, [[(int(fl.in_prompt[0]), int(fl.in_len[0]))] if i == g else []
                                                     for i in range(fl.n_inst)]))
    assert extended.q[g] == pytest.approx(sim.q[g] + fl.coef["delta"][c] * fl.in_prompt[0], rel=1e-12)
    assert extended.d[g] == pytest.approx(sim.d[g] + fl.coef["beta"][c] + fl.coef["gamma"][c] * fl.in_prompt[0], rel=1e-12)
    others = np.arange(fl.n_inst) != g
    assert np.array_equal(extended.q[others], sim.q[others]) and np.array_equal(extended.d[others], sim.d[others])
    np.testing.assert_array_equal(seen[1][1], extended.pair_T(fl.in_prompt[1:2], fl.in_len[1:2]))
    # following someone else's commits: the second request sees the state those commits made
    forced = np.array([(g + 1) % fl.n_inst, 0], dtype=np.int32)
    _, seen_f = oracle.route_with_feedback(fl, fl.in_prompt[:2], fl.in_len[:2], D[:2], chunk=1, follow=forced)
    assert not np.array_equal(seen_f[1][1], seen[1][1])


# --------------------------------------------------------------------------- batch cap (Sec. 3.1's memory bound on concurrency)
@pytest.mark.parametrize("seed", range(8))
def test_batch_cap_matches_brute_force_replay(seed):
    rng = np.random.default_rng(600 + seed)
    coefs, inst_class, actives, queued = random_tiny(rng, n_inst=4, max_n=8)
    # more queued requests than the default helper makes, so that the queue really waits
    queued = [[(int(rng.integers(1, 50)), int(rng.integers(1, 21))) for _ in range(int(rng.integers(0, 7)))]
              for _ in range(4)]
    f = make(coefs, inst_class, actives, queued)
    f.batch_cap = np.array([int(rng.integers(1, len(actives[g]) + len(queued[g]) + 3)) for g in range(4)], np.int32)
    sim = oracle.simulate(f)
    reqs = [(int(rng.integers(1, 60)), int(rng.integers(1, 31)), int(rng.integers(0, 2))) for _ in range(10)]
    hits = (np.arange(11, dtype=np.int32) * 4, np.tile(np.arange(4, dtype=np.int32), 10),
            np.repeat(np.array([r[2] * (r[0] // 2) for r in reqs], dtype=np.int32), 4))
    T = sim.pair_T([r[0] for r in reqs], [r[1] for r in reqs], hits=hits)
    waited = False
    for g in range(4):
        co, cap = coefs[inst_class[g]], int(f.batch_cap[g])
        fin, admitted, first = brute.replay_capped(co, actives[g], queued[g], cap)
        got = np.concatenate([sim.act_finish[f.act_off[g]:f.act_off[g + 1]],
                              sim.q_finish[f.q_off[g]:f.q_off[g + 1]]])
        np.testing.assert_allclose(got, np.array(fin, dtype=np.float64), rtol=1e-12)
        assert sim.d[g] == pytest.approx(co[1] if first is None else first, rel=1e-12)
        waited |= any(a > 0 for a in admitted)
        for r, (c0, ln, hit) in enumerate(reqs):
            want, when = brute.latency_if_routed_capped(co, actives[g], queued[g], cap, c0, ln, hit * (c0 // 2))
            assert T[r, g] == pytest.approx(want, rel=1e-11)
            assert sim.q[g] == pytest.approx(when, rel=1e-12, abs=1e-15)
    assert waited or seed > 3


def test_batch_cap_one_is_a_single_server_queue():
    """cap = 1: requests run alone, one after the other; every finish time is a sum of solo latencies."""
    co = (0.01, 1.0, 0.1, 0.001)
    solo = lambda ctx, L: L * (co[1] + co[2]) + co[3] * (ctx * L + L * (L - 1) / 2)
    f = make([co], [0], [[(10, 2, 3)]], [[(5, 4), (7, 2), (3, 6)]])
    f.batch_cap = np.array([1], np.int32)
    sim = oracle.simulate(f)
    t = solo(12, 3)
    assert sim.act_finish[0] == pytest.approx(t, rel=1e-13)
    for j, (P, L) in enumerate([(5, 4), (7, 2), (3, 6)]):
        t += co[0] * P + solo(P, L)
        assert sim.q_finish[j] == pytest.approx(t, rel=1e-13)
    assert sim.q[0] == pytest.approx(t, rel=1e-13)          # a newcomer is admitted when the last one is done
    assert sim.d[0] == pytest.approx(co[1] + co[2] + co[3] * 12, rel=1e-13)
    T = sim.pair_T([8], [5])
    assert T[0, 0] == pytest.approx(t + co[0] * 8 + solo(8, 5), rel=1e-13)


def test_batch_cap_limits(tiny):
    fl, sim = tiny
    from copy import copy
    n_g = np.diff(fl.act_off) + np.diff(fl.q_off)
    roomy = copy(fl)
    roomy.batch_cap = (n_g + 1).astype(np.int32)           # room for everybody and a newcomer: no cap at all
    s2 = oracle.simulate(roomy)
    assert np.array_equal(s2.act_finish, sim.act_finish) and np.array_equal(s2.q, sim.q) and np.array_equal(s2.d, sim.d)
    assert np.array_equal(s2.pair_T(fl.in_prompt, fl.in_len), sim.pair_T(fl.in_prompt, fl.in_len))
    # a tighter cap never lets a newcomer in earlier
    prev = sim.q
    for shrink in (0, 4, 16, 40):
        capped = copy(fl)
        capped.batch_cap = np.maximum(1, n_g - shrink).astype(np.int32)
        q = oracle.simulate(capped).q
        assert np.all(q >= prev - 1e-12)
        prev = q
    # exactly full: the newcomer waits for the first departure
    full = copy(fl)
    full.batch_cap = n_g.astype(np.int32)
    sf = oracle.simulate(full)
    first_departure = np.array([min(np.concatenate([sf.act_finish[fl.act_off[g]:fl.act_off[g + 1]],
                                                    sf.q_finish[fl.q_off[g]:fl.q_off[g + 1]]])) for g in range(fl.n_inst)])
    np.testing.assert_allclose(sf.q, first_departure, rtol=1e-13)
