"""GPU parity on the degenerate and extreme inputs of the path, and the error
behaviour of the C interface.  Custom fleets are plain namespaces with the
array attributes of workloads.Fleet."""
from types import SimpleNamespace

import numpy as np
import pytest

import oracle
from paper_2605_16867_amd import binding, workloads
from tests import parity
from tests.fleets import CLASSES, fleet, rand_entries, solo, two_equal_minima_in_one_lane

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["auto", "grouped"])
def scoring_layout(request):
    """Every test here runs twice: with the library choosing how a batch is scored
    (few pairs: a thread per pair; many: grouped by length), and always grouped."""
    parity.SMALL_BATCH_PAIRS = None if request.param == "auto" else 0
    yield
    parity.SMALL_BATCH_PAIRS = None


def test_empty_and_queue_only_instances():
    rng = np.random.default_rng(0)
    acts = [rand_entries(rng, 70), np.zeros((0, 3)), np.zeros((0, 3)), rand_entries(rng, 1),
            rand_entries(rng, 300)]
    queued = [[], [], [(500, 40), (900, 7)], [], [(128, 4096)]]
    inc = np.stack([rng.integers(128, 2049, 500), np.clip(np.rint(rng.lognormal(5, 1, 500)), 1, 4096)], 1)
    bud = rng.uniform(1.0, 8.0, 500) * solo(inc[:, 0], inc[:, 1])
    fl = fleet([0, 1, 2, 0, 1], acts, queued, inc, bud)
    sim = oracle.simulate(fl)
    fl.act_budget = (sim.act_finish * rng.uniform(0.5, 1.5, len(sim.act_finish))).astype(np.float32)
    rep = parity.run_and_check(fl)
    assert rep["route_n"] == 500 and 0 < rep["flag_frac"] < 1


def test_all_instances_empty():
    inc = [(100, 1), (2048, 4096), (1, 1)]
    fl = fleet([0, 1, 1, 2], [[], [], [], []], [[], [], [], []], inc,
               [solo(100, 1), solo(2048, 4096) * 3, 0.0])
    parity.run_and_check(fl)


def test_identical_instances_tie_to_lowest_index():
    rng = np.random.default_rng(1)
    e = rand_entries(rng, 100)
    inc = np.stack([rng.integers(128, 2049, 64), rng.integers(1, 2000, 64)], 1)
    # huge budgets: all feasible, equal d_g -> instance 0; zero budgets: fallback, equal T -> instance 0
    for scale in (1e6, 0.0):
        fl = fleet([1, 1, 1, 1, 1, 1], [e] * 6, [[]] * 6, inc, scale * solo(inc[:, 0], inc[:, 1]))
        parity.run_and_check(fl)
    d = parity.upload(fl)
    import torch
    h = parity.make_handle(fl)
    fin = torch.empty(len(fl.act_prompt), dtype=torch.float32, device="cuda:0")
    h.gr_build_status(d["act_off"], d["act_prompt"], d["act_gen"], d["act_rem"], d["q_off"],
                      d["q_prompt"], d["q_len"], fin)
    inst = torch.empty(64, dtype=torch.int32, device="cuda:0")
    sl = torch.empty(64, dtype=torch.float32, device="cuda:0")
    ex = torch.zeros(64, dtype=torch.int32, device="cuda:0")
    h.gr_score_route(d["in_prompt"], d["in_len"], d["in_budget"], inst, sl, exclude_inst=ex)
    torch.cuda.synchronize()
    assert (inst.cpu().numpy() == 1).all()       # instance 0 excluded: next lowest index
    h.close()


def test_equal_minima_at_two_positions_of_one_lane_go_to_the_lowest_index():
    """Two different instances, 64 positions apart in capability order (the same lane of the
    scoring wave), with the same latency bit for bit and smaller than everybody else's: the
    fallback choice is the lower index, whichever comes first in capability order."""
    for between in (63, 127, 191):
        fl = two_equal_minima_in_one_lane(between)
        rep = parity.run_and_check(fl)
        assert rep["route_exact_ties"] == 48 and rep["route_ambiguous"] == 0 and rep["route_differ"] == 0
        # the same with either of the two barred: the other one
        M = len(fl.inst_class)
        for ex in (0, M - 1):
            rep = parity.run_and_check(fl, exclude=np.full(len(fl.in_prompt), ex, dtype=np.int32))
            assert rep["route_ambiguous"] == 0 and rep["route_differ"] == 0


def test_single_instance_and_everything_excluded():
    rng = np.random.default_rng(2)
    inc = [(300, 50), (700, 10)]
    fl = fleet([0], [rand_entries(rng, 10)], [[]], inc, [1e9, 0.0])
    parity.run_and_check(fl)
    rep = parity.run_and_check(fl, exclude=np.array([0, 0], dtype=np.int32))
    assert rep["route_n"] == 2
    # a risk scan on one instance has no other instance to go to: targets are -1
    fl.act_budget = np.zeros(10, dtype=np.float32)
    parity.run_and_check(fl)


def test_exclusion_of_the_would_be_choice():
    """Excluding exactly the instance Alg. 1 would have picked forces the second pass."""
    fl = workloads.make_fleet(workloads.spec("mid", slo_scale=2.0, seed=11))
    sim = oracle.simulate(fl)
    first = sim.route(fl.in_prompt, fl.in_len, fl.in_budget.astype(np.float64))
    rep = parity.run_and_check(fl, exclude=first.inst)
    assert 0.05 < rep["route_feasible_frac"] < 1.0


def test_one_length_many_requests_and_all_lengths_distinct():
    rng = np.random.default_rng(3)
    acts = [rand_entries(rng, int(n)) for n in rng.integers(1, 400, 70)]
    cls = rng.integers(0, 3, 70)
    n = 5000
    same = np.stack([rng.integers(128, 2049, n), np.full(n, 137)], 1)
    fl = fleet(cls, acts, [[]] * 70, same, rng.uniform(0.5, 30, n) * solo(same[:, 0], same[:, 1]))
    parity.run_and_check(fl)
    distinct = np.stack([rng.integers(128, 2049, 4096), rng.permutation(4096) + 1], 1)
    fl = fleet(cls, acts, [[]] * 70, distinct, rng.uniform(0.5, 30, 4096) * solo(distinct[:, 0], distinct[:, 1]))
    parity.run_and_check(fl)


def test_every_tile_filling():
    """Lengths with 1 .. 70 requests each: tiles of every filling (the main pass
    runs over the requests a tile has, in eights; small tiles and full tiles
    take their minima differently), with deadlines on both sides of feasible."""
    rng = np.random.default_rng(11)
    acts = [rand_entries(rng, int(n)) for n in rng.integers(0, 120, 200)]
    cls = rng.integers(0, 3, 200)
    counts = [1, 2, 3, 4, 5, 7, 8, 9, 12, 13, 15, 16, 17, 20, 23, 24, 25, 28, 31, 32, 33, 40, 48, 63, 64, 65, 70]
    lens = np.repeat(rng.permutation(3000)[:len(counts)] + 1, counts)
    inc = np.stack([rng.integers(128, 2049, len(lens)), lens], 1)
    for scale in (0.5, 3.0, 30.0):
        fl = fleet(cls, acts, [[]] * 200, inc, rng.uniform(0.5, 2, len(lens)) * scale * solo(inc[:, 0], inc[:, 1]))
        sim = oracle.simulate(fl)
        fl.act_budget = (sim.act_finish * rng.uniform(0.5, 1.5, len(sim.act_finish))).astype(np.float32)
        parity.run_and_check(fl)


@pytest.mark.parametrize("n_inst", [6208, 8320])
def test_wide_fleets(n_inst):
    """More instances than the scoring kernel's small-workgroup variant keeps
    coefficient pairs for in LDS (larger workgroups, then global memory)."""
    rng = np.random.default_rng(n_inst)
    acts = [rand_entries(rng, int(n)) for n in rng.integers(0, 7, n_inst)]
    cls = rng.integers(0, 3, n_inst)
    inc = np.stack([rng.integers(128, 2049, 300), rng.choice([3, 50, 51, 400, 2000], 300)], 1)
    fl = fleet(cls, acts, [[]] * n_inst, inc, rng.uniform(0.8, 3, 300) * solo(inc[:, 0], inc[:, 1]))
    sim = oracle.simulate(fl)
    fl.act_budget = (sim.act_finish * rng.uniform(0.5, 1.5, len(sim.act_finish))).astype(np.float32)
    rep = parity.run_and_check(fl)
    assert rep["finish_rel_err"] < 1e-6


@pytest.mark.parametrize("n_inst,most", [(1024, 200), (1025, 200), (2048, 200), (2049, 200), (1024, 64), (500, 2048)])
def test_instances_that_share_waves(n_inst, most):
    """The status build gives an instance one, two or four waves depending on the fleet's size
    (four up to 1 024 instances, two up to 2 048) and on how many sort words a lane holds: the
    sizes either side of each switch, instances that fill their waves exactly, idle ones, queues
    that straddle the waves, and a routing with feedback on top (the rebuilds read the lists of
    routed requests the same way)."""
    rng = np.random.default_rng(n_inst + most)
    occ = rng.integers(0, most + 1, n_inst)
    occ[:4] = [most, most - 1, 0, 1]
    qn = np.minimum(rng.integers(0, 9, n_inst) * (rng.random(n_inst) > 0.5), most - occ)
    acts = [rand_entries(rng, int(n)) for n in occ]
    queued = [[(int(p), int(l)) for p, l in zip(rng.integers(1, 3000, n), rng.integers(1, 400, n))] for n in qn]
    cls = rng.integers(0, 3, n_inst)
    inc = np.stack([rng.integers(128, 2049, 200), rng.choice([3, 50, 51, 400, 2000], 200)], 1)
    fl = fleet(cls, acts, queued, inc, rng.uniform(0.8, 3, 200) * solo(inc[:, 0], inc[:, 1]))
    fl.n_inst = n_inst
    sim = oracle.simulate(fl)
    fl.act_budget = (sim.act_finish * rng.uniform(0.5, 1.5, len(sim.act_finish))).astype(np.float32)
    fl.act_rem_refreshed = np.clip(np.rint(fl.act_rem * rng.lognormal(0, 0.4, len(fl.act_rem))), 1, 4096).astype(np.int32)
    rep = parity.run_and_check(fl)
    assert rep["finish_rel_err"] < 1e-6
    if most < 2048:
        parity.run_feedback_and_check(fl, chunk=16, n_req=48)


def test_batch_cap_departures_in_groups():
    """Full batches whose departures come in groups of equal lengths: the one that
    makes room for a newcomer takes its whole group along (down to an empty batch),
    with and without a queue in front."""
    rng = np.random.default_rng(17)
    def ent(lens):
        lens = np.asarray(lens)
        return np.stack([rng.integers(128, 2049, len(lens)), rng.integers(0, 201, len(lens)), lens], 1)
    acts = [ent([50] * 20), ent([5] * 4 + [9] * 4 + [30] * 4), ent([7, 7, 7, 12, 12, 40]), ent([3] * 6),
            ent(rng.integers(1, 60, 300)), np.zeros((0, 3))]
    queued = [[], [], [(500, 20), (300, 7), (900, 7), (128, 33), (700, 5)], [(400, 3), (400, 3)],
              [(int(p), int(l)) for p, l in zip(rng.integers(128, 2049, 40), rng.integers(1, 60, 40))], [(256, 9)]]
    inc = np.stack([rng.integers(128, 2049, 200), rng.integers(1, 120, 200)], 1)
    for caps in ([10, 7, 4, 2, 200, 1], [1, 12, 6, 6, 340, 3], [20, 1, 1, 8, 100, 1]):
        fl = fleet([0, 1, 2, 0, 1, 2], acts, queued, inc, rng.uniform(0.5, 40, 200) * solo(inc[:, 0], inc[:, 1]))
        fl.batch_cap = np.asarray(caps, dtype=np.int32)
        sim = oracle.simulate(fl)
        fl.act_budget = (sim.act_finish * rng.uniform(0.7, 1.3, len(sim.act_finish))).astype(np.float32)
        parity.run_and_check(fl)


def test_special_budgets():
    rng = np.random.default_rng(4)
    acts = [rand_entries(rng, 200) for _ in range(9)]
    inc = np.stack([rng.integers(128, 2049, 8), rng.integers(1, 4097, 8)], 1)
    bud = np.array([np.inf, -np.inf, -5.0, 0.0, np.nan, 3.4e38, 1e-30, 50.0], dtype=np.float32)
    fl = fleet(rng.integers(0, 3, 9), acts, [[]] * 9, inc, bud)
    fl.act_budget = rng.choice(np.array([np.inf, -np.inf, -1.0, 0.0, 1e3], dtype=np.float32), 1800)
    # NaN budget: never feasible on either side; the classifier treats NaN like "nothing feasible"
    parity.run_and_check(fl)


def test_extreme_sizes():
    """Longest allowed lengths, most entries per instance, long prompts."""
    rng = np.random.default_rng(5)
    L = 32767
    big = np.stack([rng.integers(1, 32769, 2048), rng.integers(0, 201, 2048),
                    rng.choice([1, 2, L - 1, L], 2048)], 1)
    mid = np.stack([rng.integers(1, 32769, 2047), rng.integers(0, 201, 2047),
                    rng.integers(1, L + 1, 2047)], 1)
    inc = np.stack([rng.integers(1, 32769, 300), rng.choice([1, L, L - 1, 5000], 300)], 1)
    fl = fleet([0, 2, 1], [big, mid, np.zeros((0, 3))], [[], [(32768, L)], []], inc,
               rng.uniform(0.5, 3000, 300) * solo(inc[:, 0], inc[:, 1]), max_len=L)
    sim = oracle.simulate(fl)
    fl.act_budget = (sim.act_finish * rng.uniform(0.9, 1.1, len(sim.act_finish))).astype(np.float32)
    rep = parity.run_and_check(fl)
    assert rep["finish_rel_err"] < 1e-6


def test_error_codes_and_contract_violations():
    import torch
    dev = "cuda:0"
    co = [[1e-5], [0.01], [1e-4], [1e-8]]
    with pytest.raises(binding.GoodRouteError) as e:
        binding.Fleet(*co, [0], 4097, 4096, 10)
    assert e.value.code == -2
    with pytest.raises(binding.GoodRouteError) as e:
        binding.Fleet(*co, [0], 16, 40000, 10)
    assert e.value.code == -2
    with pytest.raises(binding.GoodRouteError) as e:
        binding.Fleet(*co, [1], 16, 100, 10)          # class id out of range
    assert e.value.code == -1
    with pytest.raises(binding.GoodRouteError) as e:
        binding.Fleet([[-1e-5]], co[1], co[2], co[3], [0], 16, 100, 10)
    assert e.value.code == -1

    h = binding.Fleet(*co, [0, 0], 4, 100, 8)
    i32 = lambda a: torch.tensor(a, dtype=torch.int32, device=dev)
    f32 = lambda n: torch.zeros(n, dtype=torch.float32, device=dev)
    req = (i32([10] * 8), i32([5] * 8), f32(8), torch.zeros(8, dtype=torch.int32, device=dev), f32(8))
    with pytest.raises(binding.GoodRouteError) as e:
        h.gr_score_route(*req)
    assert e.value.code == -4                         # no status yet
    # 3 actives on instance 0 and 5 on instance 1 (one too many), a length beyond max_len
    off, z = i32([0, 3, 8]), i32([0, 0, 0])
    fin = f32(8)
    h.gr_build_status(off, i32([10] * 8), i32([0] * 8), i32([5, 500, 7, 1, 2, 3, 4, 9]),
                      z, i32([]), i32([]), fin)
    assert h.gr_device_status() == 3                  # length clamped + entries dropped, no fault
    big = (i32([10] * 9), i32([5] * 9), f32(9), torch.zeros(9, dtype=torch.int32, device=dev), f32(9))
    with pytest.raises(binding.GoodRouteError) as e:
        h.gr_score_route(*big)
    assert e.value.code == -2
    h.gr_score_route(*req)
    torch.cuda.synchronize()
    h.close()
    h.close()                                         # idempotent


def test_zero_requests_and_zero_actives():
    import torch
    dev = "cuda:0"
    h = binding.Fleet([1e-5], [0.01], [1e-4], [1e-8], [0, 0, 0], 8, 100, 8)
    e32 = torch.zeros(0, dtype=torch.int32, device=dev)
    ef = torch.zeros(0, dtype=torch.float32, device=dev)
    eu = torch.zeros(0, dtype=torch.uint8, device=dev)
    off = torch.zeros(4, dtype=torch.int32, device=dev)
    d = torch.zeros(3, dtype=torch.float64, device=dev)
    rk = torch.full((3,), -1, dtype=torch.int32, device=dev)
    h.gr_build_status(off, e32, e32, e32, off, e32, e32, ef, None, d, rk)
    h.gr_score_route(e32, e32, ef, e32, ef)
    n = torch.full((1,), 7, dtype=torch.int32, device=dev)
    h.gr_risk_scan(off, e32, e32, e32, off, e32, e32, ef, eu, ef, e32, ef, n)
    torch.cuda.synchronize()
    assert d.cpu().tolist() == [0.01] * 3 and rk.cpu().tolist() == [0, 1, 2] and n.item() == 0
    inst = torch.full((2,), -9, dtype=torch.int32, device=dev)
    sl = torch.zeros(2, dtype=torch.float32, device=dev)
    h.gr_score_route(torch.tensor([7, 9], dtype=torch.int32, device=dev),
                     torch.tensor([3, 100], dtype=torch.int32, device=dev),
                     torch.tensor([1e9, 0.0], dtype=torch.float32, device=dev), inst, sl)
    torch.cuda.synchronize()
    assert inst.cpu().tolist() == [0, 0]
    want = 1e9 - (1e-5 * 7 + 3 * (0.01 + 1e-4) + 1e-8 * (7 * 3 + 3))
    assert abs(sl[0].item() - want) <= 1e-4 * 1e9
    h.close()


def test_cached_prefix_edge_cases():
    """Empty hit lists, zero-length and over-long prefixes, an instance named twice, ids out of
    range, a prefix on the excluded instance, a prefix that makes an infeasible instance feasible."""
    rng = np.random.default_rng(12)
    M = 9
    acts = [rand_entries(rng, int(n)) for n in rng.integers(50, 300, M)]
    n = 600
    inc = np.stack([rng.integers(128, 2049, n), rng.integers(1, 4097, n)], 1)
    fl = fleet(rng.integers(0, 3, M), acts, [[]] * M, inc, rng.uniform(0.8, 6, n) * solo(inc[:, 0], inc[:, 1]))
    off, inst, ln = [0], [], []
    for r in range(n):
        kind = r % 6
        if kind == 1:
            inst += [r % M]; ln += [0]
        elif kind == 2:
            inst += [r % M]; ln += [10 ** 6]
        elif kind == 3:
            inst += [r % M, r % M]; ln += [5, int(inc[r, 0])]
        elif kind == 4:
            inst += [-3, M, (r + 1) % M]; ln += [50, 50, 50]
        elif kind == 5:
            inst += list(range(M)); ln += [int(x) for x in rng.integers(1, inc[r, 0] + 1, M)]
        off.append(len(inst))
    hits = (np.array(off, np.int32), np.array(inst, np.int32), np.array(ln, np.int32))
    ex = np.where(np.arange(n) % 2 == 0, -1, np.arange(n) % M).astype(np.int32)
    # the reference ignores ids out of range as well: it never asks for them
    parity.run_and_check(fl, hits=hits)
    parity.run_and_check(fl, exclude=ex, hits=hits)
    none = (np.zeros(n + 1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.int32))
    rep = parity.run_and_check(fl, hits=none)
    assert rep["route_moved_by_hits"] == 0


def test_cached_prefixes_decide_when_prefill_dominates():
    """Slow prefill (delta 200x the usual), short decodes: most of T is prefill, so a cached
    prefix changes which instances are feasible and which is the least late."""
    rng = np.random.default_rng(13)
    slow_prefill = [(4e-3, 0.012, 2e-4, 2e-8), (1e-2, 0.025, 4e-4, 5e-8), (2.4e-2, 0.05, 8e-4, 1e-7)]
    M = 24
    acts = [rand_entries(rng, int(k), max_len=64) for k in rng.integers(5, 60, M)]
    n = 3000
    inc = np.stack([rng.integers(128, 2049, n), rng.integers(1, 33, n)], 1)
    fl = fleet(rng.integers(0, 3, M), acts, [[]] * M, inc,
               rng.uniform(0.5, 3.0, n) * solo(inc[:, 0], inc[:, 1], slow_prefill[0]), classes=slow_prefill)
    hits = workloads.cached_prefixes(SimpleNamespace(in_prompt=fl.in_prompt, n_inst=M), mean_hits=3.0, seed=5)
    rep = parity.run_and_check(fl, hits=hits)
    assert rep["route_moved_by_hits"] > n // 10
    ex = rng.integers(-1, M, n).astype(np.int32)
    rep = parity.run_and_check(fl, exclude=ex, hits=hits)
    assert rep["route_moved_by_hits"] > n // 10


def _random_case(rng, larger=False):
    """A small fleet with everything drawn at random: size, classes and their
    coefficients, occupancy (idle instances included), queues, the mix of
    lengths of the incoming batch, deadline scale, and which of the optional
    inputs (exclusions, cached prefixes, observed status + blend, batch caps)
    are present.  ``larger``: up to 2 050 instances, up to 2 040 held requests
    per instance (every sort width), up to 9 000 incoming requests."""
    if larger:
        return _random_larger_case(rng)
    M = int(rng.choice([1, 2, 3, 17, 64, 65, 130, 300]))
    n_class = int(rng.integers(1, 6))
    classes = [(2e-5 * f, 0.012 * f, 2e-4 * f, 2e-8 * f) for f in rng.uniform(0.5, 6.0, n_class)]
    max_len = int(rng.choice([64, 4096, 32767]))
    occ = rng.integers(0, 90, M) * (rng.random(M) > 0.15)
    acts = [np.stack([rng.integers(1, 3000, n), rng.integers(0, 300, n),
                      np.clip(np.rint(rng.lognormal(rng.uniform(1, 6), 1, n)), 1, max_len)], 1) if n else np.zeros((0, 3))
            for n in occ]
    queued = [[(int(p), int(l)) for p, l in zip(rng.integers(1, 3000, n), rng.integers(1, min(max_len, 500) + 1, n))]
              for n in rng.integers(0, 6, M) * (rng.random(M) > 0.5)]
    R = int(rng.choice([1, 5, 33, 200, 700]))
    kinds = int(rng.choice([1, 3, 40, R]))
    pool = np.clip(np.rint(rng.lognormal(rng.uniform(1, 6), 1.2, kinds)), 1, max_len)
    inc = np.stack([rng.integers(1, 4000, R), rng.choice(pool, R)], 1)
    c0 = classes[0]
    bud = rng.uniform(0.3, 3, R) * float(rng.choice([0.5, 3, 20, 300])) * solo(inc[:, 0], inc[:, 1], c0)
    special = rng.random(R)
    bud = np.where(special < 0.03, 0.0, np.where(special < 0.06, np.inf, np.where(special < 0.08, -1.0, bud)))
    return _finish_random_case(rng, fleet(rng.integers(0, n_class, M), acts, queued, inc, bud, classes=classes,
                                          max_len=max_len))


def _random_larger_case(rng):
    M = int(rng.choice([63, 64, 65, 127, 129, 256, 257, 511, 1000, 1025, 2050]))
    n_class = int(rng.integers(1, 7))
    classes = [(2e-5 * f, 0.012 * f, 2e-4 * f, 2e-8 * f) for f in rng.uniform(0.5, 6.0, n_class)]
    max_len = int(rng.choice([64, 4096, 32767]))
    top = int(rng.choice([10, 64, 65, 129, 300, 513, 1100, 2040] if M <= 300 else [10, 70, 130, 260]))
    occ = rng.integers(0, top + 1, M) * (rng.random(M) > 0.1)
    acts = [np.stack([rng.integers(1, 3000, n), rng.integers(0, 300, n),
                      np.clip(np.rint(rng.lognormal(rng.uniform(1, 6), 1, n)), 1, max_len)], 1) if n else np.zeros((0, 3))
            for n in occ]
    queued = [[(int(p), int(l)) for p, l in zip(rng.integers(1, 3000, n), rng.integers(1, min(max_len, 500) + 1, n))]
              for n in np.minimum(rng.integers(0, int(rng.choice([0, 6, 40])) + 1, M) * (rng.random(M) > 0.5), 2048 - occ)]
    R = min(int(rng.choice([1, 31, 33, 200, 700, 3000, 9000])), (1 << 24) // M)
    pool = np.clip(np.rint(rng.lognormal(rng.uniform(1, 6), 1.2, int(rng.choice([1, 3, 40, R])))), 1, max_len)
    inc = np.stack([rng.integers(1, 4000, R), rng.choice(pool, R)], 1)
    bud = rng.uniform(0.3, 3, R) * float(rng.choice([0.5, 3, 20, 300])) * solo(inc[:, 0], inc[:, 1], classes[0])
    special = rng.random(R)
    bud = np.where(special < 0.03, 0.0, np.where(special < 0.06, np.inf, np.where(special < 0.08, -1.0, bud)))
    return _finish_random_case(rng, fleet(rng.integers(0, n_class, M), acts, queued, inc, bud, classes=classes,
                                          max_len=max_len))


def _finish_random_case(rng, fl):
    M, R, max_len = len(fl.inst_class), len(fl.in_prompt), fl.max_len
    fl.n_inst = M
    sim = oracle.simulate(fl)
    fl.act_budget = (sim.act_finish * rng.uniform(0.6, 1.4, len(sim.act_finish))).astype(np.float32)
    fl.act_rem_refreshed = np.clip(np.rint(fl.act_rem * rng.lognormal(0, 0.4, len(fl.act_rem))), 1, max_len).astype(np.int32)
    kw = {}
    if rng.random() < 0.5:
        kw["exclude"] = rng.integers(-1, M, R).astype(np.int32)
    if rng.random() < 0.4:
        kw["hits"] = workloads.cached_prefixes(fl, mean_hits=float(rng.uniform(0.5, 3)), seed=int(rng.integers(1 << 30)))
    if rng.random() < 0.4:
        kw["blackbox"] = (workloads.observed_status(fl, int(rng.integers(1, 4)), seed=int(rng.integers(1 << 30))),
                          float(rng.choice([0.2, 0.5, 1.0])))
    if rng.random() < 0.4:
        fl.batch_cap = workloads.batch_caps(fl, 0.3, 1.3, seed=int(rng.integers(1 << 30)))
    return fl, kw


@pytest.mark.parametrize("seed", range(4))
def test_random_small_fleets(seed):
    rng = np.random.default_rng(1000 + seed)
    for case in range(12):
        fl, kw = _random_case(rng)
        print(f"seed {seed} case {case}: M={len(fl.inst_class)} R={len(fl.in_prompt)} "
              f"entries={len(fl.act_prompt)}+{len(fl.q_prompt)} options={sorted(kw)} "
              f"cap={getattr(fl, 'batch_cap', None) is not None}", flush=True)
        parity.run_and_check(fl, seed=seed, **kw)


@pytest.mark.parametrize("seed", range(3))
def test_random_larger_fleets(seed):
    rng = np.random.default_rng(2000 + seed)
    for case in range(10):
        fl, kw = _random_case(rng, larger=True)
        print(f"seed {seed} case {case}: M={len(fl.inst_class)} R={len(fl.in_prompt)} "
              f"entries={len(fl.act_prompt)}+{len(fl.q_prompt)} most per instance "
              f"{int(max(np.diff(fl.act_off) + np.diff(fl.q_off)))} options={sorted(kw)} "
              f"cap={getattr(fl, 'batch_cap', None) is not None}", flush=True)
        parity.run_and_check(fl, seed=seed, sample=2000 if "blackbox" in kw else None, **kw)


@pytest.mark.parametrize("capped", [False, True])
def test_feedback_routing_beyond_an_instance_s_room(capped):
    """More routed requests than an instance has room for: the surplus is still answered but no
    longer counted, the sticky bit is raised, nothing is written out of bounds (both ways of
    placing a chunk: by atomics, and in batch order under caps)."""
    import torch
    dev = "cuda:0"
    fl = workloads.make_fleet(workloads.spec("tiny", slo_scale=1.0, seed=71, n_incoming=600))
    d = parity.upload(fl, dev)
    me = int(max(np.diff(fl.act_off) + np.diff(fl.q_off)))
    h = binding.Fleet(fl.coef["delta"], fl.coef["alpha"], fl.coef["beta"], fl.coef["gamma"], fl.inst_class,
                      me + 20, parity.max_len_of(fl), 600)
    if capped:
        h.gr_set_batch_cap(np.full(fl.n_inst, 50, dtype=np.int32))
    fin = torch.zeros(len(fl.act_prompt), dtype=torch.float32, device=dev)
    h.gr_build_status(d["act_off"], d["act_prompt"], d["act_gen"], d["act_rem"], d["q_off"], d["q_prompt"], d["q_len"], fin)
    inst = torch.full((600,), -7, dtype=torch.int32, device=dev)
    slack = torch.zeros(600, dtype=torch.float32, device=dev)
    h.gr_route_feedback(200, d["in_prompt"], d["in_len"], d["in_budget"], inst, slack)
    torch.cuda.synchronize()
    g = inst.cpu().numpy()
    assert g.min() >= 0 and g.max() < fl.n_inst and np.isfinite(slack.cpu().numpy()).all()
    assert h.gr_device_status() & 2                       # entries dropped: 600 requests, room for 4 x 20
    # the handle still works: a fresh status and a routing call on it agree with the reference
    h.close()
    parity.run_and_check(workloads.make_fleet(workloads.spec("tiny", seed=71)))
