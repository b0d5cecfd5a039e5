"""CPU-only checks of the host side: the library loads and exports every entry
point the header declares, the header and the binding agree, the workload
generator is deterministic, and the choice classifier used by the GPU parity
tests accepts the reference's own answers and rejects wrong ones."""
import os
import re

import numpy as np

import oracle
from paper_2605_16867_amd import binding, workloads
from tests import parity

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "goodroute.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b(gr_[a-z_]+)\s*\(", text))


def test_library_exports_every_declared_symbol():
    lib = binding.lib()
    names = declared_functions()
    assert names == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_a_missing_library_is_an_error_not_a_fallback(monkeypatch, tmp_path):
    """The binding has no other implementation to fall back on: without the
    built library every entry point is unavailable, loudly."""
    import pytest
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libgoodroute.so"))
    with pytest.raises(ImportError):
        binding.lib()
    with pytest.raises(ImportError):
        binding.Fleet([1e-5], [0.01], [1e-4], [1e-8], [0], 8, 100, 8)
    src = open(os.path.join(ROOT, "paper_2605_16867_amd", "binding.py")).read()
    assert "oracle" not in src          # the binding never reaches for the CPU reference


def test_strerror_needs_no_gpu():
    assert binding.strerror(0) == "ok"
    assert "invalid" in binding.strerror(-1)
    assert binding.strerror(-99) == "unknown error"


def test_workloads_are_seeded_and_shaped():
    a = workloads.make_fleet(workloads.spec("mid"))
    b = workloads.make_fleet(workloads.spec("mid"))
    for k in ("act_rem", "act_budget", "in_len", "in_budget", "q_len", "act_rem_refreshed"):
        assert np.array_equal(getattr(a, k), getattr(b, k))
    assert a.n_inst == 32 and len(a.act_rem) == 32 * 256 and len(a.q_len) == 32 * 32
    assert len(a.in_len) == 4096 and a.act_rem.min() >= 1 and a.act_rem.max() <= 4096
    assert set(a.inst_class) == {0, 1, 2}
    j = workloads.make_fleet(workloads.spec("mid", occupancy_jitter=True, seed=3))
    n = np.diff(j.act_off)
    assert n.min() == 0 and n.max() <= 256 and len(j.act_rem) == j.act_off[-1]
    h = workloads.spec("heavy")
    assert h.n_class == 6 and abs(h.coef["alpha"][5] - 0.15) < 1e-12 and h.coef["alpha"][0] == 0.012


def test_classifier_accepts_reference_and_rejects_wrong_answers():
    fl = workloads.make_fleet(workloads.spec("mid", slo_scale=2.0))
    sim = oracle.simulate(fl)
    T = sim.pair_T(fl.in_prompt, fl.in_len)
    D = fl.in_budget.astype(np.float64)
    ref = sim.route(fl.in_prompt, fl.in_len, D)
    want, robust, adm, fbk = parity.classify_choices(T, D, sim.rank, None, ref.inst.astype(np.int64))
    assert np.array_equal(want, ref.inst) and adm.all()
    assert np.array_equal(fbk[fbk >= 0], ref.fallback[fbk >= 0]) and (fbk >= 0).mean() > 0.99
    assert robust.mean() > 0.99 and 0.1 < ref.fallback.mean() < 0.9
    wrong = (ref.inst.astype(np.int64) + 1) % fl.n_inst
    _, _, adm2, _ = parity.classify_choices(T, D, sim.rank, None, wrong)
    assert adm2[robust].mean() < 0.05
    # with an excluded instance the reference never returns it
    ex = ref.inst.copy()
    ref2 = sim.route(fl.in_prompt, fl.in_len, D, exclude=ex)
    assert np.all(ref2.inst != ex)
    want2, _, adm3, _ = parity.classify_choices(T, D, sim.rank, ex, ref2.inst.astype(np.int64))
    assert np.array_equal(want2, ref2.inst) and adm3.all()


def _verdicts_from_matrix(sim, c0, ln, D, ex, hits, picked):
    T = sim.pair_T(c0, ln, hits=hits)
    return parity.classify_choices(T, D, sim.rank, ex, picked)


def test_band_summary_agrees_with_the_matrix_classifier():
    """The per-request summary the C reference gives for batches of any size leads to the same
    verdicts (decided or not, acceptable or not, fallback bit) as the [n, M] classifier, for the
    reference's own answers, for wrong ones, with exclusions and with cached prefixes."""
    rng = np.random.default_rng(5)
    for scale, seed in ((1.0, 1), (2.0, 2), (8.0, 3)):
        fl = workloads.make_fleet(workloads.spec("mid", slo_scale=scale, occupancy_jitter=True, seed=seed))
        sim = oracle.simulate(fl)
        c0, ln, D = fl.in_prompt, fl.in_len, fl.in_budget.astype(np.float64)
        # deadlines moved onto the boundary of some pair so that the band is populated
        T = sim.pair_T(c0, ln)
        rows = rng.choice(len(D), 600, replace=False)
        D[rows] = T[rows, rng.integers(0, fl.n_inst, 600)] * (1 + rng.uniform(-2e-4, 2e-4, 600))
        hits = workloads.cached_prefixes(fl, mean_hits=2.0, seed=seed)
        ex = rng.integers(-1, fl.n_inst, len(D)).astype(np.int32)
        for use_ex, use_hits in ((None, None), (ex, None), (None, hits), (ex, hits)):
            ref = sim.route(c0, ln, D, exclude=use_ex, hits=use_hits)
            for picked in (ref.inst.astype(np.int64), (ref.inst.astype(np.int64) + 1) % fl.n_inst,
                           rng.integers(0, fl.n_inst, len(D)).astype(np.int64)):
                want, robust, adm, fbk = _verdicts_from_matrix(sim, c0, ln, D, use_ex, use_hits, picked)
                band = sim.band(c0, ln, D, picked, parity.EPS, exclude=use_ex, hits=use_hits)
                r2, a2, f2 = parity.judge_with_band(band, D, sim.rank, picked)
                assert np.array_equal(want, ref.inst)
                assert np.array_equal(robust, r2) and np.array_equal(adm, a2) and np.array_equal(fbk, f2)
                allowed = np.ones_like(T, dtype=bool)
                if use_ex is not None:
                    allowed[np.flatnonzero(use_ex >= 0), use_ex[use_ex >= 0]] = False
                Th = sim.pair_T(c0, ln, hits=use_hits)
                assert np.array_equal(band.picked_T, np.where(allowed[np.arange(len(D)), picked],
                                                              Th[np.arange(len(D)), picked], np.inf))
                assert np.array_equal(band.tmin, np.where(allowed, Th, np.inf).min(axis=1))
            assert 0 < (~r2).sum() < 0.2 * len(D)


def test_exact_ties_are_decided_and_go_to_the_lowest_index():
    """Two different instances with the same latency bit for bit: the fallback choice is the one
    with the lower index, and the classifiers call it decided (nothing else is acceptable)."""
    from tests.fleets import two_equal_minima_in_one_lane
    fl = two_equal_minima_in_one_lane()
    sim = oracle.simulate(fl)
    M = fl.n_inst if hasattr(fl, "n_inst") else len(fl.inst_class)
    c0, ln, D = fl.in_prompt, fl.in_len, fl.in_budget.astype(np.float64)
    assert sim.d[0] == 0.25 and sim.d[M - 1] == 0.5 and np.all(sim.d[1:M - 1] == 0.375)
    assert sim.rank[M - 1] == 0 and sim.rank[0] == M - 1          # 64 positions apart
    T = sim.pair_T(c0, ln)
    tie = ln == 8
    assert np.array_equal(T[tie, 0], T[tie, M - 1]) and np.all(T[tie, 0] == 4.0 + c0[tie] / 1024.0)
    assert np.all(T[:, 1:M - 1] > np.maximum(T[:, 0], T[:, M - 1])[:, None])
    ref = sim.route(c0, ln, D)
    tight = D < 1.0
    assert np.all(ref.inst[tight & tie] == 0)                     # equal T: lowest index
    assert np.all(ref.inst[tight & (ln < 8)] == M - 1) and np.all(ref.inst[tight & (ln > 8)] == 0)
    assert np.all(ref.inst[~tight] == M - 1) and np.all(ref.fallback == tight)
    for picked, fine in ((ref.inst.astype(np.int64), True), (np.full(len(D), M - 1, dtype=np.int64), False)):
        band = sim.band(c0, ln, D, picked, parity.EPS)
        robust, adm, _ = parity.judge_with_band(band, D, sim.rank, picked)
        want, robust_m, adm_m, _ = parity.classify_choices(T, D, sim.rank, None, picked)
        assert robust.all() and robust_m.all() and np.array_equal(want, ref.inst)
        assert np.all(band.equal[tie] == 2) and np.all(band.equal[~tie] == 1)
        assert fine == bool(np.all(picked[tight & tie] == want[tight & tie]))


def test_recorded_traffic_is_only_reported_for_unchanged_kernel_sources(tmp_path, monkeypatch):
    """bench.py takes the dominant kernel's HBM bytes from a counter summary under profiles/; the
    record carries the hash of the kernel sources and is dropped as soon as they differ."""
    import bench
    prof = tmp_path / "profiles"
    prof.mkdir()
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    for rel in bench.KERNEL_SOURCES:
        path = tmp_path / rel
        path.parent.mkdir(parents=True, exist_ok=True)
        path.write_text("// " + rel + "\n")
    good = bench.sources_sha256()
    (prof / "heavy_step_all_kernels.md").write_text(
        "# summary\n\ntraffic-record: kernel=k_tile<migrate> fetch_bytes=100 write_bytes=23 sources_sha256=" + good + "\n"
        "traffic-record: kernel=k_tile<route> fetch_bytes=7 write_bytes=1 sources_sha256=" + good + "\n")
    assert bench.recorded_traffic("heavy", "k_tile<migrate>") == (123, os.path.join("profiles", "heavy_step_all_kernels.md"))
    assert bench.recorded_traffic("heavy", "k_tile<route>")[0] == 8
    assert bench.recorded_traffic("heavy", "k_build")[0] is None           # no record for that kernel
    assert bench.recorded_traffic("large", "k_tile<route>")[0] is None     # no summary for that workload
    (tmp_path / bench.KERNEL_SOURCES[0]).write_text("// edited\n")
    value, why = bench.recorded_traffic("heavy", "k_tile<migrate>")
    assert value is None and "changed" in why
