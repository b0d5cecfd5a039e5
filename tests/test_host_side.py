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
