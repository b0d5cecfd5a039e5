"""The CPU reference under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only):
``oracle/goodroute_oracle.c`` is compiled with -fsanitize=address,undefined together with a
small driver, run on fleets that reach every function and branch of it (queues, batch caps,
empty instances, exclusions, cached prefixes named twice and over-long, lengths beyond an
instance's last request), and must (a) finish without a sanitizer report and (b) write exactly
what the ordinary build computes.  Also: the public header is plain C99."""
import os
import shutil
import subprocess

import numpy as np
import pytest

import oracle
from paper_2605_16867_amd import workloads
from tests.fleets import fleet, rand_entries

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE_C = os.path.join(ROOT, "oracle", "goodroute_oracle.c")
DRIVER_C = os.path.join(ROOT, "tests", "oracle_sanitizer_driver.c")


@pytest.fixture(scope="module")
def sanitized(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-ffp-contract=off", "-fopenmp", "-Wall", "-Wextra",
           "-o", exe, DRIVER_C, ORACLE_C, "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return exe


def i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def run_both(exe, tmp_path, fl, cap=None, exclude=None, hits=None, tag="x"):
    M, R = len(fl.inst_class), len(fl.in_prompt)
    if cap is not None:
        fl.batch_cap = i32(cap)
    sim = oracle.simulate(fl)
    D = fl.in_budget.astype(np.float64)
    rank = i32(sim.rank)
    picked = i32(np.random.default_rng(1).integers(-1, M, R))
    parts = [np.array([M, len(fl.coef["delta"]), len(fl.act_prompt), len(fl.q_prompt), R,
                       -1 if hits is None else len(hits[1]), int(cap is not None), int(exclude is not None)], np.int64)]
    parts += [np.ascontiguousarray(fl.coef[k], dtype=np.float64) for k in ("delta", "alpha", "beta", "gamma")]
    parts += [i32(fl.inst_class), i32(fl.act_off), i32(fl.act_prompt), i32(fl.act_gen), i32(fl.act_rem),
              i32(fl.q_off), i32(fl.q_prompt), i32(fl.q_len)]
    if cap is not None:
        parts.append(i32(cap))
    parts += [i32(fl.in_prompt), i32(fl.in_len), D]
    if exclude is not None:
        parts.append(i32(exclude))
    if hits is not None:
        parts += [i32(hits[0]), i32(hits[1]), i32(hits[2])]
    parts += [rank, picked]
    src, dst = str(tmp_path / f"{tag}.in"), str(tmp_path / f"{tag}.out")
    with open(src, "wb") as f:
        for p in parts:
            f.write(p.tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="4")
    r = subprocess.run([exe, src, dst], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0 and r.stderr.strip() == "", r.stderr[-3000:]

    # the ordinary build, through the Python face
    ref = sim.route(fl.in_prompt, fl.in_len, D, exclude=exclude, hits=hits)
    band = sim.band(fl.in_prompt, fl.in_len, D, picked, 1e-4, exclude=exclude, hits=hits)
    want = [sim.act_finish, sim.q_finish, sim.q, sim.d, sim.smax]
    want += [sim.step_table(g) for g in range(M)]
    want += [sim.pair_T(fl.in_prompt, fl.in_len, hits=hits), ref.inst, ref.slack, ref.fallback, ref.T,
             band.sure, band.maybe, band.tmin, band.near, band.equal, band.picked_T]
    blob = open(dst, "rb").read()
    at = 0
    for k, w in enumerate(want):
        w = np.ascontiguousarray(w)
        got = np.frombuffer(blob, dtype=w.dtype, count=w.size, offset=at).reshape(w.shape)
        at += w.nbytes
        assert np.array_equal(got, w, equal_nan=True), f"output {k} differs between the two builds"
    assert at == len(blob)


def test_reference_is_clean_under_sanitizers_and_unchanged(sanitized, tmp_path):
    rng = np.random.default_rng(0)
    # the tiny fleet of the first configuration (queues on every instance), with exclusions
    fl = workloads.make_fleet(workloads.spec("tiny"))
    run_both(sanitized, tmp_path, fl, exclude=rng.integers(-1, fl.n_inst, len(fl.in_prompt)), tag="tiny")
    # batch caps: below, at and above the number of requests held; cached prefixes
    fl = workloads.make_fleet(workloads.spec("tiny", n_queued=20, slo_scale=4.0, seed=3))
    hits = workloads.cached_prefixes(fl, mean_hits=3.0, seed=1)
    hits[2][::3] = 10 ** 6                                   # longer than the request: cut to its tokens
    if len(hits[1]) > 1:
        hits[1][1] = hits[1][0]                              # an instance named twice
    for k, cap in enumerate((1, 30, 84, 85, 1000)):
        run_both(sanitized, tmp_path, fl, cap=np.full(fl.n_inst, cap), hits=hits, tag=f"cap{k}")
    # empty and queue-only instances, one request, extreme lengths
    acts = [rand_entries(rng, 40), np.zeros((0, 3)), np.zeros((0, 3)), rand_entries(rng, 1)]
    queued = [[], [], [(500, 40), (900, 7)], [(128, 4096)]]
    inc = [(100, 1), (2048, 4096), (1, 1), (700, 5000)]       # the last one outlives every instance's requests
    fl = fleet([0, 1, 2, 0], acts, queued, inc, [0.0, 1e9, 1.0, -5.0], max_len=8192)
    run_both(sanitized, tmp_path, fl, exclude=[0, -1, 3, 1], tag="edges")
    # a single instance, everything excluded
    fl = fleet([0], [rand_entries(rng, 5)], [[]], [(300, 50), (700, 10)], [1e9, 0.0])
    run_both(sanitized, tmp_path, fl, exclude=[0, 0], tag="one")
    # a mid-size fleet: the OpenMP loops with several threads
    fl = workloads.make_fleet(workloads.spec("mid", slo_scale=2.0, occupancy_jitter=True, seed=5, n_incoming=512))
    run_both(sanitized, tmp_path, fl, tag="mid")


def test_public_header_is_plain_c99(tmp_path):
    src = tmp_path / "use_header.c"
    src.write_text('#include "goodroute.h"\nint main(void) { return GR_OK + (int)sizeof(gr_fleet *) * 0; }\n')
    r = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only",
                        "-I", os.path.join(ROOT, "include"), str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    assert shutil.which("g++") is None or subprocess.run(
        ["g++", "-std=c++11", "-fsyntax-only", "-x", "c++", "-I", os.path.join(ROOT, "include"), str(src)],
        capture_output=True, text=True).returncode == 0
