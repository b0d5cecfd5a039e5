"""GPU-vs-reference comparison shared by the GPU tests, the smoke check and the
benchmark's self-check.  Runs the three library calls through the binding on
``cuda:0`` and compares every output with ``oracle/`` on the same inputs.

Bars.  Finish times and pair latencies: relative 1e-4 (fp32 on the GPU, fp64
reference).  d_g and the capability rank: bit-exact.  Choices and flags: equal
to the reference wherever the decision does not hinge on a latency lying within
1e-4 (relative) of the deadline or of a competing latency; those few are
counted as "ambiguous" and must still be an answer that is right for some
latency within the band.
"""
from __future__ import annotations

from typing import Optional

import numpy as np

import oracle
from paper_2605_16867_amd import binding

EPS = 1e-4


def classify_choices(T, D, rank, exclude, picked):
    """T: [n, M] fp64 reference latencies; D: [n]; rank: [M]; exclude: [n] or None;
    picked: [n] instance chosen by the GPU.  Returns (want, robust, admissible):
    the reference choice, whether it is decided outside the band, and whether the
    GPU's pick is acceptable; plus the fallback bit where it does not hinge on the band
    (-1 where it does)."""
    n, M = T.shape
    T = T.copy()
    if exclude is not None:
        ok = exclude >= 0
        T[np.flatnonzero(ok), exclude[ok]] = np.inf
    order = np.argsort(rank, kind="stable")
    To = T[:, order]                                   # columns in capability order
    finite = np.isfinite(To)
    F = (To <= D[:, None]) & finite
    SF = (To * (1 + EPS) <= D[:, None]) & finite
    PF = (To * (1 - EPS) <= D[:, None]) & finite
    first = lambda m: np.where(m.any(axis=1), m.argmax(axis=1), M)
    f1, s1, p1 = first(F), first(SF), first(PF)
    Tmin = To.min(axis=1)
    # fallback: smallest T, ties to the lowest instance index
    amin = np.argmin(T, axis=1)
    want = np.where(f1 < M, order[np.minimum(f1, M - 1)], amin).astype(np.int64)
    none_allowed = ~np.isfinite(Tmin)
    want[none_allowed] = -1

    # nothing feasible: decided when every latency within 2 eps of the smallest one equals it bit
    # for bit (one instance, or exact ties, which go to the lowest index)
    with np.errstate(invalid="ignore"):
        near = (T <= (Tmin * (1 + 2 * EPS))[:, None]).sum(axis=1)
        equal = (T == Tmin[:, None]).sum(axis=1)
    robust_fb = near == equal
    robust = np.where(p1 < M, p1 == s1, robust_fb) | none_allowed

    pos = np.empty(M, dtype=np.int64)
    pos[order] = np.arange(M)
    ppos = np.where(picked >= 0, pos[np.maximum(picked, 0)], M)     # GPU pick in capability order
    rows = np.arange(n)
    pT = np.where(picked >= 0, T[rows, np.maximum(picked, 0)], np.inf)
    in_PF = (picked >= 0) & (pT * (1 - EPS) <= D) & np.isfinite(pT)
    near_min = (picked >= 0) & (pT <= Tmin * (1 + 2 * EPS))
    adm = np.where(s1 < M, in_PF & (ppos <= s1),
                   np.where(p1 < M, in_PF | near_min, near_min))
    adm = np.where(none_allowed, picked == -1, adm)
    # the "nothing was feasible" bit is fixed unless some latency sits in the band around D
    fb_known = np.where(s1 < M, 0, np.where(p1 == M, 1, -1))
    return want, robust, adm, fb_known


def check_choices(name, T, D, rank, exclude, picked, slack, rep, fallback=None):
    want, robust, adm, fb_known = classify_choices(T, D, rank, exclude, picked)
    if fallback is not None:
        known = fb_known >= 0
        assert np.array_equal(fallback[known], fb_known[known]), f"{name}: fallback bit wrong outside the band"
    bad = robust & (picked != want)
    assert not bad.any(), f"{name}: {bad.sum()} robust choices differ, first at {np.flatnonzero(bad)[:5]}"
    assert adm[~robust].all(), f"{name}: {(~adm[~robust]).sum()} ambiguous choices not admissible"
    ok = picked >= 0
    rows = np.flatnonzero(ok)
    Tp = T[rows, picked[ok]]
    got_s, want_s = slack[ok].astype(np.float64), D[ok] - Tp
    with np.errstate(invalid="ignore"):
        err = np.abs(got_s - want_s)
        tol = EPS * np.maximum(Tp, np.abs(D[ok])) + 1e-30
        fine = (err <= tol) | (got_s == want_s) | (np.isnan(got_s) & np.isnan(want_s))
    assert np.all(fine), f"{name}: {np.sum(~fine)} slacks beyond tolerance"
    rep[name + "_ambiguous"] = int((~robust).sum())
    rep[name + "_differ"] = int((picked != want).sum())
    rep[name + "_n"] = int(len(picked))
    rep[name + "_feasible_frac"] = float(np.mean((T <= D[:, None]).any(axis=1))) if len(D) else 0.0
    return want


def judge_with_band(band, D, rank, picked):
    """The same verdicts as classify_choices from the per-request summary of
    ``oracle.SimulatedFleet.band`` (no [n, M] matrix): (robust, admissible, fallback bit or -1)."""
    M = len(rank)
    s1, p1, Tmin, pT = band.sure.astype(np.int64), band.maybe.astype(np.int64), band.tmin, band.picked_T
    none_allowed = ~np.isfinite(Tmin)
    robust = np.where(p1 < M, p1 == s1, band.near == band.equal) | none_allowed
    ppos = np.where(picked >= 0, np.asarray(rank, dtype=np.int64)[np.maximum(picked, 0)], M)
    with np.errstate(invalid="ignore"):
        in_PF = np.isfinite(pT) & (pT * (1 - EPS) <= D)
        near_min = np.isfinite(pT) & (pT <= Tmin * (1 + 2 * EPS))
    adm = np.where(s1 < M, in_PF & (ppos <= s1), np.where(p1 < M, in_PF | near_min, near_min))
    adm = np.where(none_allowed, picked == -1, adm)
    fb_known = np.where(s1 < M, 0, np.where(p1 == M, 1, -1))
    return robust, adm, fb_known


def check_choices_all(name, sim, c0, ln, D, exclude, hits, picked, slack, rep, fallback=None):
    """Every request of a batch of any size against the reference's exhaustive scan:
    the reference's own choice (Alg. 1) and, per request, how firmly it stands."""
    ref = sim.route(c0, ln, D, exclude=exclude, hits=hits)
    band = sim.band(c0, ln, D, picked, EPS, exclude=exclude, hits=hits)
    want = ref.inst.astype(np.int64)
    robust, adm, fb_known = judge_with_band(band, D, sim.rank, picked)
    if fallback is not None:
        known = fb_known >= 0
        assert np.array_equal(fallback[known], fb_known[known]), f"{name}: fallback bit wrong outside the band"
        assert np.array_equal(ref.fallback[known], fb_known[known]), f"{name}: reference scan and band disagree"
    bad = robust & (picked != want)
    assert not bad.any(), f"{name}: {bad.sum()} robust choices differ, first at {np.flatnonzero(bad)[:5]}"
    assert adm[~robust].all(), f"{name}: {(~adm[~robust]).sum()} ambiguous choices not admissible"
    ok = picked >= 0
    Tp = band.picked_T[ok]
    got_s, want_s = slack[ok].astype(np.float64), D[ok] - Tp
    with np.errstate(invalid="ignore"):
        err = np.abs(got_s - want_s)
        tol = EPS * np.maximum(Tp, np.abs(D[ok])) + 1e-30
        fine = (err <= tol) | (got_s == want_s) | (np.isnan(got_s) & np.isnan(want_s))
    assert np.all(fine), f"{name}: {np.sum(~fine)} slacks beyond tolerance"
    assert np.all(slack[~ok] == 0.0)
    rep[name + "_ambiguous"] = int((~robust).sum())
    rep[name + "_differ"] = int((picked != want).sum())
    rep[name + "_n"] = int(len(picked))
    rep[name + "_exact_ties"] = int((band.equal > 1).sum())
    rep[name + "_feasible_frac"] = float(1.0 - ref.fallback.mean()) if len(D) else 0.0
    return want


def rel_err(got, want):
    want = np.asarray(want, dtype=np.float64)
    return np.abs(np.asarray(got, dtype=np.float64) - want) / np.maximum(np.abs(want), 1e-300)


def upload(fl, device="cuda:0"):
    import torch
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device)
    return {k: t(getattr(fl, k)) for k in
            ("act_off", "act_prompt", "act_gen", "act_rem", "act_rem_refreshed", "act_budget",
             "q_off", "q_prompt", "q_len", "in_prompt", "in_len", "in_budget")}


def sub_csr(hits, idx):
    """The hit lists of the requests idx, as a CSR of their own."""
    off, inst, ln = (np.asarray(x) for x in hits)
    cnt = (off[1:] - off[:-1])[idx]
    new_off = np.zeros(len(idx) + 1, dtype=np.int32)
    new_off[1:] = np.cumsum(cnt)
    take = np.concatenate([np.arange(off[i], off[i + 1]) for i in idx]) if len(idx) else np.zeros(0, np.int64)
    take = take.astype(np.int64)
    return new_off, inst[take].astype(np.int32), ln[take].astype(np.int32)


def max_len_of(fl) -> int:
    return int(fl.max_len) if hasattr(fl, "max_len") else int(fl.spec.max_len)


# How the handles of the checks below score a batch: None = the library's own choice (small
# batches pair by pair, large ones grouped by length), 0 = always grouped.  tests/conftest.py
# runs the GPU tests of the edge cases once each way.
SMALL_BATCH_PAIRS: Optional[int] = None


def make_handle(fl, max_requests: Optional[int] = None, max_entries: Optional[int] = None):
    me = int(max(np.diff(fl.act_off) + np.diff(fl.q_off)))
    h = binding.Fleet(fl.coef["delta"], fl.coef["alpha"], fl.coef["beta"], fl.coef["gamma"],
                      fl.inst_class, max(me, 1) if max_entries is None else max_entries,
                      max_len_of(fl),
                      max(len(fl.in_prompt), 1) if max_requests is None else max_requests)
    if SMALL_BATCH_PAIRS is not None:
        h.gr_set_small_batch_pairs(SMALL_BATCH_PAIRS)
    return h


def run_and_check(fl, sample: Optional[int] = None, seed: int = 0, full_T_limit: int = 1 << 25,
                  exclude=None, hits=None, blackbox=None):
    """Run the whole path on the GPU and check it.  ``sample``: number of
    requests (and of active requests) checked against the reference; None = all.
    ``hits``: (hit_off, hit_inst, hit_len) cached prefixes of the incoming requests
    (routes through gr_score_route_cached).  ``blackbox``: (rounds, weight) with
    rounds = [(ema_weight, wait, prefill, decode), ..] float32 arrays or None per term:
    fed to gr_observe, then blended in with gr_set_blend(weight)."""
    import torch
    dev = "cuda:0"
    rep = {}
    d = upload(fl, dev)
    M = len(fl.inst_class)
    na, nq, R = len(fl.act_prompt), len(fl.q_prompt), len(fl.in_prompt)
    h = make_handle(fl)
    if getattr(fl, "batch_cap", None) is not None:
        h.gr_set_batch_cap(fl.batch_cap)
    rng = np.random.default_rng(seed)
    view = lambda s, rem=None: s
    if blackbox is not None:
        rounds, lam = blackbox
        status = oracle.SmoothedStatus()
        f32t = lambda x: None if x is None else torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(dev)
        for w, ow, op, od in rounds:
            h.gr_observe(w, f32t(ow), f32t(op), f32t(od))
            status.observe(w, *[None if x is None else np.asarray(x, dtype=np.float32) for x in (ow, op, od)])
        h.gr_set_blend(lam)
        view = lambda s, rem=None: oracle.BlendedFleet(s, fl, status, lam, act_rem=rem)

    # ---- step 1: status
    fin = torch.full((na,), float("nan"), dtype=torch.float32, device=dev)
    qfin = torch.full((nq,), float("nan"), dtype=torch.float32, device=dev)
    dd = torch.zeros(M, dtype=torch.float64, device=dev)
    rk = torch.zeros(M, dtype=torch.int32, device=dev)
    h.gr_build_status(d["act_off"], d["act_prompt"], d["act_gen"], d["act_rem"],
                      d["q_off"], d["q_prompt"], d["q_len"], fin, qfin, dd, rk)
    torch.cuda.synchronize()
    sim = view(oracle.simulate(fl))
    e = rel_err(fin.cpu().numpy(), sim.act_finish)
    assert na == 0 or e.max() <= EPS, f"active finish rel err {e.max():.3g}"
    rep["finish_rel_err"] = float(e.max()) if na else 0.0
    if nq:
        e = rel_err(qfin.cpu().numpy(), sim.q_finish)
        assert e.max() <= EPS, f"queued finish rel err {e.max():.3g}"
    assert np.array_equal(dd.cpu().numpy(), sim.d), "d_g not bit-exact"
    assert np.array_equal(rk.cpu().numpy(), sim.rank), "capability rank differs"

    # ---- step 2: route
    whole = hasattr(sim, "band")       # the C reference scans a batch of any size; the numpy blend is sampled
    if R:
        ex_np = None if exclude is None else np.ascontiguousarray(exclude, dtype=np.int32)
        inst = torch.full((R,), -7, dtype=torch.int32, device=dev)
        slack = torch.zeros(R, dtype=torch.float32, device=dev)
        fb = torch.zeros(R, dtype=torch.uint8, device=dev)
        want_T = R * M <= full_T_limit
        outT = torch.zeros(R * M, dtype=torch.float32, device=dev) if want_T else None
        ex_t = None if ex_np is None else torch.from_numpy(ex_np).to(dev)
        ht = None if hits is None else [torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).to(dev) for x in hits]

        def route(c0_t, len_t, bud_t, ex_sub, h_sub, o_inst, o_slack, o_fb, o_T):
            if h_sub is None:
                h.gr_score_route(c0_t, len_t, bud_t, o_inst, o_slack, exclude_inst=ex_sub, out_fallback=o_fb, out_T=o_T)
            else:
                h.gr_score_route_cached(c0_t, len_t, bud_t, h_sub[0], h_sub[1], h_sub[2], o_inst, o_slack,
                                        exclude_inst=ex_sub, out_fallback=o_fb, out_T=o_T)
            torch.cuda.synchronize()

        route(d["in_prompt"], d["in_len"], d["in_budget"], ex_t, ht, inst, slack, fb, outT)
        g_inst, g_slack, g_fb = inst.cpu().numpy().astype(np.int64), slack.cpu().numpy(), fb.cpu().numpy()
        idx = np.arange(R) if sample is None or sample >= R else np.sort(rng.choice(R, sample, replace=False))
        D_all = fl.in_budget.astype(np.float64)
        if whole:
            check_choices_all("route", sim, fl.in_prompt, fl.in_len, D_all, ex_np, hits, g_inst, g_slack, rep,
                              fallback=g_fb)
            if hits is not None:
                rep["route_moved_by_hits"] = int((sim.route(fl.in_prompt, fl.in_len, D_all, exclude=ex_np, hits=hits).inst
                                                  != sim.route(fl.in_prompt, fl.in_len, D_all, exclude=ex_np).inst).sum())
        # every pair's latency: of the whole batch where that fits, else of a slice scored again on its own
        t_idx = (np.arange(R) if whole else idx) if want_T else np.sort(rng.choice(R, max(1, min(R, full_T_limit // M)), replace=False))
        sub_hits = None if hits is None else sub_csr(hits, t_idx)
        if not want_T:
            ti = torch.from_numpy(t_idx).to(dev)
            n_t = len(t_idx)
            s_inst = torch.full((n_t,), -7, dtype=torch.int32, device=dev)
            s_slack = torch.zeros(n_t, dtype=torch.float32, device=dev)
            s_fb = torch.zeros(n_t, dtype=torch.uint8, device=dev)
            s_T = torch.zeros(n_t * M, dtype=torch.float32, device=dev)
            route(d["in_prompt"][ti].contiguous(), d["in_len"][ti].contiguous(), d["in_budget"][ti].contiguous(),
                  None if ex_t is None else ex_t[ti].contiguous(),
                  None if sub_hits is None else [torch.from_numpy(x).to(dev) for x in sub_hits],
                  s_inst, s_slack, s_fb, s_T)
            # the same requests in a batch of their own are decided the same way
            assert np.array_equal(s_inst.cpu().numpy(), g_inst[t_idx]), "a slice of the batch is routed differently"
            assert np.array_equal(s_fb.cpu().numpy(), g_fb[t_idx])
            got_T = s_T.cpu().numpy().reshape(n_t, M)
        else:
            got_T = outT.cpu().numpy().reshape(R, M)[t_idx]
        T = sim.pair_T(fl.in_prompt[t_idx], fl.in_len[t_idx], hits=sub_hits)
        e = rel_err(got_T, T)
        assert e.max() <= EPS, f"pair latency rel err {e.max():.3g}"
        rep["pair_T_rel_err"], rep["pair_T_checked"] = float(e.max()), int(T.size)
        if not whole or len(t_idx) * M <= (1 << 24):
            # the [n, M] classifier on the same rows (the only one there is for the blended reference)
            rr = rep if not whole else {}
            want = check_choices("route", T, D_all[t_idx], sim.rank, None if ex_np is None else ex_np[t_idx],
                                 g_inst[t_idx], g_slack[t_idx], rr, fallback=g_fb[t_idx])
            ref = sim.route(fl.in_prompt[t_idx], fl.in_len[t_idx], D_all[t_idx],
                            exclude=None if ex_np is None else ex_np[t_idx], hits=sub_hits)
            if hits is not None and not whole:
                rep["route_moved_by_hits"] = int((ref.inst != sim.route(
                    fl.in_prompt[t_idx], fl.in_len[t_idx], D_all[t_idx],
                    exclude=None if ex_np is None else ex_np[t_idx]).inst).sum())
            assert np.array_equal(ref.inst, want), "reference scan and classifier disagree"

    # ---- step 3: risk scan
    if na:
        flag = torch.full((na,), 9, dtype=torch.uint8, device=dev)
        fin2 = torch.full((na,), float("nan"), dtype=torch.float32, device=dev)
        tgt = torch.full((na,), -7, dtype=torch.int32, device=dev)
        tsl = torch.full((na,), float("nan"), dtype=torch.float32, device=dev)
        nfl = torch.zeros(1, dtype=torch.int32, device=dev)
        h.gr_risk_scan(d["act_off"], d["act_prompt"], d["act_gen"], d["act_rem_refreshed"],
                       d["q_off"], d["q_prompt"], d["q_len"], d["act_budget"],
                       flag, fin2, tgt, tsl, nfl)
        torch.cuda.synchronize()
        idx = np.arange(na) if sample is None or sample >= na else np.sort(rng.choice(na, sample, replace=False))
        rs = oracle.risk_scan(fl, fl.act_rem_refreshed, fl.act_budget, only=idx,
                              view=lambda s: view(s, fl.act_rem_refreshed))
        e = rel_err(fin2.cpu().numpy(), rs.finish)
        assert e.max() <= EPS, f"risk-scan finish rel err {e.max():.3g}"
        budget = fl.act_budget.astype(np.float64)
        band = np.abs(rs.finish - budget) <= EPS * np.maximum(rs.finish, np.abs(budget))
        gflag = flag.cpu().numpy()
        assert set(np.unique(gflag)) <= {0, 1}
        bad = (gflag != rs.flag) & ~band
        assert not bad.any(), f"{bad.sum()} robust risk flags differ"
        rep["flag_ambiguous"] = int(band.sum())
        rep["flag_n"] = int(na)
        rep["flag_frac"] = float(gflag.mean())
        assert int(nfl.item()) == int(gflag.sum()), "flag count differs from flags"
        gt, gs = tgt.cpu().numpy(), tsl.cpu().numpy()
        assert np.all(gt[gflag == 0] == -1) and np.all(gs[gflag == 0] == 0.0)
        every = np.flatnonzero((gflag == 1) & (rs.flag == 1))
        both = every if whole else idx[(gflag[idx] == 1) & (rs.flag[idx] == 1)]
        if len(both):
            inst_of = (np.searchsorted(fl.act_off, both, side="right") - 1).astype(np.int32)
            c0 = fl.act_prompt[both].astype(np.int64) + fl.act_gen[both]
            if whole:
                want = check_choices_all("migrate", rs.sim, c0, fl.act_rem_refreshed[both], budget[both], inst_of,
                                         None, gt[both].astype(np.int64), gs[both], rep)
                sub = np.isin(both, idx)         # the composed reference scan names the same targets
                assert np.array_equal(want[sub], rs.target[both[sub]]), "reference scan and classifier disagree"
            else:
                T = rs.sim.pair_T(c0, fl.act_rem_refreshed[both])
                want = check_choices("migrate", T, budget[both], rs.sim.rank, inst_of,
                                     gt[both].astype(np.int64), gs[both], rep)
                assert np.array_equal(want, rs.target[both]), "reference scan and classifier disagree"
            assert np.all(gt[both] != inst_of) or M == 1
    assert h.gr_device_status() == 0, "device status bits raised on in-contract input"
    h.close()
    return rep


def run_feedback_and_check(fl, chunk: int, n_req: Optional[int] = None, exclude=None):
    """gr_route_feedback against the reference, round by round: the reference follows the
    instances the GPU committed, so every round is compared on the state the GPU really had."""
    import torch
    dev = "cuda:0"
    rep = {}
    d = upload(fl, dev)
    M = len(fl.inst_class)
    R = len(fl.in_prompt) if n_req is None else n_req
    c0, ln, D32 = fl.in_prompt[:R], fl.in_len[:R], fl.in_budget[:R]
    me = int(max(np.diff(fl.act_off) + np.diff(fl.q_off)))
    h = make_handle(fl, max_requests=max(R, 256), max_entries=min(me + R, 2048))
    if getattr(fl, "batch_cap", None) is not None:
        h.gr_set_batch_cap(fl.batch_cap)
    na = len(fl.act_prompt)
    fin = torch.zeros(na, dtype=torch.float32, device=dev)
    h.gr_build_status(d["act_off"], d["act_prompt"], d["act_gen"], d["act_rem"],
                      d["q_off"], d["q_prompt"], d["q_len"], fin)
    fin0 = fin.clone()
    inst = torch.full((R,), -7, dtype=torch.int32, device=dev)
    slack = torch.zeros(R, dtype=torch.float32, device=dev)
    fb = torch.zeros(R, dtype=torch.uint8, device=dev)
    ex_np = None if exclude is None else np.ascontiguousarray(exclude[:R], dtype=np.int32)
    h.gr_route_feedback(chunk, d["in_prompt"][:R], d["in_len"][:R], d["in_budget"][:R], inst, slack,
                        exclude_inst=None if ex_np is None else torch.from_numpy(ex_np).to(dev), out_fallback=fb)
    torch.cuda.synchronize()
    assert torch.equal(fin, fin0), "the caller's finish times were overwritten by a rebuild"
    G, S, F = inst.cpu().numpy().astype(np.int64), slack.cpu().numpy(), fb.cpu().numpy()
    D = D32.astype(np.float64)
    ref, seen = oracle.route_with_feedback(fl, c0, ln, D, chunk, exclude=ex_np, follow=G)
    amb = 0
    for k, (rows, T, rank) in enumerate(seen):
        rr = {}
        check_choices(f"round{k}", T, D[rows], rank, None if ex_np is None else ex_np[rows], G[rows], S[rows], rr,
                      fallback=F[rows])
        amb += rr[f"round{k}_ambiguous"]
    rep["rounds"], rep["ambiguous"], rep["n"] = len(seen), amb, R
    rep["instances_used"] = int(len(np.unique(G)))
    if amb == 0:        # nothing hinged on the band: the reference on its own takes the same path
        free, _ = oracle.route_with_feedback(fl, c0, ln, D, chunk, exclude=ex_np)
        assert np.array_equal(free.inst, G)
    # the handle now holds the status with every request in place: a probe batch sees it
    extra = [[] for _ in range(M)]
    for i, g in enumerate(G):
        if g >= 0:
            extra[int(g)].append((int(c0[i]), int(ln[i])))
    final = oracle.simulate(oracle._Extended(fl, extra))
    P = min(256, len(fl.in_prompt))
    pi = torch.full((P,), -7, dtype=torch.int32, device=dev)
    ps = torch.zeros(P, dtype=torch.float32, device=dev)
    h.gr_score_route(d["in_prompt"][:P], d["in_len"][:P], d["in_budget"][:P], pi, ps)
    torch.cuda.synchronize()
    check_choices("probe", final.pair_T(fl.in_prompt[:P], fl.in_len[:P]), fl.in_budget[:P].astype(np.float64),
                  final.rank, None, pi.cpu().numpy().astype(np.int64), ps.cpu().numpy(), rep)
    assert h.gr_device_status() == 0, "device status bits raised on in-contract input"
    h.close()
    return rep
