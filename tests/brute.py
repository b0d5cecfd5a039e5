"""Pure-Python brute force used only to pin the CPU reference on tiny inputs.

Written apart from ``oracle/`` on purpose: a request's latency on an instance
is found by *putting the request on the instance* (last in its queue) and
replaying the whole instance one decode step at a time with Python floats,
so it knows nothing of step tables or of the separable "own" term.  Selection
is Alg. 1 spelled out with Python lists.
"""
from __future__ import annotations


def replay(coef, active, queued):
    """coef = (delta, alpha, beta, gamma); active = [(prompt, gen, rem)];
    queued = [(prompt, len)] or [(prompt, len, cached)]: `cached` tokens of the
    prompt need no prefill (Eq. 2's hit prefix) but count as context.  Returns
    (q, first_step, finish list in the order actives then queued)."""
    delta, alpha, beta, gamma = coef
    t = 0.0
    batch = []
    for i, (p, g, r) in enumerate(active):
        batch.append({"id": i, "rem": r, "ctx": p + g})
    for j, entry in enumerate(queued):
        p, l = entry[0], entry[1]
        cached = entry[2] if len(entry) > 2 else 0
        t += delta * (p - cached)
        batch.append({"id": len(active) + j, "rem": l, "ctx": p})
    q = t
    finish = [None] * len(batch)
    first = alpha + beta * len(batch) + gamma * sum(b["ctx"] for b in batch)
    while batch:
        t += alpha + beta * len(batch) + gamma * sum(b["ctx"] for b in batch)
        for b in batch:
            b["rem"] -= 1
            b["ctx"] += 1
            if b["rem"] == 0:
                finish[b["id"]] = t
        batch = [b for b in batch if b["rem"] > 0]
    return q, first, finish


def latency_if_routed(coef, active, queued, c0, length, cached=0):
    """T(r, g) by definition: append r behind the queue and replay; `cached`
    of its c0 tokens are already on the instance."""
    _, _, finish = replay(coef, active, list(queued) + [(c0, length, cached)])
    return finish[-1]


def replay_capped(coef, active, queued, cap):
    """The same instance when at most `cap` requests may decode together: the
    queue is served in order, its head is admitted (prefilled, then put into
    the batch) whenever the batch has room, at time 0 and after every step.
    Returns (finish list in the order actives then queued, admission time of
    each queued request, duration of the first decode step or None)."""
    delta, alpha, beta, gamma = coef
    t = 0.0
    batch = [{"id": i, "rem": r, "ctx": p + g} for i, (p, g, r) in enumerate(active)]
    waiting = list(enumerate(queued))
    finish = [None] * (len(active) + len(queued))
    admitted = [None] * len(queued)
    first = None
    while batch or waiting:
        while waiting and len(batch) < cap:
            j, entry = waiting.pop(0)
            cached = entry[2] if len(entry) > 2 else 0
            admitted[j] = t
            t += delta * (entry[0] - cached)
            batch.append({"id": len(active) + j, "rem": entry[1], "ctx": entry[0]})
        if not batch:
            break
        step = alpha + beta * len(batch) + gamma * sum(b["ctx"] for b in batch)
        if first is None:
            first = step
        t += step
        for b in batch:
            b["rem"] -= 1
            b["ctx"] += 1
            if b["rem"] == 0:
                finish[b["id"]] = t
        batch = [b for b in batch if b["rem"] > 0]
    return finish, admitted, first


def latency_if_routed_capped(coef, active, queued, cap, c0, length, cached=0):
    """T(r, g) under a batch cap, by definition: r goes to the end of the queue."""
    finish, admitted, _ = replay_capped(coef, active, list(queued) + [(c0, length, cached)], cap)
    return finish[-1], admitted[-1]


def select(T, d, deadline, exclude=-1):
    """Alg. 1: feasible set, largest d_g among it, else smallest violation."""
    cand = [g for g in range(len(T)) if g != exclude]
    if not cand:
        return -1, True
    feas = [g for g in cand if T[g] <= deadline]
    if feas:
        best = max(d[g] for g in feas)
        return min(g for g in feas if d[g] == best), False
    best = min(T[g] - deadline for g in cand)
    return min(g for g in cand if T[g] - deadline == best), True
