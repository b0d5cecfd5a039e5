"""The three calls recorded into a HIP graph and replayed.

A serving loop that routes batch after batch is bound by launch cost when the
batches are small; the calls only launch kernels on the caller's stream (no
allocation, no copy, no host synchronisation, no memset node), so they can be
captured once and replayed.  Every replay is checked against the same calls
made directly, on inputs that change between replays, with the program's own
direct work and synchronisations in between.
"""
import numpy as np
import pytest

from paper_2605_16867_amd import workloads
from tests import parity

pytestmark = pytest.mark.gpu

INPUTS = ("act_prompt", "act_gen", "act_rem", "act_rem_refreshed", "act_budget", "q_prompt", "q_len",
          "in_prompt", "in_len", "in_budget")


def _outputs(torch, na, R, dev):
    z = lambda n, t: torch.zeros(n, dtype=t, device=dev)
    return dict(fin=z(na, torch.float32), inst=z(R, torch.int32), slack=z(R, torch.float32),
                fb=z(R, torch.uint8), flag=z(na, torch.uint8), fin2=z(na, torch.float32),
                tgt=z(na, torch.int32), tsl=z(na, torch.float32), nfl=z(1, torch.int32))


def _three_calls(h, d, o):
    h.gr_build_status(d["act_off"], d["act_prompt"], d["act_gen"], d["act_rem"],
                      d["q_off"], d["q_prompt"], d["q_len"], o["fin"])
    h.gr_score_route(d["in_prompt"], d["in_len"], d["in_budget"], o["inst"], o["slack"], out_fallback=o["fb"])
    h.gr_risk_scan(d["act_off"], d["act_prompt"], d["act_gen"], d["act_rem_refreshed"],
                   d["q_off"], d["q_prompt"], d["q_len"], d["act_budget"],
                   o["flag"], o["fin2"], o["tgt"], o["tsl"], o["nfl"])


@pytest.mark.parametrize("name,small_batch_pairs", [("mid", None), ("mid", 0), ("tiny", None), ("large", None)])
def test_replays_equal_direct_calls(name, small_batch_pairs):
    import torch
    dev = "cuda:0"
    # same shapes (offsets), different contents: seeds change lengths, prompts and budgets only
    fleets = [workloads.make_fleet(workloads.spec(name, seed=s, slo_scale=sc))
              for s, sc in ((0, 1.0), (1, 3.0), (2, 8.0), (3, 1.5))]
    for fl in fleets[1:]:
        assert np.array_equal(fl.act_off, fleets[0].act_off) and np.array_equal(fl.q_off, fleets[0].q_off)
        assert len(fl.in_prompt) == len(fleets[0].in_prompt)
    ups = [parity.upload(fl, dev) for fl in fleets]
    na, R = len(fleets[0].act_prompt), len(fleets[0].in_prompt)

    parity.SMALL_BATCH_PAIRS = small_batch_pairs
    try:
        h_graph, h_direct = parity.make_handle(fleets[0]), parity.make_handle(fleets[0])
    finally:
        parity.SMALL_BATCH_PAIRS = None
    d = {k: v.clone() for k, v in ups[0].items()}       # the buffers the graph reads
    o_graph, o_direct = _outputs(torch, na, R, dev), _outputs(torch, na, R, dev)

    # warm up on a side stream (first launches set kernel attributes), then record
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        _three_calls(h_graph, d, o_graph)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _three_calls(h_graph, d, o_graph)

    for rep, up in enumerate(ups[1:] + ups[:1]):
        for k in INPUTS:
            d[k].copy_(up[k])
        for v in o_graph.values():
            v.fill_(7)
        graph.replay()
        _three_calls(h_direct, up, o_direct)      # the same work made directly, on another handle
        torch.cuda.synchronize()
        for k in o_graph:
            a, b = o_graph[k].cpu().numpy(), o_direct[k].cpu().numpy()
            assert np.array_equal(a, b, equal_nan=a.dtype.kind == "f"), f"replay {rep}: {k} differs from the direct call"
        assert int(o_graph["nfl"].item()) == int(o_graph["flag"].sum().item())
    h_graph.close()
    h_direct.close()


@pytest.mark.parametrize("entry,small_batch_pairs", [("gr_score_route", None), ("gr_score_route", 0),
                                                     ("gr_score_route_noalloc", None)])
def test_a_recorded_routing_call_follows_status_builds_made_outside_the_graph(entry, small_batch_pairs):
    """Only the routing call is recorded; the status is rebuilt by direct calls between replays.
    A recorded scoring pass makes the capability order of whatever status it finds."""
    import torch
    dev = "cuda:0"
    fleets = [workloads.make_fleet(workloads.spec("mid", seed=s, slo_scale=sc, n_incoming=1024))
              for s, sc in ((0, 2.0), (1, 3.0), (2, 8.0))]
    ups = [parity.upload(fl, dev) for fl in fleets]
    na, R = len(fleets[0].act_prompt), len(fleets[0].in_prompt)
    parity.SMALL_BATCH_PAIRS = small_batch_pairs
    try:
        h_graph, h_direct = parity.make_handle(fleets[0]), parity.make_handle(fleets[0])
    finally:
        parity.SMALL_BATCH_PAIRS = None
    d = {k: v.clone() for k, v in ups[0].items()}
    o_graph, o_direct = _outputs(torch, na, R, dev), _outputs(torch, na, R, dev)

    def build(h, src, o):
        h.gr_build_status(src["act_off"], src["act_prompt"], src["act_gen"], src["act_rem"],
                          src["q_off"], src["q_prompt"], src["q_len"], o["fin"])

    def route(h, src, o):
        getattr(h, entry)(src["in_prompt"], src["in_len"], src["in_budget"], o["inst"], o["slack"], out_fallback=o["fb"])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        build(h_graph, d, o_graph)
        route(h_graph, d, o_graph)            # the capability order of this status now exists
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        route(h_graph, d, o_graph)

    for rep, up in enumerate(ups[1:] + ups[:1]):
        for k in INPUTS:
            d[k].copy_(up[k])
        for k in ("inst", "slack", "fb"):
            o_graph[k].fill_(7)
        build(h_graph, d, o_graph)            # a direct call: another status, another capability order
        graph.replay()
        build(h_direct, up, o_direct)
        route(h_direct, up, o_direct)
        torch.cuda.synchronize()
        for k in ("fin", "inst", "slack", "fb"):
            a, b = o_graph[k].cpu().numpy(), o_direct[k].cpu().numpy()
            assert np.array_equal(a, b, equal_nan=a.dtype.kind == "f"), f"replay {rep}: {k} differs from the direct call"
    assert len({tuple(workloads.make_fleet(workloads.spec("mid", seed=s)).act_rem[:8]) for s in (0, 1, 2)}) == 3
    h_graph.close()
    h_direct.close()
