"""The serving calls (siso_lookup, siso_update_hits, siso_lookup_update) never synchronise and, once warmed up, never
allocate: a loop of them can be captured in a HIP graph and replayed.  Every replay is checked
against the eager result, with eager work and synchronisations of the program between replays."""

import numpy as np
import pytest
import torch

from paper_2508_18736_amd import workloads as W
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def siso():
    from paper_2508_18736_amd import siso as m
    return m


@pytest.mark.parametrize("n,one_call", [(64, False), (300, False), (64, True), (100, True), (300, True)])
def test_lookup_and_update_in_a_graph(siso, n, one_call):
    """one_call: the step is siso_lookup_update (small batches: one kernel ends the lookup and applies the update; the
    number that marks a launch's entries on its board lives on the device, so every replay has its own)."""
    print(f"case: graph n={n} one_call={one_call}", flush=True)
    wl = W.c4_stream(n_clusters=256, per_cluster=8, batches=4, batch=n, dim=256, seed=23)
    cents = to_dev(wl.centroids, "bf16")
    batches = [to_dev(wl.queries[b * n:(b + 1) * n], "bf16") for b in range(4)]

    def eager():
        cache = siso.SisoCache(wl.dim, wl.K, siso.BF16)
        cache.load(cents)
        outs = []
        for q in batches:
            idx, sim, hit = cache.lookup(q, 0.85)
            cache.update(q, idx, hit)
            outs.append((idx.clone(), sim.clone(), hit.clone()))
        torch.cuda.synchronize()
        return outs, cache.export()

    want_outs, want_state = eager()

    cache = siso.SisoCache(wl.dim, wl.K, siso.BF16)
    q_in = torch.empty_like(batches[0])
    idx = torch.empty(n, dtype=torch.int32, device="cuda:0")
    sim = torch.empty(n, dtype=torch.float32, device="cuda:0")
    hit = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    side = torch.cuda.Stream()
    cache.set_stream(side)
    with torch.cuda.stream(side):
        cache.load(cents)
        q_in.copy_(batches[0])
        cache.lookup(q_in, 0.85, idx, sim, hit)  # warm-up: workspaces and kernel attributes are set now
        cache.update(q_in, idx, hit)
        cache.lookup_update(q_in, 0.85, idx, sim, hit)
        cache.load(cents)                         # back to the initial state
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        if one_call:
            cache.lookup_update(q_in, 0.85, idx, sim, hit)
        else:
            cache.lookup(q_in, 0.85, idx, sim, hit)
            cache.update(q_in, idx, hit)
    for b, q in enumerate(batches):
        q_in.copy_(q)                             # eager work of the program between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(idx, want_outs[b][0]) and torch.equal(hit, want_outs[b][2]), f"replay {b}"
        assert torch.equal(sim, want_outs[b][1]), f"replay {b}: similarities"
    cache.set_stream(torch.cuda.current_stream())
    got_state = cache.export()
    torch.cuda.synchronize()
    for g, w in zip(got_state, want_state):
        assert torch.equal(g, w)
    assert cache.bad_indices() == 0


@pytest.mark.parametrize("n", [64, 200])
def test_fp8_copy_and_master_in_a_graph(siso, n):
    """siso_fp8_lookup_update (an 8-bit serving copy, the bf16 master behind it) captured and replayed: outputs and the
    state of both caches after every replay are those of the eager loop of the three calls."""
    print(f"case: graph, fp8 copy with master, n={n}", flush=True)
    wl = W.c4_stream(n_clusters=256, per_cluster=8, batches=4, batch=n, dim=256, seed=29)
    cents = to_dev(wl.centroids, "bf16")
    batches = [to_dev(wl.queries[b * n:(b + 1) * n], "bf16") for b in range(4)]

    def pair():
        copy, master = siso.SisoCache(wl.dim, wl.K, siso.FP8), siso.SisoCache(wl.dim, wl.K, siso.BF16)
        return copy, master

    copy, master = pair()
    copy.load(cents)
    master.load(cents)
    want_outs = []
    for q in batches:
        idx, sim, hit = copy.lookup(q, 0.85)
        master.update(q, idx, hit)
        copy.follow(master, idx, hit)
        want_outs.append((idx.clone(), sim.clone(), hit.clone()))
    torch.cuda.synchronize()
    want_state = copy.export_fp8() + master.export()
    assert sum(int(o[2].sum().item()) for o in want_outs) > n

    copy, master = pair()
    q_in = torch.empty_like(batches[0])
    idx = torch.empty(n, dtype=torch.int32, device="cuda:0")
    sim = torch.empty(n, dtype=torch.float32, device="cuda:0")
    hit = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    side = torch.cuda.Stream()
    copy.set_stream(side)
    master.set_stream(side)
    with torch.cuda.stream(side):
        copy.load(cents)
        master.load(cents)
        q_in.copy_(batches[0])
        copy.reserve(n)
        master.reserve(n)
        copy.lookup_update_with(master, q_in, 0.85, idx, sim, hit)   # warm-up: workspaces, kernel attributes
        copy.load(cents)                                              # back to the initial state
        master.load(cents)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        copy.lookup_update_with(master, q_in, 0.85, idx, sim, hit)
    for b, q in enumerate(batches):
        q_in.copy_(q)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(idx, want_outs[b][0]) and torch.equal(hit, want_outs[b][2]), f"replay {b}"
        assert torch.equal(sim, want_outs[b][1]), f"replay {b}: similarities"
    for c in (copy, master):
        c.set_stream(torch.cuda.current_stream())
    got_state = copy.export_fp8() + master.export()
    torch.cuda.synchronize()
    for g, w in zip(got_state, want_state):
        assert torch.equal(g, w)
    assert copy.bad_indices() == 0 and master.bad_indices() == 0
