"""Pins for the LRU offload oracle, and (no GPU needed: the simulation is host code) parity of
the library's blockffn_offload_sim against it."""

import ctypes

import numpy as np
import pytest

from oracle import offload_sim as osim
from paper_2507_08771_amd import binding as B


def lists_from_sets(sets, E):
    idx = np.full((len(sets), E), -1, dtype=np.int32)
    n = np.zeros(len(sets), dtype=np.int32)
    for c, s in enumerate(sets):
        v = sorted(s)
        idx[c, :len(v)] = v
        n[c] = len(v)
    return idx, n


def random_stream(seed, n_chunks, E, p, stay=0.8):
    """Chunk sets that drift: each expert keeps its state with probability `stay`."""
    rng = np.random.default_rng(seed)
    cur = rng.random(E) < p
    out = []
    for _ in range(n_chunks):
        redraw = rng.random(E) >= stay
        cur = np.where(redraw, rng.random(E) < p, cur)
        out.append(set(np.nonzero(cur)[0].tolist()))
    return out


def loads_by_stack_distance(sets, capacity):
    """Mattson's characterisation of LRU: a touch hits iff fewer than `capacity` distinct other
    experts were touched since the previous touch of the same expert."""
    trace = [e for s in sets for e in sorted(s)]
    loads = 0
    last = {}
    for pos, e in enumerate(trace):
        if e not in last or len(set(trace[last[e] + 1:pos])) >= capacity:
            loads += 1
        last[e] = pos
    return loads


@pytest.mark.parametrize("E,n_chunks,p", [(8, 40, 0.4), (64, 60, 0.2), (130, 30, 0.1)])
def test_lru_matches_stack_distance_characterisation(E, n_chunks, p):
    sets = random_stream(E, n_chunks, E, p)
    idx, n = lists_from_sets(sets, E)
    prev = None
    for capacity in sorted({0, 1, 2, 5, E // 4, E // 2, E, E + 3}):
        loads, totals = osim.lru_offload(idx, n, capacity)
        assert totals[0] == n.sum() and totals[1] == loads.sum()
        assert totals[1] == loads_by_stack_distance(sets, capacity)
        # what was loaded and not evicted is still resident: the cache ends holding min(capacity, distinct)
        assert totals[2] == totals[1] - min(capacity, len(set().union(*sets))) if capacity else totals[2] == 0
        if prev is not None:
            assert totals[1] <= prev        # inclusion property: a larger LRU cache never loads more
        prev = totals[1]


def test_lru_closed_forms():
    E = 16
    # a cache that holds every expert only ever takes the cold loads
    sets = random_stream(1, 50, E, 0.3)
    idx, n = lists_from_sets(sets, E)
    _, totals = osim.lru_offload(idx, n, E)
    assert totals[1] == len(set().union(*sets)) and totals[2] == 0
    # identical chunks: one load per expert, then hits only
    idx, n = lists_from_sets([{1, 4, 9}] * 10, E)
    loads, totals = osim.lru_offload(idx, n, 3)
    assert loads.tolist() == [3] + [0] * 9 and totals.tolist() == [30, 3, 0]
    # a cyclic sweep over capacity + 1 experts defeats LRU completely
    idx, n = lists_from_sets([{0, 1, 2, 3, 4}] * 6, E)
    _, totals = osim.lru_offload(idx, n, 4)
    assert totals[1] == totals[0] == 30
    # alternating disjoint sets that fit together stay resident; with half the room they thrash
    idx, n = lists_from_sets([{0, 1}, {2, 3}] * 5, E)
    assert osim.lru_offload(idx, n, 4)[1][1] == 4
    assert osim.lru_offload(idx, n, 2)[1][1] == 20
    # no room at all: every touch is a load
    assert osim.lru_offload(idx, n, 0)[1].tolist() == [20, 20, 0]


def lib_offload(idx, n, capacity, per_chunk=True):
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    n = np.ascontiguousarray(n, dtype=np.int32)
    loads = np.full(len(n), -7, dtype=np.int64)
    totals = np.full(3, -7, dtype=np.int64)
    rc = B.lib().blockffn_offload_sim(idx.ctypes.data_as(ctypes.c_void_p), n.ctypes.data_as(ctypes.c_void_p),
                                      len(n), idx.shape[1], capacity,
                                      loads.ctypes.data_as(ctypes.c_void_p) if per_chunk else None,
                                      totals.ctypes.data_as(ctypes.c_void_p))
    assert rc == B.OK
    return loads, totals


@pytest.mark.parametrize("E,n_chunks,p", [(8, 40, 0.4), (64, 300, 0.2), (130, 50, 0.1), (256, 40, 0.05)])
def test_library_simulation_matches_oracle(E, n_chunks, p):
    sets = random_stream(E + 1, n_chunks, E, p)
    sets[3] = set()
    idx, n = lists_from_sets(sets, E)
    for capacity in (0, 1, 3, E // 4, E // 2, E, E + 9):
        loads, totals = lib_offload(idx, n, capacity)
        r_loads, r_totals = osim.lru_offload(idx, n, capacity)
        np.testing.assert_array_equal(loads, r_loads)
        np.testing.assert_array_equal(totals, r_totals)
    np.testing.assert_array_equal(lib_offload(idx, n, 5, per_chunk=False)[1], osim.lru_offload(idx, n, 5)[1])


def test_library_simulation_argument_checks():
    lib = B.lib()
    idx, n = lists_from_sets([{0, 1}], 4)
    totals = np.zeros(3, dtype=np.int64)
    p = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    assert lib.blockffn_offload_sim(None, p(n), 1, 4, 2, None, p(totals)) == B.ERR_INVALID
    assert lib.blockffn_offload_sim(p(idx), None, 1, 4, 2, None, p(totals)) == B.ERR_INVALID
    assert lib.blockffn_offload_sim(p(idx), p(n), 1, 4, 2, None, None) == B.ERR_INVALID
    assert lib.blockffn_offload_sim(p(idx), p(n), -1, 4, 2, None, p(totals)) == B.ERR_INVALID
    assert lib.blockffn_offload_sim(p(idx), p(n), 1, 0, 2, None, p(totals)) == B.ERR_INVALID
    assert lib.blockffn_offload_sim(p(idx), p(n), 1, 4, -1, None, p(totals)) == B.ERR_INVALID
    assert lib.blockffn_offload_sim(p(idx), p(n), 1, 300, 2, None, p(totals)) == B.ERR_UNSUPPORTED
    bad = idx.copy()
    bad[0, 1] = 7                                   # expert index outside [0, N_e)
    assert lib.blockffn_offload_sim(p(bad), p(n), 1, 4, 2, None, p(totals)) == B.ERR_INVALID
    n_bad = np.array([5], dtype=np.int32)           # more slots than experts
    assert lib.blockffn_offload_sim(p(idx), p(n_bad), 1, 4, 2, None, p(totals)) == B.ERR_INVALID
    assert lib.blockffn_offload_sim(p(idx), p(n), 0, 4, 2, None, p(totals)) == B.OK and not totals.any()
