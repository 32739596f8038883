"""The event-driven simulation behind the placement objective (Sec. 3.3 Eq. "optimal", Sec. 3.2 handler,
Sec. 5 "Settings"): the reference is pinned to hand-worked timelines and to invariants, the library must
reproduce the reference field for field, and the placement algorithms are run over it end to end."""
import ctypes

import numpy as np
import pytest

from oracle import planner as P
from oracle import simulator as S
from paper_2511_00603_amd import binding as B


def _requests(rows):
    a = np.zeros(len(rows), dtype=B.SIM_REQUEST)
    for i, (t, l, n, slo, frames) in enumerate(rows):
        a[i]["arrival_us"], a[i]["service"], a[i]["origin"], a[i]["slo_us"], a[i]["frames"] = t, l, n, slo, frames
    return a


def both(N, L, c, hop, t, max_off, placements, rows, draws):
    ref = S.simulate(N, L, c, hop, t, max_off, placements, rows, draws)
    got = B.epara_simulate(N, L, c, hop, t, max_off, placements, _requests(rows), draws)
    assert got == ref
    return ref


# ---- hand-worked timelines ---------------------------------------------------------------------

def test_one_instance_serves_in_order_and_refuses_what_would_be_late():
    c = [[10]]
    # arrivals 0, 5, 30, one frame each, 10 us per frame: finish at 10, 20 (queued behind the first), 40
    r = both(1, 1, c, 3, 100, 2, [0], [(0, 0, 0, 15, 1), (5, 0, 0, 15, 1), (30, 0, 0, 15, 1)], [[0.5, 0.5]] * 3)
    assert r == dict(satisfied=3.0, local=3, offloaded=0, timeout=0, offload_exceeded=0, insufficient=0)
    # the second one's deadline is 19 < 20: not served here, and there is nowhere else
    r = both(1, 1, c, 3, 100, 2, [0], [(0, 0, 0, 15, 1), (5, 0, 0, 14, 1), (30, 0, 0, 15, 1)], [[0.5, 0.5]] * 3)
    assert r == dict(satisfied=2.0, local=2, offloaded=0, timeout=0, offload_exceeded=0, insufficient=1)
    # a replica (the placement twice) takes it: finish at 15
    r = both(1, 1, c, 3, 100, 2, [0, 0], [(0, 0, 0, 15, 1), (5, 0, 0, 14, 1), (30, 0, 0, 15, 1)], [[0.5, 0.5]] * 3)
    assert r["satisfied"] == 3.0
    # frames multiply the service time: 3 frames = 30 us > SLO 25
    r = both(1, 1, c, 3, 100, 2, [0], [(0, 0, 0, 25, 3)], [[0.5, 0.5]])
    assert r["satisfied"] == 0.0 and r["insufficient"] == 1


def test_offload_hop_time_path_and_count():
    c = [[10, 10, 10]]
    # the service lives on server 2 only; a request entering at server 0 hops once (3 us) and finishes at 13
    r = both(3, 1, c, 3, 100, 2, [2], [(0, 0, 0, 13, 1)], [[0.0, 0.0]])
    assert r == dict(satisfied=1.0, local=1, offloaded=1, timeout=0, offload_exceeded=0, insufficient=0)
    # one microsecond less of SLO: it arrives, cannot finish in time there, and every other server either has
    # no instance or is on its path
    r = both(3, 1, c, 3, 100, 2, [2], [(0, 0, 0, 12, 1)], [[0.0, 0.0]])
    assert r == dict(satisfied=0.0, local=0, offloaded=1, timeout=0, offload_exceeded=0, insufficient=1)
    # two busy servers bounce a request until the offload count is used up:
    # instances on 1 and 2 are blocked by long requests (100 us), the third request's SLO is 20
    rows = [(0, 0, 1, 200, 10), (0, 0, 2, 200, 10), (1, 0, 0, 20, 1)]
    r = both(3, 1, c, 3, 1000, 1, [1, 2], rows, [[0.0]] * 3)
    assert r["local"] == 2 and r["offloaded"] == 1 and r["offload_exceeded"] == 1 and r["satisfied"] == 2.0
    # a slow hop makes it arrive after its deadline: timeout
    r = both(3, 1, c, 50, 1000, 2, [2], [(0, 0, 0, 20, 1)], [[0.0, 0.0]])
    assert r["timeout"] == 1 and r["satisfied"] == 0.0


def test_offloading_shares_follow_the_idle_goodput_of_the_known_window():
    # two destinations with 1 and 3 instances of equal speed: before any snapshot is known (now < 2t) the
    # shares are the theoretical goodputs, 1/4 and 3/4
    c = [[10, 10, 10]]
    placements = [1, 2, 2, 2]
    for u, dest_served in ((0.2, 1), (0.3, 2), (0.9, 2)):
        rows = [(0, 0, 0, 100, 1)]
        ref = S.simulate(3, 1, c, 1, 1000, 1, placements, rows, [[u]])
        assert ref["offloaded"] == 1 and ref["local"] == 1
        assert B.epara_simulate(3, 1, c, 1, 1000, 1, placements, _requests(rows), [[u]]) == ref
    # The known window shifts the shares.  Server 1 (one instance, 200 us per request: 5e3 per s) is too slow
    # for the SLO, server 2 (three instances, 10 us: 3e5 per s) is not, so `satisfied` tells where the request went.
    c = [[10, 200, 10]]
    u = 0.017                                               # between 5e3 / 3.05e5 = 0.0164 and 5e3 / 2.75e5 = 0.0182
    # nothing known yet (now < 2t): shares 5e3 : 3e5, the draw passes server 1 and lands on server 2
    r = both(3, 1, c, 1, 1000, 1, placements, [(250, 0, 0, 100, 1)], [[u]])
    assert r["satisfied"] == 1.0 and r["offloaded"] == 1
    # server 2 completed three requests in window 1 (t = 100): actual 3e4 per s, idle 2.7e5; the same draw now
    # stops at server 1, which cannot meet the deadline, and the offload count is used up
    rows = [(10 * i, 0, 2, 50, 1) for i in range(3)] + [(250, 0, 0, 100, 1)]
    r = both(3, 1, c, 1, 100, 1, placements, rows, [[u]] * 4)
    assert r["satisfied"] == 3.0 and r["offloaded"] == 1 and r["offload_exceeded"] == 1
    # one window later (now in [300, 400): window 2 is empty) the shares are back
    rows = [(10 * i, 0, 2, 50, 1) for i in range(3)] + [(350, 0, 0, 100, 1)]
    r = both(3, 1, c, 1, 100, 1, placements, rows, [[u]] * 4)
    assert r["satisfied"] == 4.0


# ---- invariants and the library against the reference -----------------------------------------

def _random_case(rng, n_requests):
    N, L = int(rng.integers(1, 6)), int(rng.integers(1, 4))
    c = rng.integers(0, 40, (L, N)).astype(np.int64)           # zeros: cannot run there
    placements = rng.integers(0, L * N, int(rng.integers(0, 3 * N))).tolist()
    rows = [(int(rng.integers(0, 2000)), int(rng.integers(0, L)), int(rng.integers(0, N)), int(rng.integers(0, 120)),
             int(rng.integers(1, 4))) for _ in range(n_requests)]
    max_off = int(rng.integers(0, 4))
    draws = rng.random((n_requests, max(max_off, 1)))[:, :max_off] if max_off else np.zeros((n_requests, 0))
    return N, L, c, int(rng.integers(0, 30)), int(rng.integers(1, 400)), max_off, placements, rows, draws


@pytest.mark.parametrize("seed", range(40))
def test_library_reproduces_the_reference_and_every_request_ends_exactly_once(seed):
    rng = np.random.default_rng(9000 + seed)
    N, L, c, hop, t, max_off, placements, rows, draws = _random_case(rng, int(rng.integers(0, 120)))
    r = both(N, L, c.tolist(), hop, t, max_off, placements, rows, draws.tolist())
    assert r["local"] + r["timeout"] + r["offload_exceeded"] + r["insufficient"] == len(rows)
    assert r["satisfied"] == r["local"] and r["offloaded"] <= max_off * len(rows)
    if not placements:
        assert r["satisfied"] == 0.0


def test_no_placement_no_service_and_enough_capacity_serves_everything():
    rows = [(7 * i, i % 2, i % 3, 50, 1) for i in range(60)]
    c = [[5, 5, 5], [5, 5, 5]]
    everywhere = [l * 3 + n for l in range(2) for n in range(3)]
    r = both(3, 2, c, 2, 100, 2, everywhere, rows, [[0.1, 0.2]] * 60)
    assert r["satisfied"] == 60.0 and r["offloaded"] == 0
    assert both(3, 2, c, 2, 100, 2, [], rows, [[0.1, 0.2]] * 60)["satisfied"] == 0.0


def test_error_codes():
    L = B.lib()
    cfg = B.SimConfig(None, 1, 100, 1, 1, 1, 0)
    res = B.SimResult()
    assert L.epara_simulate(None, None, 0, None, 0, None, ctypes.addressof(res)) == B.EPARA_ERR_NULL
    assert L.epara_simulate(ctypes.addressof(cfg), None, 0, None, 0, None, ctypes.addressof(res)) == B.EPARA_ERR_NULL   # no table
    c = np.array([10], dtype=np.int64)
    cfg.compute_us = c.ctypes.data
    assert L.epara_simulate(ctypes.addressof(cfg), None, 0, None, 0, None, ctypes.addressof(res)) == B.EPARA_OK
    cfg.sync_delay_us = 0
    assert L.epara_simulate(ctypes.addressof(cfg), None, 0, None, 0, None, ctypes.addressof(res)) == B.EPARA_ERR_SHAPE
    def status(**kw):
        a = dict(placements=[0], rows=[(0, 0, 0, 10, 1)], draws=[[0.5]])
        a.update(kw)
        try:
            B.epara_simulate(1, 1, [[10]], 1, 100, 1, a["placements"], _requests(a["rows"]), a["draws"])
        except B.EparaError as e:
            return e.status
        return B.EPARA_OK
    assert status() == B.EPARA_OK
    assert status(placements=[1]) == B.EPARA_ERR_SHAPE
    assert status(rows=[(0, 1, 0, 10, 1)]) == B.EPARA_ERR_SHAPE
    assert status(rows=[(0, 0, 0, 10, 0)]) == B.EPARA_ERR_SHAPE
    assert status(draws=[[1.0]]) == B.EPARA_ERR_SHAPE


# ---- placement over the simulated objective, end to end ---------------------------------------------

def test_placement_algorithms_over_the_simulated_objective():
    """Alg. 1 with phi = the simulation: library placement + library simulation against the all-Python pair,
    and against exhaustive search on an instance small enough for it."""
    rng = np.random.default_rng(4242)
    N, Lsvc = 3, 2
    c = [[8, 12, 10], [20, 15, 0]]
    rows = sorted((int(rng.integers(0, 600)), int(rng.integers(0, Lsvc)), int(rng.integers(0, N)), int(rng.integers(20, 60)), 1)
                  for _ in range(80))
    draws = rng.random((len(rows), 2))
    capacity = 2                                            # instances a server can hold: part of the caller's objective

    def feasible(theta):
        return all(sum(1 for p in theta if p % N == n) <= capacity for n in range(N))

    def phi_ref(theta):
        return S.simulate(N, Lsvc, c, 2, 100, 2, list(theta), rows, draws.tolist())["satisfied"] if feasible(theta) else -1.0

    def phi_lib(theta):
        return B.epara_simulate(N, Lsvc, c, 2, 100, 2, list(theta), _requests(rows), draws)["satisfied"] if feasible(theta) else -1.0

    X = [l * N + n for l in range(Lsvc) for n in range(N) if c[l][n] > 0]
    want = P.place_services([], X, [], phi_ref)
    got = B.epara_place_services([], X, [], phi_lib)
    assert list(got) == list(want) and len(want) > 0
    best = max(phi_ref(theta) for k in range(0, 5) for theta in __import__("itertools").combinations_with_replacement(X, k))
    assert phi_ref(want) <= best
    assert phi_ref(want) >= best / 3                        # greedy on a monotone objective: far from arbitrary
    assert phi_ref(want) > phi_ref([])
