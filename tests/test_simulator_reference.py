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
    for i, row in enumerate(rows):
        t, l, n, slo, frames = row[:5]
        a[i]["arrival_us"], a[i]["service"], a[i]["origin"], a[i]["slo_us"], a[i]["frames"] = t, l, n, slo, frames
        a[i]["fps_milli"] = row[5] if len(row) > 5 else 0
    return a


def both(N, L, c, hop, t, max_off, placements, rows, draws):
    ref = S.simulate(N, L, c, hop, t, max_off, placements, rows, draws)
    got = B.epara_simulate(N, L, c, hop, t, max_off, placements, _requests(rows), draws)
    assert got == ref
    return ref


# ---- hand-worked timelines ---------------------------------------------------------------------

def test_frequency_sensitive_streams_count_frames_in_proportion_to_the_achieved_rate():
    """Sec. 3.3: a stream of 120 frames that wants 80 fps on an instance that needs 25 ms per frame (40 fps) counts
    120 * 40 / 80 = 60; the same stream queued behind another one is served later, hence slower still; a stream
    that gets at least its rate counts every frame and no more."""
    c = [[25000]]
    r = both(1, 1, c, 0, 10 ** 6, 1, [0], [(0, 0, 0, 10 ** 9, 120, 80000)], [[0.5]])
    assert r == dict(satisfied=60.0, local=1, offloaded=0, timeout=0, offload_exceeded=0, insufficient=0)
    # a second stream arrives at the same time and waits for the first: 120 frames in 6 s = 20 fps -> 30 more
    r = both(1, 1, c, 0, 10 ** 6, 1, [0], [(0, 0, 0, 10 ** 9, 120, 80000), (0, 0, 0, 10 ** 9, 120, 80000)], [[0.5]] * 2)
    assert r["satisfied"] == 60.0 + 30.0 and r["local"] == 2
    # asked for 30 fps, gets 40: all 120 frames count, capped; a latency-sensitive request next to it counts one
    r = both(1, 1, c, 0, 10 ** 6, 1, [0, 0], [(0, 0, 0, 10 ** 9, 120, 30000), (0, 0, 0, 10 ** 9, 3, 0)], [[0.5]] * 2)
    assert r["satisfied"] == 121.0
    # a stream is refused only where no instance exists at all (and nobody else has one)
    r = both(2, 1, [[25000, 25000]], 0, 10 ** 6, 1, [], [(0, 0, 0, 10 ** 9, 10, 1000)], [[0.5]])
    assert r["satisfied"] == 0.0 and r["insufficient"] == 1

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


def test_compute_table_from_measured_passes_and_placement_over_it():
    """The lookup table c_ln (Sec. 3.3, Sec. 5 "Settings") built from a benchmark line's per-mix pass times, then
    Alg. 1 placing those services over the simulated objective: library pair = reference pair."""
    line = {"mixes": {"vit_b16_bf16_bf16": {"ms_per_step": 0.306, "requests": 75},          # the shape of bench.py's line
                      "llm_decode_bf16_bf16": {"ms_per_step": 0.221, "requests": 105},
                      "llm_prefill_bf16": {"ms_per_step": 2.816, "requests": 9}}}
    keys = ["vit_b16_bf16_bf16", "llm_decode_bf16_bf16", "llm_prefill_bf16"]
    speed = [1.0, 0.5, 0.0]                                  # this GPU, one half as fast, a server without a GPU
    c = B.compute_table_from_bench_line(line, keys, speed)
    # by hand: microseconds per request, rounded up; twice that on the slower server; 0 = cannot run
    assert c.tolist() == [[5, 9, 0], [3, 5, 0], [313, 626, 0]]
    assert c[0][0] == -(-306 // 75) and c[2][0] == -(-2816 // 9)
    assert status_of_table([0.0], [1], [1.0]) == B.EPARA_ERR_SHAPE and status_of_table([1.0], [0], [1.0]) == B.EPARA_ERR_SHAPE
    rng = np.random.default_rng(77)
    N, Lsvc = 3, 3
    rows = sorted((int(rng.integers(0, 3000)), int(rng.integers(0, Lsvc)), int(rng.integers(0, N)), int(rng.integers(300, 1500)), 1)
                  for _ in range(120))
    draws = rng.random((len(rows), 2))
    table = c.tolist()

    def feasible(theta):
        return all(sum(1 for p in theta if p % N == n) <= 2 for n in range(N))

    def phi_ref(theta):
        return S.simulate(N, Lsvc, table, 20, 500, 2, list(theta), rows, draws.tolist())["satisfied"] if feasible(theta) else -1.0

    def phi_lib(theta):
        return B.epara_simulate(N, Lsvc, c, 20, 500, 2, list(theta), _requests(rows), draws)["satisfied"] if feasible(theta) else -1.0

    X = [l * N + n for l in range(Lsvc) for n in range(N) if table[l][n] > 0]
    want = P.place_services([], X, [], phi_ref)
    got = B.epara_place_services([], X, [], phi_lib)
    assert list(got) == list(want) and len(want) > 0
    assert all(p % N != 2 for p in want)                     # nothing lands on the server that cannot run it
    assert phi_ref(want) > phi_ref([])


def status_of_table(ms, rq, speed):
    try:
        B.epara_compute_table(ms, rq, speed)
    except B.EparaError as e:
        return e.status
    return B.EPARA_OK
