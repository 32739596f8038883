"""Pins for the reference planner: invariants of the tiling rule, closed-form counts
for the decode and prefill mixes, and the worked numbers the paper prints for the
batch-accounting equations of Sec. 4.1 (tests/golden/paper_worked_numbers.txt)."""
import os

import numpy as np
import pytest

from oracle import planner as P

CLASSES = [(64, 64, 32), (P.INT32_MAX, 256, 256)]
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_worked_numbers.txt")


def coverage(groups, tiles):
    cov = [np.zeros((M, N), dtype=np.int32) for M, _K, N in groups]
    for g, m0, n0, rows, cols, _c in tiles:
        cov[g][m0:m0 + rows, n0:n0 + cols] += 1
    return cov


@pytest.mark.parametrize("groups", [
    [(4, 256, 512), (16, 256, 512)],
    [(1, 8, 10)],
    [(0, 8, 8), (65, 16, 257), (64, 32, 33), (0, 4, 4)],
    [(197, 768, 2304), (6304, 768, 3072), (255, 8, 256), (256, 8, 256), (257, 8, 255)],
])
def test_tiles_partition_every_output_exactly_once(groups):
    row_off, x_off, y_off, tiles = P.plan_groups(groups, CLASSES)
    assert row_off[0] == x_off[0] == y_off[0] == 0
    assert row_off[-1] == sum(g[0] for g in groups)
    assert x_off[-1] == sum(g[0] * g[1] for g in groups)
    assert y_off[-1] == sum(g[0] * g[2] for g in groups)
    assert all(b >= a for a, b in zip(row_off, row_off[1:]))
    for cov in coverage(groups, tiles):
        assert np.all(cov == 1)
    keys = [(t[0], t[1], t[2]) for t in tiles]
    assert keys == sorted(keys) and len(set(keys)) == len(keys)       # canonical, strictly increasing
    assert all(t[3] >= 1 and t[4] >= 1 for t in tiles)
    expect = 0
    for M, _K, N in groups:
        if M:
            _, bm, bn = CLASSES[P.pick_class(M, CLASSES)]
            expect += -(-M // bm) * -(-N // bn)
    assert len(tiles) == expect


def test_class_choice_and_empty_groups():
    assert P.pick_class(1, CLASSES) == 0 and P.pick_class(64, CLASSES) == 0 and P.pick_class(65, CLASSES) == 1
    _, _, _, tiles = P.plan_groups([(0, 4, 4)], CLASSES)
    assert tiles == []
    assert P.plan_groups([], CLASSES) == ([0], [0], [0], [])
    with pytest.raises(ValueError):
        P.plan_groups([(1, 0, 4)], CLASSES)
    with pytest.raises(ValueError):
        P.plan_groups([(1, 4, 4)], [(64, 64, 32), (64, 256, 256)])
    with pytest.raises(ValueError):
        P.plan_groups([(100, 4, 4)], [(64, 64, 32)])


def test_closed_form_counts_decode_and_prefill():
    # decode mix: 4 services, M <= 64, gate/up phase seen as N = 11008 hidden columns
    dec = [(m, 4096, 11008) for m in (1, 8, 32, 64)]
    _, _, _, t = P.plan_groups(dec, CLASSES)
    assert len(t) == 4 * (11008 // 32)
    # prefill mix: rows 4692 and 3500; gate/up phase with 128 hidden columns per tile
    pre = [(4692, 5120, 13824), (3500, 5120, 13824)]
    _, _, _, t = P.plan_groups(pre, [(64, 64, 32), (P.INT32_MAX, 256, 128)])
    assert len(t) == (19 + 14) * 108
    row_off, x_off, y_off, t = P.plan_groups([(4692, 13824, 5120), (3500, 13824, 5120)], CLASSES)
    assert len(t) == (19 + 14) * 20 and row_off == [0, 4692, 8192]
    assert x_off[-1] == 8192 * 13824 and y_off[-1] == 8192 * 5120
    last = t[19 * 20 - 1]
    assert last == (0, 18 * 256, 19 * 256, 4692 - 18 * 256, 256, 1)


@pytest.mark.parametrize("W,X", [(256, 8), (8, 8), (16, 1), (24, 4)])
def test_schedule_is_a_permutation_with_idle_padding(W, X):
    groups = [(700, 64, 900), (3, 128, 100), (300, 256, 300), (64, 32, 64)]
    _, _, _, tiles = P.plan_groups(groups, CLASSES)
    order = P.schedule_tiles(groups, CLASSES, 1, tiles, W, X, 8, 4)
    assert len(order) % W == 0
    used = [t for t in order if t >= 0]
    assert sorted(used) == list(range(len(tiles)))
    # a workgroup's list has no holes, and its panel tiles come before its streaming tiles
    for b in range(W):
        mine = order[b::W]
        live = [t for t in mine if t >= 0]
        assert mine[:len(live)] == live
        kinds = [tiles[t][5] for t in live]
        assert kinds == sorted(kinds, reverse=True)


def test_streaming_tiles_are_balanced_longest_first():
    # decode-like launch with a K too short to be split: three streaming classes, every tile of a group costs cols * K
    classes = [(16, 16, 32), (32, 32, 64), (64, 64, 128), (P.INT32_MAX, 256, 256)]
    groups = [(1, 2048, 4096), (8, 2048, 4096), (32, 2048, 4096), (64, 2048, 4096)]
    _, _, _, tiles = P.plan_groups(groups, classes)
    assert len(tiles) == 128 + 128 + 64 + 32
    W = 256
    order = P.schedule_tiles(groups, classes, 3, tiles, W, 8, 8, 4)
    cost = lambda t: 2048 * (6 * tiles[t][4] + (2 * classes[tiles[t][5]][1] if classes[tiles[t][5]][1] >= 32 else 0))     # weight columns, and activation rows at a third
    loads = [sum(cost(t) for t in order[b::W] if t >= 0) for b in range(W)]
    total = sum(cost(t) for t in range(len(tiles)))
    # greedy longest-first never exceeds the mean by more than one largest tile
    assert max(loads) <= total / W + 2048 * (6 * 128 + 128)
    assert max(loads) == 2048 * (6 * 128 + 128)             # a wide tile is all its owner gets
    # the widest tiles are visited first by whoever owns them
    firsts = [tiles[order[b]][4] for b in range(W)]
    assert sorted(firsts, reverse=True)[:32] == [128] * 32
    # the narrow table halves the widest tiles and the makespan
    narrow = classes[:2] + [(64, 64, 64)] + classes[3:]
    _, _, _, t2 = P.plan_groups(groups, narrow)
    o2 = P.schedule_tiles(groups, narrow, 3, t2, W, 8, 8, 4)
    rows = lambda bm: 2 * bm if bm >= 32 else 0
    loads2 = [sum(2048 * (6 * t2[t][4] + rows(narrow[t2[t][5]][1])) for t in o2[b::W] if t >= 0) for b in range(W)]
    assert max(loads2) <= 2048 * (6 * 64 + 128 + 6 * 32) and max(loads2) < 0.6 * max(loads)
    # gated groups stream two weight matrices: the column part of the cost doubles, the row part does not
    o2 = P.schedule_tiles([g + (True,) for g in groups], classes, 3, tiles, W, 8, 8, 4)
    gcost = lambda t: 2048 * (12 * tiles[t][4] + rows(classes[tiles[t][5]][1]))
    assert max(sum(gcost(t) for t in o2[b::W] if t >= 0) for b in range(W)) == 2048 * (12 * 128 + 128)


def test_long_k_streaming_tiles_are_visited_in_parts():
    """A single launch cuts the K of the 32- and 64-row classes' tiles in two when K >= 8192: every part once,
    items longest first, and the widest tile no longer sets the makespan."""
    classes = [(16, 16, 32, 0), (32, 32, 64, 8192), (64, 64, 128, 8192), (P.INT32_MAX, 256, 256, 0)]
    assert [P.split_parts(K, cl) for K, cl in ((4096, classes[1]), (8191, classes[2]), (8192, classes[1]), (11008, classes[2]),
                                               (11008, classes[0]), (1 << 20, (64, 64, 64)), (1 << 20, (64, 64, 64, 1 << 20)))] == \
        [1, 1, 2, 2, 1, 1, 2]
    for K, parts in ((11008, 2), (8192, 2)):
        groups = [(1, K, 4096), (8, K, 4096), (32, K, 4096), (64, K, 4096)]
        _, _, _, tiles = P.plan_groups(groups, classes)
        W = 256
        order = P.schedule_tiles(groups, classes, 3, tiles, W, 8, 8, 4)
        seen = {}
        for e in order:
            if e >= 0:
                t, j, n = P.order_decode(e)
                assert P.order_entry(t, j, n) == e
                seen.setdefault(t, []).append((j, n))
        assert sorted(seen) == list(range(len(tiles)))
        for t, v in seen.items():
            want = parts if tiles[t][5] >= 1 else 1
            assert sorted(v) == [(j, want) for j in range(want)]
        whole = lambda t: K * (6 * tiles[t][4] + (2 * classes[tiles[t][5]][1] if classes[tiles[t][5]][1] >= 32 else 0))
        def item(e):
            t, _, n = P.order_decode(e)
            return whole(t) if n == 1 else whole(t) // n + 24 * classes[tiles[t][5]][1] * tiles[t][4]
        loads = [sum(item(e) for e in order[b::W] if e >= 0) for b in range(W)]
        biggest = max(item(e) for e in order if e >= 0)
        assert max(loads) <= sum(loads) / W + biggest
        assert max(loads) < 0.8 * K * (6 * 128 + 128)       # an unsplit wide tile alone costs that
        # a chain of launches does not split
        o2 = P.schedule_chain([(groups, classes, 3, tiles), (groups, classes, 3, tiles)], W, 8, 8, 4)
        assert all(e < (1 << 24) for o in o2 for e in o)
    base, n, nbytes = P.split_layout([(64, 11008, 4096), (8, 11008, 4096), (0, 11008, 4096), (32, 8192, 100), (200, 11008, 4096), (40, 8191, 512)], classes, 3)
    assert base == [0, -1, -1, 32, -1, -1] and n == 32 + 2 and nbytes == 256 + 34 * 4 * 32768


def test_panel_tiles_of_unequal_k_are_balanced_and_equal_ones_go_round_robin():
    classes = [(64, 64, 32), (P.INT32_MAX, 256, 256)]
    # equal cost: the l-th tile of the sequence goes to die-major rank l mod W, i.e. workgroup (r mod W/X) * X + r div W/X
    groups = [(700, 64, 900), (300, 64, 300), (1000, 64, 513)]
    _, _, _, tiles = P.plan_groups(groups, classes)
    W, X = 24, 4
    order = P.schedule_tiles(groups, classes, 1, tiles, W, X, 1, 1)
    # panels of 1 x 1: inside a group the n index outermost, the m index fastest; equal K keeps the groups in order
    by_group = {g: [t for t in range(len(tiles)) if tiles[t][0] == g] for g in range(3)}
    want = []
    for g in range(3):
        TN = -(-groups[g][2] // 256); TM = -(-groups[g][0] // 256)
        want += [by_group[g][tm * TN + tn] for tn in range(TN) for tm in range(TM)]
    got = {}
    for slot, t in enumerate(order):
        if t >= 0:
            got.setdefault(slot % W, []).append(t)
    for l, t in enumerate(want):
        r = l % W
        b = (r % (W // X)) * X + r // (W // X)
        assert got[b][l // W] == t
    # unequal K: the long tiles first, one per workgroup; the short ones fill up the others, and no workgroup
    # exceeds the mean by more than one short tile... nor falls short of it by more than one long one
    groups = [(256 * 5, 3072, 256 * 3), (256 * 9, 768, 256 * 7)]
    _, _, _, tiles = P.plan_groups(groups, classes)
    W = 32
    order = P.schedule_tiles(groups, classes, 1, tiles, W, 8, 1, 4)
    loads = [sum(2040 * groups[tiles[t][0]][1] for t in order[b::W] if t >= 0) for b in range(W)]
    assert sum(loads) == 2040 * (15 * 3072 + 63 * 768)
    assert max(loads) <= sum(loads) / W + 2040 * 768 and min(loads) >= sum(loads) / W - 2040 * 3072
    rr = [0] * W                                              # plain round robin over the same sequence, for comparison
    for l in range(15 + 63):
        rr[l % W] += 2040 * (3072 if l < 15 else 768)
    assert max(loads) < max(rr)


def test_schedule_keeps_a_die_on_one_panel():
    # one group whose grid is a whole number of 8x4 panels: the 32 tiles that run together on one
    # die (slots congruent mod 8 within a round of 256) are exactly one panel
    groups = [(16 * 256, 64, 16 * 256)]
    _, _, _, tiles = P.plan_groups(groups, CLASSES)
    order = P.schedule_tiles(groups, CLASSES, 1, tiles, 256, 8, 8, 4)
    assert len(order) == 256
    for x in range(8):
        mine = [tiles[order[s]] for s in range(x, 256, 8)]
        ms = sorted({t[1] // 256 for t in mine})
        ns = sorted({t[2] // 256 for t in mine})
        assert len(ms) == 8 and len(ns) == 4 and ms[-1] - ms[0] == 7 and ns[-1] - ns[0] == 3


def test_batch_rows_accounting():
    M, first = P.batch_rows([[197] * 3, [], [5, 0, 7]])
    assert M == [591, 0, 12] and first == [[0, 197, 394], [], [0, 5, 5]]


def test_paper_worked_numbers():
    seen = 0
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, args, expect, _cite = [f.strip() for f in line.split(";", 3)]
        a = [int(v) for v in args.split()]
        if name == "dp_group_count":
            assert P.dp_group_count(*a) == int(expect)
        elif name == "inter_request_count":
            assert P.inter_request_count(*a) == int(expect)
        elif name == "satisfied_frames":
            # through the reference simulation and the library: one stream of a[0] frames that wants a[2] fps on an
            # instance that delivers a[1] fps (1e6 / a[1] us per frame, rounded to whole microseconds)
            from oracle import simulator as S
            from paper_2511_00603_amd import binding as B
            frames, achieved, wanted = a
            c = [[round(1e6 / achieved)]]
            ref = S.simulate(1, 1, c, 0, 10 ** 6, 0, [0], [(0, 0, 0, 10 ** 9, frames, 1000 * wanted)], [[]])
            req = np.zeros(1, dtype=B.SIM_REQUEST)
            req[0]["slo_us"], req[0]["frames"], req[0]["fps_milli"] = 10 ** 9, frames, 1000 * wanted
            got = B.epara_simulate(1, 1, c, 0, 10 ** 6, 0, [0], req, np.zeros((1, 0)))
            assert got == ref and ref["local"] == 1
            assert abs(ref["satisfied"] - int(expect)) < 1e-3 * int(expect)
        else:
            raise AssertionError(name)
        seen += 1
    assert seen >= 6


# ---- allocator helpers (Sec. 3.1 operator table, Sec. 4.1 MF bound, DP dealing) ----------------------

PAPER_OPERATOR_TABLE = {            # Sec. 3.1 "Performing operators to categories", the four paragraphs
    ("latency", False): {"BS", "MT"},
    ("latency", True): {"BS", "MT", "MP"},
    ("frequency", False): {"MF", "MT", "BS"},
    ("frequency", True): {"MF", "MT", "BS", "DP", "MP"},
}


def test_operator_sets_are_the_papers_four_categories():
    from paper_2511_00603_amd import binding as B
    for (cat, multi), names in PAPER_OPERATOR_TABLE.items():
        assert set(P.operator_set(cat == "frequency", multi)) == names
        bits = B.epara_operator_set(B.EPARA_CAT_FREQUENCY if cat == "frequency" else B.EPARA_CAT_LATENCY, multi)
        assert bits == sum(P.OPERATORS[n] for n in names)
    assert B.epara_operator_set(7, 0) == -1
    # DP only ever appears together with MP and MF (the fourth category)
    assert all(("DP" not in v) or {"MP", "MF"} <= v for v in PAPER_OPERATOR_TABLE.values())


def test_max_inter_frame_count_keeps_the_latency_of_a_batched_stream_within_its_requirement():
    from paper_2511_00603_amd import binding as B
    # MF frames per batch -> latency MF / fps (Sec. 4.1): at 60 fps a 66.7 ms budget admits 4 frames, 66.6 ms only 3
    assert P.max_inter_frame_count(66667, 60000) == B.epara_max_inter_frame_count(66667, 60000) == 4
    assert P.max_inter_frame_count(66666, 60000) == B.epara_max_inter_frame_count(66666, 60000) == 3
    assert B.epara_max_inter_frame_count(1, 30000) == 1                 # never below one frame
    assert B.epara_max_inter_frame_count(-1, 30000) == -1 and B.epara_max_inter_frame_count(5, 0) == -1
    rng = np.random.default_rng(5)
    for _ in range(200):
        lat, fps = int(rng.integers(0, 10**7)), int(rng.integers(1, 240001))
        mf = B.epara_max_inter_frame_count(lat, fps)
        assert mf == P.max_inter_frame_count(lat, fps)
        assert mf == 1 or (mf * 10**9 <= lat * fps < (mf + 1) * 10**9)   # MF/fps <= latency < (MF+1)/fps


def test_dp_deal_is_round_robin_over_the_stream():
    from paper_2511_00603_amd import binding as B
    per, who = B.epara_dp_deal(0, 9, 2)
    assert who.tolist() == [0, 1, 0, 1, 0, 1, 0, 1, 0] and per.tolist() == [5, 4]     # frames alternate between two groups
    rng = np.random.default_rng(6)
    for _ in range(100):
        first, n, k = int(rng.integers(0, 1000)), int(rng.integers(0, 200)), int(rng.integers(1, 9))
        per, who = B.epara_dp_deal(first, n, k)
        want_per, want_who = P.dp_deal(first, n, k)
        assert per.tolist() == want_per and who.tolist() == want_who
        assert per.sum() == n and per.max() - per.min() <= 1
        # dealing a stream in two pieces continues the rotation
        cut = int(rng.integers(0, n + 1))
        a, b = B.epara_dp_deal(first, cut, k), B.epara_dp_deal(first + cut, n - cut, k)
        assert np.array_equal(np.concatenate([a[1], b[1]]), who) and np.array_equal(a[0] + b[0], per)
    with pytest.raises(B.EparaError):
        B.epara_dp_deal(0, 5, 0)
    with pytest.raises(B.EparaError):
        B.epara_dp_deal(-1, 5, 2)
    # with the group count the paper's equation gives, every group stays within its own frame rate
    need, one = 97, 49
    k = B.epara_dp_group_count(need, one)
    per, _ = B.epara_dp_deal(0, need, k)
    assert k == 2 and per.max() <= one


# ---- service placement (Sec. 3.3, Alg. 1 and 2) ---------------------------------------------------------

def coverage_phi(requests_of, capacity, n_servers):
    """A small stand-in for the paper's objective: placement id = service * n_servers + server; a server holds at
    most `capacity` placements (later ones are ignored, as a full GPU would ignore them); phi = number of
    distinct requests covered.  Monotone and submodular, with a partition-matroid constraint inside."""
    def phi(theta):
        load, covered = {}, set()
        for x in theta:
            srv = x % n_servers
            if load.get(srv, 0) >= capacity:
                continue
            load[srv] = load.get(srv, 0) + 1
            covered |= requests_of[x]
        return float(len(covered))
    return phi


def test_alg2_on_a_modular_objective_takes_exactly_the_useful_placements_best_first():
    from paper_2511_00603_amd import binding as B
    w = {0: 3.0, 1: 0.0, 2: 5.0, 3: 1.0, 4: 0.0}
    phi = lambda theta: sum(w[x] for x in set(theta))
    cand = [0, 1, 2, 3, 4]
    # strict rule (steps S2, S3): only placements that raise phi, in descending order of gain; a set offers
    # chosen placements again, but a repeat adds nothing and ends the loop
    assert P.place_full_models(cand, True, False, [], phi) == [2, 0, 3]
    # S1 rule on a list: every listed configuration is placed, the useless ones too (gain 0 is kept), earliest first
    assert P.place_full_models(cand, False, True, [], phi) == [2, 0, 3, 1, 4]
    for is_set, keep in ((True, False), (False, True), (False, False)):
        assert B.epara_place_full_models(cand, is_set, keep, [], phi) == P.place_full_models(cand, is_set, keep, [], phi)
    # the list it starts from is kept in front
    assert B.epara_place_full_models(cand, True, False, [3], phi) == [3, 2, 0]


def test_alg2_matches_the_reference_and_the_greedy_bound_on_small_coverage_instances():
    import itertools
    from paper_2511_00603_amd import binding as B
    rng = np.random.default_rng(9)
    for trial in range(25):
        n_services, n_servers, capacity = int(rng.integers(2, 5)), int(rng.integers(1, 4)), int(rng.integers(1, 3))
        ids = [l * n_servers + n for l in range(n_services) for n in range(n_servers)]
        requests_of = {x: set(int(r) for r in rng.choice(12, size=rng.integers(0, 6), replace=False)) for x in ids}
        phi = coverage_phi(requests_of, capacity, n_servers)
        got = B.epara_place_full_models(ids, True, False, [], phi)
        assert got == P.place_full_models(ids, True, False, [], phi)
        # the best any placement list can do (one list per choice of <= capacity placements per server)
        per_server = [[x for x in ids if x % n_servers == s] for s in range(n_servers)]
        best = 0.0
        for pick in itertools.product(*[[c for k in range(capacity + 1) for c in itertools.combinations(ps, k)] for ps in per_server]):
            best = max(best, phi([x for grp in pick for x in grp]))
        assert phi(got) >= best / 2.0            # greedy on a monotone submodular objective under a matroid: at least half
        assert len(got) == len(set(got))         # a repeated placement never raises phi here, so none is kept


def test_alg1_runs_the_three_steps_in_order_and_errors_are_reported():
    from paper_2511_00603_amd import binding as B
    n_servers = 2
    requests_of = {0: {1, 2}, 1: {2, 3}, 2: {4}, 3: {1, 2, 3, 4, 5}, 100: {6, 7}, 101: set()}
    phi = coverage_phi(requests_of, 2, n_servers)
    partial, X, X_dot = [2, 101], [0, 1, 2, 3], [100, 101]
    want = P.place_services(partial, X, X_dot, phi)
    assert want[:2] == [2, 101]                  # S1 keeps both prioritised configurations, the useless one too
    assert 100 in want and want.index(100) > want.index(3)      # S3 comes after S2
    assert B.epara_place_services(partial, X, X_dot, phi) == want
    assert B.epara_place_services([], [], [], phi) == []
    with pytest.raises(B.EparaError) as e:
        B.epara_place_full_models([0, 2], True, False, [], phi, cap=1)          # two useful placements, room for one
    assert e.value.status == B.EPARA_ERR_CAPACITY
    with pytest.raises(B.EparaError) as e:
        B.epara_place_full_models([0, -1], True, False, [], phi)
    assert e.value.status == B.EPARA_ERR_SHAPE
    # an objective that never stops growing is cut off by the capacity instead of looping for ever
    with pytest.raises(B.EparaError) as e:
        B.epara_place_full_models([0], True, False, [], lambda theta: float(len(theta)), cap=50)
    assert e.value.status == B.EPARA_ERR_CAPACITY


# ---- request handling (Sec. 3.2) -----------------------------------------------------------------------

def test_handler_steps_come_in_the_papers_order():
    from paper_2511_00603_amd import binding as B
    th, ac, qu = [10.0, 8.0, 6.0], [10.0, 2.0, 3.0], [0, 0, 0]
    both = lambda *a: (B.epara_handle_request(*a), P.handle_request(*a))
    g, w = both(101, 100, True, 0, 5, th, ac, qu, 0, 10, 50, 0.3);  assert g == w == ("timeout", None)      # a late request is dropped even if it could be served
    g, w = both(100, 100, True, 9, 5, th, ac, qu, 0, 10, 50, 0.3);  assert g == w == ("local", None)        # local first, whatever the offload count
    g, w = both(0, 100, False, 5, 5, th, ac, qu, 0, 10, 50, 0.3);   assert g == w == ("offload_exceeded", None)
    g, w = both(0, 100, False, 4, 5, th, ac, qu, 0, 10, 50, 0.3);   assert g == w and g[0] == "offload" and g[1] in (1, 2)
    g, w = both(0, 100, False, 0, 5, th, th, qu, 0, 10, 50, 0.3);   assert g == w == ("insufficient", None)   # nobody has idle goodput
    g, w = both(0, 100, False, 0, 5, th, ac, [0, 61, 61], 0, 10, 50, 0.3); assert g == w == ("insufficient", None)  # queues beyond sync delay + SLO
    g, w = both(0, 100, False, 0, 5, th, ac, [0, 61, 60], 0, 10, 50, 0.99); assert g == w == ("offload", 2)
    # the deciding server never offloads to itself, however idle it is
    g, w = both(0, 100, False, 0, 5, [50.0, 1.0], [0.0, 0.5], [0, 0], 0, 10, 50, 0.0);  assert g == w == ("offload", 1)
    with pytest.raises(B.EparaError):
        B.epara_handle_request(0, 1, False, 0, 5, th, ac, qu, 3, 10, 50, 0.3)
    with pytest.raises(B.EparaError):
        B.epara_handle_request(0, 1, False, 0, 5, th, ac, qu, 0, 10, 50, 1.0)


def test_offloading_probabilities_are_the_idle_goodput_shares_of_eq_1():
    from paper_2511_00603_amd import binding as B
    # idle goodput 0 (self), 1, 0 (saturated), 3, 4 (queue too long -> excluded): shares 1/4 and 3/4
    th, ac, qu = [9.0, 5.0, 2.0, 7.0, 8.0], [1.0, 4.0, 2.0, 4.0, 4.0], [0, 0, 0, 10, 99]
    n = 4000
    picks = [B.epara_handle_request(0, 100, False, 0, 5, th, ac, qu, 0, 20, 30, (i + 0.5) / n) for i in range(n)]
    assert all(p == P.handle_request(0, 100, False, 0, 5, th, ac, qu, 0, 20, 30, (i + 0.5) / n) for i, p in enumerate(picks))
    count = {m: sum(1 for p in picks if p == ("offload", m)) for m in range(5)}
    assert count == {0: 0, 1: n // 4, 2: 0, 3: 3 * n // 4, 4: 0}
