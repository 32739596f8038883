"""Reference group planner (test infrastructure only; pure Python integers).

The allocator of the paper decides, per task, the batch shape and which services
share a GPU (Sec. 3.1: BS = requests of one service form a batch, MT = several
services run together, MF = a request may bring several frames).  On one GPU that
decision becomes: how many rows each service's batch has, where those rows sit in
a packed buffer, and which output tiles one launch has to produce.  This module
states those rules in the most literal form; the C++ planner of the library must
reproduce every integer.

Rules
-----
batch accounting   M_g = sum of rows(r) over the requests r of service g; a request's
                   first row is the running sum of the rows before it (Sec. 3.1 BS/MF;
                   Sec. 4.1, inter-request count = floor(BS / MF)).
offsets            row_off[g] = sum_{h<g} M_h,  x_off[g] = sum_{h<g} M_h*K_h,
                   y_off[g] = sum_{h<g} M_h*N_h              (each of length G+1)
tile class         the first class c with M_g <= max_M[c]
canonical tiles    for g ascending, m0 = 0, BM, 2BM, ... < M_g, n0 = 0, BN, ... < N_g:
                   (g, m0, n0, rows=min(BM, M_g-m0), cols=min(BN, N_g-n0), c)
visit order        see `schedule_tiles` (panel tiles die by die, streaming tiles longest first).
batch forming      see `request_segments` (where each request's rows go in its service's batch).
"""

INT32_MAX = 2**31 - 1


def batch_rows(request_rows_per_service):
    """M_g and per-request first rows from lists of per-request row counts."""
    M, first = [], []
    for reqs in request_rows_per_service:
        acc, starts = 0, []
        for r in reqs:
            if r < 0:
                raise ValueError("negative row count")
            starts.append(acc)
            acc += r
        M.append(acc)
        first.append(starts)
    return M, first


def request_segments(request_rows_per_service, request_row_bytes, batch_row_bytes, request_ptr_per_service, batch_ptr, to_batch):
    """The copy plan of batch forming: one (src, dst, bytes, first_chunk, group) per request, in
    request order.  A request's rows sit in the batch of its service after the rows of the
    service's earlier requests (rows of batch_row_bytes[g] bytes there, of request_row_bytes[g] in
    the request's own buffer: the two differ when the rows are quantised on the way); bytes
    counts the source side; first_chunk counts the 16-KiB chunks of all earlier segments."""
    segs, chunks = [], 0
    for g, reqs in enumerate(request_rows_per_service):
        for rb in (request_row_bytes[g], batch_row_bytes[g]):
            if rb <= 0 or rb % 16:
                raise ValueError("row size must be a positive multiple of 16 bytes")
        first = 0
        for i, rows in enumerate(reqs):
            if rows < 0:
                raise ValueError("negative row count")
            in_batch = batch_ptr[g] + first * batch_row_bytes[g]
            own = request_ptr_per_service[g][i]
            nbytes = rows * (request_row_bytes[g] if to_batch else batch_row_bytes[g])
            segs.append((own, in_batch, nbytes, chunks, g) if to_batch else (in_batch, own, nbytes, chunks, g))
            chunks += -(-nbytes // 16384)
            first += rows
    return segs, chunks


def dp_group_count(rate_required, rate_of_one_group):
    """Sec. 4.1, Eq. "DP group count" = ceil(required rate / rate of one group), integers."""
    if rate_required < 0 or rate_of_one_group <= 0:
        raise ValueError("bad rates")
    return -(-rate_required // rate_of_one_group)


def inter_request_count(batch_size, max_inter_frame_count):
    """Sec. 4.1, Eq. "inter request count" = floor(BS / max inter-frame count)."""
    if batch_size < 0 or max_inter_frame_count <= 0:
        raise ValueError("bad counts")
    return batch_size // max_inter_frame_count


OPERATORS = {"BS": 1, "MT": 2, "MP": 4, "MF": 8, "DP": 16}


def operator_set(frequency_sensitive, multi_gpu):
    """Sec. 3.1 "Performing operators to categories", the four paragraphs as a table of names."""
    if not frequency_sensitive:
        ops = ["BS", "MT"] + (["MP"] if multi_gpu else [])                 # first / second category
    else:
        ops = ["MF", "MT", "BS"] + (["DP", "MP"] if multi_gpu else [])     # third / fourth category
    return sorted(ops)


def max_inter_frame_count(latency_us, fps_milli):
    """Sec. 4.1: MF frames per batch make the latency MF / fps; the largest MF within the requirement, >= 1."""
    if latency_us < 0 or fps_milli <= 0:
        raise ValueError("bad latency or rate")
    return max(1, latency_us * fps_milli // 10**9)


def dp_deal(first_frame, n_frames, n_groups):
    """Sec. 3.1 DP: frames go to the DP groups round robin -> (frames per group, group of each frame)."""
    if n_groups <= 0 or n_frames < 0 or first_frame < 0:
        raise ValueError("bad counts")
    group = [(first_frame + j) % n_groups for j in range(n_frames)]
    return [group.count(g) for g in range(n_groups)], group


def handle_request(now_us, deadline_us, local_can_serve, offload_count, max_offload, theoretical, actual, queued_us,
                   self_index, sync_delay_us, slo_us, u):
    """Sec. 3.2, the handler's steps in the paper's order -> (decision name, destination or None).
    Offloading follows Eq. (1): among the other servers whose queued computation does not exceed
    sync delay + SLO and whose idle goodput (theoretical - actual) is positive, server m is drawn
    with probability idle_m / sum(idle); the uniform draw u is an input."""
    if now_us > deadline_us:
        return "timeout", None
    if local_can_serve:
        return "local", None
    if offload_count >= max_offload:
        return "offload_exceeded", None
    shares = []
    for m in range(len(theoretical)):
        feasible = m != self_index and queued_us[m] <= sync_delay_us + slo_us and theoretical[m] - actual[m] > 0
        shares.append(theoretical[m] - actual[m] if feasible else 0.0)
    total = 0.0
    for v in shares:
        total += v
    if not total > 0:
        return "insufficient", None
    acc, last = 0.0, None
    for m, v in enumerate(shares):
        if v <= 0:
            continue
        acc += v
        last = m
        if acc > u * total:
            break
    return "offload", last


def place_full_models(candidates, is_set, keep_equal, theta0, phi):
    """Alg. 2 (submodular placement for full models), round by round as the pseudo-code runs:
    evaluate phi(Theta + delta) for every admissible delta, collect the maximisers, add one of them
    (the earliest: the paper allows any), and stop -- dropping that addition -- as soon as phi fails
    to grow (step S1: to not shrink).  A set offers all its elements every round, a list only the
    ones not chosen yet."""
    theta = list(theta0)
    chosen_positions = set()
    while True:
        before = phi(theta)
        best_positions, best_value = [], None
        for pos, delta in enumerate(candidates):
            if not is_set and pos in chosen_positions:
                continue
            v = phi(theta + [delta])
            if best_value is None or v > best_value:
                best_positions, best_value = [pos], v
            elif v == best_value:
                best_positions.append(pos)
        if not best_positions:
            return theta
        grown = theta + [candidates[best_positions[0]]]
        ok = phi(grown) >= before if keep_equal else phi(grown) > before
        if not ok:
            return theta
        theta = grown
        chosen_positions.add(best_positions[0])


def place_services(partial, X, X_dot, phi):
    """Alg. 1 (state-aware service placement): prioritised partial configurations first (a list, kept
    while phi does not shrink), then the set of all placements, then the placements on the
    hypothetical all-GPU server."""
    theta1 = place_full_models(partial, False, True, [], phi)
    theta2 = place_full_models(X, True, False, theta1, phi)
    return place_full_models(X_dot, True, False, theta2, phi)


def pick_class(M, classes):
    for c, cl in enumerate(classes):
        if M <= cl[0]:
            return c
    raise ValueError("no tile class admits M=%d" % M)


def plan_groups(groups, classes):
    """groups: list of (M, K, N); classes: list of (max_M, BM, BN) or (max_M, BM, BN, split_K) with increasing max_M.

    Returns (row_off, x_off, y_off, tiles) with tiles a list of 6-tuples.
    """
    prev = -1
    for cl in classes:
        max_M, bm, bn = cl[:3]
        if bm <= 0 or bn <= 0 or max_M <= prev or (len(cl) > 3 and cl[3] < 0):
            raise ValueError("bad tile class table")
        prev = max_M
    row_off, x_off, y_off, tiles = [0], [0], [0], []
    for g, (M, K, N) in enumerate(groups):
        if M < 0 or K <= 0 or N <= 0:
            raise ValueError("bad group shape")
        row_off.append(row_off[-1] + M)
        x_off.append(x_off[-1] + M * K)
        y_off.append(y_off[-1] + M * N)
        if M == 0:
            continue
        c = pick_class(M, classes)
        bm, bn = classes[c][1], classes[c][2]
        for m0 in range(0, M, bm):
            for n0 in range(0, N, bn):
                tiles.append((g, m0, n0, min(bm, M - m0), min(bn, N - n0), c))
    return row_off, x_off, y_off, tiles


def split_parts(K, cls):
    """Visits a streaming tile of class cls = (max_M, BM, BN[, split_K]) is cut into: two when the class names a
    K (split_K > 0) and the group's K reaches it (see schedule_tiles)."""
    return 2 if len(cls) > 3 and cls[3] > 0 and K >= cls[3] else 1


def order_entry(tile, part, parts):
    return tile | (part << 24) | ((parts - 1) << 28)


def order_decode(entry):
    """-> (tile, part, parts) of a non-negative entry of a visit order."""
    return entry & 0xFFFFFF, (entry >> 24) & 15, ((entry >> 28) & 7) + 1


def split_layout(groups, classes, n_stream_classes):
    """-> (split_base per group, number of split tiles, workspace bytes): see epara_split_layout in the header."""
    base, n = [], 0
    for M, K, N in (g[:3] for g in groups):
        b = -1
        if M > 0:
            c = next(i for i, cl in enumerate(classes) if M <= cl[0])
            if c < n_stream_classes and split_parts(K, classes[c]) > 1:
                b = n
                n += -(-M // classes[c][1]) * -(-N // classes[c][2])
        base.append(b)
    return base, n, (0 if n == 0 else (n * 4 + 255) // 256 * 256 + n * 4 * 32768)


def split_workspace_bytes(n_split_tiles, n_panel_split_tiles):
    """Counters (4 bytes per split tile, rounded up to 256), then 4 parts of 32 KiB per streaming tile, then 4 parts
    of 256 KiB per panel tile."""
    n = n_split_tiles + n_panel_split_tiles
    return 0 if n == 0 else (n * 4 + 255) // 256 * 256 + n_split_tiles * 4 * 32768 + n_panel_split_tiles * 4 * 262144


def panel_split(groups, classes, n_stream_classes, n_workgroups):
    """-> (m, P, n_more): the last m tiles of the tile table are visited in parts of K, the first m - n_more of them in
    P parts, the others in P + 1 (m = 0: none).  Only for a launch of panel tiles alone, all of one class that names
    a split_K and of one K >= split_K, no gated group: with n tiles on W workgroups the last round holds m = n mod W
    of them.  Candidates, cost = 2040 K, a part of a tile cut in P costs cost // P + 1020000:
      (a) every tile in P = 2, 3, 4 parts: time -(-m P // W) parts one after the other;
      (b) k = 1..4 parts per workgroup, Q = k W in all, 2 m <= Q <= 4 m, Q not a multiple of m: the first m - Q % m tiles
          in P = Q // m parts, the others in P + 1; time = the most loaded of W level bins when the parts, the larger
          ones first, each go to the least loaded bin.
    The smallest time wins (in this order on ties) and must be below 9 cost // 10."""
    import heapq
    W = n_workgroups
    cls = K = None
    n = 0
    for g in groups:
        M, Kg, N = g[:3]
        if M <= 0:
            continue
        c = pick_class(M, classes)
        cl = classes[c]
        if c < n_stream_classes or (len(g) > 3 and g[3]):
            return 0, 1, 0
        if cls is not None and (c != cls or Kg != K):
            return 0, 1, 0
        if len(cl) < 4 or cl[3] <= 0 or Kg < cl[3]:
            return 0, 1, 0
        cls, K = c, Kg
        n += -(-M // cl[1]) * -(-N // cl[2])
    if cls is None or n % W == 0:
        return 0, 1, 0
    m, cost = n % W, 2040 * K
    best, parts, more = cost * 9 // 10, 1, 0
    for P in (2, 3, 4):
        t = -(-m * P // W) * (cost // P + 1020000)
        if t < best:
            best, parts, more = t, P, 0
    for k in (1, 2, 3, 4):
        Q = k * W
        if Q < 2 * m or Q > 4 * m or Q % m == 0:
            continue
        base, extra = divmod(Q, m)
        bins = [0] * W
        heapq.heapify(bins)
        t = 0
        for i in range(Q):
            item = cost // base + 1020000 if i < (m - extra) * base else cost // (base + 1) + 1020000
            load = heapq.heappop(bins) + item
            heapq.heappush(bins, load)
            t = max(t, load)
        if t < best:
            best, parts, more = t, base, extra
    return (m, parts, more) if parts > 1 else (0, 1, 0)


def schedule_tiles(groups, classes, n_stream_classes, tiles, n_workgroups, n_xcd, panel_m, panel_n):
    """Visit order of the persistent workgroups.

    groups: (M, K, N) or (M, K, N, gated) tuples.  Workgroup b of a launch of W = n_workgroups
    visits slots b, b+W, b+2W, ... and the hardware places workgroup b on compute die
    b mod n_xcd.  Every workgroup gets a list of tiles; slot j*W + b is the j-th entry of
    workgroup b (-1 = idle), the order has W * (longest list) entries.  The first
    n_stream_classes classes are weight-streaming classes, the others panel classes.

    1. Panel tiles.  Classes by descending BM*BN (ties: lower class first); inside a class the
       groups by descending K (ties: lower group first); inside a group the tile grid TM x TN
       is cut into panels of panel_m x panel_n tiles, panels taken with the n-panel index
       outermost, and inside a panel the m index runs fastest.  Each tile of that sequence goes to the
       workgroup with the smallest accumulated cost (a panel tile costs 2040 * K); among equally loaded
       workgroups the one of smallest die-major rank, rank r standing for workgroup (r mod (W/X)) * X + r div (W/X).
       Tiles of equal cost therefore go round robin, the l-th to rank l mod W, and the W/X tiles that run
       together on one die are consecutive in the sequence; a workgroup that got a long-K tile gets fewer
       of the short ones.  In a single launch the last m tiles of the table may be left out of this sequence
       and visited in P parts of K instead (panel_split): their parts follow, tile by tile and part by part,
       each an item of cost 2040 * K // P + 1020000 (P: that tile's number of parts) under the same rule, entry
       tile | part << 24 | (P - 1) << 28.
    2. Streaming tiles, longest first.  cost = K * (6 * cols * (2 if gated) + (2 * BM if BM >= 32 else 0))
       for a streaming tile (weight columns streamed from HBM, plus the activation rows re-read from L2
       at a third of that price, free for the 16-row class), 2040 * K for a panel tile.  In a single launch a
       streaming tile of a class (max_M, BM, BN, split_K) with split_K > 0 and K >= split_K is visited in P = 2 parts of K, each an
       item of cost // P + 24 * BM * cols (* 2 if gated) whose order entry is tile | part << 24 | (P - 1) << 28.
       Items by descending cost (ties: lower tile index, then lower part) each go to the workgroup with the
       smallest accumulated cost (ties: lower workgroup), after that workgroup's panel tiles.
    """
    return schedule_chain([(groups, classes, n_stream_classes, tiles)], n_workgroups, n_xcd, panel_m, panel_n)[0]


def schedule_chain(phases, n_workgroups, n_xcd, panel_m, panel_n):
    """Visit orders of a chain of launches run by one kernel, phase after phase in every workgroup.

    phases: list of (groups, classes, n_stream_classes, tiles).  The rule of schedule_tiles with the
    workgroup loads shared by all phases: step 1 phase by phase on the accumulated loads; step 2 once over the streaming tiles of all phases (ties of equal cost: earlier
    phase, then lower tile index), each tile joining its workgroup's list of its own phase.
    Returns one order per phase (W * longest list of that phase entries).
    """
    import heapq
    W, X = n_workgroups, n_xcd
    if W <= 0 or X <= 0 or W % X != 0 or panel_m <= 0 or panel_n <= 0:
        raise ValueError("bad schedule parameters")
    per = W // X
    lists = [[[] for _ in range(W)] for _ in phases]
    load = [0] * W
    rank_heap = [(0, r) for r in range(W)]                   # (load, die-major rank); rank r = workgroup (r mod per) * X + r div per
    stream = []
    n_panel_split, panel_parts, panel_more = panel_split(*phases[0][:3], W) if len(phases) == 1 else (0, 1, 0)
    for p, (groups, classes, n_stream_classes, tiles) in enumerate(phases):
        if not 0 <= n_stream_classes <= len(classes):
            raise ValueError("bad number of streaming classes")
        first = {}
        for t, tile in enumerate(tiles):
            first.setdefault(tile[0], t)
        panel_classes = sorted(range(n_stream_classes, len(classes)), key=lambda c: (-classes[c][1] * classes[c][2], c))
        for c in panel_classes:
            members = sorted({t[0] for t in tiles if t[5] == c}, key=lambda g: (-groups[g][1], g))
            bm, bn = classes[c][1], classes[c][2]
            for g in members:
                M, K, N = groups[g][:3]
                TM, TN = -(-M // bm), -(-N // bn)
                for pn in range(0, TN, panel_n):
                    for pm in range(0, TM, panel_m):
                        for tn in range(pn, min(pn + panel_n, TN)):
                            for tm in range(pm, min(pm + panel_m, TM)):
                                t = first[g] + tm * TN + tn
                                if t >= len(tiles) - n_panel_split:      # visited in parts, after the whole tiles
                                    continue
                                _, r = heapq.heappop(rank_heap)
                                x, i = divmod(r, per)
                                b = i * X + x
                                lists[p][b].append(t)
                                load[b] += 2040 * K
                                heapq.heappush(rank_heap, (load[b], r))
        for t in range(len(tiles) - n_panel_split, len(tiles)):    # the parts: tile by tile, part by part, same rule
            parts_t = panel_parts + (1 if t >= len(tiles) - panel_more else 0)      # the last panel_more tiles: one part more
            each = 2040 * groups[tiles[t][0]][1] // parts_t + 1020000
            for j in range(parts_t):
                _, r = heapq.heappop(rank_heap)
                x, i = divmod(r, per)
                b = i * X + x
                lists[p][b].append(order_entry(t, j, parts_t))
                load[b] += each
                heapq.heappush(rank_heap, (load[b], r))
        for t, tile in enumerate(tiles):
            if tile[5] < n_stream_classes:
                g = groups[tile[0]]
                gated = len(g) > 3 and bool(g[3])
                bm = classes[tile[5]][1]
                cost = g[1] * (6 * tile[4] * (2 if gated else 1) + (2 * bm if bm >= 32 else 0))
                parts = split_parts(g[1], classes[tile[5]]) if len(phases) == 1 else 1
                if parts == 1:
                    stream.append((-cost, p, t, 0, t))
                else:                                            # a split tile: one item per part of K
                    each = cost // parts + 24 * bm * tile[4] * (2 if gated else 1)
                    stream += [(-each, p, t, j, order_entry(t, j, parts)) for j in range(parts)]
    stream.sort()
    heap = [(load[b], b) for b in range(W)]
    heapq.heapify(heap)
    for negcost, p, _, _, entry in stream:
        ld, b = heapq.heappop(heap)
        lists[p][b].append(entry)
        heapq.heappush(heap, (ld - negcost, b))
    orders = []
    for p, (groups, classes, n_stream_classes, tiles) in enumerate(phases):
        assert sum(len(v) for v in lists[p]) >= len(tiles)
        longest = max(len(v) for v in lists[p])
        order = [-1] * (longest * W)
        for b in range(W):
            for j, t in enumerate(lists[p][b]):
                order[j * W + b] = t
        orders.append(order)
    return orders


def chain_waits(producer_tiles, counter_base, producer):
    """What each group of a phase waits for: (counter, need) = (counter_base + q, number of tiles of
    group q in the phase before) for producer[g] = q >= 0, (-1, 0) otherwise."""
    count = {}
    for tile in producer_tiles:
        count[tile[0]] = count.get(tile[0], 0) + 1
    return [(-1, 0) if q < 0 else (counter_base + q, count.get(q, 0)) for q in producer]
