"""Reference event-driven simulation of one placement period (test infrastructure only).

What the placement objective phi(Theta) of Sec. 3.3 counts: the requests of a period that the request
handler of Sec. 3.2 gets served within their SLO, for a given placement list.  As in the paper's
large-scale evaluation, nothing is executed: a request served by service l on server n occupies one
instance of that placement for frames * c_ln microseconds, c_ln taken from a table (Sec. 3.3; Sec. 5
"Settings"), and an offload hop costs a fixed transmission time.  Plain Python integers and floats,
events in (time, sequence) order; the handler decision itself is oracle.planner.handle_request.

The readings this simulation takes where the paper leaves the model open:
  * a placement id l * N + n adds one instance of service l on server n; an instance serves one request
    at a time, in the order the handler assigned them;
  * "locally placed services suffice" = the instance of (l, n) that is free first would finish the
    request by its deadline (arrival + SLO); the request is then bound to that instance at once;
  * state synchronisation is periodic with period t (the sync delay): at time j*t every server
    publishes, per service, how many requests it completed in ((j-1)t, jt] and when its first
    instance will be free; others know snapshot J = floor(now / t) - 1 (none yet: zeros).  Theoretical
    goodput of (l, m) = instances / c_lm, actual = completions of the known window / t, both per second;
    the expected computation queued = max(0, first free time - J*t);
  * a request is never offloaded to a server it has already visited (the recorded path);
  * a latency-sensitive request (required rate 0) counts as one satisfied request when it is served (it is
    only bound to an instance if it meets its deadline);
  * a frequency-sensitive request (required rate > 0 frames per second) is a stream of `frames` frames, each
    of which counts as a request (Sec. 3.3: 120 frames wanted at 60 fps but served at 30 fps count
    120 * 30 / 60 = 60).  "Locally sufficient" for it = an instance of (l, n) exists: the stream is bound to the
    instance that is free first, whatever rate that gives (a saturated instance serves it late, hence
    slowly); achieved rate = frames / (finish - arrival); satisfied = frames * min(1, achieved / required).
"""
import heapq

from . import planner


def simulate(n_servers, n_services, compute_us, hop_us, sync_delay_us, max_offload, placements, requests, draws):
    """compute_us[l][n]; requests: list of (arrival_us, service, origin, slo_us, frames[, fps_milli]) with
    fps_milli = 1000 * the required frame rate of a frequency-sensitive request (0 or absent: latency-sensitive);
    draws[r][k]: the uniform draw of request r's k-th offloading decision.
    -> dict(satisfied, local, offloaded, timeout, offload_exceeded, insufficient)."""
    N, t = n_servers, sync_delay_us
    free, log, done = {}, {}, {}
    for p in placements:
        l, n = divmod(p, N)
        free.setdefault((l, n), []).append(0)
    out = dict(satisfied=0.0, local=0, offloaded=0, timeout=0, offload_exceeded=0, insufficient=0)
    heap = [(req[0], i, i, req[2], 0, (req[2],)) for i, req in enumerate(requests)]
    heapq.heapify(heap)
    seq = len(requests)
    while heap:
        now, _, r, n, hops, path = heapq.heappop(heap)
        arrival, l, _origin, slo, frames = requests[r][:5]
        fps_milli = requests[r][5] if len(requests[r]) > 5 else 0
        deadline = arrival + slo
        local_ok, slot, finish = False, -1, 0
        inst = free.get((l, n))
        if inst and compute_us[l][n] > 0:
            slot = min(range(len(inst)), key=lambda i: (inst[i], i))
            finish = max(now, inst[slot]) + frames * compute_us[l][n]
            local_ok = finish <= deadline or fps_milli > 0
        J = now // t - 1
        theoretical, actual, queued = [0.0] * N, [0.0] * N, [0] * N
        for m in range(N):
            k = len(free.get((l, m), ()))
            if k == 0 or compute_us[l][m] <= 0 or m in path:
                continue                                    # idle goodput 0: never a destination
            theoretical[m] = k * 1e6 / compute_us[l][m]
            if J >= 1:
                actual[m] = done.get((l, m, J), 0) * 1e6 / t
                first_free = 0
                for when, value in log.get((l, m), ()):
                    if when <= J * t:
                        first_free = value
                queued[m] = max(0, first_free - J * t)
        u = draws[r][hops] if hops < max_offload else 0.0
        decision, dest = planner.handle_request(now, deadline, local_ok, hops, max_offload, theoretical, actual, queued,
                                                n, t, slo, u)
        if decision == "local":
            inst[slot] = finish
            log.setdefault((l, n), []).append((now, min(inst)))
            bucket = -(-finish // t)
            done[(l, n, bucket)] = done.get((l, n, bucket), 0) + 1
            out["local"] += 1
            if fps_milli > 0:
                achieved = frames * 1e6 / (finish - arrival)            # frames per second over the whole stream
                out["satisfied"] += frames * min(1.0, achieved / (fps_milli / 1000.0))
            else:
                out["satisfied"] += 1.0
        elif decision == "offload":
            out["offloaded"] += 1
            heapq.heappush(heap, (now + hop_us, seq, r, dest, hops + 1, path + (dest,)))
            seq += 1
        else:
            out[decision] += 1
    return out
