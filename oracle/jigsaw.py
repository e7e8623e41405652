"""Iteration-level placement of data-parallel training tasks (oracle side, test infrastructure).

Sec. 3 of the paper: a job is a chain of iterations, an iteration is one task per worker, and iteration i + 1 of a
job may start only when every task of its iteration i has ended.  Under SPB the tasks of one iteration differ in
run time (and memory), so the scheduler places TASKS, not whole gangs: all ready tasks sit in a priority queue
keyed by the product of the task's GPU resource and its run time (largest first); the task taken from the queue
goes to the device on which it can start EARLIEST, where a device other than the one that ran the same worker in
the previous iteration can start it no sooner than `gamma * model_size` after the previous iteration ended (the
model has to be moved there first).  A device runs one task at a time; a task may fill a gap between tasks
placed earlier.  The baseline of the same section is gang scheduling: the workers of an iteration start together
on as many devices and the devices are held until the slowest worker is done.

Plain Python, float64, quadratic scans written for reading, not for speed.

Readings where the paper is silent:
  * the priority is resource * run time as they come (the paper normalises both, by constants of the cluster,
    which does not change the order); ties go to the smaller (job, iteration, worker);
  * a device is exclusive in time; the resource figure only orders the queue and must not exceed `capacity`;
  * the first iteration of a job pays the start-up delay on every device (nothing is resident anywhere yet) and is
    released at the job's arrival time;
  * moving the model occupies the network, not the device: the device may run other tasks meanwhile;
  * between devices that offer the same start the one that ran this worker last wins, then the lowest index;
  * gang baseline: an iteration is placed at the earliest time at which enough devices are free for the slowest
    worker's run time; a worker keeps its previous device when that one is free then, the others take the free
    devices of lowest index and need the start-up delay; iterations are ordered by (sum of resources) * (slowest
    run time), ties to the smaller (job, iteration).
"""
from __future__ import annotations


def _free(busy, t, d):
    """True when [t, t + d) meets none of the half-open busy intervals."""
    return all(not (s < t + d and t < e) for s, e in busy)


def _earliest_gap(busy, t0, d):
    """Earliest t >= t0 such that [t, t + d) is free: t0 itself or the end of a busy interval."""
    for t in sorted([t0] + [e for _s, e in busy if e > t0]):
        if _free(busy, t, d):
            return t
    raise AssertionError("unreachable: the end of the last interval is always free")


def _check(jobs, n_machines, capacity):
    if n_machines < 1:
        raise ValueError("at least one device")
    for j, job in enumerate(jobs):
        w = len(job["durations"])
        if w < 1 or len(job["resources"]) != w:
            raise ValueError(f"job {j}: one duration and one resource per worker")
        if any(not d > 0 for d in job["durations"]) or any(r < 0 or r > capacity for r in job["resources"]):
            raise ValueError(f"job {j}: durations must be positive, resources within [0, capacity]")
        if job["iterations"] < 0 or job["arrival"] < 0 or job["model_size"] < 0:
            raise ValueError(f"job {j}: negative iterations, arrival or model size")


def schedule(jobs, n_machines: int, gamma: float = 0.0, capacity: float = 1.0, gang: bool = False):
    """jobs: list of dict(arrival, iterations, model_size, durations[w], resources[w]).

    Returns (placements, makespan); a placement is a dict(job, iteration, worker, machine, start, end, held_until,
    moved): the task computes during [start, end) and its device is taken during [start, held_until).
    """
    _check(jobs, n_machines, capacity)
    if gang:
        return _schedule_gang(jobs, n_machines, gamma)
    busy = [[] for _ in range(n_machines)]
    last_machine = {}                      # (job, worker) -> device of the previous iteration
    release = {}                           # (job, iteration) -> earliest start of its tasks
    pending = {}                           # (job, iteration) -> tasks not placed yet
    ends = {}                              # (job, iteration) -> ends of the placed tasks
    queue = []
    for j, job in enumerate(jobs):
        if job["iterations"] > 0:
            release[(j, 0)] = float(job["arrival"])
            pending[(j, 0)] = len(job["durations"])
            ends[(j, 0)] = []
            queue += [(j, 0, w) for w in range(len(job["durations"]))]
    out = []
    while queue:
        # largest resource * run time first
        queue.sort(key=lambda t: (-(jobs[t[0]]["resources"][t[2]] * jobs[t[0]]["durations"][t[2]]), t[0], t[1], t[2]))
        j, i, w = queue.pop(0)
        job = jobs[j]
        d = float(job["durations"][w])
        prev = last_machine.get((j, w))
        best = None
        for m in range(n_machines):
            ready = release[(j, i)] + (0.0 if (i > 0 and m == prev) else gamma * job["model_size"])
            start = _earliest_gap(busy[m], ready, d)
            key = (start, 0 if m == prev else 1, m)
            if best is None or key < best[0]:
                best = (key, m, start)
        _key, m, start = best
        end = start + d
        busy[m].append((start, end))
        out.append(dict(job=j, iteration=i, worker=w, machine=m, start=start, end=end, held_until=end,
                        moved=bool(i > 0 and m != prev)))
        last_machine[(j, w)] = m
        ends[(j, i)].append(end)
        pending[(j, i)] -= 1
        if pending[(j, i)] == 0 and i + 1 < job["iterations"]:
            release[(j, i + 1)] = max(ends[(j, i)])
            pending[(j, i + 1)] = len(job["durations"])
            ends[(j, i + 1)] = []
            queue += [(j, i + 1, w2) for w2 in range(len(job["durations"]))]
    return out, max([p["end"] for p in out], default=0.0)


def _schedule_gang(jobs, n_machines, gamma):
    busy = [[] for _ in range(n_machines)]
    last_machine = {}
    out = []
    queue = [(j, 0, float(job["arrival"])) for j, job in enumerate(jobs) if job["iterations"] > 0]
    for j, job in enumerate(jobs):
        if len(job["durations"]) > n_machines:
            raise ValueError(f"job {j}: a gang of {len(job['durations'])} workers needs as many devices")
    while queue:
        queue.sort(key=lambda t: (-(sum(jobs[t[0]]["resources"]) * max(jobs[t[0]]["durations"])), t[0], t[1]))
        j, i, rel = queue.pop(0)
        job = jobs[j]
        n_workers = len(job["durations"])
        slowest = float(max(job["durations"]))
        moved_ready = rel + gamma * job["model_size"]
        candidates = sorted({rel, moved_ready} | {e for b in busy for _s, e in b if e > rel})
        placed = None
        for t in candidates:
            free = [m for m in range(n_machines) if _free(busy[m], t, slowest)]
            assign = {}
            for w in range(n_workers):                      # a worker keeps its device when that one is free at t
                prev = last_machine.get((j, w)) if i > 0 else None
                if prev is not None and prev in free:
                    assign[w] = prev
                    free.remove(prev)
            rest = [w for w in range(n_workers) if w not in assign]
            if rest and (t < moved_ready or len(free) < len(rest)):
                continue
            for w, m in zip(rest, free):                    # the others move: lowest free indices
                assign[w] = m
            placed = (t, assign)
            break
        assert placed is not None, "the end of the last busy interval is a candidate at which every device is free"
        t, assign = placed
        for w in range(n_workers):
            m = assign[w]
            prev = last_machine.get((j, w)) if i > 0 else None
            busy[m].append((t, t + slowest))
            out.append(dict(job=j, iteration=i, worker=w, machine=m, start=t, end=t + float(job["durations"][w]),
                            held_until=t + slowest, moved=bool(i > 0 and m != prev)))
            last_machine[(j, w)] = m
        if i + 1 < job["iterations"]:
            queue.append((j, i + 1, t + slowest))
    return out, max([p["held_until"] for p in out], default=0.0)
