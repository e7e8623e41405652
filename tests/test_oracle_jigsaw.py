"""Pins of the scheduling oracle (oracle/jigsaw.py) against what Sec. 3 of the paper and the mathematics fix:
the worked example of the section's text, hand-computed placements, the invariants of a valid schedule, the
critical path and the work bound, and the brute-force optimum on tiny instances (longest-first list scheduling
of independent tasks stays within 4/3 - 1/(3 M) of it)."""
import itertools
import random

import pytest

from oracle import jigsaw


def job(durations, iterations=1, arrival=0.0, model_size=0.0, resources=None):
    return dict(arrival=arrival, iterations=iterations, model_size=model_size, durations=list(durations),
                resources=list(resources) if resources is not None else [1.0] * len(durations))


def by_task(placements):
    return {(p["job"], p["iteration"], p["worker"]): p for p in placements}


def check_valid(jobs, n_machines, gamma, placements):
    """Every task once, nothing overlaps on a device, iterations in order, start-up delays respected."""
    t = by_task(placements)
    assert len(t) == len(placements) == sum(len(j["durations"]) * j["iterations"] for j in jobs)
    for m in range(n_machines):
        held = sorted((p["start"], p["held_until"]) for p in placements if p["machine"] == m)
        for (s0, e0), (s1, _e1) in zip(held, held[1:]):
            assert e0 <= s1 + 1e-12, f"device {m}: [{s0}, {e0}) overlaps a task starting at {s1}"
    for (j, i, w), p in t.items():
        jb = jobs[j]
        assert 0 <= p["machine"] < n_machines
        assert p["end"] == p["start"] + jb["durations"][w] and p["held_until"] >= p["end"]
        rel = jb["arrival"] if i == 0 else max(t[(j, i - 1, v)]["held_until"] for v in range(len(jb["durations"])))
        stays = i > 0 and t[(j, i - 1, w)]["machine"] == p["machine"]
        assert p["moved"] == (i > 0 and not stays)
        assert p["start"] >= rel + (0.0 if stays else gamma * jb["model_size"]) - 1e-12


def test_example_of_the_section_three_devices_two_jobs():
    """Workers of 0.3 s, 0.6 s and 1 s next to a second job: placed task by task the second job's work fills the
    devices the short workers free; as a gang the first job holds all three devices for 1 s (Sec. 3)."""
    jobs = [job([0.3, 0.6, 1.0]), job([0.5])]
    placed, makespan = jigsaw.schedule(jobs, 3)
    t = by_task(placed)
    # queue order by resource * time: 1.0, 0.6, 0.5, 0.3
    assert (t[(0, 0, 2)]["machine"], t[(0, 0, 2)]["start"]) == (0, 0.0)
    assert (t[(0, 0, 1)]["machine"], t[(0, 0, 1)]["start"]) == (1, 0.0)
    assert (t[(1, 0, 0)]["machine"], t[(1, 0, 0)]["start"]) == (2, 0.0)
    assert (t[(0, 0, 0)]["machine"], t[(0, 0, 0)]["start"]) == (2, 0.5)
    assert makespan == 1.0
    gang, gang_makespan = jigsaw.schedule(jobs, 3, gang=True)
    g = by_task(gang)
    assert {g[(0, 0, w)]["start"] for w in range(3)} == {0.0} and {g[(0, 0, w)]["held_until"] for w in range(3)} == {1.0}
    assert g[(1, 0, 0)]["start"] == 1.0 and gang_makespan == 1.5
    check_valid(jobs, 3, 0.0, placed)
    check_valid(jobs, 3, 0.0, gang)


def test_next_iteration_waits_for_the_slowest_worker_and_stays_on_its_device():
    jobs = [job([1.0, 2.0], iterations=3, model_size=4.0)]
    placed, makespan = jigsaw.schedule(jobs, 2, gamma=0.5)
    t = by_task(placed)
    # iteration 0 pays the start-up delay of 2 everywhere; afterwards both workers stay where they are
    assert t[(0, 0, 1)]["start"] == 2.0 and t[(0, 0, 0)]["start"] == 2.0
    for i in (1, 2):
        assert t[(0, i, 0)]["start"] == t[(0, i, 1)]["start"] == 2.0 + 2.0 * i
        assert not t[(0, i, 0)]["moved"] and not t[(0, i, 1)]["moved"]
    assert makespan == 8.0
    check_valid(jobs, 2, 0.5, placed)


def test_moving_is_chosen_only_when_it_starts_the_task_earlier():
    # job 1 (two long workers, placed first: bigger) takes devices 0 and 1 from 0.2 on; job 0's first iteration
    # slips in before it on device 0; for its second iteration staying means waiting for job 1
    big = job([5.0, 5.0], arrival=0.2)
    small = job([0.1], iterations=2, model_size=1.0)
    placed, _ = jigsaw.schedule([small, big], 3, gamma=0.05)
    t = by_task(placed)
    assert (t[(0, 0, 0)]["machine"], t[(0, 0, 0)]["start"]) == (0, 0.05)
    assert t[(0, 1, 0)]["moved"] and t[(0, 1, 0)]["machine"] == 2          # ready there at 0.15 + 0.05
    assert t[(0, 1, 0)]["start"] == pytest.approx(0.2, abs=1e-15)
    check_valid([small, big], 3, 0.05, placed)
    # with a start-up delay longer than job 1, everything of job 0 comes after it and staying is never worse
    placed, _ = jigsaw.schedule([small, big], 3, gamma=10.0)
    t = by_task(placed)
    assert t[(0, 0, 0)]["start"] == 10.0 and not t[(0, 1, 0)]["moved"] and t[(0, 1, 0)]["start"] == 10.1
    # two devices only: moving to device 1 would start at 5.2 as well; the tie goes to the device it ran on
    placed, _ = jigsaw.schedule([small, big], 2, gamma=0.05)
    t = by_task(placed)
    assert not t[(0, 1, 0)]["moved"] and t[(0, 1, 0)]["start"] == 5.2


def test_short_task_fills_a_gap_before_a_later_reservation():
    # job 1 arrives late and is placed first (bigger); job 0's short task must slip in before it
    jobs = [job([1.0]), job([4.0], arrival=2.0, resources=[1.0])]
    placed, makespan = jigsaw.schedule(jobs, 1)
    t = by_task(placed)
    assert t[(1, 0, 0)]["start"] == 2.0 and t[(0, 0, 0)]["start"] == 0.0 and makespan == 6.0
    jobs = [job([3.0]), job([4.0], arrival=2.0)]          # 3 does not fit into [0, 2): it goes behind
    placed, makespan = jigsaw.schedule(jobs, 1)
    assert by_task(placed)[(0, 0, 0)]["start"] == 6.0 and makespan == 9.0


def test_single_job_runs_along_its_critical_path():
    rng = random.Random(3)
    for _ in range(20):
        w = rng.randint(1, 5)
        jobs = [job([rng.uniform(0.1, 2.0) for _ in range(w)], iterations=rng.randint(1, 6))]
        for gang in (False, True):
            placed, makespan = jigsaw.schedule(jobs, w, gang=gang)
            check_valid(jobs, w, 0.0, placed)
            assert makespan == pytest.approx(jobs[0]["iterations"] * max(jobs[0]["durations"]), rel=1e-12)


def test_one_device_does_all_the_work_back_to_back():
    rng = random.Random(4)
    jobs = [job([rng.uniform(0.1, 1.0) for _ in range(rng.randint(1, 3))], iterations=rng.randint(1, 4)) for _ in range(5)]
    placed, makespan = jigsaw.schedule(jobs, 1)
    check_valid(jobs, 1, 0.0, placed)
    assert makespan == pytest.approx(sum(sum(j["durations"]) * j["iterations"] for j in jobs), rel=1e-12)


def test_random_mixes_are_valid_and_respect_the_lower_bounds():
    rng = random.Random(5)
    for case in range(30):
        n_machines = rng.randint(1, 6)
        jobs = []
        for _ in range(rng.randint(1, 6)):
            w = rng.randint(1, min(4, n_machines))
            jobs.append(job([rng.uniform(0.05, 1.5) for _ in range(w)], iterations=rng.randint(0, 4),
                            arrival=rng.uniform(0.0, 2.0), model_size=rng.uniform(0.0, 3.0),
                            resources=[rng.uniform(0.1, 1.0) for _ in range(w)]))
        gamma = rng.choice([0.0, 0.05, 0.5])
        for gang in (False, True):
            placed, makespan = jigsaw.schedule(jobs, n_machines, gamma=gamma, gang=gang)
            check_valid(jobs, n_machines, gamma, placed)
            work = sum(sum(j["durations"]) * j["iterations"] for j in jobs)
            path = max([j["arrival"] + j["iterations"] * max(j["durations"]) for j in jobs if j["iterations"]], default=0.0)
            assert makespan >= max(work / n_machines, path) - 1e-9 or not placed


def test_longest_first_stays_within_the_classical_bound_of_the_brute_force_optimum():
    rng = random.Random(6)
    for _ in range(25):
        n_machines = rng.randint(2, 3)
        durations = [rng.uniform(0.1, 1.0) for _ in range(rng.randint(2, 7))]
        jobs = [job([d]) for d in durations]                     # independent single-task jobs, equal resources
        _placed, makespan = jigsaw.schedule(jobs, n_machines)
        best = min(max(sum(d for d, m in zip(durations, a) if m == k) for k in range(n_machines))
                   for a in itertools.product(range(n_machines), repeat=len(durations)))
        assert best - 1e-12 <= makespan <= (4.0 / 3.0 - 1.0 / (3.0 * n_machines)) * best + 1e-12


def test_argument_errors():
    with pytest.raises(ValueError):
        jigsaw.schedule([job([1.0])], 0)
    with pytest.raises(ValueError):
        jigsaw.schedule([job([0.0])], 1)
    with pytest.raises(ValueError):
        jigsaw.schedule([job([1.0], resources=[2.0])], 1)
    with pytest.raises(ValueError):
        jigsaw.schedule([job([1.0, 1.0])], 1, gang=True)
    assert jigsaw.schedule([], 3) == ([], 0.0)
    assert jigsaw.schedule([job([1.0], iterations=0)], 3) == ([], 0.0)
