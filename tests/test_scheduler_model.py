"""The scheduling rule of the dispatcher on a CPU model (tests/scheduler_model.py): publication order,
W workers claiming in that order, workers that wait once they hold a unit.  The first version of the
rule (hold back only large dependent tasks) lets every worker park behind small tasks whose
dependency is published after them; the rule the kernel implements cannot: whatever a worker waits
for lies before its own unit in the unit ring."""
import numpy as np
import pytest

import scheduler_model as M


@pytest.mark.parametrize("workers", [3, 8, 767])
def test_large_only_rule_parks_every_worker_behind_a_held_task(workers):
    # the producer keeps every worker busy for a few rounds; meanwhile the consumers are published
    tasks = M.producer_with_dependants(n_consumers=workers + 5, producer_chunks=3 * workers)
    r = M.simulate(tasks, workers, "large_only")
    assert r.deadlock and r.parked == workers          # every worker holds a consumer of the unpublished task
    assert r.completed == 1                            # only the producer ever finished
    # fewer consumers than workers: one workgroup is left to run the held task, and the stream drains
    r = M.simulate(M.producer_with_dependants(n_consumers=workers - 1, producer_chunks=3 * workers), workers, "large_only")
    assert not r.deadlock


def test_large_only_rule_parks_on_a_chain_of_small_links_too():
    r = M.simulate(M.chain_behind_held_task(n_links=6, link_chunks=4), 16, "large_only")
    assert r.deadlock and r.parked == 16


@pytest.mark.parametrize("workers", [1, 3, 8, 767])
def test_published_deps_rule_drains_the_same_streams(workers):
    for tasks in (M.producer_with_dependants(n_consumers=workers + 5, producer_chunks=3 * workers),
                  M.producer_with_dependants(n_consumers=1500, consumer_chunks=3),
                  M.chain_behind_held_task(n_links=300, link_chunks=4)):
        r = M.simulate(tasks, workers, "published_deps")
        assert not r.deadlock and r.completed == len(tasks) and r.order_violations == 0
        assert r.held >= 2                             # the small dependants joined the pending list behind the held task


@pytest.mark.parametrize("seed", range(8))
def test_published_deps_rule_never_parks_on_random_dags(seed):
    rng = np.random.default_rng(seed)
    tasks = M.random_dag(rng, 700)
    for workers, pend_max, lookahead in ((3, 128, 64), (7, 64, 8192), (40, 128, 512)):
        r = M.simulate(tasks, workers, "published_deps", pend_max=pend_max, lookahead=lookahead)
        assert not r.deadlock and r.completed == len(tasks) and r.order_violations == 0


def test_random_dags_do_park_under_the_large_only_rule():
    """The random streams are hard enough to show the fault of the first rule (so the test above can fail)."""
    hits = 0
    for seed in range(8):
        tasks = M.random_dag(np.random.default_rng(seed), 700)
        hits += M.simulate(tasks, 5, "large_only").deadlock
    assert hits >= 1


def test_the_gpu_regression_stream_is_one_the_large_only_rule_parks_on():
    """tests/parity_cases.producer_with_dependants, with the chunk counts the host really packs
    (gpuos_task_plan): under the first rule every one of 767 workers ends up parked; under the rule
    the kernel implements the stream drains."""
    import parity_cases as C
    from helpers import HostPools
    from paper_2604_17861_amd import runtime as R
    s = C.producer_with_dependants()
    hp = HostPools(s)
    impl = s.impl_for()
    tasks = []
    for i in range(len(s)):
        path, nchunks, _, _ = R.task_plan(hp.tasks, i, int(impl[i]))
        tasks.append(M.Task(nchunks, tuple(int(d) for d in s.tasks["dep"][i]), False))
    assert tasks[0].nchunks > 4 and tasks[1].nchunks > 4 and all(t.nchunks == 1 for t in tasks[2:1202]) and tasks[1202].nchunks == 4
    # the dispatcher is fast against a 2M-element task: give it enough passes per chunk-time to publish the consumers
    r = M.simulate(tasks, 767, "large_only", disp_passes=32)
    assert r.deadlock and r.parked == 767
    r = M.simulate(tasks, 767, "published_deps", disp_passes=32)
    assert not r.deadlock and r.completed == len(tasks)
    assert r.held == 128          # the pending list fills behind the held task; dequeuing pauses until it is published
