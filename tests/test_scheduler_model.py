"""The scheduling rule of the dispatcher on a CPU model (tests/scheduler_model.py): publication order,
W workers claiming in that order and holding up to `stash` units each, workers that wait once
everything they hold waits.  The first version of the
rule (hold back only large dependent tasks) lets every worker park behind small tasks whose
dependency is published after them; the rule the kernel implements cannot: whatever a worker waits
for lies before its own unit in the unit ring."""
import numpy as np
import pytest

import scheduler_model as M


@pytest.mark.parametrize("workers,stash", [(3, 1), (8, 1), (767, 1), (3, 8), (8, 8), (767, 8)])
def test_large_only_rule_parks_every_worker_behind_a_held_task(workers, stash):
    # the producer keeps every worker busy for a few rounds; meanwhile the consumers are published
    room = workers * stash                              # units the workgroups can hold between them
    tasks = M.producer_with_dependants(n_consumers=room + 5, producer_chunks=3 * room)
    # (the dispatcher publishes faster than the workers claim: 64 records per pass, several passes per chunk-time)
    r = M.simulate(tasks, workers, "large_only", stash=stash, disp_passes=8 * stash)
    assert r.deadlock and r.parked == workers          # every slot of every worker holds a consumer of the unpublished task
    assert r.completed == 1                            # only the producer ever finished
    # fewer consumers than slots: one is left to run the held task, and the stream drains
    r = M.simulate(M.producer_with_dependants(n_consumers=room - 1, producer_chunks=3 * room), workers, "large_only", stash=stash, disp_passes=8 * stash)
    assert not r.deadlock


def test_large_only_rule_parks_on_a_chain_of_small_links_too():
    r = M.simulate(M.chain_behind_held_task(n_links=6, link_chunks=4), 16, "large_only", stash=1)
    assert r.deadlock and r.parked == 16
    r = M.simulate(M.chain_behind_held_task(n_links=6, link_chunks=4), 2, "large_only", stash=8)
    assert r.deadlock and r.parked == 2


@pytest.mark.parametrize("workers,stash", [(1, 1), (3, 1), (8, 8), (767, 1), (767, 8)])
def test_published_deps_rule_drains_the_same_streams(workers, stash):
    for tasks in (M.producer_with_dependants(n_consumers=workers * stash + 5, producer_chunks=3 * workers),
                  M.producer_with_dependants(n_consumers=1500, consumer_chunks=3),
                  M.chain_behind_held_task(n_links=300, link_chunks=4)):
        r = M.simulate(tasks, workers, "published_deps", stash=stash)
        assert not r.deadlock and r.completed == len(tasks) and r.order_violations == 0
        assert r.held >= 2                             # the small dependants joined the pending list behind the held task


@pytest.mark.parametrize("seed", range(8))
def test_published_deps_rule_never_parks_on_random_dags(seed):
    rng = np.random.default_rng(seed)
    tasks = M.random_dag(rng, 700)
    for workers, pend_max, lookahead, stash in ((3, 128, 64, 1), (7, 64, 8192, 8), (40, 128, 512, 8), (2, 128, 8192, 3)):
        r = M.simulate(tasks, workers, "published_deps", pend_max=pend_max, lookahead=lookahead, stash=stash)
        assert not r.deadlock and r.completed == len(tasks) and r.order_violations == 0


def test_random_dags_do_park_under_the_large_only_rule():
    """The random streams are hard enough to show the fault of the first rule (so the test above can fail)."""
    hits = 0
    for seed in range(8):
        tasks = M.random_dag(np.random.default_rng(seed), 700)
        hits += M.simulate(tasks, 5, "large_only", stash=1).deadlock
        hits += M.simulate(tasks, 2, "large_only", stash=3).deadlock
    assert hits >= 1


def _planned(s):
    from helpers import HostPools
    from paper_2604_17861_amd import runtime as R
    hp = HostPools(s)
    impl = s.impl_for()
    return [M.Task(R.task_plan(hp.tasks, i, int(impl[i]))[1], tuple(int(d) for d in s.tasks["dep"][i]), False) for i in range(len(s))]


def test_the_gpu_regression_streams_are_ones_the_large_only_rule_parks_on():
    """tests/parity_cases.producer_with_dependants, with the chunk counts the host really packs
    (gpuos_task_plan).  1,200 consumers: under the first rule, with one unit per workgroup (the kernel
    the fault was found in), every one of 767 workers ends up parked.  6,400 consumers, more than 767
    workgroups can hold at eight units each: the same with the units a workgroup holds today.  Under
    the rule the kernel implements both drain."""
    import parity_cases as C
    tasks = _planned(C.producer_with_dependants())
    assert tasks[0].nchunks > 4 and tasks[1].nchunks > 4 and all(t.nchunks == 1 for t in tasks[2:1202]) and tasks[1202].nchunks == 4
    # the dispatcher is fast against a 2M-element task: give it enough passes per chunk-time to publish the consumers
    r = M.simulate(tasks, 767, "large_only", disp_passes=32, stash=1)
    assert r.deadlock and r.parked == 767
    for stash in (1, 8):
        r = M.simulate(tasks, 767, "published_deps", disp_passes=32, stash=stash)
        assert not r.deadlock and r.completed == len(tasks)
        assert r.held == 128      # the pending list fills behind the held task; dequeuing pauses until it is published
    tasks = _planned(C.producer_with_dependants(n_consumers=6400))
    assert all(t.nchunks == 1 for t in tasks[2:6402])
    # (every consumer is published while the producer still runs: a timing the rule must not depend on)
    r = M.simulate(tasks, 767, "large_only", disp_passes=256, stash=8)
    assert r.deadlock and r.parked == 767
    r = M.simulate(tasks, 767, "published_deps", disp_passes=256, stash=8)
    assert not r.deadlock and r.completed == len(tasks) and r.held == 128
