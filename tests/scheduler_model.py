"""A CPU model of the device-side scheduler: the order in which the dispatcher publishes work
units, W worker workgroups that claim units strictly in publication order and hold up to `stash` of
them each (a workgroup whose unit must wait claims the next one and runs whatever it holds that is
ready), and workers that can only wait once everything they hold has an incomplete dependency.  TEST INFRASTRUCTURE: it executes no
operator; it answers one question about a task stream: can every worker end up parked behind work
that is published after the units they hold (a deadlock of the resident kernel)?

The dispatcher's rules modelled here (csrc/gpuos_kernels.hip, run_dispatcher):
  * records are dequeued in ticket order, at most `batch` per pass, only while fewer than `lookahead`
    published units are unclaimed and while the pending list has room for the pass;
  * a FENCE task is dequeued alone at the head of a pass, after the pending list has drained and every
    earlier ticket has completed;
  * a task that is HELD goes to the pending list (ticket order) and is published, flagged "dependencies
    resolved", once all its dependencies have completed; every other task is published at once and a
    worker that claims one of its units waits for the dependencies itself;
  * which tasks are held is the `rule`:
      "large_only"  (the first version of the scheduler): dependent tasks of more than `small`
                    chunks whose dependencies are incomplete;
      "published_deps" (the rule the kernel implements): those, and every dependent task that names a
                    task which is itself not yet published (on the pending list, or held earlier in
                    the same pass).  Publication order then respects dependency order: a worker only
                    ever waits for units that lie before its own in the unit ring.
"""
from collections import namedtuple

Task = namedtuple("Task", "nchunks deps fence")      # deps: back-distances (0 = none)
Result = namedtuple("Result", "deadlock rounds parked completed held order_violations")


def simulate(tasks, workers, rule, batch=64, pend_max=128, lookahead=8192, small=4, disp_passes=8, stash=8, max_rounds=10 ** 7):
    """One round = the time a worker takes for one chunk; the dispatcher makes `disp_passes` passes in
    that time (a pass over 64 records takes a few microseconds, a chunk of 16K elements tens).  A
    worker claims at most one unit and runs at most one unit per round.  stash=1 is the kernel as it
    first was: one unit per workgroup, which then sits on it."""
    n = len(tasks)
    done = [False] * n
    chunks_done = [0] * n
    published = [False] * n
    units = []                    # (ticket, waits): publication order == claim order
    claim = 0
    pending = []                  # tickets, ticket order
    mirrored = 0
    holding = [[] for _ in range(workers)]    # unit indices a worker holds, oldest first
    held_total = 0
    violations = 0
    completed = 0
    floor = 0                     # every ticket below it is done

    def deps_of(t):
        return [t - d for d in tasks[t].deps if d and d <= t]

    def complete(t):
        return all(done[d] for d in deps_of(t))

    def publish(t, waits):
        published[t] = True
        for _ in range(tasks[t].nchunks):
            units.append((t, waits))

    for rnd in range(max_rounds):
        progress = False
        for _pass in range(disp_passes):
            # ---- dispatcher pass ----
            ready = [t for t in pending if complete(t)][:batch]
            for t in ready:
                pending.remove(t)
                publish(t, False)
                progress = True
            room = pend_max - len(pending)
            take = min(batch, n - mirrored, room)
            if len(units) - claim >= lookahead:
                take = 0
            if take > 0:
                for i in range(1, take):                       # a FENCE starts a pass of its own
                    if tasks[mirrored + i].fence:
                        take = i
                        break
                while floor < mirrored and done[floor]:
                    floor += 1
                if tasks[mirrored].fence and (pending or floor < mirrored):
                    take = 0                                   # the fence waits (the dispatcher keeps serving the pending list)
            held_in_pass = set()
            for t in range(mirrored, mirrored + take):
                tk = tasks[t]
                deps = deps_of(t)
                hold = False
                if deps:
                    if tk.nchunks > small:
                        hold = not complete(t)
                    elif rule == "published_deps":
                        hold = any((not published[d]) or d in held_in_pass for d in deps)
                if hold:
                    pending.append(t)
                    held_in_pass.add(t)
                    held_total += 1
                else:
                    publish(t, bool(deps) and tk.nchunks <= small)
                progress = True
            mirrored += take
        # ---- workers ----
        for w in range(workers):
            if len(holding[w]) < stash and claim < len(units):
                holding[w].append(claim)
                claim += 1
                progress = True
        for w in range(workers):
            ran = False
            for u in holding[w]:
                t, waits = units[u]
                if not complete(t):
                    if not waits:
                        violations += 1                    # a "resolved" unit whose dependencies are not complete
                    continue                               # stays held
                if ran:
                    continue
                ran = True
                chunks_done[t] += 1
                if chunks_done[t] == tasks[t].nchunks:
                    done[t] = True
                    completed += 1
                holding[w].remove(u)
                progress = True
                break
        if completed == n:
            return Result(False, rnd + 1, 0, completed, held_total, violations)
        if not progress:
            parked = sum(1 for h in holding if len(h) == stash)
            return Result(True, rnd + 1, parked, completed, held_total, violations)
    raise RuntimeError("model did not finish")


def producer_with_dependants(n_consumers, producer_chunks=64, dependent_chunks=16, consumer_chunks=1):
    """One large task, a large task that depends on it (held back while the first one runs), then
    n_consumers small tasks that each depend on the held one: the stream shape of a big producer and
    per-row consumers."""
    tasks = [Task(producer_chunks, (0, 0, 0), False), Task(dependent_chunks, (1, 0, 0), False)]
    for k in range(n_consumers):
        tasks.append(Task(consumer_chunks, (k + 1, 0, 0), False))
    return tasks


def chain_behind_held_task(n_links, link_chunks=4):
    """A held large task followed by a chain of small links, each depending on the previous one."""
    tasks = [Task(64, (0, 0, 0), False), Task(16, (1, 0, 0), False)]
    for _ in range(n_links):
        tasks.append(Task(link_chunks, (1, 0, 0), False))
    return tasks


def random_dag(rng, n_tasks, max_dist=200, p_fence=0.02):
    tasks = []
    for t in range(n_tasks):
        nchunks = int(rng.choice([1, 1, 2, 4, 5, 8, 40, 300]))
        deps = [0, 0, 0]
        for k in range(int(rng.integers(0, 4))):
            if t > 0:
                deps[k] = int(rng.integers(1, min(t, max_dist) + 1))
        tasks.append(Task(nchunks, tuple(deps), bool(rng.random() < p_fence)))
    return tasks
