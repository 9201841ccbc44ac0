"""Visibility inside a kernel that never ends.  The eight dies of the GPU have one second-level
cache each, not coherent with one another for ordinary accesses, and the persistent kernel never
reaches the kernel boundary where they are written back and invalidated: every hand-off of data from
one workgroup to another rests on the cache policy the kernel's accesses carry (stores write
through, loads do not hit stale lines) and on the done-word protocol.  This is the soak test of that:
a million producer -> consumer hand-offs whose consumer was claimed by another workgroup, mostly on
another die, while the producer was still running, over buffers that are rewritten every other link
(so a reader that kept a line of the previous contents would be caught), with integer payloads that
make one stale word anywhere show at the end of its chain."""
import numpy as np
import pytest

from paper_2604_17861_amd import runtime as R
from paper_2604_17861_amd import streams as S

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("push_ring,n_chains,length", [(1, 256, 4096), (0, 256, 4096), (1, 8, 32768), (0, 8, 32768)])
def test_a_million_handoffs_between_workgroups(push_ring, n_chains, length):
    """256 chains round-robin: a million hand-offs, nearly all to another workgroup, seven in eight to
    another die.  8 chains: a quarter of a million hand-offs in which the consumer's workgroup is
    already waiting on the done word while the producer still writes (the tightest hand-off there is)."""
    from gpu_helpers import DevicePools
    import oracle
    from helpers import HostPools
    numel = 1024
    s = S.handoff_chains(n_chains, length, numel)
    assert len(s) == (1 << 20 if n_chains == 256 else 1 << 18)
    dp = DevicePools(s)
    print("handoffs: %d tasks, ring in %s memory" % (len(s), "device" if push_ring else "host"), flush=True)
    with R.Runtime(0, idle_exit_ms=30000, wait_timeout_ms=30000, push_ring=push_ring, trace_entries=1 << 20,
                   completion_log=1 << 20) as rt:
        rt.register_table(s.table)
        assert rt.peek_queue().push_ring == push_ring
        rt.submit_from_threads(dp.tasks, 1, 64, 1)
        rt.wait()
        comps = rt.completions(0, len(s))
        tr = rt.trace(0, len(s))
    assert np.all(comps["status"] == 0)
    # who handed over to whom: the workgroup that finished link t-1 and the one that ran link t
    wg = tr["workgroup"].astype(np.int64).reshape(length, n_chains)
    other_wg = wg[1:] != wg[:-1]
    other_die = (wg[1:] % 8) != (wg[:-1] % 8)                 # workgroups are dealt round-robin over the 8 dies
    started_before = tr["t_start"].reshape(length, n_chains)[1:] < tr["t_done"].reshape(length, n_chains)[:-1]
    print("hand-offs %d: to another workgroup %d, to another die %d, consumer claimed while the producer ran %d"
          % (other_wg.size, other_wg.sum(), other_die.sum(), started_before.sum()), flush=True)
    if n_chains == 256:
        assert other_wg.sum() >= 1_000_000 and other_die.sum() >= 800_000
    else:
        assert started_before.sum() >= 100_000 and other_die.sum() >= 150_000
    # the end of every chain: x0 + the sum of the operands it was given, exactly
    a0 = s.pools[0].host_image().view(np.int32).reshape(n_chains, numel)
    ops = s.pools[2].host_image().view(np.int32).reshape(-1, numel)
    which = s.info["which"]                                    # [link, chain]
    want = a0.astype(np.int64)
    counts = np.zeros((n_chains, ops.shape[0]), np.int64)
    for c in range(n_chains):
        counts[c] = np.bincount(which[:, c], minlength=ops.shape[0])
    want = (want + counts @ ops.astype(np.int64)).astype(np.uint64).astype(np.uint32).view(np.int32)     # wrap-around
    got = dp.download([0])[0].view(np.int32).reshape(n_chains, numel)          # an even number of links: the result is in buffer A
    bad = np.nonzero((got != want).any(axis=1))[0]
    assert bad.size == 0, "first chain with a wrong end: %d (element %d)" % (bad[0], np.nonzero(got[bad[0]] != want[bad[0]])[0][0])
    # ... and the sequential oracle on the same stream, a sample of whole chains (every link of them)
    hp = HostPools(s)
    impl = s.impl_for()
    for c in (0, n_chains // 3, n_chains - 1):
        idx = np.arange(c, len(s), n_chains)
        sub = np.ascontiguousarray(hp.tasks[idx])
        st = oracle.run_stream(sub, np.ascontiguousarray(impl[idx]))
        assert np.all(st == 0)
        assert np.array_equal(hp.arrays[0].view(np.int32).reshape(n_chains, numel)[c], got[c]), c
