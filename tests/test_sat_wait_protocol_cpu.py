"""A CPU model of the grid-wide wait of hb_sat2d's one-launch kernel, run with FEWER execution slots
than workgroups (workgroups that are not resident together), tiny wait limits and random delays.

The protocol under test, in the kernel's own steps: every workgroup publishes its region's sums,
arrives (leaf counters, root counter, the last arrival raises `go`), then polls `go` a bounded
number of times.  A workgroup that stops waiting marks its region in `todo`, raises `late`, looks at
`go` once more and leaves if it is still down.  A workgroup that gets past the wait reads `late`
and, if it is set, claims marked regions one by one and finishes them.  Claims to check: every
thread ends (no workgroup ever waits without bound), every region is finished at least once, and no
region is finished before every workgroup has published its sums.
"""
import random
import threading
import time

import pytest


class Grid:
    def __init__(self, nwg, slots, wait_limit, seed):
        self.nwg, self.wait_limit = nwg, wait_limit
        self.slots = threading.Semaphore(slots)          # compute-unit residency
        self.mu = threading.Lock()                       # one lock = the memory side serving one access at a time
        self.nleaf = min(nwg, 16)
        self.leaf = [0] * self.nleaf
        self.root = 0
        self.go = 0
        self.late = 0
        self.todo = [0] * nwg
        self.published = [False] * nwg
        self.finished = [0] * nwg
        self.errors = []
        self.rng = random.Random(seed)

    def pause(self):
        if self.rng.random() < 0.3:
            time.sleep(self.rng.random() * 2e-4)

    def finish(self, region):
        with self.mu:
            if not all(self.published):
                self.errors.append(f"region {region} finished before every workgroup had published")
            self.finished[region] += 1

    def workgroup(self, wg):
        self.slots.acquire()
        try:
            self.pause()
            with self.mu:
                self.published[wg] = True
            lf = wg % self.nleaf
            leaf_target = (self.nwg - lf + self.nleaf - 1) // self.nleaf
            with self.mu:
                self.leaf[lf] += 1
                last_leaf = self.leaf[lf] == leaf_target
            if last_leaf:
                with self.mu:
                    self.root += 1
                    last = self.root == self.nleaf
                if last:
                    with self.mu:
                        self.go = 1
            passed, polls = True, 0
            while True:
                with self.mu:
                    if self.go:
                        break
                polls += 1
                if polls > self.wait_limit:
                    passed = False
                    break
                self.pause()
            if not passed:
                with self.mu:
                    self.todo[wg] = 1
                    self.late = 1
                self.pause()
                with self.mu:
                    go = self.go
                    if go and self.todo[wg] == 1:
                        self.todo[wg] = 2
                if not go:
                    return                                # leaves; a finisher takes the region
            with self.mu:
                late = self.late
            self.pause()
            self.finish(wg)
            if not late:
                return
            while True:
                claimed = -1
                with self.mu:
                    for r in range(self.nwg):
                        if self.todo[r] == 1:
                            self.todo[r] = 2
                            claimed = r
                            break
                if claimed < 0:
                    return
                self.pause()
                self.finish(claimed)
        finally:
            self.slots.release()


@pytest.mark.parametrize("nwg,slots,wait_limit", [(1, 1, 0), (16, 16, 50), (40, 7, 3), (40, 7, 0), (97, 5, 1),
                                                  (256, 16, 2), (64, 64, 0), (33, 1, 5)])
def test_wait_protocol_ends_and_finishes_every_region(nwg, slots, wait_limit):
    for seed in range(3):
        g = Grid(nwg, slots, wait_limit, seed)
        threads = [threading.Thread(target=g.workgroup, args=(w,), daemon=True) for w in range(nwg)]
        order = list(range(nwg))
        g.rng.shuffle(order)
        for i in order:
            threads[i].start()
        for t in threads:
            t.join(timeout=30)
            assert not t.is_alive(), "a workgroup never ended"
        assert not g.errors, g.errors[0]
        assert all(n >= 1 for n in g.finished), f"unfinished regions: {[r for r, n in enumerate(g.finished) if n == 0]}"
        assert g.go == 1 and g.root == g.nleaf and sum(g.leaf) == nwg
