"""A thread-per-workgroup model of the stage-ordered kernel's barrier protocol (CPU only).

The kernel (csrc/fq_staged.hip) separates two stages by a grid-wide barrier built from plain
device-scope atomics: 128 arrival counters that count up through the launch (workgroup b adds to
counter b % 128; after stage s counter l must hold (s + 1) * |{b : b % 128 = l}|), an abort flag, a
sticky count of launches that gave up, and a count of finished workgroups whose last arrival puts
counters and flag back to zero.  This model runs the same steps with one Python thread per
workgroup and checks what the kernel relies on:
  - no workgroup reads a stage's input before every workgroup has written the previous stage,
  - a bounded wait that runs out makes EVERY workgroup leave, whatever the others are doing,
  - after any launch, completed or given up, the sync words are clean for the next launch.
"""
import random
import threading
import time

import pytest

N_COUNTERS = 128


class SyncWords:
    """The plan's sync words; every access is one atomic operation (a lock stands in for the
    memory system's atomicity)."""

    def __init__(self):
        self.lock = threading.Lock()
        self.counter = [0] * N_COUNTERS
        self.abort = 0
        self.gave_up = 0
        self.done = 0

    def add(self, name, idx=None, v=1):
        with self.lock:
            if idx is None:
                old = getattr(self, name)
                setattr(self, name, old + v)
            else:
                old = getattr(self, name)[idx]
                getattr(self, name)[idx] = old + v
            return old

    def exchange(self, name, v):
        with self.lock:
            old = getattr(self, name)
            setattr(self, name, v)
            return old

    def snapshot(self):
        """What one poll of the wavefront sees: every counter and the flag (the lanes' loads are
        issued together; each word is read atomically, and the protocol does not rely on more)."""
        with self.lock:
            return list(self.counter), self.abort

    def load(self, name, idx=None):
        with self.lock:
            return getattr(self, name) if idx is None else getattr(self, name)[idx]

    def store(self, name, v, idx=None):
        with self.lock:
            if idx is None:
                setattr(self, name, v)
            else:
                getattr(self, name)[idx] = v


def members(G, l):
    return (G - l + N_COUNTERS - 1) // N_COUNTERS


def wait_stage(sync, s, G, wait_limit):
    it = 0
    while True:
        vals, aborted = sync.snapshot()
        if aborted:
            return False
        if all(vals[l] >= (s + 1) * members(G, l) for l in range(N_COUNTERS)):
            return True
        if it >= wait_limit:
            if sync.exchange("abort", 1) == 0:     # the first to give up counts the launch
                sync.add("gave_up")
            return False
        it += 1
        time.sleep(0.0001)


def workgroup(b, G, n_stages, sync, wait_limit, written, violations, delay, start_gate=None):
    if start_gate is not None:
        start_gate.wait()
    rng = random.Random(b)
    for s in range(n_stages):
        if delay:
            time.sleep(rng.random() * delay)
        written[s][b] = True                       # this workgroup's rows of stage s, write-through
        if s + 1 == n_stages:
            break
        sync.add("counter", b % N_COUNTERS)        # arrival, after the stores are acknowledged
        if not wait_stage(sync, s, G, wait_limit):
            break
        if not all(written[s]):                    # stage s + 1 reads what stage s wrote
            violations.append((b, s))
    if sync.add("done") == G - 1:                  # last one out puts the words back
        for l in range(N_COUNTERS):
            sync.store("counter", 0, l)
        sync.store("abort", 0)
        sync.store("done", 0)


def launch(G, n_stages, sync, wait_limit=10 ** 9, delay=0.0, late=()):
    written = [[False] * G for _ in range(n_stages)]
    violations = []
    gate = threading.Event()
    threads = [threading.Thread(target=workgroup,
                                args=(b, G, n_stages, sync, wait_limit, written, violations, delay,
                                      gate if b in late else None))
               for b in range(G)]
    for t in threads:
        t.start()
    return threads, gate, written, violations


def join_all(threads, timeout=60):
    for t in threads:
        t.join(timeout)
        assert not t.is_alive(), "a workgroup never left the kernel"


def clean(sync):
    return sync.counter == [0] * N_COUNTERS and sync.abort == 0 and sync.done == 0


@pytest.mark.parametrize("G,n_stages", [(1, 5), (7, 9), (32, 4), (45, 6), (140, 3)])
def test_stages_are_ordered_and_words_end_clean(G, n_stages):
    sync = SyncWords()
    for _ in range(3):                             # replays on the same words, as a HIP graph would
        threads, _, written, violations = launch(G, n_stages, sync, delay=0.0002)
        join_all(threads)
        assert violations == []
        assert all(all(w) for w in written)
        assert clean(sync) and sync.gave_up == 0


def test_counter_targets_cover_every_workgroup():
    for G in range(1, 300):
        assert sum(members(G, l) for l in range(N_COUNTERS)) == G
        for l in range(N_COUNTERS):
            assert members(G, l) == len([b for b in range(G) if b % N_COUNTERS == l])


def test_a_wait_that_runs_out_lets_everyone_leave_and_the_next_launch_is_clean():
    G, n_stages = 12, 6
    sync = SyncWords()
    # workgroups 3 and 7 are not resident until the others have given up
    threads, gate, written, violations = launch(G, n_stages, sync, wait_limit=50, late=(3, 7))
    for b, t in enumerate(threads):
        if b not in (3, 7):
            t.join(60)
            assert not t.is_alive()
    assert sync.gave_up == 1 and sync.abort == 1   # the flag stays up until the last one is out
    gate.set()                                     # the late ones start, see the flag, leave
    join_all(threads)
    assert violations == []
    assert not all(written[n_stages - 1])          # the launch did not finish its work
    assert clean(sync)
    gave_up = sync.gave_up
    threads, _, written, violations = launch(G, n_stages, sync, delay=0.0002)
    join_all(threads)
    assert violations == [] and all(all(w) for w in written)
    assert clean(sync) and sync.gave_up == gave_up


def test_zero_wait_limit_never_hangs():
    # the host-forced condition of the GPU test: with no polls allowed a wait succeeds only if
    # everyone has already arrived; whatever happens, everyone leaves and the words end clean
    for seed in range(5):
        G, n_stages = 9, 4
        sync = SyncWords()
        threads, _, _, violations = launch(G, n_stages, sync, wait_limit=0, delay=0.0003 * seed)
        join_all(threads)
        assert violations == []
        assert clean(sync)
