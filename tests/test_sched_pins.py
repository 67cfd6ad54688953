"""Pins for the oracle of the token-wise precision switching (Sec. 4.4, Alg. 1): a hand-worked
run, invariants that the method's description fixes, and a brute-force recomputation of the
sliding average."""
import math
import os

import numpy as np

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sched_hand_case.txt")


def test_hand_worked_run():
    pple, expect = None, None
    for line in open(GOLDEN):
        if line.startswith("ppple:"):
            pple = [float(v) for v in line.split(":")[1].split()]
        if line.startswith("switch_tokens:"):
            expect = [int(v) for v in line.split(":")[1].split()]
    bits = np.full(8, 8, dtype=np.int32)
    s = oracle.Scheduler(bits, [(5, 4), (2, 4), (7, 4)], window=3, thre=2.1)
    fired = []
    for t, p in enumerate(pple):
        if s.step(math.log(p)):
            fired.append(t)
    assert fired == expect
    assert list(s.ev_token) == expect
    assert list(bits) == [8, 8, 4, 8, 8, 4, 8, 4]
    assert s.next_event == 3


def _run(entropies, n_entries, events, window, thre, per_trigger=1):
    bits = np.full(n_entries, 8, dtype=np.int32)
    s = oracle.Scheduler(bits, events, window=window, thre=thre, per_trigger=per_trigger)
    history = []
    for h in entropies:
        history.append((s.step(float(h)), bits.copy(), s.last_mean))
    return s, history


def test_invariants_on_random_run():
    # PPLE decaying with the token index, as the paper observes (Sec. 4.2, Fig. 5), plus noise
    n, T, window = 32, 3000, 20
    noise = synth.normal_f32(0, "sched/pins/noise", T, 0.3)
    H = (np.log(40.0) - 1.5 * np.arange(T) / T + noise).astype(np.float32)
    events = [(int(e), 4) for e in np.random.default_rng(0).permutation(n)]
    thre = 25.0
    s, hist = _run(H, n, events, window, thre)
    pple = np.exp(H.astype(np.float64))
    last_switch = -1
    n_switched = 0
    for t, (applied, bits, mean) in enumerate(hist):
        if applied:
            # never before a full window of tokens generated since the previous switch
            assert t - last_switch >= window
            # brute force: the average that triggered is the mean of the last `window` PPLEs
            assert abs(mean - pple[t - window + 1:t + 1].mean()) < 1e-9 * mean
            assert mean < thre
            # exactly the next entry of the order went to 4 bits
            assert applied == 1
            assert bits[events[n_switched][0]] == 4
            n_switched += 1
            last_switch = t
        else:
            # no switch: either the window is still filling, or the average is not below
            # the threshold, or every event has fired
            since = t - last_switch
            if since >= window and n_switched < len(events):
                assert pple[t - window + 1:t + 1].mean() >= thre * (1 - 1e-12)
        # bit-widths only ever go down, and only entries already reached in the order change
        assert (bits == 4).sum() == n_switched
    assert 0 < n_switched <= n
    # precision is never raised again and unswitched entries keep their width
    final = hist[-1][1]
    for i, (e, _) in enumerate(events):
        assert final[e] == (4 if i < n_switched else 8)


def test_never_switches_above_threshold_and_ladder():
    H = np.full(200, math.log(10.0), dtype=np.float32)
    s, hist = _run(H, 4, [(0, 4), (1, 4)], window=20, thre=9.99)
    assert all(a == 0 for a, _, _ in hist)
    # below the threshold from the start: one trigger per full window, per_trigger events each,
    # over a 16 -> 8 -> 4 ladder given as events
    bits = np.full(3, 16, dtype=np.int32)
    ladder = [(0, 8), (1, 8), (2, 8), (0, 4), (1, 4), (2, 4)]
    s = oracle.Scheduler(bits, ladder, window=5, thre=11.0, per_trigger=2)
    fired = [t for t in range(40) if s.step(math.log(10.0))]
    assert fired == [4, 9, 14]
    assert list(s.ev_token) == [4, 4, 9, 9, 14, 14]
    assert list(bits) == [4, 4, 4]


def test_threshold_from_prefill_is_mean_ppl_of_last_positions():
    H = np.log(np.array([100, 50, 8, 4, 2, 1], dtype=np.float64)).astype(np.float32)
    s = oracle.Scheduler(np.zeros(1, dtype=np.int32), [], window=20)
    s.threshold_from_prefill(H, 3)
    assert abs(s.thre - (4 + 2 + 1) / 3) < 1e-6
    s.threshold_from_prefill(H, 100)  # more than there are: all of them
    assert abs(s.thre - 165 / 6) < 1e-5
