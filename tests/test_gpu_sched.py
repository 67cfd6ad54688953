"""GPU parity of the device-side precision scheduler (Sec. 4.4, Alg. 1) against the oracle:
the switch decisions are integers and must agree exactly -- which event fired at which
token, and the bit-width array after every run."""
import math

import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2506_12024_amd as fq
from gpu_util import DEV, to_dev

pytestmark = pytest.mark.gpu


def _gpu_run(H, n_entries, events, window, thre, per_trigger, start_bits=8, prefill=None):
    ev = np.asarray(events, dtype=np.int32).reshape(-1, 2)
    ev_entry = to_dev(np.ascontiguousarray(ev[:, 0]))
    ev_bits = to_dev(np.ascontiguousarray(ev[:, 1]))
    bits = torch.full((n_entries,), start_bits, dtype=torch.int32, device=DEV)
    ev_token = torch.full((max(len(ev), 1),), -1, dtype=torch.int32, device=DEV)
    state = torch.zeros(fq.fq_sched_state_bytes(window), dtype=torch.uint8, device=DEV)
    fq.fq_sched_init(state, window, thre, per_trigger, ev_entry, ev_bits, len(ev), bits, ev_token)
    if prefill is not None:
        pf = to_dev(prefill[0])
        fq.fq_sched_threshold_from_prefill(state, pf, pf.numel(), prefill[1])
    H_dev = to_dev(H)
    for t in range(len(H)):
        fq.fq_sched_step(state, H_dev[t:t + 1])
    next_event, tokens, thre_out, last_mean = fq.fq_sched_peek(state)
    return bits.cpu().numpy(), ev_token.cpu().numpy()[:len(ev)], next_event, tokens, thre_out, last_mean


def test_hand_case_on_gpu():
    pple = [4, 4, 1, 1, 1, 1, 1, 1, 3, 3, 3, 1, 1, 1]
    H = np.log(np.array(pple, dtype=np.float64)).astype(np.float32)
    bits, ev_token, ne, tokens, _, _ = _gpu_run(H, 8, [(5, 4), (2, 4), (7, 4)], 3, 2.1, 1)
    assert list(ev_token) == [3, 6, 12]
    assert list(bits) == [8, 8, 4, 8, 8, 4, 8, 4]
    assert ne == 3 and tokens == len(pple)


@pytest.mark.parametrize("window,per_trigger,thre,T", [(20, 1, 25.0, 3000), (20, 3, 30.0, 2500), (7, 2, 22.0, 800)])
def test_scheduler_matches_oracle(window, per_trigger, thre, T):
    n = 224
    noise = synth.normal_f32(0, "sched/par/noise/%d" % window, T, 0.3)
    H = (np.log(40.0) - 1.5 * np.arange(T) / T + noise).astype(np.float32)
    events = [(int(e), 4) for e in np.random.default_rng(window).permutation(n)]
    ref_bits = np.full(n, 8, dtype=np.int32)
    ref = oracle.Scheduler(ref_bits, events, window=window, thre=thre, per_trigger=per_trigger)
    for h in H:
        ref.step(float(h))
    bits, ev_token, ne, tokens, thre_out, last_mean = _gpu_run(H, n, events, window, thre, per_trigger)
    assert ne == ref.next_event and 0 < ne
    assert tokens == T
    assert np.array_equal(ev_token, ref.ev_token)
    assert np.array_equal(bits, ref_bits)
    assert thre_out == thre
    assert abs(last_mean - ref.last_mean) <= 1e-12 * ref.last_mean


def test_ladder_and_threshold_from_prefill():
    # FP16 -> INT8 -> INT4 ladder as a list of events; threshold = mean PPLE of the last
    # 20 of 64 prefill positions
    n, T = 12, 600
    prefill_H = (np.log(30.0) + synth.normal_f32(1, "sched/par/prefill", 64, 0.2)).astype(np.float32)
    H = (np.log(30.0) - 1.2 * np.arange(T) / T + synth.normal_f32(1, "sched/par/dec", T, 0.2)).astype(np.float32)
    events = [(e, 8) for e in range(n)] + [(e, 4) for e in range(n)]
    ref_bits = np.full(n, 16, dtype=np.int32)
    ref = oracle.Scheduler(ref_bits, events, window=20, thre=0.0, per_trigger=2)
    ref.threshold_from_prefill(prefill_H, 20)
    for h in H:
        ref.step(float(h))
    bits, ev_token, ne, tokens, thre_out, _ = _gpu_run(H, n, events, 20, 0.0, 2, start_bits=16,
                                                       prefill=(prefill_H, 20))
    assert abs(thre_out - ref.thre) <= 1e-12 * ref.thre
    assert ne == ref.next_event and ne > 0
    assert np.array_equal(ev_token, ref.ev_token)
    assert np.array_equal(bits, ref_bits)


def test_scheduler_drives_a_plan_without_host_round_trip():
    # entropy kernel -> scheduler step -> plan, all on one stream, the bit-width array never
    # leaves the device; the linears must follow the oracle's decisions token by token
    from gpu_util import make_layer
    N, K, T, V = 64, 1024, 60, 2048
    layers, xs, ys, packs, xs_np = [], [], [], [], []
    for i in range(3):
        w = synth.weight(0, "sched/plan/w%d" % i, N, K, 0.02)
        layer, packed = make_layer(w, (4, 8))
        x = synth.activations(0, "sched/plan/x%d" % i, 1, K)
        layers.append(layer); packs.append(packed); xs_np.append(x)
        xs.append(to_dev(x)); ys.append(torch.zeros((1, N), dtype=torch.float16, device=DEV))
    ws = torch.empty(fq.Plan.workspace_bytes(3), dtype=torch.uint8, device=DEV)
    plan = fq.Plan(layers, xs, ys, 1, ws)
    # logits whose entropy falls over time: scale up a fixed random vector
    base = synth.normal_f32(0, "sched/plan/logits", V, 1.0)
    logits = np.stack([base * (0.5 + 0.05 * t) for t in range(T)]).astype(np.float32)
    H_ref, _ = oracle.entropy_kl(logits)
    events = [(1, 4), (0, 4), (2, 4)]
    ref_bits = np.full(3, 8, dtype=np.int32)
    thre = float(np.exp(H_ref[T // 3]))
    ref = oracle.Scheduler(ref_bits, events, window=5, thre=thre, per_trigger=1)
    logits_dev = to_dev(logits)
    H_dev = torch.zeros(T, dtype=torch.float32, device=DEV)
    bits = torch.full((3,), 8, dtype=torch.int32, device=DEV)
    ev = np.asarray(events, dtype=np.int32)
    ev_entry, ev_bits = to_dev(np.ascontiguousarray(ev[:, 0])), to_dev(np.ascontiguousarray(ev[:, 1]))
    state = torch.zeros(fq.fq_sched_state_bytes(5), dtype=torch.uint8, device=DEV)
    fq.fq_sched_init(state, 5, thre, 1, ev_entry, ev_bits, 3, bits, None)
    y_hist = []
    for t in range(T):
        plan.run(bits)
        y_hist.append([y.clone() for y in ys])
        fq.fq_entropy_kl(logits_dev[t], None, 1, V, H_dev[t:t + 1], None)
        fq.fq_sched_step(state, H_dev[t:t + 1])
    torch.cuda.synchronize()
    switched = 0
    for t in range(T):
        # the plan of token t ran with the bit-widths decided after token t-1
        for i in range(3):
            b = int(ref_bits[i])
            c, s, z = (p.cpu().numpy() for p in packs[i][b])
            y_ref = oracle.linear(xs_np[i], c, s, z, b).astype(np.float64)
            got = y_hist[t][i].cpu().numpy().astype(np.float64)
            assert np.abs(got - y_ref).max() <= 2e-3 * np.abs(y_ref).max(), (t, i, b)
        # feed the oracle the entropy the GPU produced (checked against the oracle's own below)
        assert abs(H_dev[t].item() - H_ref[t]) <= 1e-4 * abs(H_ref[t]) + 1e-7
        switched += ref.step(float(H_ref[t]))
    assert switched == 3 and np.array_equal(bits.cpu().numpy(), ref_bits)


def test_events_outside_the_array_are_passed_over():
    # a replacement order ranked over more linears than the plan has, and an event with no valid
    # bit-width: neither may write anything; the guard words around the array stay as they were
    pple = [1.0] * 12
    H = np.log(np.array(pple, dtype=np.float64)).astype(np.float32)
    n = 4
    guard = torch.full((n + 8,), 77, dtype=torch.int32, device=DEV)
    bits = guard[4:4 + n]
    bits.fill_(8)
    ev = np.array([(1, 4), (9, 4), (-3, 4), (2, 5), (3, 4)], dtype=np.int32)
    ev_entry, ev_bits = to_dev(np.ascontiguousarray(ev[:, 0])), to_dev(np.ascontiguousarray(ev[:, 1]))
    ev_token = torch.full((len(ev),), -1, dtype=torch.int32, device=DEV)
    state = torch.zeros(fq.fq_sched_state_bytes(2), dtype=torch.uint8, device=DEV)
    fq.fq_sched_init(state, 2, 5.0, 1, ev_entry, ev_bits, len(ev), bits, ev_token, entries=n)
    H_dev = to_dev(H)
    for t in range(len(H)):
        fq.fq_sched_step(state, H_dev[t:t + 1])
    next_event, tokens, _, _ = fq.fq_sched_peek(state)
    assert next_event == len(ev) and tokens == len(pple)
    assert guard.cpu().tolist() == [77] * 4 + [8, 4, 8, 4] + [77] * 4
    assert ev_token.cpu().tolist() == [1, -2, -2, -2, 9]
