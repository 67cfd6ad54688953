"""The split entropy / KL reduction (Sec. 3.1, Eq. (5): a few rows of a large vocabulary) and the
fused output layer (Alg. 1: logits, entropy and next token in one pass) combine their workgroups'
partial results in static device arrays of the library, of which every stream owns a copy: calls
that overlap on different streams must give what the same calls give one after the other.  This
file uses up the copies of the process (sixteen streams per device) and is therefore collected
after the other files that call these two entry points."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2506_12024_amd as fq
from gpu_util import DEV, to_dev

pytestmark = pytest.mark.gpu


def test_calls_overlapping_on_streams_match_serial_calls():
    n_streams, reps = 4, 24
    R, V, K, M = 6, 32000, 1024, 2
    Vh = 20000
    a = [to_dev(synth.logits_pair(3, "banks/ent/%d" % s, R, V)[0]) for s in range(n_streams)]
    b = [to_dev(synth.logits_pair(3, "banks/ent/%d" % s, R, V)[1]) for s in range(n_streams)]
    w = [to_dev(synth.weight(3, "banks/w/%d" % s, Vh, K, 0.03)) for s in range(n_streams)]
    x = [to_dev(synth.activations(3, "banks/x/%d" % s, M, K)) for s in range(n_streams)]

    def outputs():
        return ([torch.full((reps, R), float("nan"), device=DEV) for _ in range(n_streams)],
                [torch.full((reps, R), float("nan"), device=DEV) for _ in range(n_streams)],
                [torch.full((reps, M), float("nan"), device=DEV) for _ in range(n_streams)],
                [torch.full((reps, M), -1, dtype=torch.int32, device=DEV) for _ in range(n_streams)])

    # one after the other on the current stream
    H0, KL0, HL0, AM0 = outputs()
    for s in range(n_streams):
        for i in range(reps):
            fq.fq_entropy_kl(a[s], b[s], R, V, H0[s][i], KL0[s][i])
            fq.fq_lm_head_entropy(x[s], w[s], M, Vh, K, None, HL0[s][i], AM0[s][i])
    torch.cuda.synchronize()
    # the same calls interleaved over four streams
    H1, KL1, HL1, AM1 = outputs()
    streams = [torch.cuda.Stream() for _ in range(n_streams)]
    for i in range(reps):
        for s in range(n_streams):
            fq.fq_entropy_kl(a[s], b[s], R, V, H1[s][i], KL1[s][i], stream=streams[s])
            fq.fq_lm_head_entropy(x[s], w[s], M, Vh, K, None, HL1[s][i], AM1[s][i], stream=streams[s])
    torch.cuda.synchronize()
    for s in range(n_streams):
        assert torch.equal(H0[s], H1[s]) and torch.equal(KL0[s], KL1[s]), s
        assert torch.equal(HL0[s], HL1[s]) and torch.equal(AM0[s], AM1[s]), s
        assert torch.isfinite(H1[s]).all() and torch.isfinite(HL1[s]).all()
    H_ref, KL_ref = oracle.entropy_kl(a[0].cpu().numpy(), b[0].cpu().numpy())
    assert np.all(np.abs(H1[0][reps - 1].cpu().numpy() - H_ref) <= 1e-4 * np.abs(H_ref) + 1e-7)
    assert np.all(np.abs(KL1[0][reps - 1].cpu().numpy() - KL_ref) <= 1e-4 * np.abs(KL_ref) + 1e-7)


def test_more_streams_than_copies():
    # every further stream: the entropy call takes its path without scratch (same results to the
    # tolerance), the output layer refuses
    R, V, K, M, Vh = 3, 32000, 512, 1, 3000
    a_np, b_np = synth.logits_pair(4, "banks/more", R, V)
    H_ref, KL_ref = oracle.entropy_kl(a_np, b_np)
    a, b = to_dev(a_np), to_dev(b_np)
    w, x = to_dev(synth.weight(4, "banks/more/w", Vh, K, 0.03)), to_dev(synth.activations(4, "banks/more/x", M, K))
    refused = 0
    keep = []
    for i in range(fq.FQ_SCRATCH_BANKS + 3):
        st = torch.cuda.Stream()
        keep.append(st)
        H = torch.full((R,), float("nan"), device=DEV)
        KL = torch.full((R,), float("nan"), device=DEV)
        fq.fq_entropy_kl(a, b, R, V, H, KL, stream=st)
        HL = torch.full((M,), float("nan"), device=DEV)
        try:
            fq.fq_lm_head_entropy(x, w, M, Vh, K, None, HL, None, stream=st)
        except fq.FlexqError as e:
            refused += 1
            assert e.code == -6  # FQ_ERR_HIP
        st.synchronize()
        assert np.all(np.abs(H.cpu().numpy() - H_ref) <= 1e-4 * np.abs(H_ref) + 1e-7), i
        assert np.all(np.abs(KL.cpu().numpy() - KL_ref) <= 1e-4 * np.abs(KL_ref) + 1e-7), i
    assert refused >= 3
