"""Full-size parity, in the launch configuration bench.py times: the whole synthetic stack
is resident, one plan launch runs every linear with device-side bit-widths, and sampled
outputs are recomputed one by one by the CPU oracle from regenerated weight rows (the input
generator can reproduce any row alone; quantization is per row and group, so a row can be
quantized alone too).  Properties that hold at any size cover the rest: every output is
written and finite."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2506_12024_amd as fq
import bench
from gpu_util import DEV, to_dev

pytestmark = pytest.mark.gpu

TOL_Y = 2e-3


def _check_stack(st, steps, n_entries, rows_per_entry, rng):
    n = len(st.layers)
    for step in steps:
        for y in st.ys:
            y.fill_(float("nan"))
        st.run_linears(step)
        torch.cuda.synchronize()
        pattern = st.patterns[step % bench.N_PATTERNS]
        # any-size property: every output of every linear was written and is finite
        for y in st.ys:
            assert torch.isfinite(y.float()).all()
        for e in rng.choice(n, size=n_entries, replace=False):
            li, mname, K, N = st.entries[e]
            bits = int(pattern[e])
            y = st.ys[e].cpu().numpy().astype(np.float64)      # [M][N]
            ymax = np.abs(y).max()
            x = synth.activations(bench.SEED, st.xname(li, mname), st.M, K)
            rows = sorted(set([0, N - 1] + list(rng.integers(0, N, size=rows_per_entry))))
            for r in rows:
                w_row = synth.weight(bench.SEED, st.wname(li, mname), N, K, st.std, outlier_p=st.outl,
                                     row0=int(r), rows=1)
                if bits == 16:
                    y_ref = oracle.linear(x, w_row, None, None, 16)
                else:
                    c, s, z = oracle.quantize(w_row, bits)
                    # the resident packed row is bit-identical to the oracle's
                    cg, sg, zg = st.layers[e]._keep[bits]
                    row_bytes = K * bits // 8
                    assert np.array_equal(cg[r * row_bytes:(r + 1) * row_bytes].cpu().numpy(), c[0])
                    assert np.array_equal(sg[r * (K // 128):(r + 1) * (K // 128)].cpu().numpy(), s[0])
                    assert np.array_equal(zg[r * (K // 128):(r + 1) * (K // 128)].cpu().numpy(), z[0])
                    y_ref = oracle.linear(x, c, s, z, bits)
                err = np.abs(y[:, r] - y_ref[:, 0].astype(np.float64)).max()
                assert err <= TOL_Y * ymax, (step, e, mname, bits, r, err, ymax)
        # the step's entropy / KL
        st.run_entropy(step)
        torch.cuda.synchronize()
        i, M = step % bench.N_PATTERNS, st.M
        a, b = st.logits_host
        H_ref, KL_ref = oracle.entropy_kl(a[i * M:(i + 1) * M], b[i * M:(i + 1) * M])
        H = st.H[i].cpu().numpy().astype(np.float64)
        KL = st.KL[i].cpu().numpy().astype(np.float64)
        assert np.all(np.abs(H - H_ref) <= 1e-4 * np.abs(H_ref) + 1e-7)
        assert np.all(np.abs(KL - KL_ref) <= 1e-4 * np.abs(KL_ref) + 1e-7)


def test_llama7b_stack_batch1_mixed_w4_w8():
    st = bench.Stack("llama7b", M=1, bit_choices=(4, 8))
    _check_stack(st, steps=(0, 77), n_entries=28, rows_per_entry=6, rng=np.random.default_rng(0))


def test_llama7b_stack_batch1_bits_2_4_8():
    st = bench.Stack("llama7b", M=1, bit_choices=(2, 4, 8))
    _check_stack(st, steps=(11,), n_entries=28, rows_per_entry=5, rng=np.random.default_rng(3))


def test_llama7b_stack_batch16_bits_4_8_16():
    st = bench.Stack("llama7b", M=16, bit_choices=(4, 8, 16))
    _check_stack(st, steps=(3,), n_entries=21, rows_per_entry=4, rng=np.random.default_rng(1))


@pytest.mark.parametrize("M", [4, 32])
def test_llama7b_stack_batch_sweep_bits_4_8_16(M):
    # the other batch sizes of the sweep (one and two batch tiles of the streaming kernel)
    st = bench.Stack("llama7b", M=M, bit_choices=(4, 8, 16))
    _check_stack(st, steps=(9,), n_entries=14, rows_per_entry=3, rng=np.random.default_rng(10 + M))


def test_llama7b_stack_batch16_bits_2_4_8():
    # a plan of the streaming kernel's size whose layers hold 2-bit copies: two kernels per launch
    st = bench.Stack("llama7b", M=16, bit_choices=(2, 4, 8))
    _check_stack(st, steps=(2,), n_entries=21, rows_per_entry=3, rng=np.random.default_rng(5))


def test_llama13b_stack_batch8_outliers():
    st = bench.Stack("llama13b", M=8, bit_choices=(4, 8))
    _check_stack(st, steps=(5,), n_entries=21, rows_per_entry=4, rng=np.random.default_rng(2))


@pytest.mark.parametrize("N,K", [(28672, 8192), (8192, 28672)])
def test_prefill_slice_sampled_outputs(N, K):
    M = 2048
    name = "full/prefill/%dx%d" % (N, K)
    w = synth.weight(0, name + "/w", N, K, 0.015)
    x = synth.activations(0, name + "/x", M, K)
    w_dev, x_dev = to_dev(w), to_dev(x)
    y = torch.empty((M, N), dtype=torch.float16, device=DEV)
    rng = np.random.default_rng(3)
    for bits in (4, 8):
        cb, sb, zb = fq.fq_packed_sizes(N, K, bits)
        c = torch.empty(cb, dtype=torch.uint8, device=DEV)
        s = torch.empty(sb // 4, dtype=torch.float32, device=DEV)
        z = torch.empty(zb, dtype=torch.uint8, device=DEV)
        fq.fq_quantize(w_dev, N, K, bits, 128, c, s, z)
        layer = fq.Layer(N, K).attach(bits, c, s, z)
        y.fill_(float("nan"))
        fq.fq_linear(layer, bits, x_dev, M, y)
        torch.cuda.synchronize()
        assert torch.isfinite(y.float()).all()
        ymax = float(y.float().abs().max())
        for n in [0, N - 1] + list(rng.integers(0, N, size=10)):
            cr, sr, zr = oracle.quantize(w[n:n + 1], bits)
            ms = [0, M - 1] + list(rng.integers(0, M, size=6))
            y_ref = oracle.linear(x[ms], cr, sr, zr, bits)[:, 0].astype(np.float64)
            got = y[ms, int(n)].cpu().numpy().astype(np.float64)
            assert np.abs(got - y_ref).max() <= TOL_Y * ymax, (bits, n)
        del c, s, z, layer


def test_batched_entropy_kl_full_size_sampled_rows():
    R, V = 2048, 128256
    a, b = synth.logits_pair(0, "full/entropy", R, V)
    a_dev, b_dev = to_dev(a), to_dev(b)
    H = torch.full((R,), float("nan"), device=DEV)
    KL = torch.full((R,), float("nan"), device=DEV)
    fq.fq_entropy_kl(a_dev, b_dev, R, V, H, KL)
    torch.cuda.synchronize()
    assert torch.isfinite(H).all() and torch.isfinite(KL).all()
    assert (KL >= 0).all() and (H > 0).all() and (H < np.log(V)).all()
    rows = [0, R - 1] + list(np.random.default_rng(4).integers(0, R, size=14))
    H_ref, KL_ref = oracle.entropy_kl(a[rows], b[rows])
    Hn = H.cpu().numpy().astype(np.float64)[rows]
    KLn = KL.cpu().numpy().astype(np.float64)[rows]
    assert np.all(np.abs(Hn - H_ref) <= 1e-4 * np.abs(H_ref) + 1e-7)
    assert np.all(np.abs(KLn - KL_ref) <= 1e-4 * np.abs(KL_ref) + 1e-7)


@pytest.mark.parametrize("N,K", [(28672, 8192), (8192, 28672)])
def test_w8a8_slice_sampled_outputs(N, K):
    """The W8A8 prefill at the benchmark's shapes: activation codes and scales of sampled tokens
    bit-exact, group sums exact everywhere, sampled outputs against the oracle."""
    M = 2048
    name = "full/prefill/%dx%d" % (N, K)
    w = synth.weight(0, name + "/w", N, K, 0.015)
    x = synth.activations(0, name + "/x", M, K)
    w_dev, x_dev = to_dev(w), to_dev(x)
    cb, sb, zb = fq.fq_packed_sizes(N, K, 8)
    c = torch.empty(cb, dtype=torch.uint8, device=DEV)
    s = torch.empty(sb // 4, dtype=torch.float32, device=DEV)
    z = torch.empty(zb, dtype=torch.uint8, device=DEV)
    fq.fq_quantize(w_dev, N, K, 8, 128, c, s, z)
    layer = fq.Layer(N, K).attach(8, c, s, z)
    xq = torch.empty((M, K), dtype=torch.int8, device=DEV)
    sx = torch.empty(M, dtype=torch.float32, device=DEV)
    xsum = torch.empty((K // 128, M), dtype=torch.int32, device=DEV)
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
    fq.fq_quantize_act(x_dev, M, K, xq, sx, xsum)
    fq.fq_linear_w8a8(layer, xq, sx, xsum, M, y)
    torch.cuda.synchronize()
    assert torch.isfinite(y.float()).all()
    rng = np.random.default_rng(5)
    ms = [0, M - 1] + list(rng.integers(0, M, size=6))
    xq_ref, sx_ref = oracle.quantize_act(x[ms])
    assert np.array_equal(xq[ms].cpu().numpy(), xq_ref)
    assert np.array_equal(sx[ms].cpu().numpy().view(np.uint32), sx_ref.view(np.uint32))
    sums = xq.view(M, K // 128, 128).sum(dim=2, dtype=torch.int32).t()
    assert torch.equal(xsum, sums)
    ymax = float(y.float().abs().max())
    for n in [0, N - 1] + list(rng.integers(0, N, size=10)):
        cr, sr, zr = oracle.quantize(w[n:n + 1], 8)
        y_ref = oracle.linear_w8a8(xq_ref, sx_ref, cr, sr, zr)[:, 0].astype(np.float64)
        got = y[ms, int(n)].cpu().numpy().astype(np.float64)
        assert np.abs(got - y_ref).max() <= TOL_Y * ymax, n
