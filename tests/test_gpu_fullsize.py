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


# Cost model of the batch-1 plan kernel's work partition (a byte of 8-bit codes costs 200, a 4-bit
# byte 230, a 2-bit group 0.73 and a 3-bit group 0.95 of a 4-bit one; units of 16 rows; one slice of
# the total per workgroup; two workgroups per compute unit, three or four when 30 % or 90 % of the
# cost is at 2 or 3 bits).  Only used to AIM samples at the rows where one
# workgroup's share ends and the next begins: if the kernel's table changes, the rows checked here
# are still valid samples, merely no longer the boundary ones.
def _unit_cost(K, bits):
    groups = K // 128
    return {2: groups * (64 * 230 * 730 // 1000), 3: groups * (64 * 230 * 950 // 1000), 4: groups * 64 * 230,
            8: groups * 128 * 200, 16: groups * 256 * 200}[bits]


def _partition_boundary_rows(entries, pattern, cus):
    """{entry: rows on either side of every cut that falls inside it}, cuts as the kernel places
    them: workgroup b starts at cost b C / G."""
    units = [(N + 15) // 16 for (_, _, K, N) in entries]
    ucost = [_unit_cost(K, int(b)) for (_, _, K, N), b in zip(entries, pattern)]
    incl = np.cumsum([u * c for u, c in zip(units, ucost)], dtype=np.int64)
    C = int(incl[-1])
    low = sum(u * c for u, c, b in zip(units, ucost, pattern) if int(b) in (2, 3))
    workgroups = cus * (4 if low * 10 >= C * 9 else 3 if low * 10 >= C * 3 else 2)
    out = {}
    for b in range(1, workgroups):
        t = b * C // workgroups
        e = int(np.searchsorted(incl, t, side="right"))
        excl = int(incl[e] - units[e] * ucost[e])
        row = 16 * ((t - excl) // ucost[e])
        N = entries[e][3]
        out.setdefault(e, set()).update(r for r in (row - 1, row, row + 15, row + 16) if 0 <= r < N)
    return out


def _check_rows(st, e, rows, bits, y):
    """Outputs y[:, rows] of entry e against the oracle, which regenerates and quantizes each weight
    row alone; the error is normalised by the largest oracle output computed for this call."""
    li, mname, K, N = st.entries[e]
    x = synth.activations(bench.SEED, st.xname(li, mname), st.M, K)
    refs = []
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
        refs.append(y_ref[:, 0].astype(np.float64))
    refs = np.stack(refs, axis=1)                               # [M][rows]
    ref_max = np.abs(refs).max()
    err = np.abs(y[:, rows] - refs).max(axis=0)
    worst = int(np.argmax(err))
    assert err[worst] <= TOL_Y * ref_max, (e, mname, bits, rows[worst], err[worst], ref_max)


def _check_stack(st, steps, n_entries, rows_per_entry, rng, boundary_entries=0):
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
            N = st.entries[e][3]
            y = st.ys[e].cpu().numpy().astype(np.float64)      # [M][N]
            rows = sorted(set([0, N - 1] + [int(r) for r in rng.integers(0, N, size=rows_per_entry)]))
            _check_rows(st, e, rows, int(pattern[e]), y)
        if boundary_entries:
            # the rows where the plan kernel's cost partition hands over from one workgroup to the next
            cuts = _partition_boundary_rows(st.entries, pattern, torch.cuda.get_device_properties(0).multi_processor_count)
            for e in rng.choice(sorted(cuts), size=min(boundary_entries, len(cuts)), replace=False):
                y = st.ys[e].cpu().numpy().astype(np.float64)
                _check_rows(st, int(e), sorted(cuts[int(e)])[:12], int(pattern[e]), y)
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
    _check_stack(st, steps=(0, 77), n_entries=28, rows_per_entry=6, rng=np.random.default_rng(0), boundary_entries=10)


def test_llama7b_stack_batch1_bits_4_8_16():
    # the three-way draw of the batch sweep, at batch 1
    st = bench.Stack("llama7b", M=1, bit_choices=(4, 8, 16))
    _check_stack(st, steps=(21,), n_entries=28, rows_per_entry=5, rng=np.random.default_rng(7), boundary_entries=8)


def test_llama13b_stack_batch1_outliers():
    st = bench.Stack("llama13b", M=1, bit_choices=(4, 8))
    _check_stack(st, steps=(6, 130), n_entries=21, rows_per_entry=5, rng=np.random.default_rng(8), boundary_entries=8)


def test_llama7b_stack_batch1_bits_2_4_8():
    st = bench.Stack("llama7b", M=1, bit_choices=(2, 4, 8))
    _check_stack(st, steps=(11,), n_entries=28, rows_per_entry=5, rng=np.random.default_rng(3), boundary_entries=8)


def test_llama7b_stack_batch16_bits_4_8_16():
    st = bench.Stack("llama7b", M=16, bit_choices=(4, 8, 16))
    _check_stack(st, steps=(3,), n_entries=21, rows_per_entry=4, rng=np.random.default_rng(1))


@pytest.mark.parametrize("M", [4, 32])
def test_llama7b_stack_batch_sweep_bits_4_8_16(M):
    # the other batch sizes of the sweep (one and two batch tiles of the streaming kernel)
    st = bench.Stack("llama7b", M=M, bit_choices=(4, 8, 16))
    _check_stack(st, steps=(9,), n_entries=14, rows_per_entry=3, rng=np.random.default_rng(10 + M))


def test_llama7b_stack_batch16_bits_2_4_8():
    # a plan of the streaming kernel's size whose layers hold 2-bit copies, served in the same launch
    st = bench.Stack("llama7b", M=16, bit_choices=(2, 4, 8))
    _check_stack(st, steps=(2,), n_entries=21, rows_per_entry=3, rng=np.random.default_rng(5))


def test_llama7b_stack_batch16_bits_3_4_8():
    # a plan of the streaming kernel's size whose layers hold 3-bit copies: the register-fed kernel
    # in 128-row tiles serves every entry
    st = bench.Stack("llama7b", M=16, bit_choices=(3, 4, 8))
    _check_stack(st, steps=(4,), n_entries=21, rows_per_entry=3, rng=np.random.default_rng(6))


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
        # sampled weight rows x sampled tokens, the error normalised by the largest oracle output
        # computed for this call
        ns = [0, N - 1] + [int(n) for n in rng.integers(0, N, size=10)]
        ms = [0, M - 1] + [int(m) for m in rng.integers(0, M, size=30)]
        refs, gots = [], []
        for n in ns:
            cr, sr, zr = oracle.quantize(w[n:n + 1], bits)
            refs.append(oracle.linear(x[ms], cr, sr, zr, bits)[:, 0].astype(np.float64))
            gots.append(y[ms, n].cpu().numpy().astype(np.float64))
        refs, gots = np.stack(refs), np.stack(gots)
        assert np.abs(gots - refs).max() <= TOL_Y * np.abs(refs).max(), (bits, np.abs(gots - refs).max(), np.abs(refs).max())
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


@pytest.mark.parametrize("per_row", [False, True])
@pytest.mark.parametrize("N,K", [(28672, 8192), (8192, 28672)])
def test_w8a8_slice_sampled_outputs(N, K, per_row):
    """The W8A8 prefill at the benchmark's shapes, with groups of 128 and with one scale per weight
    row: activation codes and scales of sampled tokens bit-exact, group sums exact everywhere,
    sampled outputs against the oracle."""
    M = 2048
    group = K if per_row else 128
    name = "full/prefill/%dx%d" % (N, K)
    w = synth.weight(0, name + "/w", N, K, 0.015)
    x = synth.activations(0, name + "/x", M, K)
    w_dev, x_dev = to_dev(w), to_dev(x)
    cb, sb, zb = fq.fq_packed_sizes(N, K, 8, group)
    c = torch.empty(cb, dtype=torch.uint8, device=DEV)
    s = torch.empty(sb // 4, dtype=torch.float32, device=DEV)
    z = torch.empty(zb, dtype=torch.uint8, device=DEV)
    fq.fq_quantize(w_dev, N, K, 8, group, c, s, z)
    layer = fq.Layer(N, K, group).attach(8, c, s, z)
    xq = torch.empty((M, K), dtype=torch.int8, device=DEV)
    sx = torch.empty(M, dtype=torch.float32, device=DEV)
    xsum = torch.empty((K // 128, M), dtype=torch.int32, device=DEV)
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
    fq.fq_quantize_act(x_dev, M, K, xq, sx, xsum)
    fq.fq_linear_w8a8(layer, xq, sx, xsum, M, y)
    torch.cuda.synchronize()
    assert torch.isfinite(y.float()).all()
    rng = np.random.default_rng(5)
    ms = [0, M - 1] + [int(m) for m in rng.integers(0, M, size=30)]
    xq_ref, sx_ref = oracle.quantize_act(x[ms])
    assert np.array_equal(xq[ms].cpu().numpy(), xq_ref)
    assert np.array_equal(sx[ms].cpu().numpy().view(np.uint32), sx_ref.view(np.uint32))
    sums = xq.view(M, K // 128, 128).sum(dim=2, dtype=torch.int32).t()
    assert torch.equal(xsum, sums)
    refs, gots = [], []
    for n in [0, N - 1] + [int(n) for n in rng.integers(0, N, size=10)]:
        cr, sr, zr = oracle.quantize(w[n:n + 1], 8, group=group)
        refs.append(oracle.linear_w8a8(xq_ref, sx_ref, cr, sr, zr, group=group)[:, 0].astype(np.float64))
        gots.append(y[ms, n].cpu().numpy().astype(np.float64))
    refs, gots = np.stack(refs), np.stack(gots)
    assert np.abs(gots - refs).max() <= TOL_Y * np.abs(refs).max(), (np.abs(gots - refs).max(), np.abs(refs).max())
