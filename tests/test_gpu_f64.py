"""GPU parity of the fp64 tasks (the paper's own element type) against the fp64 oracle.

Tolerance: both sides round every product once to fp64; the oracle then accumulates in
long double, the GPU in fp64 in its own order.  A sum of K fp64 terms in any order is
within (K - 1) * 2^-53 * sum|term| of the exact sum; the discount factor 1 - dis[j]
rounded once and the fused p * (1 - dis) add at most 2 * 2^-53 per term.  With K <= 4096
in these cases the bound is below 5e-13; the tests use 1e-12.  COUNT_GT is an integer
count and is compared bit for bit, as are all tasks on dyadic data whose every partial
sum is exactly representable.
"""
import numpy as np
import pytest

import oracle
from parity import worst_ratio

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

TOL_F64 = 1e-12
TASKS = [0, 1, 2, 3]
FORMS = [0, 1, 2, 3]


@pytest.fixture(scope="module")
def am():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2305_08872_amd as am
    am.load_library()
    return am


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def make_case(form, M, N, K, seed, exact=False):
    g = np.random.Generator(np.random.PCG64(seed))
    if exact:
        A = g.integers(-8, 9, (M, K)).astype(np.float64)
        B = g.integers(-8, 9, (K, N)).astype(np.float64)
    else:
        A = g.standard_normal((M, K)) * 2
        B = g.standard_normal((K, N)) * 2
    shape = {0: (N,), 1: (M,), 2: (1,), 3: (M, N)}[form]
    th = (g.integers(-24, 25, shape) / 2.0) if exact else g.standard_normal(shape) * 3
    dis = (g.integers(0, 9, N) / 8.0) if exact else g.uniform(0, 1, N)
    R_in = g.integers(-5, 6, (M, N)).astype(np.float64)
    return A, B, np.asarray(th, dtype=np.float64), np.asarray(dis, dtype=np.float64), R_in


def run(am, task, form, dA, dB, th, dis, dR):
    am.amulet_mmlike_f64(task, dA, dB, dev(th) if task else None, dev(dis) if task == 1 else None, dR,
                         thres_form=form)
    torch.cuda.synchronize()
    return dR.cpu().numpy()


def check(R, R_ref, ab, R_in, task, what):
    if task == 3:
        assert np.array_equal(R, R_ref), what
        return
    w = worst_ratio(R, R_ref, ab, R_in, ulp=2.0 ** -52)
    assert w <= TOL_F64, "%s: worst |diff|/sum|term| = %.3e" % (what, w)


# several tiles (16 x 128) in both directions, ragged M, N and K (K % 16 and K % 2 != 0)
SIZES = [(70, 300, 37), (33, 513, 100), (129, 1030, 77), (3, 5, 2), (16, 128, 16), (17, 129, 1),
         (64, 256, 4096)]


@pytest.mark.parametrize("task", TASKS)
@pytest.mark.parametrize("form", FORMS)
def test_f64_forms_and_ragged_sizes(am, task, form):
    if task == 0 and form != 0:
        pytest.skip("the identity task has no threshold operand")
    for idx, (M, N, K) in enumerate(SIZES):
        A, B, th, dis, R_in = make_case(form, M, N, K, 7000 + 64 * task + 8 * form + idx)
        print("case f64", task, form, M, N, K, flush=True)
        R_ref, ab, _ = oracle.mmlike_f64_general(task, A, B, th, dis, R_in, thres_form=form)
        R = run(am, task, form, dev(A), dev(B), th, dis, dev(R_in))
        check(R, R_ref, ab, R_in, task, "task %d form %d %dx%dx%d" % (task, form, M, N, K))


@pytest.mark.parametrize("task", TASKS)
def test_f64_exact_dyadic_data_with_ties(am, task):
    """Small integers and thresholds on multiples of 1/2: products hit thresholds exactly
    (strict >), and every sum is exact in fp64, so the result is bit-exact in any order."""
    for form in ([0] if task == 0 else FORMS):
        M, N, K = 50, 260, 45
        A, B, th, dis, R_in = make_case(form, M, N, K, 7700 + 8 * task + form, exact=True)
        if task:
            if form == 2:
                th = np.array([6.0])   # a value integer products do hit
            thb = (th[None, None, :] if form == 0 else th[:, None, None] if form == 1 else
                   th.reshape(1, 1, 1) if form == 2 else th[:, None, :])
            ties = np.sum((A[:, :, None] * B[None, :, :]) == thb)
            assert ties > 0
        R_ref, _, _ = oracle.mmlike_f64_general(task, A, B, th, dis, R_in, thres_form=form)
        R = run(am, task, form, dev(A), dev(B), th, dis, dev(R_in))
        assert np.array_equal(R, R_ref), (task, form)


@pytest.mark.parametrize("task", TASKS)
def test_f64_strided_and_unaligned_operands(am, task):
    """Row pitches larger than the row, odd pitches and views that start 8 bytes off a
    16-byte boundary (the scalar path instead of the 16-byte one)."""
    M, N, K = 37, 301, 53
    A, B, th, dis, R_in = make_case(0, M, N, K, 7800 + task)
    R_ref, ab, _ = oracle.mmlike_f64_general(task, A, B, th, dis, R_in)
    for pad_a, pad_b, pad_r, off in [(3, 5, 7, 0), (0, 1, 1, 1), (2, 2, 2, 1), (0, 0, 0, 0)]:
        bufA = torch.zeros(M, K + pad_a + off, dtype=torch.float64, device="cuda")
        bufB = torch.zeros(K, N + pad_b + off, dtype=torch.float64, device="cuda")
        bufR = torch.full((M, N + pad_r + off), -77.0, dtype=torch.float64, device="cuda")
        dA, dB, dR = bufA[:, off:off + K], bufB[:, off:off + N], bufR[:, off:off + N]
        dA.copy_(dev(A)); dB.copy_(dev(B)); dR.copy_(dev(R_in))
        print("case f64 strided", task, pad_a, pad_b, pad_r, off, flush=True)
        am.amulet_mmlike_f64(task, dA, dB, dev(th) if task else None, dev(dis) if task == 1 else None, dR)
        torch.cuda.synchronize()
        check(dR.cpu().numpy(), R_ref, ab, R_in, task, "strided %r" % ((pad_a, pad_b, pad_r, off),))
        full = bufR.cpu().numpy()
        assert np.all(full[:, :off] == -77.0) and np.all(full[:, off + N:] == -77.0), "wrote outside R"


def test_f64_accumulates_into_R_and_special_thresholds(am):
    M, N, K = 40, 200, 64
    A, B, th, dis, R_in = make_case(0, M, N, K, 7900)
    dA, dB = dev(A), dev(B)
    # thres = +inf: nothing is over it, DISCOUNT and BOOST reduce to the plain product, COUNT_GT to 0
    inf = np.full(N, np.inf)
    ident, ab, _ = oracle.mmlike_f64_general(0, A, B, None, None, R_in)
    for task in (1, 2):
        R = run(am, task, 0, dA, dB, inf, dis, dev(R_in))
        assert worst_ratio(R, ident, ab, R_in, ulp=2.0 ** -52) <= TOL_F64
    R = run(am, 3, 0, dA, dB, inf, dis, dev(R_in))
    assert np.array_equal(R, R_in)
    # thres = -inf: every product is over it
    R = run(am, 3, 0, dA, dB, -inf, dis, dev(R_in))
    assert np.array_equal(R, R_in + K)
    # two calls accumulate
    dR = dev(R_in)
    am.amulet_mmlike_f64(1, dA, dB, dev(th), dev(dis), dR)
    am.amulet_mmlike_f64(1, dA, dB, dev(th), dev(dis), dR)
    torch.cuda.synchronize()
    once, ab1, _ = oracle.mmlike_f64_general(1, A, B, th, dis, R_in)
    twice, ab2, _ = oracle.mmlike_f64_general(1, A, B, th, dis, once)
    assert worst_ratio(dR.cpu().numpy(), twice, ab1 + ab2, R_in, ulp=2.0 ** -51) <= TOL_F64


def test_f64_argument_errors_and_empty(am):
    z = torch.zeros(4, 4, dtype=torch.float64, device="cuda")
    v = torch.zeros(4, dtype=torch.float64, device="cuda")
    with pytest.raises(am.AmuletError):
        am.amulet_mmlike_f64(7, z, z, v, v, z)
    lib = am.load_library()
    assert lib.amulet_mmlike_f64(1, 9, 4, 4, 4, z.data_ptr(), 4, z.data_ptr(), 4, v.data_ptr(), 0, v.data_ptr(),
                                 z.data_ptr(), 4, None) == -1   # unknown threshold form
    assert lib.amulet_mmlike_f64(1, 0, 4, 4, 4, z.data_ptr(), 4, z.data_ptr(), 4, None, 0, v.data_ptr(),
                                 z.data_ptr(), 4, None) == -3   # thres missing
    assert lib.amulet_mmlike_f64(1, 0, 4, 4, 4, z.data_ptr(), 3, z.data_ptr(), 4, v.data_ptr(), 0,
                                 v.data_ptr(), z.data_ptr(), 4, None) == -4   # lda < K
    # empty problems are accepted and leave R untouched
    R = torch.full((4, 4), 3.0, dtype=torch.float64, device="cuda")
    e = torch.zeros(4, 0, dtype=torch.float64, device="cuda")
    am.amulet_mmlike_f64(1, e, torch.zeros(0, 4, dtype=torch.float64, device="cuda"), v, v, R)
    torch.cuda.synchronize()
    assert torch.all(R == 3.0)


@pytest.mark.parametrize("name", ["f64_discount_4096", "f64_boost_2048", "f64_identity_4096"])
def test_f64_named_workloads_full_size_sampled(am, name):
    """The bench's fp64 workloads at full size, in the launch configuration the bench times;
    the oracle recomputes a seeded sample of whole rows and whole columns."""
    import amulet_workloads as wl
    spec, A, B, P = wl.make(name)
    task, M, N, K = spec["task"], spec["M"], spec["N"], spec["K"]
    th = None if P is None else P[0]
    dis = None if (P is None or P.shape[0] < 2) else P[1]
    print(name, "gpu run", flush=True)
    dR = torch.zeros(M, N, dtype=torch.float64, device="cuda")
    am.amulet_mmlike_f64(task, dev(A), dev(B), None if th is None else dev(th), None if dis is None else dev(dis), dR)
    torch.cuda.synchronize()
    R = dR.cpu().numpy()
    g = np.random.Generator(np.random.PCG64(4244))
    rows = np.sort(g.choice(M, 12, replace=False)); rows[0], rows[-1] = 0, M - 1
    cols = np.sort(g.choice(N, 12, replace=False)); cols[0], cols[-1] = 0, N - 1
    print(name, "oracle rows", flush=True)
    R_ref, ab, _ = oracle.mmlike_f64_general(task, np.ascontiguousarray(A[rows]), B, th, dis)
    assert worst_ratio(R[rows], R_ref, ab) <= TOL_F64
    print(name, "oracle cols", flush=True)
    R_ref, ab, _ = oracle.mmlike_f64_general(task, A, np.ascontiguousarray(B[:, cols]),
                                             None if th is None else th[cols], None if dis is None else dis[cols])
    assert worst_ratio(R[:, cols], R_ref, ab) <= TOL_F64
    if task == 0:
        # whole-matrix property: column sums of R equal (column sums of A) @ B
        ref = A.sum(0) @ B
        scale = np.abs(A).sum(0) @ np.abs(B)
        assert np.max(np.abs(R.sum(0) - ref) / scale) < 1e-12


def test_vector_alu_probes_report_plausible_rates(am):
    """The register-only loops behind the bench's measured ceilings: every instruction mix gives
    a rate between 5 and 80 T products/s (the chip issues 78.6 T lane-operations/s), the pure
    FMA mix the highest; an unknown mix or wave count is refused."""
    rates = [am.amulet_probe_valu(mix, 4) for mix in (0, 1, 2, 3)]
    assert all(5e12 < r < 80e12 for r in rates), rates
    assert rates[0] == max(rates)
    for bad in ((4, 4), (-1, 4), (1, 0), (1, 9)):
        with pytest.raises(am.AmuletError):
            am.amulet_probe_valu(*bad)


def test_matrix_core_probe_reports_a_plausible_rate(am):
    macs = am.amulet_probe_mfma_i8(4)
    # between a tenth of and the whole nominal int8 peak (2.5e15 multiply-adds per second)
    assert 2.5e14 < macs < 2.6e15
    with pytest.raises(am.AmuletError):
        am.amulet_probe_mfma_i8(0)


@pytest.mark.parametrize("task", TASKS)
@pytest.mark.parametrize("tA,tB", [(True, False), (False, True), (True, True)])
def test_f64_transposed_operands(am, task, tA, tB):
    """A stored K x M and / or B stored N x K (the transposed variants of the test queries), over
    ragged sizes, all threshold forms, aligned and 8-byte-offset views."""
    for idx, (M, N, K) in enumerate([(70, 300, 37), (33, 513, 100), (129, 130, 77), (3, 5, 2), (64, 256, 64),
                                     (5, 129, 1)]):
        form = (idx + task) % 4 if task else 0
        A, B, th, dis, R_in = make_case(form, M, N, K, 8000 + 50 * task + idx)
        As = np.ascontiguousarray(A.T) if tA else A
        Bs = np.ascontiguousarray(B.T) if tB else B
        print("case f64 trans", task, tA, tB, form, M, N, K, flush=True)
        R_ref, ab, _ = oracle.mmlike_f64_general(task, As, Bs, th, dis, R_in, thres_form=form, trans_a=tA,
                                                 trans_b=tB)
        # the oracle's transposed form against its own row-major form (same arithmetic, other indexing)
        R_rm, _, _ = oracle.mmlike_f64_general(task, A, B, th, dis, R_in, thres_form=form)
        assert np.array_equal(R_ref, R_rm)
        off = idx % 2
        bufA = torch.zeros(As.shape[0], As.shape[1] + off, dtype=torch.float64, device="cuda")
        bufB = torch.zeros(Bs.shape[0], Bs.shape[1] + off, dtype=torch.float64, device="cuda")
        dA, dB = bufA[:, off:], bufB[:, off:]
        dA.copy_(dev(As)); dB.copy_(dev(Bs))
        dR = dev(R_in)
        am.amulet_mmlike_f64(task, dA, dB, dev(th) if task else None, dev(dis) if task == 1 else None, dR,
                             thres_form=form, trans_a=tA, trans_b=tB)
        torch.cuda.synchronize()
        check(dR.cpu().numpy(), R_ref, ab, R_in, task, "trans %r %r task %d %dx%dx%d" % (tA, tB, task, M, N, K))


@pytest.mark.parametrize("task", TASKS)
def test_f64_few_tiles_long_k_split_over_workgroups(am, task):
    """Tiny M x N with a long K: K is split over several workgroups per tile, which add their
    parts to R with fp64 atomics (vector-ALU kernel and matrix-core identity kernel)."""
    for idx, (M, N, K, trans) in enumerate([(64, 64, 5000, False), (20, 300, 1037, False), (130, 260, 777, True),
                                            (5, 5, 4096, False)]):
        form = (idx + task) % 4 if task else 0
        A, B, th, dis, R_in = make_case(form, M, N, K, 8300 + 10 * task + idx)
        As = np.ascontiguousarray(A.T) if trans else A
        Bs = np.ascontiguousarray(B.T) if trans else B
        R_ref, ab, _ = oracle.mmlike_f64_general(task, As, Bs, th, dis, R_in, thres_form=form, trans_a=trans,
                                                 trans_b=trans)
        print("f64 split-K case", task, form, M, N, K, trans, flush=True)
        dR = dev(R_in)
        am.amulet_mmlike_f64(task, dev(As), dev(Bs), dev(th) if task else None, dev(dis) if task == 1 else None, dR,
                             thres_form=form, trans_a=trans, trans_b=trans)
        torch.cuda.synchronize()
        check(dR.cpu().numpy(), R_ref, ab, R_in, task, "f64 split-K task %d %dx%dx%d" % (task, M, N, K))
    A, B, th, dis, R_in = make_case(0, 48, 200, 1500, 8400 + task, exact=True)
    R_ref, _, _ = oracle.mmlike_f64_general(task, A, B, th, dis, R_in)
    dR = dev(R_in)
    am.amulet_mmlike_f64(task, dev(A), dev(B), dev(th) if task else None, dev(dis) if task == 1 else None, dR)
    torch.cuda.synchronize()
    assert np.array_equal(dR.cpu().numpy(), R_ref)


@pytest.mark.parametrize("task", [1, 3])
def test_last_round_of_workgroups_split_over_k(am, task):
    """More tiles than the chip holds workgroups at once (1176 tiles of 16 x 128 against 1024),
    with a last round far from full: those tiles run once per k range and add their parts to R
    atomically.  Ragged in M, N and K; every output is checked."""
    M, N, K = 770, 3050, 1100
    A, B, th, dis, R_in = make_case(0, M, N, K, seed=880 + task, exact=(task == 3))
    print("f64 tail-split case", task, M, N, K, flush=True)
    R_ref, ab, _ = oracle.mmlike_f64_general(task, A, B, th, dis if task == 1 else None, R_in)
    R = run(am, task, 0, dev(A), dev(B), th, dis, dev(R_in))
    check(R, R_ref, ab, R_in, task, "f64 tail split task %d" % task)


def test_identity_last_round_of_tiles_split_over_k(am):
    """fp64 matrix-core identity kernel with a few more tiles than compute units (275 of
    128 x 128 against 256): the last round's tiles run once per k range (fp64 atomics)."""
    M, N, K = 1300, 3200, 1100
    A, B, th, dis, R_in = make_case(0, M, N, K, seed=890)
    print("f64 identity tail-split case", M, N, K, flush=True)
    R_ref, ab, _ = oracle.mmlike_f64_general(0, A, B, None, None, R_in)
    R = run(am, 0, 0, dev(A), dev(B), th, dis, dev(R_in))
    check(R, R_ref, ab, R_in, 0, "f64 identity tail split")


@pytest.mark.parametrize("task", [1, 2, 3])
def test_rows_of_A_with_a_colliding_pitch_go_through_lds(am, task):
    """A row-major fp64 A whose row pitch is a multiple of 32 KiB (a view of a wider array, pitch
    64 KiB) takes the kernel variant that stages A through LDS: every threshold form, ragged
    sizes, a K remainder, a split K and a split last round."""
    cases = [(70, 300, 37), (129, 1030, 77), (3, 5, 2), (64, 256, 1100), (770, 3050, 600)]
    for idx, (M, N, K) in enumerate(cases):
        form = idx % 4
        A, B, th, dis, R_in = make_case(form, M, N, K, seed=8300 + 10 * task + idx, exact=(task == 3))
        R_ref, ab, _ = oracle.mmlike_f64_general(task, A, B, th, dis if task == 1 else None, R_in, thres_form=form)
        wide = torch.zeros((M, 8192), dtype=torch.float64, device="cuda")        # pitch 64 KiB
        dA = wide[:, :K]
        dA.copy_(dev(A))
        assert am.amulet_pitch_collides(8192, 8)
        print("f64 A through LDS", task, form, M, N, K, flush=True)
        R = run(am, task, form, dA, dev(B), th, dis, dev(R_in))
        check(R, R_ref, ab, R_in, task, "f64 A through LDS task %d form %d %dx%dx%d" % (task, form, M, N, K))


@pytest.mark.parametrize("task", [1, 2, 3])
@pytest.mark.parametrize("shape", range(6))
def test_f64_every_shape_on_ragged_sizes(am, task, shape):
    """Every point of the fp64 shape grid (tile 16 x 128 or 32 x 128, K whole or in 2 or 4 parts per
    tile): ragged sizes, every threshold form, row-major and transposed operands, one case long
    enough in K for the forced split to apply, and exact data bit for bit."""
    assert am.amulet_f64_shape_count() == 6 and am.amulet_f64_shape_name(shape) != "invalid"
    cases = [(70, 300, 37, False, False), (33, 513, 100, True, False), (129, 130, 77, False, True),
             (3, 5, 2, True, True), (40, 260, 700, False, False), (65, 129, 333, True, True)]
    for idx, (M, N, K, tA, tB) in enumerate(cases):
        form = (idx + task + shape) % 4
        A, B, th, dis, R_in = make_case(form, M, N, K, 9000 + 100 * task + 10 * shape + idx)
        As = np.ascontiguousarray(A.T) if tA else A
        Bs = np.ascontiguousarray(B.T) if tB else B
        print("case f64 shape", task, shape, form, M, N, K, tA, tB, flush=True)
        R_ref, ab, _ = oracle.mmlike_f64_general(task, As, Bs, th, dis, R_in, thres_form=form, trans_a=tA, trans_b=tB)
        dR = dev(R_in)
        am.amulet_mmlike_f64(task, dev(As), dev(Bs), dev(th), dev(dis) if task == 1 else None, dR,
                             thres_form=form, trans_a=tA, trans_b=tB, shape=shape)
        torch.cuda.synchronize()
        check(dR.cpu().numpy(), R_ref, ab, R_in, task, "f64 shape %d task %d %dx%dx%d" % (shape, task, M, N, K))
    A, B, th, dis, R_in = make_case(0, 48, 200, 1500, 9900 + task, exact=True)
    R_ref, _, _ = oracle.mmlike_f64_general(task, A, B, th, dis, R_in)
    dR = dev(R_in)
    am.amulet_mmlike_f64(task, dev(A), dev(B), dev(th), dev(dis) if task == 1 else None, dR, shape=shape)
    torch.cuda.synchronize()
    assert np.array_equal(dR.cpu().numpy(), R_ref)
    with pytest.raises(am.AmuletError):
        am.amulet_mmlike_f64(task, dev(A), dev(B), dev(th), dev(dis) if task == 1 else None, dR, shape=6)


def test_f64_adaptive_execution_trials_contribute_to_the_result(am, monkeypatch):
    """In-flight adaptive execution in fp64: the trial slabs are rows of the caller's R computed
    with different shapes, the rest runs with the winner, and the whole R must match the oracle
    (general form: thres[i], transposed A).  The winner is cached for the size bucket and used by
    a later plain call; the identity task and small tasks run whole, without trials."""
    monkeypatch.setenv("AMULET_ADAPTIVE_MIN_TASK_MS", "0")   # (a task of about a millisecond: lift the one-trial limit)
    M, N, K = 8192, 4096, 160
    form, tA = 1, True
    A, B, th, dis, R_in = make_case(form, M, N, K, 9950)
    As = np.ascontiguousarray(A.T)
    R_ref, ab, _ = oracle.mmlike_f64_general(1, As, B, th, dis, R_in, thres_form=form, trans_a=tA)
    am.amulet_clear_selections()
    dA, dB, dth, ddis = dev(As), dev(B), dev(th), dev(dis)
    dR = dev(R_in)
    chosen, trials = am.amulet_mmlike_f64_adaptive(1, dA, dB, dth, ddis, dR, thres_form=form, trans_a=tA)
    torch.cuda.synchronize()
    print("f64 adaptive chose", chosen, am.amulet_f64_shape_name(chosen), "after", trials, "trials", flush=True)
    assert 0 <= chosen < am.amulet_f64_shape_count() and trials >= 4   # the default, the k axis, one more tile
    check(dR.cpu().numpy(), R_ref, ab, R_in, 1, "f64 adaptive")
    assert am.amulet_selected_shape_f64(1, M, N, K) == chosen
    assert am.amulet_selected_shape_f64(1, M - 3, N - 1, K) == chosen      # same size bucket
    dR2 = dev(R_in)
    am.amulet_mmlike_f64(1, dA, dB, dth, ddis, dR2, thres_form=form, trans_a=tA)
    torch.cuda.synchronize()
    check(dR2.cpu().numpy(), R_ref, ab, R_in, 1, "f64 plain after adaptive")
    # too small for three slabs: no trials, still the whole result
    A, B, th, dis, R_in = make_case(0, 300, 260, 50, 9951)
    R_ref, ab, _ = oracle.mmlike_f64_general(2, A, B, th, None, R_in)
    dR = dev(R_in)
    chosen, trials = am.amulet_mmlike_f64_adaptive(2, dev(A), dev(B), dev(th), None, dR)
    torch.cuda.synchronize()
    assert trials == 0
    check(dR.cpu().numpy(), R_ref, ab, R_in, 2, "f64 adaptive small")
    # identity: one matrix-core kernel, no trials
    R_ref, ab, _ = oracle.mmlike_f64_general(0, A, B, None, None, R_in)
    dR = dev(R_in)
    chosen, trials = am.amulet_mmlike_f64_adaptive(0, dev(A), dev(B), None, None, dR)
    torch.cuda.synchronize()
    assert trials == 0
    check(dR.cpu().numpy(), R_ref, ab, R_in, 0, "f64 adaptive identity")
    am.amulet_clear_selections()


@pytest.mark.parametrize("tA,tB", [(False, False), (True, False), (False, True), (True, True)])
def test_f64_identity_streamed_kernel_on_every_size(am, tA, tB):
    """The fp64 matrix-core identity kernel that streams its operands HBM -> LDS (128 x 128 and
    64 x 64 tiles) runs on operands
    of any size and alignment with at least one 8-k stage, in any of the four operand layouts.  Cases: fewer stages than the ring holds, one tile, several tiles with padded pitches
    and a non-zero R_in, few tiles with a long K (every tile split over workgroups), a few more
    tiles than compute units (the last round's tiles split), and exact data bit for bit.  Every
    output is checked."""
    cases = [(128, 128, 8, 0), (128, 128, 24, 0), (256, 384, 200, 2), (128, 256, 4096, 0), (1408, 3200, 1104, 6),
             # M and N that are not whole tiles: fewer rows than a tile, one more row or unit than
             # whole tiles, odd sizes (streamed only where the operand's lines run along k), a split
             # K with edge tiles, a split last round with edge tiles
             (100, 130, 64, 0), (257, 258, 200, 2), (129, 131, 32, 0), (60, 4098, 4096, 0), (1300, 3202, 1104, 6),
             # K that is no whole number of 8-k stages: one stage and a bit, padded pitches, a split K,
             # a split last round, together with edge tiles
             (128, 128, 12, 0), (256, 384, 202, 2), (128, 256, 4102, 0), (1408, 3200, 1106, 6), (100, 130, 1034, 0),
             # odd sizes and pitches: rows that are not 16-byte aligned, edges that cut a two-line
             # unit, tiles of one line (129 = 128 + 1), the smallest operands the kernel takes
             (129, 131, 17, 0), (257, 259, 203, 1), (127, 129, 1001, 0), (3, 5, 24, 0), (2, 2, 8, 0), (130, 133, 1037, 3),
             (1301, 3203, 1109, 0),
             # around the 64 x 64 tile: one tile and one stage, a line more than whole tiles, fewer
             # stages than its ring holds plus a tail, few tiles with a long K
             (64, 64, 8, 0), (65, 67, 17, 0), (190, 70, 50, 2), (192, 320, 2100, 0)]
    for idx, (M, N, K, pad) in enumerate(cases):
        A, B, th, dis, R_in = make_case(0, M, N, K, 9960 + idx)
        As = np.ascontiguousarray(A.T) if tA else A
        Bs = np.ascontiguousarray(B.T) if tB else B
        R_ref, ab, _ = oracle.mmlike_f64_general(0, As, Bs, None, None, R_in, trans_a=tA, trans_b=tB)
        bufA = torch.full((As.shape[0], As.shape[1] + pad), float("nan"), dtype=torch.float64, device="cuda")
        bufA[:, :As.shape[1]] = dev(As)
        bufB = torch.full((Bs.shape[0], Bs.shape[1] + pad), float("nan"), dtype=torch.float64, device="cuda")
        bufB[:, :Bs.shape[1]] = dev(Bs)
        for shape in (1, 0, -1):   # (the identity task reads the shape's tile index: 128 x 128, 64 x 64, the rule)
            print("f64 identity streamed", tA, tB, M, N, K, pad, shape, flush=True)
            dR = dev(R_in)
            am.amulet_mmlike_f64(0, bufA[:, :As.shape[1]], bufB[:, :Bs.shape[1]], None, None, dR, trans_a=tA, trans_b=tB,
                                 shape=shape)
            torch.cuda.synchronize()
            check(dR.cpu().numpy(), R_ref, ab, R_in, 0, "f64 identity streamed %dx%dx%d shape %d" % (M, N, K, shape))
    A, B, th, dis, R_in = make_case(0, 256, 256, 1600, 9970, exact=True)
    As = np.ascontiguousarray(A.T) if tA else A
    Bs = np.ascontiguousarray(B.T) if tB else B
    R_ref, _, _ = oracle.mmlike_f64_general(0, As, Bs, None, None, R_in, trans_a=tA, trans_b=tB)
    for shape in (1, 0):
        dR = dev(R_in)
        am.amulet_mmlike_f64(0, dev(As), dev(Bs), None, None, dR, trans_a=tA, trans_b=tB, shape=shape)
        torch.cuda.synchronize()
        assert np.array_equal(dR.cpu().numpy(), R_ref), shape


@pytest.mark.parametrize("task,M,N,K", [(1, 64, 128, 20000), (3, 770, 3050, 1100), (0, 1536, 1536, 2048), (0, 300, 300, 4096)])
def test_f64_deterministic_mode_gives_the_same_bits_twice(am, task, M, N, K):
    """fp64 sizes whose default launch splits K (few tiles, a nearly empty last round, the streamed
    and the register-staged identity kernel): with the deterministic mode on, two runs agree bit
    for bit and match the oracle; so does the default mode, to the tolerance."""
    A, B, th, dis, R_in = make_case(0, M, N, K, 9980 + task)
    R_ref, ab, _ = oracle.mmlike_f64_general(task, A, B, th if task else None, dis if task == 1 else None, R_in)
    was = am.amulet_get_deterministic()
    try:
        am.amulet_set_deterministic(True)
        R1 = run(am, task, 0, dev(A), dev(B), th, dis, dev(R_in))
        R2 = run(am, task, 0, dev(A), dev(B), th, dis, dev(R_in))
    finally:
        am.amulet_set_deterministic(was)
    assert np.array_equal(R1, R2)
    check(R1, R_ref, ab, R_in, task, "f64 deterministic mode, task %d" % task)
    R3 = run(am, task, 0, dev(A), dev(B), th, dis, dev(R_in))
    check(R3, R_ref, ab, R_in, task, "f64 default mode, task %d" % task)
