"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle
element by element on the same seeded inputs."""
import numpy as np
import pytest

import amulet_workloads as wl
import oracle
from parity import TOL_F32, assert_parity_f32

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

NPAR = {0: 0, 1: 2, 2: 1, 3: 1}
TASKS = [0, 1, 2, 3]


@pytest.fixture(scope="module")
def am():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2305_08872_amd as am
    am.load_library()  # raises if the HIP library is missing: there is no fallback
    return am


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def rand_case(task, M, N, K, seed):
    g = np.random.Generator(np.random.PCG64(seed))
    A = (g.standard_normal((M, K)) * 2).astype(np.float32)
    B = (g.standard_normal((K, N)) * 2).astype(np.float32)
    rows = []
    if NPAR[task] >= 1:
        rows.append(g.standard_normal(N).astype(np.float32) * 3)
    if NPAR[task] == 2:
        rows.append(g.uniform(0, 1, N).astype(np.float32))
    params = np.stack(rows) if rows else None
    R_in = g.standard_normal((M, N)).astype(np.float32) * 5
    return A, B, params, R_in


def run_gpu(am, task, A, B, params, R_in, shape=None):
    dA, dB, dR = dev(A), dev(B), dev(R_in)
    dP = dev(params) if params is not None else None
    if shape is None:
        am.amulet_mmlike_f32(task, dA, dB, dP, dR)
    else:
        am.amulet_mmlike_f32_shape(task, shape, dA, dB, dP, dR)
    torch.cuda.synchronize()
    return dR.cpu().numpy()


# several tiles in each direction plus ragged tails in M, N and K for every shape
ODD_SHAPES = [(70, 300, 37), (33, 513, 100), (1, 1, 1), (129, 1030, 77), (5, 257, 16), (64, 512, 8), (40, 520, 700)]


@pytest.mark.parametrize("task", TASKS)
@pytest.mark.parametrize("shape", range(20))
def test_every_shape_on_ragged_sizes(am, task, shape):
    if shape >= am.amulet_shape_count(task):
        pytest.skip("task %d has no shape %d" % (task, shape))
    for idx, (M, N, K) in enumerate(ODD_SHAPES):
        A, B, params, R_in = rand_case(task, M, N, K, seed=1000 + 17 * task + idx)
        print("case", task, shape, M, N, K, flush=True)
        R_ref, ab, _ = oracle.mmlike_f32(task, A, B, params, R_in)
        R = run_gpu(am, task, A, B, params, R_in, shape)
        if task == 3 and K < 128:   # (a count added to a fractional R_in in several parts is rounded once per part)
            assert np.array_equal(R, R_ref), (task, shape, M, N, K)
        else:
            assert_parity_f32(R, R_ref, ab, R_in, what="task %d shape %d %dx%dx%d" % (task, shape, M, N, K))


@pytest.mark.parametrize("task", TASKS)
def test_strided_and_unaligned_operands(am, task):
    M, N, K = 45, 301, 53
    A, B, params, R_in = rand_case(task, M, N, K, seed=77 + task)
    R_ref, ab, _ = oracle.mmlike_f32(task, A, B, params, R_in)
    # lda = K + 3, ldb = N + 2 (odd pitch: no 16-byte rows), ldr = N + 5, all sliced from bigger buffers
    bigA = torch.zeros(M, K + 3, device="cuda"); bigA[:, :K] = dev(A)
    bigB = torch.full((K, N + 2), 7.0, device="cuda"); bigB[:, :N] = dev(B)
    bigR = torch.full((M, N + 5), -3.0, device="cuda"); bigR[:, :N] = dev(R_in)
    dP = dev(params) if params is not None else None
    am.amulet_mmlike_f32(task, bigA[:, :K], bigB[:, :N], dP, bigR[:, :N])
    torch.cuda.synchronize()
    out = bigR.cpu().numpy()
    assert np.all(out[:, N:] == -3.0)  # nothing written beyond column N
    if task == 3:
        assert np.array_equal(out[:, :N], R_ref)
    else:
        assert_parity_f32(out[:, :N], R_ref, ab, R_in, what="strided task %d" % task)
    # offset base pointer: 4-byte but not 16-byte aligned B and R
    flatB = torch.zeros(K * N + 1, device="cuda"); flatB[1:] = dev(B).reshape(-1)
    flatR = torch.zeros(M * N + 3, device="cuda"); flatR[3:] = dev(R_in).reshape(-1)
    am.amulet_mmlike_f32(task, dev(A), flatB[1:].view(K, N), dP, flatR[3:].view(M, N))
    torch.cuda.synchronize()
    out2 = flatR[3:].view(M, N).cpu().numpy()
    if task == 3:
        assert np.array_equal(out2, R_ref)
    else:
        assert_parity_f32(out2, R_ref, ab, R_in, what="unaligned task %d" % task)


def test_exact_data_is_bit_exact_for_all_tasks(am):
    # every product, term and partial sum is a small dyadic rational: any order of
    # fp32 summation is exact, so the GPU must equal the oracle bit for bit (ties included)
    for task in TASKS:
        A, B, params = wl.small_exact(97, 700, 83, seed=5 + task, n_param=NPAR[task])
        R_in = np.zeros((97, 700), np.float32)
        R_ref, _, _ = oracle.mmlike_f32(task, A, B, params, R_in)
        for shape in (0, 3, 7, 8):
            if shape >= am.amulet_shape_count(task):
                continue
            R = run_gpu(am, task, A, B, params, R_in, shape)
            assert np.array_equal(R, R_ref), (task, shape)


def test_infinite_thresholds_and_zero_result_invariants(am):
    M, N, K = 40, 520, 130
    A, B, _, R_in = rand_case(1, M, N, K, seed=9)
    g = np.random.Generator(np.random.PCG64(10))
    dis = g.uniform(0, 1, N).astype(np.float32)
    inf = np.full(N, np.inf, np.float32)
    # thres = +inf: discount and boost are plain matmul (the oracle's identity result), count is zero
    R_ref, ab, _ = oracle.mmlike_f32(0, A, B, None, R_in)
    assert_parity_f32(run_gpu(am, 0, A, B, None, R_in), R_ref, ab, R_in, what="identity")
    assert_parity_f32(run_gpu(am, 1, A, B, np.stack([inf, dis]), R_in), R_ref, ab, R_in,
                      what="discount thres=+inf")
    assert_parity_f32(run_gpu(am, 2, A, B, inf[None], R_in), R_ref, ab, R_in, what="boost thres=+inf")
    assert np.array_equal(run_gpu(am, 3, A, B, inf[None], R_in), R_in)
    # thres = -inf: count is K; discount with dis = 1 leaves R exactly unchanged
    assert np.array_equal(run_gpu(am, 3, A, B, -inf[None], np.zeros_like(R_in)), np.full((M, N), K, np.float32))
    P = np.stack([-inf, np.ones(N, np.float32)])
    assert np.array_equal(run_gpu(am, 1, A, B, P, R_in), R_in)
    # boost with thres = -inf is +inf everywhere, as in the oracle
    R_ref, ab, _ = oracle.mmlike_f32(2, A, B, -inf[None], R_in)
    assert np.array_equal(run_gpu(am, 2, A, B, -inf[None], R_in), R_ref)


def test_negative_thresholds_and_k_tail_without_padding(am):
    # g(0) = -thres for boost with thres < 0 and 1 for count: a zero-padded K tail would show
    for K in (1, 7, 17, 31):
        A = np.zeros((20, K), np.float32)
        B = np.ones((K, 300), np.float32)
        th = np.full((1, 300), -2.0, np.float32)
        R0 = np.zeros((20, 300), np.float32)
        assert np.array_equal(run_gpu(am, 2, A, B, th, R0), np.full((20, 300), 2.0 * K, np.float32))
        assert np.array_equal(run_gpu(am, 3, A, B, th, R0), np.full((20, 300), float(K), np.float32))


def test_predicate_on_rounded_product(am):
    a = np.float32(1 + 2.0 ** -12)
    p32 = np.float32(a * a)
    A = np.full((3, 5), a, np.float32)
    B = np.full((5, 260), a, np.float32)
    th = np.full((1, 260), p32, np.float32)   # exact product exceeds thres, rounded product equals it
    R0 = np.zeros((3, 260), np.float32)
    assert not run_gpu(am, 3, A, B, th, R0).any()
    R = run_gpu(am, 1, A, B, np.concatenate([th, np.full((1, 260), 0.5, np.float32)]), R0)
    R_ref, _, _ = oracle.mmlike_f32(1, A, B, np.concatenate([th, np.full((1, 260), 0.5, np.float32)]), R0)
    assert np.array_equal(R, R_ref)


def test_boost_at_a_straddling_threshold_stays_inside_the_tolerance(am):
    """The boost task is evaluated with fused operations on the unrounded product (its g is
    continuous in p), so at a threshold that the exact product exceeds and the rounded product
    only equals, a term may differ from the oracle's rounded-product term by one rounding of p:
    inside the tolerance, not necessarily the same bits."""
    a = np.float32(1 + 2.0 ** -12)
    p32 = np.float32(a * a)
    A = np.full((3, 5), a, np.float32)
    B = np.full((5, 260), a, np.float32)
    th = np.full((1, 260), p32, np.float32)
    R0 = np.zeros((3, 260), np.float32)
    R = run_gpu(am, 2, A, B, th, R0)
    R_ref, ab, _ = oracle.mmlike_f32(2, A, B, th, R0)
    assert_parity_f32(R, R_ref, ab, what="boost at a straddling threshold")
    # the oracle itself does not trigger here (tie on the rounded product): its result is the plain sum
    assert np.array_equal(R_ref, oracle.mmlike_f32(0, A, B, None, R0)[0])


def test_empty_dimensions_are_noops(am):
    R = torch.full((4, 6), 2.5, device="cuda")
    am.amulet_mmlike_f32(1, torch.zeros(4, 0, device="cuda"), torch.zeros(0, 6, device="cuda"),
                         torch.zeros(2, 6, device="cuda"), R)
    torch.cuda.synchronize()
    assert torch.all(R == 2.5)


@pytest.mark.parametrize("shape", [None, 4, 5])
@pytest.mark.parametrize("task", [1, 3])
def test_last_round_of_workgroups_split_over_k(am, task, shape):
    """More tiles than the chip holds workgroups at once, with a last round at most half full:
    the launcher runs those last tiles as a second launch that splits K (atomic adds into R).
    Ragged in M, N and K; every output is checked (a tile run twice, or not at all, shows)."""
    M, N, K = 770, 6100, 1100      # 25 x 24 tiles of 32 x 256 (600 > 512), 49 x 24 of 16 x 256 (1176 > 1024)
    A, B, params, R_in = rand_case(task, M, N, K, seed=640 + task)
    if task == 3:
        # a split tile's count reaches R in several adds: exact as long as R holds integers
        # (a fractional R_in would be rounded once per add instead of once)
        R_in = np.rint(R_in)
    print("tail-split case", task, shape, M, N, K, flush=True)
    R_ref, ab, _ = oracle.mmlike_f32(task, A, B, params, R_in)
    R = run_gpu(am, task, A, B, params, R_in, shape)
    if task == 3:
        assert np.array_equal(R, R_ref)
    else:
        assert_parity_f32(R, R_ref, ab, R_in, what="tail split, task %d shape %s" % (task, shape))


# ---- join count -----------------------------------------------------------------
@pytest.mark.parametrize("shape", [None, 0, 1, 2, 3, 4, 5, 6, 7, 8])
def test_count_i8_bit_exact_ragged(am, shape):
    for idx, (M, N, K) in enumerate([(70, 300, 37), (129, 1030, 77), (1, 1, 1), (257, 129, 1000), (64, 64, 64),
                                       (300, 272, 128), (512, 256, 192), (256, 512, 64), (384, 768, 448),
                                       (768, 512, 320), (1000, 1300, 256), (513, 257, 64)]):
        g = np.random.Generator(np.random.PCG64(300 + idx))
        A = g.integers(-128, 128, (M, K)).astype(np.int8)
        B = g.integers(-128, 128, (K, N)).astype(np.int8)
        R_in = g.integers(-1000, 1000, (M, N)).astype(np.int32)
        R_ref, _ = oracle.count_i8(A, B, R_in)
        dR = dev(R_in)
        if shape is None:
            am.amulet_count_i8(dev(A), dev(B), dR)
        else:
            am.amulet_count_i8_shape(shape, dev(A), dev(B), dR)
        torch.cuda.synchronize()
        assert np.array_equal(dR.cpu().numpy(), R_ref), (M, N, K)


@pytest.mark.parametrize("shape", [None, 1, 3, 5, 6, 7, 8])
def test_count_i8_few_tiles_long_k_split_over_workgroups(am, shape):
    """Tiny M x N with a long K: K is split over several workgroups per tile, which add their parts
    to R with integer atomics (exact in any order), in the streamed and the register-staged kernels."""
    for idx, (M, N, K) in enumerate([(128, 256, 8192), (256, 256, 4096), (100, 300, 5000), (256, 512, 3000)]):
        g = np.random.Generator(np.random.PCG64(350 + idx))
        A = g.integers(-128, 128, (M, K)).astype(np.int8)
        B = g.integers(-128, 128, (K, N)).astype(np.int8)
        R_in = g.integers(-1000, 1000, (M, N)).astype(np.int32)
        R_ref, _ = oracle.count_i8(A, B, R_in)
        dR = dev(R_in)
        print("i8 split-K case", shape, M, N, K, flush=True)
        if shape is None:
            am.amulet_count_i8(dev(A), dev(B), dR)
        else:
            am.amulet_count_i8_shape(shape, dev(A), dev(B), dR)
        torch.cuda.synchronize()
        assert np.array_equal(dR.cpu().numpy(), R_ref), (M, N, K)


@pytest.mark.parametrize("phases", ["1,0,1,0", "2,2,2,8", "8,2,2,16", "4,1,8,16", "16,3,4,12"])
@pytest.mark.parametrize("shape", [8, 108, 208, None])
def test_count_i8_persistent_workgroups(am, shape, phases, monkeypatch):
    """Sizes large enough for the persistent streamed kernels (every workgroup walks at least two
    tiles of its XCD's part), with ragged edges around the whole-tile interior and a K of five
    stages, so that a workgroup's first tile is summed in two passes (2 + 3 stages, or 1 + 4 ...
    by phase).  Phase arrangements "slot groups, stages between them, XCD modulus, XCD span in
    sixteenths of K" (none, coarse, the default, fine, odd), full int8 value range, non-zero R_in,
    bit-exact; the row and column checksums cover the whole matrix, sampled rows and columns go
    against the oracle.  Shape 108: shape 8 on a tile count that is no whole number of rounds
    (22 x 32 tiles: an XCD's workgroups walk 2 or 3 tiles); 208: shape 8 on 23 x 23 tiles, which no
    cut into 8 rectangular parts covers (the XCDs walk equal runs of one panel order, 66 or 67 tiles
    each, the last place of some holding no tile)."""
    monkeypatch.setenv("AMULET_I8_PHASES", phases)
    M, N, K = {8: (8192 + 77, 4096 + 33, 320), 108: (5632 + 5, 8192 + 1, 320), 208: (5888 + 3, 5888 + 9, 320),
               None: (8192, 8192, 320)}[shape]
    if shape in (108, 208):
        shape = 8
    g = np.random.Generator(np.random.PCG64(377 + (shape or 0)))
    A = g.integers(-128, 128, (M, K)).astype(np.int8)
    B = g.integers(-128, 128, (K, N)).astype(np.int8)
    dR = torch.full((M, N), 7, dtype=torch.int32, device="cuda")
    print("i8 persistent case", shape, phases, M, N, K, flush=True)
    if shape is None:
        assert am.amulet_selected_shape(am.AMULET_TASK_COUNT_I8, M, N, K) == 8   # the default at this size
        am.amulet_count_i8(dev(A), dev(B), dR)
    else:
        am.amulet_count_i8_shape(shape, dev(A), dev(B), dR)
    torch.cuda.synchronize()
    R = dR.cpu().numpy()
    rows = np.sort(g.choice(M, 40, replace=False)); rows[0], rows[-1] = 0, M - 1
    cols = np.sort(g.choice(N, 40, replace=False)); cols[0], cols[-1] = 0, N - 1
    R_ref, _ = oracle.count_i8(np.ascontiguousarray(A[rows]), B, np.full((len(rows), N), 7, np.int32))
    assert np.array_equal(R[rows], R_ref)
    R_ref, _ = oracle.count_i8(A, np.ascontiguousarray(B[:, cols]), np.full((M, len(cols)), 7, np.int32))
    assert np.array_equal(R[:, cols], R_ref)
    A64, B64 = A.astype(np.int64), B.astype(np.int64)
    assert np.array_equal(R.astype(np.int64).sum(1), A64 @ B64.sum(1) + 7 * N)
    assert np.array_equal(R.astype(np.int64).sum(0), A64.sum(0) @ B64 + 7 * M)


@pytest.mark.parametrize("case", [
    # (shape, M, N, K): the persistent streamed kernel (a workgroup's first tile in two passes: the
    # first stores, the second adds), the one-tile streamed kernels, a streamed interior with
    # register-staged edge strips, the register-staged kernels with ragged sizes and unaligned K,
    # few tiles with a long K (K split: R cleared, then atomic adds), the plain loop, the default
    (8, 8192, 8192, 320), (7, 1024, 2048, 192), (6, 640, 1280, 128), (8, 8192 + 77, 4096 + 33, 320),
    (1, 777, 999, 130), (4, 300, 500, 77), (5, 513, 257, 64), (3, 256, 256, 4096), (6, 256, 512, 8192),
    (0, 70, 90, 33), (-1, 2048, 2048, 256), (-1, 100, 100, 3)])
def test_count_i8_assign_writes_the_counts_whatever_R_held(am, case):
    """amulet_count_i8_assign: R = A . B exactly, with R full of other values beforehand (and the
    padding of R's rows untouched); against the oracle with a zero R_in, whole matrix for the small
    cases, sampled rows and columns plus whole-matrix checksums for the large ones.  K = 0 gives
    zeros; a second call gives the same R again (nothing accumulates)."""
    shape, M, N, K = case
    g = np.random.Generator(np.random.PCG64(431 + M + K))
    A = g.integers(-128, 128, (M, K)).astype(np.int8)
    B = g.integers(-128, 128, (K, N)).astype(np.int8)
    pad = 4
    buf = torch.full((M, N + pad), -123456, dtype=torch.int32, device="cuda")
    dR = buf[:, :N]
    print("i8 assign case", case, flush=True)
    dA, dB = dev(A), dev(B)
    for _ in range(2):
        am.amulet_count_i8_assign(dA, dB, dR, shape=shape)
    torch.cuda.synchronize()
    full = buf.cpu().numpy()
    assert np.all(full[:, N:] == -123456), "wrote outside R"
    R = full[:, :N]
    if M * N * K <= 300 * 500 * 4096:
        R_ref, _ = oracle.count_i8(A, B, np.zeros((M, N), np.int32))
        assert np.array_equal(R, R_ref)
    else:
        rows = np.sort(g.choice(M, 24, replace=False)); rows[0], rows[-1] = 0, M - 1
        cols = np.sort(g.choice(N, 24, replace=False)); cols[0], cols[-1] = 0, N - 1
        R_ref, _ = oracle.count_i8(np.ascontiguousarray(A[rows]), B, np.zeros((len(rows), N), np.int32))
        assert np.array_equal(R[rows], R_ref)
        R_ref, _ = oracle.count_i8(A, np.ascontiguousarray(B[:, cols]), np.zeros((M, len(cols)), np.int32))
        assert np.array_equal(R[:, cols], R_ref)
        A64, B64 = A.astype(np.int64), B.astype(np.int64)
        assert np.array_equal(R.astype(np.int64).sum(1), A64 @ B64.sum(1))
        assert np.array_equal(R.astype(np.int64).sum(0), A64.sum(0) @ B64)
    # an empty sum
    am.amulet_count_i8_assign(dA[:, :0], dB[:0, :], dR, shape=shape)
    torch.cuda.synchronize()
    full = buf.cpu().numpy()
    assert np.all(full[:, :N] == 0) and np.all(full[:, N:] == -123456)


@pytest.mark.parametrize("phases", ["8,2,2,16", "4,1,8,16"])
def test_count_i8_assign_with_phased_workgroups(am, phases, monkeypatch):
    """The R = form runs the persistent kernel's workgroups in step by default; with phases forced, a
    workgroup sums its first tile in two passes, of which the first stores and the second adds to
    what the first stored.  Exact, from an R full of other values (sampled rows and columns, whole
    matrix checksums)."""
    monkeypatch.setenv("AMULET_I8_PHASES", phases)
    M, N, K = 8192, 8192, 320
    g = np.random.Generator(np.random.PCG64(433))
    A = g.integers(-128, 128, (M, K)).astype(np.int8)
    B = g.integers(-128, 128, (K, N)).astype(np.int8)
    dR = torch.full((M, N), 99, dtype=torch.int32, device="cuda")
    print("i8 assign phased", phases, flush=True)
    am.amulet_count_i8_assign(dev(A), dev(B), dR, shape=8)
    torch.cuda.synchronize()
    R = dR.cpu().numpy()
    rows = np.sort(g.choice(M, 24, replace=False)); rows[0], rows[-1] = 0, M - 1
    cols = np.sort(g.choice(N, 24, replace=False)); cols[0], cols[-1] = 0, N - 1
    R_ref, _ = oracle.count_i8(np.ascontiguousarray(A[rows]), B, np.zeros((len(rows), N), np.int32))
    assert np.array_equal(R[rows], R_ref)
    R_ref, _ = oracle.count_i8(A, np.ascontiguousarray(B[:, cols]), np.zeros((M, len(cols)), np.int32))
    assert np.array_equal(R[:, cols], R_ref)
    A64, B64 = A.astype(np.int64), B.astype(np.int64)
    assert np.array_equal(R.astype(np.int64).sum(1), A64 @ B64.sum(1))
    assert np.array_equal(R.astype(np.int64).sum(0), A64.sum(0) @ B64)


def test_count_i8_adaptive_execution_trials_contribute_to_the_result(am, monkeypatch):
    """In-flight adaptive execution of the join count: slabs of rows of the caller's R are computed
    by different matrix-core kernels, the rest by the fastest; the whole R must be the exact count
    (sampled rows and columns against the oracle, whole-matrix row and column checksums).  The
    winner is cached; a problem too small for two slabs runs whole, without trials."""
    monkeypatch.setenv("AMULET_ADAPTIVE_MIN_TASK_MS", "0")   # (a sub-millisecond task: lift the no-trials limit)
    M, N, K = 12288, 16384, 128
    g = np.random.Generator(np.random.PCG64(391))
    A = g.integers(-128, 128, (M, K)).astype(np.int8)
    B = g.integers(-128, 128, (K, N)).astype(np.int8)
    dR = torch.full((M, N), 7, dtype=torch.int32, device="cuda")
    am.amulet_clear_selections()
    chosen, trials = am.amulet_count_i8_adaptive(dev(A), dev(B), dR)
    torch.cuda.synchronize()
    print("i8 adaptive chose", chosen, am.amulet_shape_name(am.AMULET_TASK_COUNT_I8, chosen), "after", trials, "trials", flush=True)
    assert 1 <= chosen < am.amulet_shape_count(am.AMULET_TASK_COUNT_I8) and trials >= 3
    assert am.amulet_selected_shape(am.AMULET_TASK_COUNT_I8, M, N, K) == chosen
    R = dR.cpu().numpy()
    rows = np.sort(g.choice(M, 48, replace=False)); rows[0], rows[-1] = 0, M - 1
    cols = np.sort(g.choice(N, 24, replace=False)); cols[0], cols[-1] = 0, N - 1
    R_ref, _ = oracle.count_i8(np.ascontiguousarray(A[rows]), B, np.full((len(rows), N), 7, np.int32))
    assert np.array_equal(R[rows], R_ref)
    R_ref, _ = oracle.count_i8(A, np.ascontiguousarray(B[:, cols]), np.full((M, len(cols)), 7, np.int32))
    assert np.array_equal(R[:, cols], R_ref)
    A64, B64 = A.astype(np.int64), B.astype(np.int64)
    assert np.array_equal(R.astype(np.int64).sum(1), A64 @ B64.sum(1) + 7 * N)
    assert np.array_equal(R.astype(np.int64).sum(0), A64.sum(0) @ B64 + 7 * M)
    del R, dR
    am.amulet_clear_selections()
    # too small for two slabs: the whole count with the built-in shape, no trials
    A, B = A[:300, :100], B[:100, :500]
    R_in = g.integers(-1000, 1000, (300, 500)).astype(np.int32)
    dR = dev(R_in)
    chosen, trials = am.amulet_count_i8_adaptive(dev(A), dev(B), dR)
    torch.cuda.synchronize()
    assert trials == 0
    R_ref, _ = oracle.count_i8(np.ascontiguousarray(A), np.ascontiguousarray(B), R_in)
    assert np.array_equal(dR.cpu().numpy(), R_ref)


@pytest.mark.parametrize("tA,tB", [(True, False), (False, True), (True, True), (False, False)])
def test_count_i8_transposed_operands(am, tA, tB):
    """A stored K x M and / or B stored N x K: transposed into the lent workspace, then the
    row-major kernels.  Ragged and whole-tile sizes, padded pitches, non-zero R_in; bit-exact."""
    for idx, (M, N, K, pad) in enumerate([(70, 300, 37, 0), (129, 1030, 77, 5), (256, 512, 128, 0),
                                           (1, 1, 1, 0), (300, 70, 1000, 16), (512, 1024, 640, 0)]):
        g = np.random.Generator(np.random.PCG64(420 + idx))
        A = g.integers(-128, 128, (M, K)).astype(np.int8)
        B = g.integers(-128, 128, (K, N)).astype(np.int8)
        R_in = g.integers(-1000, 1000, (M, N)).astype(np.int32)
        R_ref, _ = oracle.count_i8(A, B, R_in)
        As, Bs = (A.T.copy() if tA else A), (B.T.copy() if tB else B)
        bufA = torch.full((As.shape[0], As.shape[1] + pad), 55, dtype=torch.int8, device="cuda")
        bufB = torch.full((Bs.shape[0], Bs.shape[1] + pad), 66, dtype=torch.int8, device="cuda")
        bufA[:, :As.shape[1]] = dev(As)
        bufB[:, :Bs.shape[1]] = dev(Bs)
        need = am.amulet_count_i8_workspace_bytes(tA, tB, M, N, K)
        assert (need == 0) == (not tA and not tB)
        ws = torch.empty(need + 1, dtype=torch.int8, device="cuda")[:need] if need else None
        dR = dev(R_in)
        print("i8 transposed", tA, tB, M, N, K, pad, flush=True)
        am.amulet_count_i8_general(bufA[:, :As.shape[1]], bufB[:, :Bs.shape[1]], dR, ws, trans_a=tA, trans_b=tB)
        torch.cuda.synchronize()
        assert np.array_equal(dR.cpu().numpy(), R_ref), (tA, tB, M, N, K)
        if need:
            with pytest.raises(am.AmuletError) as err:
                am.amulet_count_i8_general(bufA[:, :As.shape[1]], bufB[:, :Bs.shape[1]], dR, ws[:need - 1],
                                           trans_a=tA, trans_b=tB)
            assert err.value.code == -8
            with pytest.raises(am.AmuletError) as err:
                am.amulet_count_i8_general(bufA[:, :As.shape[1]], bufB[:, :Bs.shape[1]], dR, None,
                                           trans_a=tA, trans_b=tB)
            assert err.value.code == -3


@pytest.mark.parametrize("tA,tB", [(False, False), (True, False), (False, True), (True, True)])
def test_count_i8_repacked_operands(am, tA, tB):
    """With the larger workspace the general entry point re-pitches operands whose rows are not
    16-byte aligned and pads a K that is not a multiple of 64 with zeros: same counts, bit for bit.
    The workspace starts out poisoned, the operands sit at odd byte offsets inside larger buffers,
    and sizes span whole streamed tiles plus ragged edges."""
    for idx, (M, N, K, pad, off) in enumerate([(300, 777, 1000, 3, 1), (512, 1024, 640, 0, 0), (257, 513, 63, 5, 7),
                                               (640, 600, 1030, 1, 3), (1, 1, 1, 0, 1), (520, 530, 129, 2, 0)]):
        g = np.random.Generator(np.random.PCG64(470 + idx))
        A = g.integers(-128, 128, (M, K)).astype(np.int8)
        B = g.integers(-128, 128, (K, N)).astype(np.int8)
        R_in = g.integers(-1000, 1000, (M, N)).astype(np.int32)
        R_ref, _ = oracle.count_i8(A, B, R_in)
        As, Bs = (A.T.copy() if tA else A), (B.T.copy() if tB else B)

        def place(X, fill):     # X at byte offset `off` of a buffer with row pitch cols + pad
            r, c = X.shape
            flat = torch.full((off + r * (c + pad) + 16,), fill, dtype=torch.int8, device="cuda")
            view = flat[off:off + r * (c + pad)].view(r, c + pad)[:, :c]
            view.copy_(dev(X))
            return view

        vA, vB = place(As, 55), place(Bs, 66)
        need = am.amulet_count_i8_repack_workspace_bytes(M, N, K)
        assert need >= am.amulet_count_i8_workspace_bytes(tA, tB, M, N, K)
        ws = torch.full((need,), 77, dtype=torch.int8, device="cuda")
        assert ws.data_ptr() % 16 == 0
        dR = dev(R_in)
        print("i8 repacked", tA, tB, M, N, K, pad, off, flush=True)
        am.amulet_count_i8_general(vA, vB, dR, ws, trans_a=tA, trans_b=tB)
        torch.cuda.synchronize()
        assert np.array_equal(dR.cpu().numpy(), R_ref), (tA, tB, M, N, K)


def test_count_i8_aligned_ragged_edges(am):
    """Aligned operands (rows on 16-byte boundaries, N a whole number of 16-byte units) whose M and N
    are not whole tiles: the edge workgroups load through range-checked buffers instead of the
    guarded loader.  Every matrix-core shape, full int8 range, non-zero R, K with and without a
    partial last stage; the operands sit inside larger poisoned buffers."""
    for idx, (M, N, K) in enumerate([(300, 400, 1008), (257, 528, 1024), (130, 272, 960), (700, 1296, 2048),
                                     (129, 16, 64), (513, 784, 1040)]):
        g = np.random.Generator(np.random.PCG64(480 + idx))
        A = g.integers(-128, 128, (M, K)).astype(np.int8)
        B = g.integers(-128, 128, (K, N)).astype(np.int8)
        R_in = g.integers(-1000, 1000, (M, N)).astype(np.int32)
        R_ref, _ = oracle.count_i8(A, B, R_in)
        bufA = torch.full((M + 3, K + 32), 99, dtype=torch.int8, device="cuda")
        bufB = torch.full((K + 3, N + 48), -77, dtype=torch.int8, device="cuda")
        bufA[:M, :K] = dev(A)
        bufB[:K, :N] = dev(B)
        for shape in range(1, am.amulet_shape_count(100)):
            for (vA, vB) in ((dev(A), dev(B)), (bufA[:M, :K], bufB[:K, :N])):
                dR = dev(R_in)
                print("i8 aligned ragged", M, N, K, shape, vA.stride(0), vB.stride(0), flush=True)
                am.amulet_count_i8_shape(shape, vA, vB, dR)
                torch.cuda.synchronize()
                assert np.array_equal(dR.cpu().numpy(), R_ref), (M, N, K, shape)


def test_count_i8_long_ragged_k(am):
    """Aligned operands with a long K that is not a whole number of 64-byte stages (so the last
    stage of every tile is partial), M and N ragged as well: default shape and both shapes that
    stream whole-stage problems."""
    for idx, (M, N, K) in enumerate([(260, 272, 4100), (512, 512, 4159), (300, 528, 4097)]):
        g = np.random.Generator(np.random.PCG64(490 + idx))
        A = g.integers(-128, 128, (M, K)).astype(np.int8)
        B = g.integers(-128, 128, (K, N)).astype(np.int8)
        R_in = g.integers(-1000, 1000, (M, N)).astype(np.int32)
        R_ref, _ = oracle.count_i8(A, B, R_in)
        bufA = torch.full((M, (K + 15) // 16 * 16 + 16), 99, dtype=torch.int8, device="cuda")
        bufA[:, :K] = dev(A)
        for shape in (-1, 6, 7):
            dR = dev(R_in)
            print("i8 long ragged K", M, N, K, shape, flush=True)
            if shape < 0:
                am.amulet_count_i8(bufA[:, :K], dev(B), dR)
            else:
                am.amulet_count_i8_shape(shape, bufA[:, :K], dev(B), dR)
            torch.cuda.synchronize()
            assert np.array_equal(dR.cpu().numpy(), R_ref), (M, N, K, shape)


def test_count_i8_strided(am):
    M, N, K = 50, 130, 75
    A, B = wl.join_indicator(M, N, K, seed=8, density=0.3)
    R_ref, _ = oracle.count_i8(A, B)
    bigA = torch.zeros(M, K + 5, dtype=torch.int8, device="cuda"); bigA[:, :K] = dev(A)
    bigB = torch.ones(K, N + 3, dtype=torch.int8, device="cuda"); bigB[:, :N] = dev(B)
    bigR = torch.full((M, N + 1), 9, dtype=torch.int32, device="cuda"); bigR[:, :N] = 0
    am.amulet_count_i8(bigA[:, :K], bigB[:, :N], bigR[:, :N])
    torch.cuda.synchronize()
    out = bigR.cpu().numpy()
    assert np.array_equal(out[:, :N], R_ref) and np.all(out[:, N] == 9)


# ---- the named workloads ----------------------------------------------------------
def test_cfg0_discount_256_full(am):
    spec, A, B, P = wl.make("cfg0_discount_256")
    R_ref, ab, _ = oracle.mmlike_f32(spec["task"], A, B, P)
    R = run_gpu(am, spec["task"], A, B, P, np.zeros_like(R_ref))
    assert_parity_f32(R, R_ref, ab, what="cfg0")


def test_cfg1_boost_2048_full(am):
    spec, A, B, P = wl.make("cfg1_boost_2048")
    R = run_gpu(am, spec["task"], A, B, P, np.zeros((2048, 2048), np.float32))
    print("cfg1: oracle on the full 2048^3 matrix", flush=True)
    R_ref, ab, _ = oracle.mmlike_f32(spec["task"], A, B, P)
    assert_parity_f32(R, R_ref, ab, what="cfg1")


def _sampled_rows_cols(am, name, n_rows=24, n_cols=24):
    """Full-size run in the default launch configuration; the oracle recomputes a
    seeded sample of whole rows and whole columns one by one."""
    spec, A, B, P = wl.make(name)
    M, N, K = spec["M"], spec["N"], spec["K"]
    print(name, "gpu run", flush=True)
    R = run_gpu(am, spec["task"], A, B, P, np.zeros((M, N), np.float32))
    g = np.random.Generator(np.random.PCG64(4242))
    rows = np.sort(g.choice(M, n_rows, replace=False))
    rows[0], rows[-1] = 0, M - 1
    cols = np.sort(g.choice(N, n_cols, replace=False))
    cols[0], cols[-1] = 0, N - 1
    print(name, "oracle rows", flush=True)
    R_ref, ab, _ = oracle.mmlike_f32(spec["task"], np.ascontiguousarray(A[rows]), B, P)
    w1 = assert_parity_f32(R[rows], R_ref, ab, what=name + " rows")
    print(name, "oracle cols", flush=True)
    Pc = None if P is None else np.ascontiguousarray(P[:, cols])
    R_ref, ab, _ = oracle.mmlike_f32(spec["task"], A, np.ascontiguousarray(B[:, cols]), Pc)
    w2 = assert_parity_f32(R[:, cols], R_ref, ab, what=name + " cols")
    print(name, "worst ratio", max(w1, w2), flush=True)
    return R, A, B, P


def test_cfg2_identity_4096_sampled(am):
    R, A, B, _ = _sampled_rows_cols(am, "cfg2_identity_4096")
    # whole-matrix property: column sums of R equal (column sums of A) @ B
    ref = A.astype(np.float64).sum(0) @ B.astype(np.float64)
    scale = np.abs(A).astype(np.float64).sum(0) @ np.abs(B).astype(np.float64)
    assert np.max(np.abs(R.astype(np.float64).sum(0) - ref) / scale) < 1e-5


def test_cfg4_discount_rect_sampled(am):
    _sampled_rows_cols(am, "cfg4_discount_16384x2048x8192", n_rows=12, n_cols=6)


def test_headline_discount_8192_sampled(am):
    _sampled_rows_cols(am, "headline_discount_8192", n_rows=12, n_cols=12)


def test_headline_discount_8192_whole_matrix_closed_form(am):
    """The headline size in the default launch configuration on operands whose result has a
    closed form: A = B = 1, thres = 0.5, dis = 0.5, so every product is 1, triggers, and adds
    exactly 0.5; every one of the 8192^2 outputs must equal R_in + K / 2 bit for bit (integer
    R_in).  A tile computed twice, skipped, or fed a wrong k range shows."""
    M = N = K = 8192
    dA = torch.ones(M, K, device="cuda")
    dB = torch.ones(K, N, device="cuda")
    dP = torch.full((2, N), 0.5, device="cuda")
    g = torch.Generator(device="cuda").manual_seed(5)
    dR = torch.randint(-3, 4, (M, N), device="cuda", generator=g).float()
    want = dR + K / 2
    print("headline closed form: gpu run", flush=True)
    am.amulet_mmlike_f32(1, dA, dB, dP, dR)
    torch.cuda.synchronize()
    assert torch.equal(dR, want)


def test_query3_count_gt_4096_sampled(am):
    """Query 3 at the paper's square size: integer counts, so sampled rows and columns must
    match the oracle bit for bit (and they pass assert_parity_f32 a fortiori)."""
    spec, A, B, P = wl.make("query3_count_gt_4096")
    M, N = spec["M"], spec["N"]
    R = run_gpu(am, spec["task"], A, B, P, np.zeros((M, N), np.float32))
    g = np.random.Generator(np.random.PCG64(4343))
    rows = np.sort(g.choice(M, 24, replace=False))
    rows[0], rows[-1] = 0, M - 1
    cols = np.sort(g.choice(N, 24, replace=False))
    cols[0], cols[-1] = 0, N - 1
    R_ref, _, _ = oracle.mmlike_f32(spec["task"], np.ascontiguousarray(A[rows]), B, P)
    assert np.array_equal(R[rows], R_ref)
    R_ref, _, _ = oracle.mmlike_f32(spec["task"], A, np.ascontiguousarray(B[:, cols]), np.ascontiguousarray(P[:, cols]))
    assert np.array_equal(R[:, cols], R_ref)
    assert 0 < R.mean() < spec["K"]          # neither never nor always triggered


def test_cfg3_join_count_full_size_sampled(am):
    spec, A, B, _ = wl.make("cfg3_count_i8_8192x8192x4096")
    M, N = spec["M"], spec["N"]
    dR = torch.zeros(M, N, dtype=torch.int32, device="cuda")
    am.amulet_count_i8(dev(A), dev(B), dR)
    torch.cuda.synchronize()
    R = dR.cpu().numpy()
    g = np.random.Generator(np.random.PCG64(4243))
    rows = np.sort(g.choice(M, 32, replace=False)); rows[0], rows[-1] = 0, M - 1
    cols = np.sort(g.choice(N, 32, replace=False)); cols[0], cols[-1] = 0, N - 1
    R_ref, _ = oracle.count_i8(np.ascontiguousarray(A[rows]), B)
    assert np.array_equal(R[rows], R_ref)
    R_ref, _ = oracle.count_i8(A, np.ascontiguousarray(B[:, cols]))
    assert np.array_equal(R[:, cols], R_ref)
    # whole-matrix checksum: sum_j R[i][j] = sum_k A[i][k] * (sum_j B[k][j]), exact in int64
    assert np.array_equal(R.astype(np.int64).sum(1), A.astype(np.int64) @ B.astype(np.int64).sum(1))
    assert np.array_equal(R.astype(np.int64).sum(0), A.astype(np.int64).sum(0) @ B.astype(np.int64))


def test_join_count_odd_full_size_repacked_and_in_place_sampled(am):
    """The join count at 8191 x 8191 x 4095 (nothing aligned, nothing a whole tile or stage), in
    place and through the repacking workspace, in the launch configurations the library picks
    at that size: sampled rows and columns against the oracle, and the whole-matrix checksums."""
    M, N, K = 8191, 8191, 4095
    A, B = wl.join_indicator(M, N, K, seed=31, density=0.05)
    g = np.random.Generator(np.random.PCG64(4244))
    rows = np.sort(g.choice(M, 16, replace=False)); rows[0], rows[-1] = 0, M - 1
    cols = np.sort(g.choice(N, 16, replace=False)); cols[0], cols[-1] = 0, N - 1
    R_rows, _ = oracle.count_i8(np.ascontiguousarray(A[rows]), B)
    R_cols, _ = oracle.count_i8(A, np.ascontiguousarray(B[:, cols]))
    row_sums = A.astype(np.int64) @ B.astype(np.int64).sum(1)
    col_sums = A.astype(np.int64).sum(0) @ B.astype(np.int64)
    dA, dB = dev(A), dev(B)
    ws = torch.full((am.amulet_count_i8_repack_workspace_bytes(M, N, K),), 77, dtype=torch.int8, device="cuda")
    for how in ("in place", "repacked"):
        dR = torch.zeros(M, N, dtype=torch.int32, device="cuda")
        print("join count odd full size", how, flush=True)
        if how == "in place":
            am.amulet_count_i8(dA, dB, dR)
        else:
            am.amulet_count_i8_general(dA, dB, dR, ws)
        torch.cuda.synchronize()
        R = dR.cpu().numpy()
        assert np.array_equal(R[rows], R_rows), how
        assert np.array_equal(R[:, cols], R_cols), how
        assert np.array_equal(R.astype(np.int64).sum(1), row_sums), how
        assert np.array_equal(R.astype(np.int64).sum(0), col_sums), how


def test_tune_picks_a_valid_shape_and_result_still_matches(am):
    M, N, K = 512, 1024, 256
    chosen = am.amulet_tune(1, M, N, K)
    assert 0 <= chosen < am.amulet_shape_count(1)
    assert am.amulet_selected_shape(1, M, N, K) == chosen
    A, B, P = wl.retail(M, N, K, seed=21)
    R_ref, ab, _ = oracle.mmlike_f32(1, A, B, P)
    R = run_gpu(am, 1, A, B, P, np.zeros_like(R_ref))
    assert_parity_f32(R, R_ref, ab, what="after tune")
    am.amulet_clear_selections()


def test_tuned_choice_serves_the_whole_size_bucket(am):
    """The selection cache is keyed by size buckets of 256: a choice tuned at one size is the
    one used at neighbouring sizes of the same bucket, and not beyond."""
    am.amulet_clear_selections()
    chosen = am.amulet_tune(1, 512, 1024, 256)
    assert am.amulet_selected_shape(1, 500, 1000, 250) == chosen
    assert am.amulet_selected_shape(1, 257, 769, 1) == chosen
    am.amulet_clear_selections()
    assert am.amulet_selected_shape(1, 512, 1024, 256) == am.amulet_selected_shape(1, 500, 1000, 250)


def test_refused_launch_leaves_R_untouched_and_nothing_cached(am):
    """Launches refused on the host (the library's test seam): every compute call reports the
    failure, R keeps its contents, and neither amulet_tune nor the adaptive call caches a shape
    that never ran."""
    M, N, K = 4096, 4096, 512
    A, B, P = wl.retail(M, N, K, seed=77)
    dA, dB, dP = dev(A), dev(B), dev(P)
    dR = torch.full((M, N), 3.0, device="cuda")
    am.amulet_clear_selections()
    before = am.amulet_selected_shape(1, M, N, K)
    try:
        am.amulet_debug_fail_launches(1)
        with pytest.raises(am.AmuletError) as e:
            am.amulet_mmlike_f32(1, dA, dB, dP, dR)
        assert e.value.code == -5
        am.amulet_debug_fail_launches(1 << 20)
        with pytest.raises(am.AmuletError) as e:
            am.amulet_tune(1, M, N, K)
        assert e.value.code == -5
        with pytest.raises(am.AmuletError) as e:
            am.amulet_mmlike_f32_adaptive(1, dA, dB, dP, dR)
        assert e.value.code == -5
        with pytest.raises(am.AmuletError):
            am.amulet_count_i8(torch.ones(256, 64, dtype=torch.int8, device="cuda"),
                               torch.ones(64, 256, dtype=torch.int8, device="cuda"),
                               torch.zeros(256, 256, dtype=torch.int32, device="cuda"))
    finally:
        am.amulet_debug_fail_launches(0)
    torch.cuda.synchronize()
    assert torch.all(dR == 3.0)
    assert am.amulet_selected_shape(1, M, N, K) == before
    # and the library works as before once the seam is off
    am.amulet_mmlike_f32(1, dA, dB, dP, dR)
    torch.cuda.synchronize()
    rows = np.arange(0, M, 257)
    R_ref, ab, _ = oracle.mmlike_f32(1, np.ascontiguousarray(A[rows]), B, P, np.full((len(rows), N), 3.0, np.float32))
    assert_parity_f32(dR.cpu().numpy()[rows], R_ref, ab, np.full((len(rows), N), 3.0, np.float32), what="after the seam")


@pytest.mark.parametrize("task,M,N,K", [(1, 256, 256, 256), (2, 64, 64, 20000), (1, 770, 6100, 1100), (0, 300, 300, 4096),
                                        (0, 1536, 1536, 2048)])   # the last: whole tiles, the streamed identity kernel
def test_deterministic_mode_gives_the_same_bits_twice(am, task, M, N, K):
    """Sizes whose default launch splits K (few tiles; a nearly empty last round): with the
    deterministic mode on, two runs agree bit for bit and match the oracle to the tolerance."""
    A, B, params, R_in = rand_case(task, M, N, K, seed=900 + task)
    R_ref, ab, _ = oracle.mmlike_f32(task, A, B, params, R_in)
    was = am.amulet_get_deterministic()
    try:
        am.amulet_set_deterministic(True)
        R1 = run_gpu(am, task, A, B, params, R_in)
        R2 = run_gpu(am, task, A, B, params, R_in)
    finally:
        am.amulet_set_deterministic(was)
    assert np.array_equal(R1, R2)
    assert_parity_f32(R1, R_ref, ab, R_in, what="deterministic mode, task %d" % task)
    R3 = run_gpu(am, task, A, B, params, R_in)   # default mode: split K, same tolerance
    assert_parity_f32(R3, R_ref, ab, R_in, what="default mode, task %d" % task)
