"""GPU parity for the general test-query form: threshold operand forms and transposed
operand storage, against the oracle's general form on the same seeded inputs."""
import numpy as np
import pytest

import oracle
from parity import assert_parity_f32

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

FORMS = [0, 1, 2, 3]
TASKS = [1, 2, 3]


@pytest.fixture(scope="module")
def am():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2305_08872_amd as am
    am.load_library()
    return am


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def make_case(task, form, tA, tB, M, N, K, seed, exact=False):
    g = np.random.Generator(np.random.PCG64(seed))
    if exact:
        A = g.integers(-8, 9, (M, K)).astype(np.float32)
        B = g.integers(-8, 9, (K, N)).astype(np.float32)
    else:
        A = (g.standard_normal((M, K)) * 2).astype(np.float32)
        B = (g.standard_normal((K, N)) * 2).astype(np.float32)
    shape = {0: (N,), 1: (M,), 2: (1,), 3: (M, N)}[form]
    th = (g.integers(-24, 25, shape) / 2.0).astype(np.float32) if exact else \
        (g.standard_normal(shape) * 3).astype(np.float32)
    dis = (g.integers(0, 9, N) / 8.0).astype(np.float32) if exact else g.uniform(0, 1, N).astype(np.float32)
    R_in = (g.integers(-5, 6, (M, N))).astype(np.float32)
    As = np.ascontiguousarray(A.T) if tA else A
    Bs = np.ascontiguousarray(B.T) if tB else B
    return As, Bs, th, dis, R_in


def run(am, task, form, tA, tB, As, Bs, th, dis, R_in, shape=-1):
    dR = dev(R_in)
    am.amulet_mmlike_f32_general(task, dev(As), dev(Bs), dev(th) if task else None,
                                 dev(dis) if task == 1 else None, dR,
                                 thres_form=form, trans_a=tA, trans_b=tB, shape=shape)
    torch.cuda.synchronize()
    return dR.cpu().numpy()


SIZES = [(70, 300, 37), (33, 513, 100), (129, 1030, 77), (3, 5, 2)]


@pytest.mark.parametrize("task", TASKS)
@pytest.mark.parametrize("form", FORMS)
def test_threshold_forms_all_shapes(am, task, form):
    for shape in range(8):
        M, N, K = SIZES[shape % len(SIZES)]
        As, Bs, th, dis, R_in = make_case(task, form, False, False, M, N, K, 2000 + 40 * task + 8 * form + shape)
        print("case", task, form, shape, M, N, K, flush=True)
        R_ref, ab, _ = oracle.mmlike_f32_general(task, As, Bs, th, dis, R_in, thres_form=form)
        R = run(am, task, form, False, False, As, Bs, th, dis, R_in, shape)
        if task == 3:
            assert np.array_equal(R, R_ref), (task, form, shape)
        else:
            assert_parity_f32(R, R_ref, ab, R_in, what="task %d form %d shape %d" % (task, form, shape))


@pytest.mark.parametrize("task", [0, 1, 2, 3])
@pytest.mark.parametrize("tA,tB", [(True, False), (False, True), (True, True)])
def test_transposed_operands(am, task, tA, tB):
    for idx, (M, N, K) in enumerate(SIZES + [(64, 512, 64)]):
        for shape in ((0, 7) if idx % 2 == 0 else (2, 5)):
            form = (idx + shape) % 4 if task else 0
            As, Bs, th, dis, R_in = make_case(task, form, tA, tB, M, N, K, 3000 + 50 * task + idx)
            print("case", task, tA, tB, shape, M, N, K, flush=True)
            R_ref, ab, _ = oracle.mmlike_f32_general(task, As, Bs, th, dis, R_in, thres_form=form,
                                                     trans_a=tA, trans_b=tB)
            R = run(am, task, form, tA, tB, As, Bs, th, dis, R_in, shape)
            if task == 3:
                assert np.array_equal(R, R_ref), (task, tA, tB, shape, M, N, K)
            else:
                assert_parity_f32(R, R_ref, ab, R_in, what="task %d tA %d tB %d %dx%dx%d" % (task, tA, tB, M, N, K))


def test_exact_data_bit_exact_all_forms_and_layouts(am):
    for task in TASKS:
        for form in FORMS:
            for tA, tB in ((False, False), (True, True)):
                As, Bs, th, dis, R_in = make_case(task, form, tA, tB, 50, 520, 45, 4000 + task * 9 + form, exact=True)
                R_ref, _, _ = oracle.mmlike_f32_general(task, As, Bs, th, dis, R_in, thres_form=form,
                                                        trans_a=tA, trans_b=tB)
                R = run(am, task, form, tA, tB, As, Bs, th, dis, R_in)
                assert np.array_equal(R, R_ref), (task, form, tA, tB)


def test_transposed_strided_unaligned(am):
    M, N, K = 37, 290, 53
    task, form = 2, 1
    As, Bs, th, dis, R_in = make_case(task, form, True, True, M, N, K, 5000)
    R_ref, ab, _ = oracle.mmlike_f32_general(task, As, Bs, th, dis, R_in, thres_form=form, trans_a=True, trans_b=True)
    bigA = torch.zeros(K, M + 3, device="cuda"); bigA[:, :M] = dev(As)     # lda = M + 3 (odd pitch)
    bigB = torch.zeros(N, K + 1, device="cuda"); bigB[:, :K] = dev(Bs)     # ldb = K + 1
    dR = dev(R_in)
    am.amulet_mmlike_f32_general(task, bigA[:, :M], bigB[:, :K], dev(th), None, dR, thres_form=form,
                                 trans_a=True, trans_b=True)
    torch.cuda.synchronize()
    assert_parity_f32(dR.cpu().numpy(), R_ref, ab, R_in, what="transposed strided")


@pytest.mark.parametrize("tA,tB", [(True, False), (False, True), (True, True)])
def test_identity_transposed_on_the_matrix_cores(am, tA, tB):
    """The matrix-core identity kernel (shape 8; what the default falls back to for these layouts) with transposed operands: ragged
    and multi-tile sizes, odd pitches (scalar path) and aligned ones (16-byte path)."""
    for idx, (M, N, K) in enumerate([(70, 300, 37), (129, 1030, 77), (3, 5, 2), (256, 256, 64), (200, 136, 100),
                                     (130, 129, 17)]):
        As, Bs, th, dis, R_in = make_case(0, 0, tA, tB, M, N, K, 5200 + idx)
        R_ref, ab, _ = oracle.mmlike_f32_general(0, As, Bs, None, None, R_in, trans_a=tA, trans_b=tB)
        for pad in (0, 3):
            bufA = torch.zeros(As.shape[0], As.shape[1] + pad, device="cuda"); bufA[:, :As.shape[1]] = dev(As)
            bufB = torch.zeros(Bs.shape[0], Bs.shape[1] + pad, device="cuda"); bufB[:, :Bs.shape[1]] = dev(Bs)
            for shape in (8, 9, 10, 11, 12, -1):   # 10, 11, 12: the streamed kernels where the size allows it
                print("identity trans", tA, tB, M, N, K, pad, shape, flush=True)
                dR = dev(R_in)
                am.amulet_mmlike_f32_general(0, bufA[:, :As.shape[1]], bufB[:, :Bs.shape[1]], None, None, dR,
                                             trans_a=tA, trans_b=tB, shape=shape)
                torch.cuda.synchronize()
                assert_parity_f32(dR.cpu().numpy(), R_ref, ab, R_in, what="identity trans %r %r" % (tA, tB))


def test_identity_aligned_ragged_edges_on_the_matrix_cores(am):
    """Aligned row-major operands (16-byte aligned rows, N a multiple of 4) whose M and N are not
    whole tiles: the edge workgroups of the matrix-core kernel load through range-checked buffers.
    The operands sit inside larger buffers filled with NaN, so anything read from outside them
    that reached an existing output would show."""
    for idx, (M, N, K) in enumerate([(300, 400, 1008), (257, 528, 1024), (130, 272, 96), (513, 784, 1040),
                                     (129, 4, 16), (700, 1296, 208)]):
        As, Bs, th, dis, R_in = make_case(0, 0, False, False, M, N, K, 5300 + idx)
        R_ref, ab, _ = oracle.mmlike_f32_general(0, As, Bs, None, None, R_in)
        bufA = torch.full((M + 3, K + 8), float("nan"), device="cuda"); bufA[:M, :K] = dev(As)
        bufB = torch.full((K + 3, N + 12), float("nan"), device="cuda"); bufB[:K, :N] = dev(Bs)
        for shape in (8, 9, 10, 11, 12, -1):   # 10, 11, 12: the streamed kernels where the size allows it
            for (vA, vB) in ((dev(As), dev(Bs)), (bufA[:M, :K], bufB[:K, :N])):
                print("identity aligned ragged", M, N, K, shape, vA.stride(0), vB.stride(0), flush=True)
                dR = dev(R_in)
                am.amulet_mmlike_f32_general(0, vA, vB, None, None, dR, shape=shape)
                torch.cuda.synchronize()
                assert_parity_f32(dR.cpu().numpy(), R_ref, ab, R_in, what="identity aligned ragged %d" % shape)


def test_adaptive_execution_trials_contribute_to_the_result(am, monkeypatch):
    import amulet_workloads as wl
    monkeypatch.setenv("AMULET_ADAPTIVE_MIN_TASK_MS", "0")   # (a sub-millisecond task: lift the one-trial limit)
    M, N, K = 8192, 8192, 48
    A, B, P = wl.retail(M, N, K, seed=31)
    R_in = np.ones((M, N), np.float32)
    dR = dev(R_in)
    am.amulet_clear_selections()
    chosen, trials = am.amulet_mmlike_f32_adaptive(1, dev(A), dev(B), dev(P), dR)
    torch.cuda.synchronize()
    assert 0 <= chosen < am.amulet_shape_count(1)
    assert trials >= 3                      # two depths, then at least one step along the tile axis
    assert am.amulet_selected_shape(1, M, N, K) == chosen
    R_ref, ab, _ = oracle.mmlike_f32(1, A, B, P, R_in)
    assert_parity_f32(dR.cpu().numpy(), R_ref, ab, R_in, what="adaptive execution")
    # a task too small for trial slabs still runs, with the default shape and no trials
    A2, B2, P2 = wl.retail(40, 300, 50, seed=32)
    dR2 = torch.zeros(40, 300, device="cuda")
    _, t2 = am.amulet_mmlike_f32_adaptive(1, dev(A2), dev(B2), dev(P2), dR2)
    torch.cuda.synchronize()
    assert t2 == 0
    R_ref, ab, _ = oracle.mmlike_f32(1, A2, B2, P2)
    assert_parity_f32(dR2.cpu().numpy(), R_ref, ab, what="adaptive, small")
    # identity: the matrix-core kernel takes part in the trials
    A3 = np.random.Generator(np.random.PCG64(5)).standard_normal((8192, 40)).astype(np.float32)
    B3 = np.random.Generator(np.random.PCG64(6)).standard_normal((40, 8192)).astype(np.float32)
    dR3 = torch.zeros(8192, 8192, device="cuda")
    c3, t3 = am.amulet_mmlike_f32_adaptive(0, dev(A3), dev(B3), None, dR3)
    torch.cuda.synchronize()
    R_ref, ab, _ = oracle.mmlike_f32(0, A3, B3, None)
    assert_parity_f32(dR3.cpu().numpy(), R_ref, ab, what="adaptive identity")
    assert t3 >= 1 and c3 in (8, 9, 10, 11)   # only the matrix-core shapes are tried for the dense contraction
    am.amulet_clear_selections()


@pytest.mark.parametrize("task,form,tA,tB", [(1, 1, False, False), (2, 3, True, False), (3, 2, False, True), (1, 0, True, True)])
def test_adaptive_execution_of_the_general_form(am, task, form, tA, tB, monkeypatch):
    """In-flight adaptive execution with the other threshold operand forms and transposed layouts:
    trials on row slabs of the caller's R (rows of a transposed A are columns of its storage, the
    rows of thres[i] / thres[i][j] move with the slab), K long enough for the k axis's split
    points to act; the whole R against the oracle.  (The task takes about a millisecond, which an
    adaptive call would not spend more than one trial on: the limit is lifted for the test.)"""
    monkeypatch.setenv("AMULET_ADAPTIVE_MIN_TASK_MS", "0")
    M, N, K = 8192, 8192, 300
    g = np.random.Generator(np.random.PCG64(700 + task))
    A = g.integers(0, 10, (M, K)).astype(np.float32)
    B = g.uniform(1, 100, (K, N)).astype(np.float32)
    th = {0: g.uniform(100, 500, N), 1: g.uniform(100, 500, M), 2: np.array([250.0]),
          3: g.uniform(100, 500, (M, N))}[form].astype(np.float32)
    dis = g.uniform(0.05, 0.3, N).astype(np.float32)
    R_in = np.rint(g.standard_normal((M, N)) * 3).astype(np.float32)
    dR = dev(R_in)
    am.amulet_clear_selections()
    print("adaptive general", task, form, tA, tB, flush=True)
    chosen, trials = am.amulet_mmlike_f32_adaptive_general(
        task, dev(A.T) if tA else dev(A), dev(B.T) if tB else dev(B), dev(th), dev(dis) if task == 1 else None, dR,
        thres_form=form, trans_a=tA, trans_b=tB)
    torch.cuda.synchronize()
    assert 0 <= chosen < am.amulet_shape_count(task) and trials >= 6   # the default shape, then the whole k axis
    assert am.amulet_selected_shape(task, M, N, K) == chosen
    R_ref, ab, _ = oracle.mmlike_f32_general(task, A, B, th, dis if task == 1 else None, R_in, thres_form=form)
    if task == 3:
        assert np.array_equal(dR.cpu().numpy(), R_ref)
    else:
        assert_parity_f32(dR.cpu().numpy(), R_ref, ab, R_in, what="adaptive general form")
    am.amulet_clear_selections()


@pytest.mark.parametrize("task", [0, 1, 2, 3])
def test_few_tiles_long_k_split_over_workgroups(am, task):
    """Tiny M x N with a long K: the launcher splits K over several workgroups per tile, which add
    their parts to R atomically.  Checked for every vector-ALU shape, ragged K, non-zero R_in, a
    transposed layout and data whose sums are exact in any order (bit-exact then)."""
    cases = [(64, 64, 5000, False), (20, 300, 1037, False), (130, 260, 777, True), (5, 5, 4096, False)]
    for idx, (M, N, K, trans) in enumerate(cases):
        for shape in (4, 0, 5, 7) + ((8, 9, 10, 11) if task == 0 else ()):   # 8-11: the matrix-core identity kernels
            form = (idx + shape) % 4 if task else 0
            As, Bs, th, dis, R_in = make_case(task, form, trans, trans, M, N, K, 6100 + 10 * task + idx)
            R_ref, ab, _ = oracle.mmlike_f32_general(task, As, Bs, th, dis, R_in, thres_form=form, trans_a=trans,
                                                     trans_b=trans)
            print("split-K case", task, form, shape, M, N, K, trans, flush=True)
            R = run(am, task, form, trans, trans, As, Bs, th, dis, R_in, shape)
            if task == 3:
                assert np.array_equal(R, R_ref), (task, form, shape, M, N, K)
            else:
                assert_parity_f32(R, R_ref, ab, R_in, what="split-K task %d shape %d %dx%dx%d" % (task, shape, M, N, K))
    # exact data: small integers and half-integer thresholds, every partial sum exact in fp32
    As, Bs, th, dis, R_in = make_case(task, 0, False, False, 48, 200, 1500, 6200 + task, exact=True)
    R_ref, _, _ = oracle.mmlike_f32_general(task, As, Bs, th, dis, R_in)
    R = run(am, task, 0, False, False, As, Bs, th, dis, R_in)
    assert np.array_equal(R, R_ref)


@pytest.mark.parametrize("trans", [False, True])
def test_identity_last_round_of_tiles_split_over_k(am, trans):
    """Matrix-core identity kernels with a few more tiles than compute units (275 tiles of
    128 x 128 against 256): the tiles of the nearly empty last round run once per k range and
    add their parts to R atomically.  Ragged M, N, K; every output checked; the 256 x 256
    shape (77 tiles: fewer than half the compute units, every tile split) rides along."""
    M, N, K = 1300, 3200, 1100
    As, Bs, th, dis, R_in = make_case(0, 0, trans, trans, M, N, K, 6400 + int(trans))
    R_ref, ab, _ = oracle.mmlike_f32_general(0, As, Bs, None, None, R_in, trans_a=trans, trans_b=trans)
    for shape in (8, 9, 10, 11, 12, -1):   # 10, 11, 12: the streamed kernels where the size allows it
        print("identity tail split", trans, shape, M, N, K, flush=True)
        R = run(am, 0, 0, trans, trans, As, Bs, th, dis, R_in, shape)
        assert_parity_f32(R, R_ref, ab, R_in, what="identity tail split shape %d" % shape)


@pytest.mark.parametrize("tA,tB", [(False, False), (True, False), (False, True), (True, True)])
def test_identity_streamed_kernel_on_every_size(am, tA, tB):
    """The matrix-core identity kernel that streams its operands HBM -> LDS (shapes 10, 11: 128 x
    128 tiles, rings of 3 and 4 stages; 12: 64 x 64 tiles, ring of 6) runs on operands of any size and alignment with at least one 16-k stage, in
    any of the four operand layouts.  Cases: fewer stages than the ring holds,
    one tile, several tiles with padded pitches and a non-zero R_in, few tiles with a long K (every
    tile split over workgroups), and a few more tiles than compute units (the last round's tiles
    split).  Every output is checked against the oracle; data whose sums are exact must match
    bit for bit."""
    cases = [(128, 128, 16, 0), (128, 128, 32, 0), (256, 384, 208, 4), (128, 256, 4096, 0), (1408, 3200, 1104, 8),
             # M and N that are not whole tiles (edge tiles fetch clamped lines and write back only
             # what exists): fewer rows than a tile, one more row or unit than whole tiles, sizes
             # that are no multiple of four (streamed only where the operand's lines run along k),
             # a split K with edge tiles, a split last round with edge tiles
             (100, 132, 64, 0), (257, 260, 208, 4), (130, 131, 32, 0), (60, 4100, 4096, 0), (1300, 3204, 1104, 8),
             # K that is no whole number of 16-k stages (the k past the last whole stage are multiplied
             # from values each lane fetches itself): one stage and a bit, padded pitches, a split K,
             # a split last round, together with edge tiles
             (128, 128, 20, 0), (256, 384, 204, 4), (128, 256, 4100, 0), (1408, 3200, 1108, 8), (100, 132, 1036, 0),
             # odd sizes and pitches: rows that are not 16-byte aligned (16-byte pieces fetched at
             # 4-byte aligned addresses), edges that cut a four-line unit, tiles with fewer than four
             # lines (129 = 128 + 1), the smallest operands the kernel takes
             (129, 131, 33, 0), (257, 259, 211, 1), (127, 129, 1001, 0), (5, 7, 48, 0), (4, 4, 16, 0), (130, 133, 1037, 3),
             (1301, 3203, 1109, 0),
             # around the 64 x 64 tile: one tile and one stage, a line more than whole tiles, a K of
             # fewer stages than its ring holds plus a tail, few tiles with a long K
             (64, 64, 16, 0), (65, 67, 33, 0), (190, 70, 100, 2), (192, 320, 2100, 0)]
    for idx, (M, N, K, pad) in enumerate(cases):
        As, Bs, th, dis, R_in = make_case(0, 0, tA, tB, M, N, K, 6500 + idx)
        R_ref, ab, _ = oracle.mmlike_f32_general(0, As, Bs, None, None, R_in, trans_a=tA, trans_b=tB)
        bufA = torch.full((As.shape[0], As.shape[1] + pad), float("nan"), device="cuda"); bufA[:, :As.shape[1]] = dev(As)
        bufB = torch.full((Bs.shape[0], Bs.shape[1] + pad), float("nan"), device="cuda"); bufB[:, :Bs.shape[1]] = dev(Bs)
        for shape in (10, 11, 12):
            print("identity streamed", tA, tB, M, N, K, pad, shape, flush=True)
            dR = dev(R_in)
            am.amulet_mmlike_f32_general(0, bufA[:, :As.shape[1]], bufB[:, :Bs.shape[1]], None, None, dR,
                                         trans_a=tA, trans_b=tB, shape=shape)
            torch.cuda.synchronize()
            assert_parity_f32(dR.cpu().numpy(), R_ref, ab, R_in, what="identity streamed %d %dx%dx%d" % (shape, M, N, K))
    As, Bs, th, dis, R_in = make_case(0, 0, tA, tB, 256, 256, 1600, 6600, exact=True)
    R_ref, _, _ = oracle.mmlike_f32_general(0, As, Bs, None, None, R_in, trans_a=tA, trans_b=tB)
    for shape in (10, 11, 12):
        R = run(am, 0, 0, tA, tB, As, Bs, None, None, R_in, shape)
        assert np.array_equal(R, R_ref), shape


@pytest.mark.parametrize("task", TASKS)
def test_rows_of_A_with_a_colliding_pitch_go_through_lds(am, task):
    """A row-major A whose row pitch is a multiple of 32 KiB (here 64 KiB: a view of a wider
    array) takes the kernel variant that stages A through LDS.  Every shape (those without
    the variant run their usual kernel), every threshold form, ragged M, N and K, a K
    remainder, a split K (few tiles, long K) and a split last round; A unaligned as well."""
    cases = [(70, 300, 37, 0), (129, 1030, 77, 0), (33, 513, 100, 1), (3, 5, 2, 0), (64, 512, 1100, 0),
             (770, 6100, 600, 0)]
    for idx, (M, N, K, off) in enumerate(cases):
        form = idx % 4 if task else 0
        As, Bs, th, dis, R_in = make_case(task, form, False, False, M, N, K, 7300 + 10 * task + idx)
        R_ref, ab, _ = oracle.mmlike_f32_general(task, As, Bs, th, dis, R_in, thres_form=form)
        wide = torch.zeros((M * 16384 + 4,), device="cuda")[off:off + M * 16384].view(M, 16384)   # pitch 64 KiB
        dA = wide[:, :K]
        dA.copy_(dev(As))
        assert am.amulet_pitch_collides(dA.stride(0) if M > 1 else 16384, 4)
        for shape in ((-1, 4, 5, 0, 1, 2) if idx < 5 else (-1, 4, 5)):
            dR = dev(R_in)
            print("A through LDS", task, form, shape, M, N, K, off, flush=True)
            am.amulet_mmlike_f32_general(task, dA, dev(Bs), dev(th) if task else None, dev(dis) if task == 1 else None,
                                         dR, thres_form=form, shape=shape)
            torch.cuda.synchronize()
            R = dR.cpu().numpy()
            if task == 3:
                assert np.array_equal(R, R_ref), (task, form, shape, M, N, K)
            else:
                assert_parity_f32(R, R_ref, ab, R_in, what="A through LDS task %d shape %d %dx%dx%d" % (task, shape, M, N, K))


def test_compute_calls_can_be_captured_in_a_graph(am):
    """Compute calls only enqueue kernels on the caller's stream (no allocation, no sync, no
    memset), so a sequence of them can be captured once and replayed: three tasks of different
    kinds (split-K vector-ALU, matrix-core identity, int8 join count) in one graph, replayed
    several times with eager work in between, every replay checked against the oracle."""
    g = np.random.Generator(np.random.PCG64(77))
    M, N, K = 96, 512, 320
    As, Bs, th, dis, R_in = make_case(1, 0, False, False, M, N, K, 6400)
    dA, dB, dth, ddis = dev(As), dev(Bs), dev(th), dev(dis)
    A8 = g.integers(-3, 4, (128, 256)).astype(np.int8); B8 = g.integers(-3, 4, (256, 256)).astype(np.int8)
    dA8, dB8 = dev(A8), dev(B8)
    R1 = torch.zeros(M, N, device="cuda"); R0 = torch.zeros(M, N, device="cuda")
    R8 = torch.zeros(128, 256, dtype=torch.int32, device="cuda")

    def enqueue():
        am.amulet_mmlike_f32_general(1, dA, dB, dth, ddis, R1)
        am.amulet_mmlike_f32_general(0, dA, dB, None, None, R0)
        am.amulet_count_i8(dA8, dB8, R8)

    enqueue()                       # eager warm-up: one-time kernel attributes are set outside the capture
    torch.cuda.synchronize()
    R1.zero_(); R0.zero_(); R8.zero_()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue()
    ref1, ab1, _ = oracle.mmlike_f32_general(1, As, Bs, th, dis, None)
    ref0, ab0, _ = oracle.mmlike_f32_general(0, As, Bs, None, None, None)
    ref8, _ = oracle.count_i8(A8, B8)
    for replay in range(1, 4):
        graph.replay()
        torch.cuda.synchronize()
        scratch = torch.rand(256, 256, device="cuda") @ torch.rand(256, 256, device="cuda")   # eager work between replays
        torch.cuda.synchronize()
        del scratch
        # R accumulates: after `replay` replays it holds replay x the single-call result
        assert_parity_f32(R1.cpu().numpy(), replay * ref1, replay * ab1, what="graph replay %d discount" % replay)
        assert_parity_f32(R0.cpu().numpy(), replay * ref0, replay * ab0, what="graph replay %d identity" % replay)
        assert np.array_equal(R8.cpu().numpy(), replay * ref8)
