"""GPU parity where the output has more than 2^31 elements, so that an element offset
i * ldr + j no longer fits 32 bits: every kernel family must index R (and the wide operand)
in 64 bits.  K is short, so the launches are quick; the oracle checks sampled whole rows,
among them the last ones, whose offsets are the largest."""
import numpy as np
import pytest

import oracle
from parity import assert_parity_f32, worst_ratio

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

M, N, K = 46400, 46400, 24            # M * N = 2.153e9 > 2^31 = 2.147e9
ROWS = np.array([0, 1, 255, 256, M // 2 + 3, 46336, M - 3, M - 2, M - 1])


@pytest.fixture(scope="module")
def am():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2305_08872_amd as am
    am.load_library()
    return am


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def sampled_rows(dR):
    return dR[torch.from_numpy(ROWS).cuda()].cpu().numpy()


def test_offsets_really_exceed_32_bits():
    assert M * N > 2 ** 31 and (ROWS[-1] * N + N - 1) > 2 ** 31


@pytest.mark.parametrize("task", [0, 1, 2, 3])
def test_f32_tasks_beyond_2_31_outputs(am, task):
    g = np.random.Generator(np.random.PCG64(9100 + task))
    A = (g.standard_normal((M, K)) * 2).astype(np.float32)
    B = (g.standard_normal((K, N)) * 2).astype(np.float32)
    thres = (g.standard_normal(N) * 2).astype(np.float32)
    dis = g.uniform(0, 1, N).astype(np.float32)
    params = {0: None, 1: np.stack([thres, dis]), 2: thres[None, :], 3: thres[None, :]}[task]
    print("f32 task", task, M, N, K, flush=True)
    dR = torch.full((M, N), 1.5, dtype=torch.float32, device="cuda")
    am.amulet_mmlike_f32(task, dev(A), dev(B), dev(params) if params is not None else None, dR)
    torch.cuda.synchronize()
    R = sampled_rows(dR)
    del dR
    R_in = np.full((len(ROWS), N), 1.5, np.float32)
    R_ref, ab, _ = oracle.mmlike_f32(task, A[ROWS], B, params, R_in)
    if task == 3:
        assert np.array_equal(R, R_ref)
    else:
        assert_parity_f32(R, R_ref, ab, R_in, what="f32 task %d, 2^31+ outputs" % task)


@pytest.mark.parametrize("task", [0, 1])
def test_f64_tasks_beyond_2_31_outputs(am, task):
    g = np.random.Generator(np.random.PCG64(9200 + task))
    A = g.standard_normal((M, K)) * 2
    B = g.standard_normal((K, N)) * 2
    thres = g.standard_normal(N) * 2
    dis = g.uniform(0, 1, N)
    print("f64 task", task, M, N, K, flush=True)
    dR = torch.full((M, N), -2.0, dtype=torch.float64, device="cuda")
    am.amulet_mmlike_f64(task, dev(A), dev(B), dev(thres) if task else None, dev(dis) if task == 1 else None, dR)
    torch.cuda.synchronize()
    R = sampled_rows(dR)
    del dR
    R_in = np.full((len(ROWS), N), -2.0)
    R_ref, ab, _ = oracle.mmlike_f64_general(task, A[ROWS], B, thres if task else None,
                                            dis if task == 1 else None, R_in)
    assert worst_ratio(R, R_ref, ab, R_in) <= 1e-12


def test_count_i8_beyond_2_31_outputs(am):
    g = np.random.Generator(np.random.PCG64(9300))
    Kc = 64                                   # whole 64-byte stages: the streamed kernel takes the interior
    A = g.integers(-128, 128, (M, Kc)).astype(np.int8)
    B = g.integers(-128, 128, (Kc, N)).astype(np.int8)
    print("count_i8", M, N, Kc, flush=True)
    dR = torch.full((M, N), 7, dtype=torch.int32, device="cuda")
    am.amulet_count_i8(dev(A), dev(B), dR)
    torch.cuda.synchronize()
    R = sampled_rows(dR)
    del dR
    R_ref, _ = oracle.count_i8(A[ROWS], B, np.full((len(ROWS), N), 7, np.int32))
    assert np.array_equal(R, R_ref)


def test_elementwise_threshold_and_transposed_operands_beyond_2_31(am):
    """thres[i][j] is itself an M x N array (offsets past 2^31), and A stored K x M makes the
    row index the fast one of a wide operand."""
    g = np.random.Generator(np.random.PCG64(9400))
    At = (g.standard_normal((K, M)) * 2).astype(np.float32)      # A stored transposed
    Bt = (g.standard_normal((N, K)) * 2).astype(np.float32)      # B stored transposed
    print("f32 general boost, thres[i][j], both transposed", M, N, K, flush=True)
    dT = torch.full((M, N), 0.25, dtype=torch.float32, device="cuda")
    dR = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    am.amulet_mmlike_f32_general(2, dev(At), dev(Bt), dT, None, dR, thres_form=3, trans_a=True, trans_b=True)
    torch.cuda.synchronize()
    R = sampled_rows(dR)
    del dR, dT
    R_ref, ab, _ = oracle.mmlike_f32_general(2, np.ascontiguousarray(At[:, ROWS]), Bt,
                                            np.full((len(ROWS), N), 0.25, np.float32), None,
                                            np.zeros((len(ROWS), N), np.float32),
                                            thres_form=3, trans_a=True, trans_b=True)
    assert_parity_f32(R, R_ref, ab, None, what="general boost, 2^31+ outputs")


MAX_DIM = 2 ** 31 - 2 ** 16 - 1      # the largest extent the library accepts


@pytest.mark.parametrize("task", [1, 3])
def test_largest_accepted_row_count(am, task):
    """M at the library's limit (N = 1, K = 2): 67 million row tiles in one launch.  Operands are
    written on the device from a short period pattern; sampled rows, the last one among them,
    are checked against the oracle."""
    M, N, K = MAX_DIM, 1, 2
    lib = am.load_library()
    assert lib.amulet_mmlike_f32(task, M + 1, N, K, 16, K, 16, N, 16, 16, N, None) == -7   # one more is refused
    period = torch.tensor([[-3.0, 0.5], [1.0, 2.0], [2.5, -1.0], [0.25, 4.0], [7.0, 0.0], [-0.5, -0.5], [1.5, 3.0]],
                          device="cuda")
    reps = (M + 6) // 7
    dA = period.repeat(reps, 1)[:M]
    B = np.array([[2.0], [1.5]], np.float32)
    params = np.array([[1.0], [0.25]], np.float32)[: (2 if task == 1 else 1)]
    dR = torch.full((M, N), 1.0, dtype=torch.float32, device="cuda")
    print("max M", task, M, N, K, flush=True)
    am.amulet_mmlike_f32(task, dA, dev(B), dev(params), dR)
    torch.cuda.synchronize()
    rows = np.array([0, 1, 2, 3, 4, 5, 6, 7, 2 ** 24 + 1, 2 ** 30 + 5, M - 8, M - 3, M - 2, M - 1])
    idx = torch.from_numpy(rows).cuda()
    R = dR[idx].cpu().numpy()
    A_rows = dA[idx].cpu().numpy()
    assert np.array_equal(A_rows, period.cpu().numpy()[rows % 7])      # the rows are what the pattern says
    R_ref, ab, _ = oracle.mmlike_f32(task, A_rows, B, params, np.ones((len(rows), 1), np.float32))
    assert np.array_equal(R, R_ref)                                     # two exact products per output
    assert float(dR.sum(dtype=torch.float64)) == float(M) + (M // 7) * float((R_ref[:7] - 1).sum()) + \
        float((R_ref[:M % 7] - 1).sum())


def test_largest_accepted_column_count(am):
    """N at the library's limit (M = 1, K = 3): 8.4 million column tiles, thresholds and discounts
    per column."""
    M, N, K = 1, MAX_DIM, 3
    pat = torch.tensor([1.0, -2.0, 0.5, 3.0, 0.25, -1.5, 2.0, 4.0, -0.75, 1.25, 6.0], device="cuda")
    reps = (N + 10) // 11
    dB = torch.stack([pat.repeat(reps)[:N], pat.flip(0).repeat(reps)[:N], (pat * 0.5).repeat(reps)[:N]])
    dP = torch.stack([(pat * 0.5).repeat(reps)[:N], (pat.abs() / 8).repeat(reps)[:N]]).contiguous()
    A = np.array([[2.0, -1.0, 4.0]], np.float32)
    dR = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    print("max N", M, N, K, flush=True)
    am.amulet_mmlike_f32(1, dev(A), dB, dP, dR)
    torch.cuda.synchronize()
    cols = np.array([0, 1, 5, 10, 11, 255, 256, 2 ** 24 + 3, 2 ** 30 + 7, N - 257, N - 256, N - 2, N - 1])
    idx = torch.from_numpy(cols).cuda()
    R = dR[:, idx].cpu().numpy()
    B_cols = dB[:, idx].cpu().numpy()
    P_cols = dP[:, idx].cpu().numpy()
    R_ref, ab, _ = oracle.mmlike_f32(1, A, B_cols, P_cols, np.zeros((1, len(cols)), np.float32))
    assert_parity_f32(R, R_ref, ab, None, what="max N")


def test_largest_accepted_row_count_other_kernels(am):
    """The same extent through the other kernel families: identity on the matrix cores, the
    fp64 vector-ALU kernel and the int8 join count (each with its own workgroup size, so its own
    number of launches)."""
    M = MAX_DIM
    rows = np.array([0, 1, 2, 3, 4, 5, 6, 7, 2 ** 24 + 1, 2 ** 30 + 5, M - 130, M - 8, M - 3, M - 2, M - 1])
    idx = torch.from_numpy(rows).cuda()
    period = torch.tensor([[-3.0, 0.5], [1.0, 2.0], [2.5, -1.0], [0.25, 4.0], [7.0, 0.0], [-0.5, -0.5], [1.5, 3.0]],
                          device="cuda")
    reps = (M + 6) // 7
    # fp32 identity (matrix cores)
    dA = period.repeat(reps, 1)[:M]
    B = np.array([[2.0], [1.5]], np.float32)
    dR = torch.full((M, 1), 1.0, dtype=torch.float32, device="cuda")
    print("max M identity f32", flush=True)
    am.amulet_mmlike_f32(0, dA, dev(B), None, dR)
    torch.cuda.synchronize()
    R_ref, _, _ = oracle.mmlike_f32(0, dA[idx].cpu().numpy(), B, None, np.ones((len(rows), 1), np.float32))
    assert np.array_equal(dR[idx].cpu().numpy(), R_ref)
    del dR, dA
    # fp64 discount
    dA64 = period.double().repeat(reps, 1)[:M]
    dR64 = torch.full((M, 1), 1.0, dtype=torch.float64, device="cuda")
    print("max M discount f64", flush=True)
    am.amulet_mmlike_f64(1, dA64, dev(B.astype(np.float64)), dev(np.array([1.0])), dev(np.array([0.25])), dR64)
    torch.cuda.synchronize()
    R_ref, _, _ = oracle.mmlike_f64_general(1, dA64[idx].cpu().numpy(), B.astype(np.float64), np.array([1.0]),
                                            np.array([0.25]), np.ones((len(rows), 1)))
    assert np.array_equal(dR64[idx].cpu().numpy(), R_ref)
    del dR64, dA64
    # int8 join count
    pat8 = torch.tensor([[3, -1], [0, 7], [-128, 127], [5, 5], [1, 0], [-7, 2], [100, -100]], dtype=torch.int8,
                        device="cuda")
    dA8 = pat8.repeat(reps, 1)[:M]
    B8 = np.array([[2], [-3]], np.int8)
    dR8 = torch.full((M, 1), 7, dtype=torch.int32, device="cuda")
    print("max M count_i8", flush=True)
    am.amulet_count_i8(dA8, dev(B8), dR8)
    torch.cuda.synchronize()
    R_ref, _ = oracle.count_i8(dA8[idx].cpu().numpy(), B8, np.full((len(rows), 1), 7, np.int32))
    assert np.array_equal(dR8[idx].cpu().numpy(), R_ref)


def test_largest_accepted_inner_dimension(am):
    """K at the library's limit (M = N = 1): one tile whose K loop is split over a thousand
    workgroups.  COUNT_GT with one product in a thousand above the threshold, so the count
    (about 2.1 million) is exact in fp32 and has a closed form."""
    K = MAX_DIM
    pat = torch.full((1000,), 0.5, device="cuda")
    pat[137] = 2.0
    dA = pat.repeat((K + 999) // 1000)[:K].view(1, K)
    dB = torch.ones((K, 1), device="cuda")
    dR = torch.zeros((1, 1), device="cuda")
    print("max K", K, flush=True)
    am.amulet_mmlike_f32(3, dA, dB, dev(np.array([[1.0]], np.float32)), dR)
    torch.cuda.synchronize()
    expected = K // 1000 + (1 if K % 1000 > 137 else 0)       # the k with k % 1000 == 137
    assert expected < 2 ** 24
    assert float(dR[0, 0]) == float(expected)
    # the oracle on the first and the last 5000 k agrees with the closed form used above
    for k0 in (0, K - 5000):
        A_part = dA[:, k0:k0 + 5000].cpu().numpy()
        R_ref, _, _ = oracle.mmlike_f32(3, A_part, np.ones((5000, 1), np.float32), np.array([[1.0]], np.float32))
        assert R_ref[0, 0] == sum(1 for k in range(k0, k0 + 5000) if k % 1000 == 137)
