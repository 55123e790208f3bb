"""Every output sums every k exactly once, whatever the launch plan: with A and B all ones the
result has a closed form that holds at any size (R_in + K for the identity tasks and the join
count; R_in + K for the count task with a threshold below 1, R_in for one above), exact in every
element type.  A tile or a k range covered twice, or not at all, by one of the launchers'
plans (split K, split last round, several launches for a long grid, edge strips) shows as a
wrong integer.  Sizes are drawn at random (seeded) over the ranges where those plans change."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def am():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2305_08872_amd as am
    am.load_library()
    return am


def sizes(seed, n):
    g = np.random.Generator(np.random.PCG64(seed))
    out = []
    for _ in range(n):
        kind = g.integers(0, 4)
        if kind == 0:      # mid sizes: one to a few rounds of workgroups, K long enough to split
            M, N, K = g.integers(600, 5000), g.integers(600, 5000), g.integers(256, 3000)
        elif kind == 1:    # few tiles, long K
            M, N, K = g.integers(1, 400), g.integers(1, 700), g.integers(1000, 20000)
        elif kind == 2:    # tall or wide
            M, N, K = g.integers(1, 200), g.integers(3000, 40000), g.integers(1, 700)
            if g.integers(0, 2):
                M, N = N, M
        else:              # tiny and ragged
            M, N, K = g.integers(1, 300), g.integers(1, 300), g.integers(1, 300)
        out.append((int(M), int(N), int(K)))
    return out


def check_constant(R, expected, what):
    bad = (R != expected).nonzero()
    assert bad.numel() == 0, "%s: %d outputs differ from %r, first at %r with %r" % (
        what, bad.shape[0], expected, bad[0].tolist(), R[tuple(bad[0].tolist())].item())


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_every_k_of_every_output_once_fp32(am, seed):
    for (M, N, K) in sizes(seed, 40):
        A = torch.ones((M, K), device="cuda")
        B = torch.ones((K, N), device="cuda")
        low = torch.full((1, N), 0.5, device="cuda")
        high = torch.full((1, N), 1.5, device="cuda")
        print("cover f32", M, N, K, flush=True)
        for task, P, expected in ((3, low, 3.0 + K), (3, high, 3.0), (0, None, 3.0 + K),
                                  (1, torch.cat([low, torch.full((1, N), 0.5, device="cuda")]), 3.0 + 0.5 * K)):
            R = torch.full((M, N), 3.0, device="cuda")
            am.amulet_mmlike_f32(task, A, B, P, R)
            torch.cuda.synchronize()
            check_constant(R, expected, "f32 task %d %dx%dx%d" % (task, M, N, K))
        # transposed storage of the same ones
        R = torch.full((M, N), 3.0, device="cuda")
        am.amulet_mmlike_f32_general(3, A.t().contiguous(), B.t().contiguous(), low.view(-1), None, R,
                                     trans_a=True, trans_b=True)
        torch.cuda.synchronize()
        check_constant(R, 3.0 + K, "f32 count, both transposed %dx%dx%d" % (M, N, K))


@pytest.mark.parametrize("seed", [21, 22])
def test_every_k_of_every_output_once_fp64(am, seed):
    for (M, N, K) in sizes(seed, 30):
        A = torch.ones((M, K), dtype=torch.float64, device="cuda")
        B = torch.ones((K, N), dtype=torch.float64, device="cuda")
        low = torch.full((N,), 0.5, dtype=torch.float64, device="cuda")
        half = torch.full((N,), 0.5, dtype=torch.float64, device="cuda")
        print("cover f64", M, N, K, flush=True)
        for task, th, dis, expected in ((3, low, None, 3.0 + K), (0, None, None, 3.0 + K), (1, low, half, 3.0 + 0.5 * K),
                                        (2, low, None, 3.0 + 1.5 * K)):
            R = torch.full((M, N), 3.0, dtype=torch.float64, device="cuda")
            am.amulet_mmlike_f64(task, A, B, th, dis, R)
            torch.cuda.synchronize()
            check_constant(R, expected, "f64 task %d %dx%dx%d" % (task, M, N, K))


@pytest.mark.parametrize("seed", [31, 32])
def test_every_k_of_every_output_once_join_count(am, seed):
    for (M, N, K) in sizes(seed, 40):
        A = torch.ones((M, K), dtype=torch.int8, device="cuda")
        B = torch.ones((K, N), dtype=torch.int8, device="cuda")
        print("cover i8", M, N, K, flush=True)
        for shape in (None, 3, 4, 6, 7):
            R = torch.full((M, N), -5, dtype=torch.int32, device="cuda")
            if shape is None:
                am.amulet_count_i8(A, B, R)
            else:
                am.amulet_count_i8_shape(shape, A, B, R)
            torch.cuda.synchronize()
            check_constant(R, K - 5, "i8 shape %s %dx%dx%d" % (shape, M, N, K))
