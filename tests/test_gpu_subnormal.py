"""GPU parity on products in the subnormal range of the element type: the product is one IEEE
multiply, subnormal results included, and the predicate looks at that value (a kernel that
flushed subnormals to zero would decide `p > 0` differently and drop the terms from the sum)."""
import numpy as np
import pytest

import oracle
from parity import assert_parity_f32, worst_ratio

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def am():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2305_08872_amd as am
    am.load_library()
    return am


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def subnormal_case(dtype, M, N, K, seed):
    """Operands whose products straddle the smallest normal number of `dtype`: some products are
    normal, most subnormal, some round to zero; thresholds at 0, at subnormal values and at
    the smallest normal number."""
    g = np.random.Generator(np.random.PCG64(seed))
    tiny = np.finfo(dtype).tiny                                  # smallest normal
    A = (g.uniform(0.5, 2.0, (M, K)) * g.choice([-1.0, 1.0], (M, K)) * np.sqrt(tiny)).astype(dtype)
    B = (g.uniform(0.5, 2.0, (K, N)) * np.sqrt(tiny) * g.choice([1.0, 1e-3, 1e-6, 1e-9], (K, N))).astype(dtype)
    thres = (g.choice([0.0, -0.0, 1e-3, 1e-6, 0.25, 1.0, -1e-4], N) * tiny).astype(dtype)
    dis = g.uniform(0, 1, N).astype(dtype)
    return A, B, thres, dis


@pytest.mark.parametrize("task", [0, 1, 2, 3])
def test_f32_subnormal_products(am, task):
    for idx, (M, N, K) in enumerate([(70, 300, 37), (64, 512, 128)]):
        A, B, thres, dis = subnormal_case(np.float32, M, N, K, 9500 + 10 * task + idx)
        p = A[:, :, None].astype(np.float32) * B[None, :, :]        # the products themselves (data check only)
        sub = (p != 0) & (np.abs(p) < np.finfo(np.float32).tiny)
        assert sub.mean() > 0.3, "the case must really be subnormal"
        params = {0: None, 1: np.stack([thres, dis]), 2: thres[None, :], 3: thres[None, :]}[task]
        R_ref, ab, _ = oracle.mmlike_f32(task, A, B, params, None)
        for shape in ([None, 8, 4] if task == 0 else [None]):       # identity: matrix cores and vector ALU
            dR = torch.zeros((M, N), device="cuda")
            print("subnormal f32", task, shape, M, N, K, flush=True)
            if shape is None:
                am.amulet_mmlike_f32(task, dev(A), dev(B), dev(params) if params is not None else None, dR)
            else:
                am.amulet_mmlike_f32_shape(task, shape, dev(A), dev(B), None, dR)
            torch.cuda.synchronize()
            R = dR.cpu().numpy()
            if task == 3:
                assert np.array_equal(R, R_ref), "predicate on subnormal products differs"
            else:
                assert_parity_f32(R, R_ref, ab, None, what="subnormal f32 task %d shape %s" % (task, shape))


@pytest.mark.parametrize("task", [0, 1, 3])
def test_f64_subnormal_products(am, task):
    M, N, K = 70, 300, 37
    A, B, thres, dis = subnormal_case(np.float64, M, N, K, 9600 + task)
    R_ref, ab, _ = oracle.mmlike_f64_general(task, A, B, thres if task else None, dis if task == 1 else None, None)
    dR = torch.zeros((M, N), dtype=torch.float64, device="cuda")
    print("subnormal f64", task, M, N, K, flush=True)
    am.amulet_mmlike_f64(task, dev(A), dev(B), dev(thres) if task else None, dev(dis) if task == 1 else None, dR)
    torch.cuda.synchronize()
    R = dR.cpu().numpy()
    if task == 3:
        assert np.array_equal(R, R_ref), "predicate on subnormal products differs"
    else:
        assert worst_ratio(R, R_ref, ab, None) <= 1e-12
