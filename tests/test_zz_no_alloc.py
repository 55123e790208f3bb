"""The entry point that allocates nothing (amulet_count_i8_static): its result against the
existing entry point with a lent workspace (amulet_count_i8_general) and against the oracle, bit
for bit, on two calls in a row that share the library's static scratch array, the second
smaller than the first."""
import ctypes

import numpy as np
import pytest

import amulet_workloads as wl
import oracle

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


def one_case(am, M, N, K, tA, tB, seed):
    A, B = wl.join_indicator(M, N, K, seed=seed, density=0.2)
    g = np.random.Generator(np.random.PCG64(seed))
    R_in = g.integers(-5, 6, size=(M, N)).astype(np.int32)
    R_ref, _ = oracle.count_i8(A, B, R_in)
    dA = dev(A.T) if tA else dev(A)
    dB = dev(B.T) if tB else dev(B)
    # the existing entry point, with a workspace torch allocated
    ws = torch.full((am.amulet_count_i8_repack_workspace_bytes(M, N, K),), 55, dtype=torch.int8, device="cuda")
    R_general = dev(R_in)
    am.amulet_count_i8_general(dA, dB, R_general, ws, trans_a=tA, trans_b=tB)
    # the entry point under test
    R_static = dev(R_in)
    print("static join count", M, N, K, tA, tB, flush=True)
    am.amulet_count_i8_static(dA, dB, R_static, trans_a=tA, trans_b=tB)
    torch.cuda.synchronize()
    assert torch.equal(R_static, R_general)
    assert np.array_equal(R_static.cpu().numpy(), R_ref)


def test_two_calls_in_a_row_share_the_static_scratch(am):
    # first call: transposed A, nothing aligned, K not whole stages: both operands are copied
    one_case(am, 1000, 1300, 1111, True, False, seed=61)
    # second call, smaller, other layout: the array still holds the first call's copies
    one_case(am, 300, 272, 130, False, True, seed=62)
    # a third one that needs no copy at all (aligned, whole tiles, whole stages)
    one_case(am, 512, 512, 256, False, False, seed=63)


def test_sizes_beyond_the_static_scratch_are_refused(am):
    lib = am.load_library()
    one = ctypes.c_void_p(256)   # never read: the size check comes first
    assert lib.amulet_count_i8_static(0, 0, 8191, 8191, 4095, one, 4095, one, 8191, one, 8191, None) == -8
    assert am.amulet_strerror(-8).startswith("workspace")
    assert lib.amulet_count_i8_static(0, 0, 0, 5, 5, None, 5, None, 5, None, 5, None) == 0
