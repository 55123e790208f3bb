"""GPU tests of packing (Sec. 3.1): the strided copy is exact, and a call that packs gives
the plain call's result (the same kernels on the same values) and the oracle's."""
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


@pytest.mark.parametrize("dtype", [torch.int8, torch.float32, torch.float64])
def test_pack_copies_every_element_and_nothing_else(am, dtype):
    g = torch.Generator(device="cuda").manual_seed(5)
    for rows, cols, ld_src, ld_dst, off in [(37, 1000, 1024, 1056, 0), (5, 3, 3, 4, 0), (300, 257, 300, 263, 1),
                                             (70000, 16, 16, 48, 0), (3, 70001, 70016, 70048, 0), (1, 1, 1, 1, 0)]:
        print("pack", dtype, rows, cols, ld_src, ld_dst, off, flush=True)
        src_store = torch.randint(-100, 100, (rows * ld_src + off,), device="cuda", generator=g).to(dtype)
        src = src_store[off:].view(rows, ld_src)[:, :cols]
        dst_store = torch.full((rows * ld_dst + off,), 77, device="cuda").to(dtype)
        dst = dst_store[off:].view(rows, ld_dst)[:, :cols]
        am.amulet_pack(src, dst)
        torch.cuda.synchronize()
        assert torch.equal(dst, src)
        if ld_dst > cols:   # the gaps between packed rows are not written
            assert torch.all(dst_store[off:].view(rows, ld_dst)[:, cols:] == 77)


def colliding_view(rows, cols, dtype):
    """rows x cols view whose row pitch (64 KiB) collides."""
    ld = 65536 // torch.empty((), dtype=dtype).element_size()
    store = torch.zeros((rows, ld), dtype=dtype, device="cuda")
    return store[:, :cols]


@pytest.mark.parametrize("task", [0, 1, 2, 3])
def test_f32_autopack_equals_plain_call_and_oracle(am, task):
    M, N, K = 150, 300, 101   # K below the split-K limit: one workgroup per tile, fixed sum order
    g = np.random.Generator(np.random.PCG64(4200 + task))
    A = (g.standard_normal((M, K)) * 2).astype(np.float32)
    B = (g.standard_normal((K, N)) * 2).astype(np.float32)
    thres = (g.standard_normal(N) * 2).astype(np.float32)
    dis = g.uniform(0, 1, N).astype(np.float32)
    R_in = g.standard_normal((M, N)).astype(np.float32)
    dA = colliding_view(M, K, torch.float32)
    dA.copy_(dev(A))
    assert am.amulet_pitch_collides(dA.stride(0), 4)
    dT, dD = (dev(thres) if task else None), (dev(dis) if task == 1 else None)
    need = am.amulet_autopack_workspace_bytes(4, M, K)
    assert need == M * am.amulet_packed_ld(K, 4) * 4
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    R_plain, R_pack, R_nows = dev(R_in), dev(R_in), dev(R_in)
    am.amulet_mmlike_f32_general(task, dA, dev(B), dT, dD, R_plain)
    am.amulet_mmlike_f32_autopack(task, dA, dev(B), dT, dD, R_pack, ws)
    am.amulet_mmlike_f32_autopack(task, dA, dev(B), dT, dD, R_nows, None)
    torch.cuda.synchronize()
    assert torch.equal(R_pack, R_plain) and torch.equal(R_nows, R_plain)
    R_ref, ab, _ = oracle.mmlike_f32_general(task, A, B, thres if task else None, dis if task == 1 else None, R_in)
    if task == 3:
        assert np.array_equal(R_pack.cpu().numpy(), R_ref)
    else:
        assert_parity_f32(R_pack.cpu().numpy(), R_ref, ab, R_in, what="autopack task %d" % task)
    if task:   # the vector-ALU tasks pack: a workspace one byte short is refused
        with pytest.raises(am.AmuletError) as err:
            am.amulet_mmlike_f32_autopack(task, dA, dev(B), dT, dD, R_pack, ws[:need - 1])
        assert err.value.code == -8
        packed = ws.view(torch.float32).view(M, am.amulet_packed_ld(K, 4))[:, :K]
        assert torch.equal(packed, dA)   # the workspace holds the packed A


def test_f32_autopack_leaves_other_layouts_alone(am):
    """A transposed A, or a pitch that does not collide, is read in place: the workspace stays
    untouched and may be too small."""
    M, N, K = 64, 256, 100
    g = np.random.Generator(np.random.PCG64(4300))
    A = (g.standard_normal((M, K)) * 2).astype(np.float32)
    B = (g.standard_normal((K, N)) * 2).astype(np.float32)
    thres = (g.standard_normal(N) * 2).astype(np.float32)
    ws = torch.full((16,), 9, dtype=torch.uint8, device="cuda")
    R_ref, ab, _ = oracle.mmlike_f32_general(2, A, B, thres, None, None)
    R1 = torch.zeros((M, N), device="cuda")
    am.amulet_mmlike_f32_autopack(2, dev(A), dev(B), dev(thres), None, R1, ws)            # pitch 400 bytes
    At = colliding_view(K, M, torch.float32)
    At.copy_(dev(A.T.copy()))
    R2 = torch.zeros((M, N), device="cuda")
    am.amulet_mmlike_f32_autopack(2, At, dev(B), dev(thres), None, R2, ws, trans_a=True)  # transposed A
    torch.cuda.synchronize()
    assert torch.all(ws == 9)
    assert_parity_f32(R1.cpu().numpy(), R_ref, ab, None, what="autopack, no collision")
    assert_parity_f32(R2.cpu().numpy(), R_ref, ab, None, what="autopack, transposed A")


@pytest.mark.parametrize("task", [0, 1, 3])
def test_f64_autopack_equals_plain_call_and_oracle(am, task):
    M, N, K = 70, 260, 101    # K below the split-K limit: fixed sum order
    g = np.random.Generator(np.random.PCG64(4400 + task))
    A = g.standard_normal((M, K)) * 2
    B = g.standard_normal((K, N)) * 2
    thres = g.standard_normal(N) * 2
    dis = g.uniform(0, 1, N)
    R_in = g.standard_normal((M, N))
    dA = colliding_view(M, K, torch.float64)
    dA.copy_(dev(A))
    dT, dD = (dev(thres) if task else None), (dev(dis) if task == 1 else None)
    ws = torch.empty(am.amulet_autopack_workspace_bytes(8, M, K), dtype=torch.uint8, device="cuda")
    R_plain, R_pack = dev(R_in), dev(R_in)
    am.amulet_mmlike_f64(task, dA, dev(B), dT, dD, R_plain)
    am.amulet_mmlike_f64_autopack(task, dA, dev(B), dT, dD, R_pack, ws)
    torch.cuda.synchronize()
    assert torch.equal(R_pack, R_plain)
    R_ref, ab, _ = oracle.mmlike_f64_general(task, A, B, thres if task else None, dis if task == 1 else None, R_in)
    if task == 3:
        assert np.array_equal(R_pack.cpu().numpy(), R_ref)
    else:
        assert worst_ratio(R_pack.cpu().numpy(), R_ref, ab, R_in) <= 1e-12
    if task:
        with pytest.raises(am.AmuletError) as err:
            am.amulet_mmlike_f64_autopack(task, dA, dev(B), dT, dD, R_pack, ws[:16])
        assert err.value.code == -8
