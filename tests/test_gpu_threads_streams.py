"""Host threads and streams: compute calls from several host threads at once, each on its own
stream, and calls given an explicit stream that is not the current one."""
import threading

import numpy as np
import pytest

import oracle
from parity import assert_parity_f32

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


def case(task, M, N, K, seed):
    g = np.random.Generator(np.random.PCG64(seed))
    A = (g.standard_normal((M, K)) * 2).astype(np.float32)
    B = (g.standard_normal((K, N)) * 2).astype(np.float32)
    thres = (g.standard_normal(N) * 3).astype(np.float32)
    dis = g.uniform(0, 1, N).astype(np.float32)
    params = {0: None, 1: np.stack([thres, dis]), 2: thres[None, :], 3: thres[None, :]}[task]
    return A, B, params


def test_calls_from_several_host_threads_on_their_own_streams(am):
    """Eight threads, each with its own stream, task and size, ten calls each (R accumulates, so
    the expected result is ten times one call's terms); one of them also tunes, which takes the
    selector's lock and allocates, while the others launch."""
    specs = [(t % 4, 100 + 37 * t, 300 + 64 * t, 90 + 11 * t) for t in range(8)]   # K below 128: fixed sum order
    inputs = [case(task, M, N, K, 3100 + i) for i, (task, M, N, K) in enumerate(specs)]
    refs = [oracle.mmlike_f32(spec[0], A, B, P, None) for spec, (A, B, P) in zip(specs, inputs)]
    results, errors = [None] * len(specs), []

    def worker(i):
        try:
            task, M, N, K = specs[i]
            A, B, P = inputs[i]
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                dA, dB = dev(A), dev(B)
                dP = dev(P) if P is not None else None
                dR = torch.zeros((M, N), device="cuda")
                if i == 3:
                    am.amulet_tune(task, M, N, K, stream=stream)
                for _ in range(10):
                    am.amulet_mmlike_f32(task, dA, dB, dP, dR, stream=stream)
                stream.synchronize()
                results[i] = dR.cpu().numpy()
        except Exception as e:   # reported by the main thread
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(len(specs))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for i, (spec, (R_ref, ab, _)) in enumerate(zip(specs, refs)):
        if spec[0] == 3:
            assert np.array_equal(results[i], 10 * R_ref), spec
        else:
            assert_parity_f32(results[i], 10 * R_ref.astype(np.float64), 10 * ab, None, what="thread %d %r" % (i, spec))


def test_explicit_stream_that_is_not_the_current_one(am):
    """The work goes to the stream that is passed, not to torch's current stream: a long
    kernel is queued on the side stream first, the call follows it there, and the default
    stream sees the result only after waiting for the side stream."""
    task, M, N, K = 1, 512, 1024, 100
    A, B, P = case(task, M, N, K, 3200)
    R_ref, ab, _ = oracle.mmlike_f32(task, A, B, P, None)
    dA, dB, dP = dev(A), dev(B), dev(P)
    dR = torch.zeros((M, N), device="cuda")
    big = torch.rand(4096, 4096, device="cuda")
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for _ in range(20):
            big = big @ big * 1e-4                      # keeps the side stream busy for a while
    am.amulet_mmlike_f32(task, dA, dB, dP, dR, stream=side)   # current stream here is the default one
    done = torch.cuda.Event()
    done.record(side)
    torch.cuda.current_stream().wait_event(done)
    out = dR.clone()
    torch.cuda.synchronize()
    assert_parity_f32(out.cpu().numpy(), R_ref, ab, None, what="explicit stream")
