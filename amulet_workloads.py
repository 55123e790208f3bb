"""Seeded synthetic inputs for the matrix-multiplication-like tasks.

This module only draws numbers: it holds none of the method's arithmetic, and
it is the one module both the CPU oracle's tests and the GPU path's tests and
bench read their inputs from.  Every array comes from numpy's PCG64 generator
seeded with the stated seed, so a (name, seed, shape) triple always names the
same data.

The paper does not publish its input data or value distributions (Sec. 6 only
gives matrix orders), so the recipes below stand in for its two scenarios: the
retail one (A = units bought, B = list prices, per-seller threshold and
discount; Sec. 1, Fig. 1) and the signal one (A = observation weights, B =
feature strengths, per-location threshold; Sec. 1, Fig. 2), plus a plain
matmul and a 0/1 join-indicator pair for the join-as-matmul case.
"""
from __future__ import annotations

import numpy as np

IDENTITY, DISCOUNT, BOOST, COUNT_GT = 0, 1, 2, 3
TASK_NAMES = {IDENTITY: "identity", DISCOUNT: "discount", BOOST: "boost", COUNT_GT: "count_gt"}


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def retail(M: int, N: int, K: int, seed: int):
    """Discount-task inputs: A integer unit counts 0..9 (as fp32), B prices in
    [1, 100), thres[j] in [100, 500), dis[j] in [0.05, 0.3]."""
    g = _rng(seed)
    A = g.integers(0, 10, size=(M, K)).astype(np.float32)
    B = g.uniform(1.0, 100.0, size=(K, N)).astype(np.float32)
    thres = g.uniform(100.0, 500.0, size=N).astype(np.float32)
    dis = g.uniform(0.05, 0.3, size=N).astype(np.float32)
    return A, B, np.stack([thres, dis])


def signal(M: int, N: int, K: int, seed: int):
    """Boost-task inputs: A, B i.i.d. standard normal, thres[j] = |N(0,1)| + 1."""
    g = _rng(seed)
    A = g.standard_normal(size=(M, K), dtype=np.float32)
    B = g.standard_normal(size=(K, N), dtype=np.float32)
    thres = (np.abs(g.standard_normal(size=N, dtype=np.float32)) + np.float32(1.0)).astype(np.float32)
    return A, B, thres[None, :]


def uniform_pm1(M: int, N: int, K: int, seed: int):
    """Plain-matmul inputs: A, B uniform in [-1, 1)."""
    g = _rng(seed)
    A = (g.random(size=(M, K), dtype=np.float32) * np.float32(2.0) - np.float32(1.0)).astype(np.float32)
    B = (g.random(size=(K, N), dtype=np.float32) * np.float32(2.0) - np.float32(1.0)).astype(np.float32)
    return A, B, None


def join_indicator(M: int, N: int, K: int, seed: int, density: float = 0.05):
    """Join-count inputs: 0/1 int8 indicator matrices, entries Bernoulli(density)."""
    g = _rng(seed)
    A = (g.random(size=(M, K), dtype=np.float32) < density).astype(np.int8)
    B = (g.random(size=(K, N), dtype=np.float32) < density).astype(np.int8)
    return A, B


def price_counts(M: int, N: int, K: int, seed: int):
    """Count-over-threshold inputs (Query 3's retail reading): the retail A, B
    with a per-seller threshold around the paper's constant 100."""
    g = _rng(seed)
    A = g.integers(0, 10, size=(M, K)).astype(np.float32)
    B = g.uniform(1.0, 100.0, size=(K, N)).astype(np.float32)
    thres = g.uniform(50.0, 150.0, size=N).astype(np.float32)
    return A, B, thres[None, :]


def small_exact(M: int, N: int, K: int, seed: int, n_param: int):
    """Small-integer / dyadic data on which every product, comparison operand
    and term is exact in fp32 and in double: A, B integers in [-8, 8], thres
    multiples of 1/2 in [-12, 12] (so ties p == thres occur), dis multiples of
    1/8 in [0, 1]."""
    g = _rng(seed)
    A = g.integers(-8, 9, size=(M, K)).astype(np.float32)
    B = g.integers(-8, 9, size=(K, N)).astype(np.float32)
    rows = []
    if n_param >= 1:
        rows.append((g.integers(-24, 25, size=N) / 2.0).astype(np.float32))
    if n_param >= 2:
        rows.append((g.integers(0, 9, size=N) / 8.0).astype(np.float32))
    params = np.stack(rows) if rows else None
    return A, B, params


# The named workloads the build is measured and parity-checked on.
CONFIGS = {
    "cfg0_discount_256": dict(task=DISCOUNT, M=256, N=256, K=256, seed=0, gen="retail"),
    "cfg1_boost_2048": dict(task=BOOST, M=2048, N=2048, K=2048, seed=1, gen="signal"),
    "cfg2_identity_4096": dict(task=IDENTITY, M=4096, N=4096, K=4096, seed=2, gen="uniform_pm1"),
    "cfg3_count_i8_8192x8192x4096": dict(task="count_i8", M=8192, N=8192, K=4096, seed=3,
                                         gen="join_indicator"),
    "cfg4_discount_16384x2048x8192": dict(task=DISCOUNT, M=16384, N=2048, K=8192, seed=4,
                                          gen="retail"),
    "headline_discount_8192": dict(task=DISCOUNT, M=8192, N=8192, K=8192, seed=4, gen="retail"),
    # Query 3 (count of products over a threshold) on the retail data, the paper's square size
    "query3_count_gt_4096": dict(task=COUNT_GT, M=4096, N=4096, K=4096, seed=8, gen="price_counts"),
    # the paper's own element type (its listings are double): same recipes, widened to fp64
    "f64_discount_4096": dict(task=DISCOUNT, M=4096, N=4096, K=4096, seed=5, gen="retail", dtype="f64"),
    "f64_boost_2048": dict(task=BOOST, M=2048, N=2048, K=2048, seed=6, gen="signal", dtype="f64"),
    "f64_identity_4096": dict(task=IDENTITY, M=4096, N=4096, K=4096, seed=7, gen="uniform_pm1", dtype="f64"),
    # a plain matmul of few tiles (64 of 128 x 128 for 256 compute units): the 64 x 64 identity tiles
    "identity_1024": dict(task=IDENTITY, M=1024, N=1024, K=1024, seed=9, gen="uniform_pm1"),
    "f64_identity_1024": dict(task=IDENTITY, M=1024, N=1024, K=1024, seed=10, gen="uniform_pm1", dtype="f64"),
}

_GENS = {"retail": retail, "signal": signal, "uniform_pm1": uniform_pm1,
         "join_indicator": join_indicator, "price_counts": price_counts}


def make(name: str):
    """Return (spec, A, B, params) for a named workload; params is None where
    the task takes none (and absent for the int8 join count)."""
    spec = dict(CONFIGS[name])
    out = _GENS[spec["gen"]](spec["M"], spec["N"], spec["K"], spec["seed"])
    if spec["gen"] == "join_indicator":
        A, B = out
        return spec, A, B, None
    A, B, params = out
    if spec.get("dtype") == "f64":
        A, B = A.astype(np.float64), B.astype(np.float64)
        params = None if params is None else params.astype(np.float64)
    return spec, A, B, params
