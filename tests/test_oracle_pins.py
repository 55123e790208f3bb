"""Pins for the CPU oracle: it is checked against things other than itself.

 - a 3x3 example worked by hand from the paper's printed task definitions;
 - an exact rational evaluation of the printed C text, bool-times-value and
   all, on tiny exact data (must match bit for bit);
 - the invariants the formulas imply (special cases reducing to numpy's
   matmul, closed forms, linearity in R_in);
 - the reading "product rounded once to fp32, compared strictly".
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

import amulet_workloads as wl
import oracle

TASKS_F32 = [oracle.IDENTITY, oracle.DISCOUNT, oracle.BOOST, oracle.COUNT_GT]
NPAR = {oracle.IDENTITY: 0, oracle.DISCOUNT: 2, oracle.BOOST: 1, oracle.COUNT_GT: 1}


# --------------------------------------------------------------------------
# 1. hand-worked example (tests/golden/worked_3x3.json)
# --------------------------------------------------------------------------
@pytest.fixture(scope="module")
def worked(golden_dir):
    with open(os.path.join(golden_dir, "worked_3x3.json")) as f:
        return json.load(f)


def test_worked_example_all_tasks(worked):
    A = np.array(worked["A"], np.float32)
    B = np.array(worked["B"], np.float32)
    th = np.array(worked["thres"], np.float32)
    dis = np.array(worked["dis"], np.float32)
    R, ab, _ = oracle.mmlike_f32(oracle.IDENTITY, A, B, None)
    assert R.tolist() == worked["identity"]
    R, ab, _ = oracle.mmlike_f32(oracle.DISCOUNT, A, B, np.stack([th, dis]))
    assert R.tolist() == worked["discount"]
    assert ab.tolist() == worked["discount"]  # every term is >= 0 here
    R, ab, _ = oracle.mmlike_f32(oracle.BOOST, A, B, th[None])
    assert R.tolist() == worked["boost"]
    c = np.full((1, 3), worked["count_gt_const"], np.float32)
    R, ab, _ = oracle.mmlike_f32(oracle.COUNT_GT, A, B, c)
    assert R.tolist() == worked["count_gt"]
    Rj, _ = oracle.count_i8(np.array(worked["join_A"], np.int8), np.array(worked["join_B"], np.int8))
    assert Rj.tolist() == worked["join_count"]


def test_worked_example_accumulates_into_R(worked):
    A = np.array(worked["A"], np.float32)
    B = np.array(worked["B"], np.float32)
    P = np.array([worked["thres"], worked["dis"]], np.float32)
    R0 = np.arange(9, dtype=np.float32).reshape(3, 3) * 1000
    R, _, _ = oracle.mmlike_f32(oracle.DISCOUNT, A, B, P, R0)
    assert R.tolist() == (np.array(worked["discount"]) + R0).tolist()


# --------------------------------------------------------------------------
# 2. exact rational evaluation of the printed loop text
# --------------------------------------------------------------------------
def _literal_fraction(task, A, B, params, R_in):
    """The C text of Fig. 1 / Fig. 2 / Query 3 evaluated in exact rationals:
    the comparison yields 0 or 1 and MULTIPLIES the remaining factors, left to
    right, with A[i][k]*B[k][j] re-evaluated at each occurrence."""
    M, K = A.shape
    N = B.shape[1]
    fa = [[Fraction(float(x)) for x in row] for row in A]
    fb = [[Fraction(float(x)) for x in row] for row in B]
    fp = [[Fraction(float(x)) for x in row] for row in params] if params is not None else None
    R = [[Fraction(float(R_in[i][j])) for j in range(N)] for i in range(M)]
    S = [[Fraction(0) for _ in range(N)] for _ in range(M)]
    for i in range(M):
        for j in range(N):
            for k in range(K):
                if task == oracle.IDENTITY:
                    t = fa[i][k] * fb[k][j]
                elif task == oracle.DISCOUNT:
                    t = fa[i][k] * fb[k][j] - int(fa[i][k] * fb[k][j] > fp[0][j]) * fa[i][k] * fb[k][j] * fp[1][j]
                elif task == oracle.BOOST:
                    t = fa[i][k] * fb[k][j] + int(fa[i][k] * fb[k][j] > fp[0][j]) * (fa[i][k] * fb[k][j] - fp[0][j])
                else:
                    t = Fraction(int(fa[i][k] * fb[k][j] > fp[0][j]))
                R[i][j] += t
                S[i][j] += abs(t)
    return R, S


@pytest.mark.parametrize("task", TASKS_F32)
@pytest.mark.parametrize("shape", [(1, 1, 1), (2, 3, 4), (5, 7, 3), (8, 8, 8), (3, 1, 6), (1, 6, 5)])
def test_matches_exact_rational_literal(task, shape):
    M, N, K = shape
    A, B, params = wl.small_exact(M, N, K, seed=100 + task * 7 + M * N * K, n_param=NPAR[task])
    R_in = (np.arange(M * N, dtype=np.float32).reshape(M, N) - 3.0) * 0.5
    R, ab, _ = oracle.mmlike_f32(task, A, B, params, R_in)
    Rf, Sf = _literal_fraction(task, A, B, params, R_in)
    for i in range(M):
        for j in range(N):
            # every value is a small dyadic rational: exact in fp32 and fp64
            assert Fraction(float(R[i, j])) == Rf[i][j], (i, j)
            assert Fraction(float(ab[i, j])) == Sf[i][j], (i, j)


def test_small_exact_data_has_ties_and_both_branches():
    # the exact-data pin is only worth something if both predicate outcomes and ties occur
    A, B, params = wl.small_exact(8, 8, 8, seed=100 + 1 * 7 + 512, n_param=2)
    P = A[:, :, None] * B[None, :, :]
    th = params[0][None, None, :]
    assert (P > th).any() and (P < th).any() and (P == th).any()


# --------------------------------------------------------------------------
# 3. reductions to numpy's matmul, closed forms, invariants
# --------------------------------------------------------------------------
def _rand(M, N, K, seed):
    g = np.random.Generator(np.random.PCG64(seed))
    A = g.standard_normal((M, K)).astype(np.float32) * 3
    B = g.standard_normal((K, N)).astype(np.float32) * 3
    return g, A, B


def _matmul_of_rounded_products(A, B):
    """sum_k fl32(a*b) in double, by a broadcast tensor (an independent route)."""
    P = (A[:, :, None] * B[None, :, :]).astype(np.float32)  # fp32 multiply, M x K x N
    return P.astype(np.float64).sum(axis=1), P


def test_identity_is_numpy_matmul_on_integer_data():
    g = np.random.Generator(np.random.PCG64(5))
    A = g.integers(-20, 21, (13, 17)).astype(np.float32)
    B = g.integers(-20, 21, (17, 11)).astype(np.float32)
    R, ab, _ = oracle.mmlike_f32(oracle.IDENTITY, A, B, None)
    assert np.array_equal(R, (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float32))
    assert np.array_equal(ab, np.abs(A.astype(np.int64))[:, :, None].__mul__(np.abs(B.astype(np.int64))[None]).sum(1))


def test_identity_close_to_double_gemm():
    _, A, B = _rand(37, 29, 53, 6)
    R, ab, _ = oracle.mmlike_f32(oracle.IDENTITY, A, B, None)
    ref = A.astype(np.float64) @ B.astype(np.float64)
    # each product is rounded to fp32 once (2^-24 relative), the result once more
    assert np.all(np.abs(R - ref) <= 2.0 ** -23 * ab + 1e-30)


@pytest.mark.parametrize("task", [oracle.DISCOUNT, oracle.BOOST])
def test_thres_plus_inf_is_plain_matmul(task):
    g, A, B = _rand(9, 12, 31, 7)
    rows = [np.full(12, np.inf, np.float32)]
    if task == oracle.DISCOUNT:
        rows.append(g.uniform(0, 1, 12).astype(np.float32))
    R, ab, _ = oracle.mmlike_f32(task, A, B, np.stack(rows))
    Ri, abi, _ = oracle.mmlike_f32(oracle.IDENTITY, A, B, None)
    assert np.array_equal(R, Ri) and np.array_equal(ab, abi)


def test_count_gt_thres_plus_inf_is_zero_and_minus_inf_is_K():
    _, A, B = _rand(4, 5, 19, 8)
    R, _, _ = oracle.mmlike_f32(oracle.COUNT_GT, A, B, np.full((1, 5), np.inf, np.float32))
    assert not R.any()
    R, _, _ = oracle.mmlike_f32(oracle.COUNT_GT, A, B, np.full((1, 5), -np.inf, np.float32))
    assert np.all(R == 19)


def test_discount_dis_one_thres_minus_inf_leaves_R_unchanged():
    g, A, B = _rand(6, 7, 41, 9)
    R_in = g.standard_normal((6, 7)).astype(np.float32)
    P = np.stack([np.full(7, -np.inf, np.float32), np.ones(7, np.float32)])
    R, ab, _ = oracle.mmlike_f32(oracle.DISCOUNT, A, B, P, R_in)
    assert np.array_equal(R, R_in)
    assert not ab.any()


def test_discount_dis_zero_is_plain_matmul():
    g, A, B = _rand(6, 7, 41, 10)
    P = np.stack([g.standard_normal(7).astype(np.float32), np.zeros(7, np.float32)])
    R, _, _ = oracle.mmlike_f32(oracle.DISCOUNT, A, B, P)
    Ri, _, _ = oracle.mmlike_f32(oracle.IDENTITY, A, B, None)
    assert np.array_equal(R, Ri)


def test_discount_thres_minus_inf_scales_matmul_by_one_minus_dis():
    g, A, B = _rand(6, 7, 41, 11)
    dis = g.uniform(0.0, 1.0, 7).astype(np.float32)
    P = np.stack([np.full(7, -np.inf, np.float32), dis])
    R, ab, _ = oracle.mmlike_f32(oracle.DISCOUNT, A, B, P)
    S, _ = _matmul_of_rounded_products(A, B)
    ref = (1.0 - dis.astype(np.float64))[None, :] * S
    assert np.all(np.abs(R - ref) <= 2.0 ** -23 * np.abs(ref) + 1e-12 * ab + 1e-30)


def test_discount_closed_form_matmul_minus_dis_times_masked_sum():
    g, A, B = _rand(11, 13, 23, 12)
    th = g.standard_normal(13).astype(np.float32) * 4
    dis = g.uniform(0.0, 1.0, 13).astype(np.float32)
    R, ab, _ = oracle.mmlike_f32(oracle.DISCOUNT, A, B, np.stack([th, dis]))
    S, P = _matmul_of_rounded_products(A, B)
    mask = P > th[None, None, :]
    assert mask.any() and (~mask).any()
    hi = np.where(mask, P.astype(np.float64), 0.0).sum(axis=1)
    ref = S - dis.astype(np.float64)[None, :] * hi
    assert np.all(np.abs(R - ref) <= 2.0 ** -23 * np.abs(ref) + 1e-12 * ab + 1e-30)
    ab_ref = np.where(mask, np.abs(P.astype(np.float64) * (1 - dis.astype(np.float64))[None, None, :]),
                      np.abs(P.astype(np.float64))).sum(axis=1)
    assert np.allclose(ab, ab_ref, rtol=1e-12, atol=0)


def test_boost_closed_form_matmul_plus_relu_sum():
    g, A, B = _rand(11, 13, 23, 13)
    th = g.standard_normal(13).astype(np.float32) * 4
    R, ab, _ = oracle.mmlike_f32(oracle.BOOST, A, B, th[None])
    S, P = _matmul_of_rounded_products(A, B)
    relu = np.maximum(P.astype(np.float64) - th.astype(np.float64)[None, None, :], 0.0).sum(axis=1)
    ref = S + relu
    assert np.all(np.abs(R - ref) <= 2.0 ** -23 * np.abs(ref) + 1e-12 * ab + 1e-30)
    Ri, _, _ = oracle.mmlike_f32(oracle.IDENTITY, A, B, None)
    assert np.all(R >= Ri)  # the boosted part is never negative


def test_boost_thres_below_every_product_is_2AB_minus_K_T():
    g, A, B = _rand(5, 6, 17, 14)
    T = np.float32(-1000.0)
    R, _, _ = oracle.mmlike_f32(oracle.BOOST, A, B, np.full((1, 6), T, np.float32))
    S, _ = _matmul_of_rounded_products(A, B)
    ref = 2.0 * S - 17 * float(T)
    assert np.all(np.abs(R - ref) <= 2.0 ** -23 * np.abs(ref))


def test_count_gt_counts_products_over_threshold_by_tensor():
    g, A, B = _rand(9, 10, 33, 15)
    th = g.standard_normal(10).astype(np.float32)
    R, ab, _ = oracle.mmlike_f32(oracle.COUNT_GT, A, B, th[None])
    _, P = _matmul_of_rounded_products(A, B)
    ref = (P > th[None, None, :]).sum(axis=1)
    assert np.array_equal(R, ref.astype(np.float32)) and np.array_equal(ab, ref.astype(np.float64))


def test_join_count_is_integer_matmul_and_query3_on_indicator_data():
    A, B = wl.join_indicator(37, 29, 211, seed=16, density=0.2)
    R, _ = oracle.count_i8(A, B)
    ref = A.astype(np.int64) @ B.astype(np.int64)
    assert ref.max() > 3 and np.array_equal(R, ref.astype(np.int32))
    Rq, _, _ = oracle.mmlike_f32(oracle.COUNT_GT, A.astype(np.float32), B.astype(np.float32),
                                 np.full((1, 29), 0.5, np.float32))
    assert np.array_equal(Rq, ref.astype(np.float32))
    # row-sum checksum: sum_j R[i][j] = sum_k A[i][k] * (sum_j B[k][j])
    assert np.array_equal(R.sum(1), A.astype(np.int64) @ B.astype(np.int64).sum(1))


def test_count_i8_full_int8_range_and_R_in():
    g = np.random.Generator(np.random.PCG64(17))
    A = g.integers(-128, 128, (7, 300)).astype(np.int8)
    B = g.integers(-128, 128, (300, 5)).astype(np.int8)
    R_in = g.integers(-10 ** 6, 10 ** 6, (7, 5)).astype(np.int32)
    R, _ = oracle.count_i8(A, B, R_in)
    assert np.array_equal(R, (A.astype(np.int64) @ B.astype(np.int64) + R_in).astype(np.int32))


def test_count_i8_reports_int32_overflow():
    A = np.full((1, 4), 127, np.int8)
    B = np.full((4, 1), 127, np.int8)
    with pytest.raises(OverflowError):
        oracle.count_i8(A, B, np.array([[2 ** 31 - 10]], np.int32))


@pytest.mark.parametrize("task", TASKS_F32)
def test_linear_in_R_in(task):
    g, A, B = _rand(5, 6, 20, 18 + task)
    params = None
    if NPAR[task]:
        params = np.stack([g.standard_normal(6).astype(np.float32)] +
                          ([g.uniform(0, 1, 6).astype(np.float32)] if NPAR[task] == 2 else []))
    X = (g.integers(-50, 50, (5, 6)) * 4096).astype(np.float32)
    R0, _, _ = oracle.mmlike_f32(task, A, B, params)
    RX, _, _ = oracle.mmlike_f32(task, A, B, params, X)
    assert np.all(np.abs(RX.astype(np.float64) - (X.astype(np.float64) + R0)) <=
                  2.0 ** -23 * np.abs(RX) + 2.0 ** -23 * np.abs(R0))


def test_operands_are_not_transposed_and_strides_are_honoured():
    # non-square, asymmetric data: swapping or transposing an operand changes the result
    g = np.random.Generator(np.random.PCG64(19))
    Abig = g.integers(-5, 6, (4, 9)).astype(np.float32)
    Bbig = g.integers(-5, 6, (9, 8)).astype(np.float32)
    A = Abig[:, :7]       # lda = 9 > K = 7
    B = Bbig[:7, :5]      # ldb = 8 > N = 5
    R, _, _ = oracle.mmlike_f32(oracle.IDENTITY, A, B, None)
    assert np.array_equal(R, (A.astype(np.int64) @ B.astype(np.int64)).astype(np.float32))
    th = np.array([1, -2, 3, 0, 5], np.float32)
    Rb, _, _ = oracle.mmlike_f32(oracle.BOOST, A, B, th[None])
    P = A[:, :, None].astype(np.float64) * B[None].astype(np.float64)
    assert np.array_equal(Rb, (P + np.maximum(P - th[None, None], 0)).sum(1).astype(np.float32))


def test_param_is_indexed_by_column_j_not_row_i():
    A = np.ones((3, 1), np.float32) * 10
    B = np.ones((1, 3), np.float32)
    th = np.array([5, 20, 5], np.float32)
    dis = np.array([0.5, 0.5, 0.25], np.float32)
    R, _, _ = oracle.mmlike_f32(oracle.DISCOUNT, A, B, np.stack([th, dis]))
    assert R.tolist() == [[5.0, 10.0, 7.5]] * 3


# --------------------------------------------------------------------------
# 4. the compared product is the fp32-rounded one, compared strictly
# --------------------------------------------------------------------------
def test_predicate_uses_the_fp32_rounded_product():
    a = np.float32(1 + 2.0 ** -12)
    exact = float(a) * float(a)                 # 1 + 2^-11 + 2^-24, exact in double
    p32 = np.float32(a * a)                     # ties-to-even drops the 2^-24
    assert exact > float(p32) and float(p32) == 1 + 2.0 ** -11
    A = np.array([[a]], np.float32)
    B = np.array([[a]], np.float32)
    th = np.array([[p32]], np.float32)          # exact product > thres, rounded product == thres
    R, _, _ = oracle.mmlike_f32(oracle.COUNT_GT, A, B, th)
    assert R[0, 0] == 0.0
    R, _, _ = oracle.mmlike_f32(oracle.DISCOUNT, A, B, np.array([[p32], [0.5]], np.float32))
    assert R[0, 0] == p32                       # not discounted
    # one ulp lower threshold: now it triggers
    lo = np.nextafter(p32, np.float32(0))
    R, _, _ = oracle.mmlike_f32(oracle.COUNT_GT, A, B, np.array([[lo]], np.float32))
    assert R[0, 0] == 1.0
    R, _, _ = oracle.mmlike_f32(oracle.BOOST, A, B, np.array([[lo]], np.float32))
    assert R[0, 0] == np.float32(float(p32) + (float(p32) - float(lo)))


def test_negative_threshold_boosts_zero_products():
    # g(0) = -thres when thres < 0: zero padding of K would be wrong
    A = np.zeros((2, 5), np.float32)
    B = np.ones((5, 2), np.float32)
    R, _, _ = oracle.mmlike_f32(oracle.BOOST, A, B, np.array([[-2.0, 3.0]], np.float32))
    assert R.tolist() == [[10.0, 0.0]] * 2


def test_empty_K_and_threads_do_not_change_result():
    A = np.zeros((3, 0), np.float32)
    B = np.zeros((0, 4), np.float32)
    R_in = np.arange(12, dtype=np.float32).reshape(3, 4)
    R, ab, _ = oracle.mmlike_f32(oracle.BOOST, A, B, np.zeros((1, 4), np.float32), R_in)
    assert np.array_equal(R, R_in) and not ab.any()
    A, B, P = wl.retail(33, 20, 50, seed=3)
    R1, ab1, u1 = oracle.mmlike_f32(oracle.DISCOUNT, A, B, P, threads=1)
    R4, ab4, u4 = oracle.mmlike_f32(oracle.DISCOUNT, A, B, P, threads=4)
    assert u1 == 1 and u4 == 4
    assert np.array_equal(R1, R4) and np.array_equal(ab1, ab4)


def test_subnormal_products_are_kept_not_flushed():
    """Powers of two, so every value below is exact and known without computing it:
    2^-100 * 2^-40 = 2^-140 is a subnormal fp32 number, 2^-100 * 2^-60 = 2^-160 rounds to 0.
    The predicate sees the subnormal product (it is > 0 and > 2^-141, not > 2^-139), the sums
    keep it, and the fp64 oracle does the same at 2^-1040."""
    A = np.array([[2.0 ** -100, 2.0 ** -100]], np.float32)
    B = np.array([[2.0 ** -40, 2.0 ** -40, 2.0 ** -40], [2.0 ** -60, 2.0 ** -60, 2.0 ** -60]], np.float32)
    thres = np.array([0.0, 2.0 ** -141, 2.0 ** -139], np.float32)
    cnt, _, _ = oracle.mmlike_f32(3, A, B, thres[None, :])
    assert cnt.tolist() == [[1.0, 1.0, 0.0]]
    ident, ab, _ = oracle.mmlike_f32(0, A, B, None)
    assert ident.tolist() == [[2.0 ** -140] * 3] and ab.tolist() == [[2.0 ** -140] * 3]
    dis = np.array([0.5, 0.5, 0.5], np.float32)
    disc, _, _ = oracle.mmlike_f32(1, A, B, np.stack([thres, dis]))
    assert disc.tolist() == [[2.0 ** -141, 2.0 ** -141, 2.0 ** -140]]
    A64 = np.array([[2.0 ** -1000]])
    B64 = np.array([[2.0 ** -40, 2.0 ** -40]])
    t64 = np.array([2.0 ** -1041, 2.0 ** -1039])
    c64, _, _ = oracle.mmlike_f64_general(3, A64, B64, t64, None, None)
    assert c64.tolist() == [[1.0, 0.0]]
    i64, _, _ = oracle.mmlike_f64_general(0, A64, B64, None, None, None)
    assert i64.tolist() == [[2.0 ** -1040, 2.0 ** -1040]]
