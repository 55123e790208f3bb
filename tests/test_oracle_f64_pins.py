"""Pins for the fp64 oracle (the paper's own element type): hand-worked example, exact-rational
evaluation of the printed text, reductions to numpy routines, and the reading "the compared
product is the fp64-rounded one"."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

TASKS = [oracle.IDENTITY, oracle.DISCOUNT, oracle.BOOST, oracle.COUNT_GT]
FORMS = [oracle.THRES_COL, oracle.THRES_ROW, oracle.THRES_CONST, oracle.THRES_ELEM]


def test_worked_examples_in_double(golden_dir):
    with open(os.path.join(golden_dir, "worked_3x3.json")) as f:
        base = json.load(f)
    with open(os.path.join(golden_dir, "worked_3x3_forms.json")) as f:
        g = json.load(f)
    A = np.array(base["A"], np.float64)
    B = np.array(base["B"], np.float64)
    dis = np.array(base["dis"], np.float64)
    R, ab, _ = oracle.mmlike_f64_general(oracle.IDENTITY, A, B)
    assert R.tolist() == base["identity"]
    for key, task in (("discount", oracle.DISCOUNT), ("boost", oracle.BOOST)):
        R, ab, _ = oracle.mmlike_f64_general(task, A, B, base["thres"], dis)
        assert R.tolist() == base[key] and R.dtype == np.float64
    for form, th, want in ((oracle.THRES_ROW, g["thres_row"], g["row"]),
                           (oracle.THRES_CONST, [g["thres_const"]], g["const"]),
                           (oracle.THRES_ELEM, g["thres_elem"], g["elem"])):
        for key, task in (("discount", oracle.DISCOUNT), ("boost", oracle.BOOST), ("count_gt", oracle.COUNT_GT)):
            R, _, _ = oracle.mmlike_f64_general(task, A, B, th, dis, thres_form=form)
            assert R.tolist() == want[key], (form, key)


@pytest.mark.parametrize("task", TASKS)
@pytest.mark.parametrize("form", FORMS)
@pytest.mark.parametrize("tA,tB", [(False, False), (True, True)])
def test_f64_matches_exact_rational_literal(task, form, tA, tB):
    M, N, K = 4, 5, 6
    g = np.random.Generator(np.random.PCG64(900 + 31 * task + 7 * form + tA))
    # dyadic data with more bits than fp32 holds: exact in double only
    A = (g.integers(-2 ** 20, 2 ** 20, size=(K, M) if tA else (M, K)) / 2.0 ** 12).astype(np.float64)
    B = (g.integers(-2 ** 20, 2 ** 20, size=(N, K) if tB else (K, N)) / 2.0 ** 12).astype(np.float64)
    shape = {oracle.THRES_COL: (N,), oracle.THRES_ROW: (M,), oracle.THRES_CONST: (1,), oracle.THRES_ELEM: (M, N)}[form]
    th = (g.integers(-2 ** 14, 2 ** 14, size=shape) / 8.0).astype(np.float64)
    dis = (g.integers(0, 9, size=N) / 8.0).astype(np.float64)
    R_in = g.integers(-9, 10, size=(M, N)).astype(np.float64)
    R, ab, _ = oracle.mmlike_f64_general(task, A, B, th, dis, R_in, thres_form=form, trans_a=tA, trans_b=tB)
    F = lambda x: Fraction(float(x))
    for i in range(M):
        for j in range(N):
            t = F({oracle.THRES_COL: lambda: th[j], oracle.THRES_ROW: lambda: th[i],
                   oracle.THRES_CONST: lambda: th[0], oracle.THRES_ELEM: lambda: th[i][j]}[form]())
            acc, sab = F(R_in[i][j]), Fraction(0)
            for k in range(K):
                a = F(A[k][i]) if tA else F(A[i][k])
                b = F(B[j][k]) if tB else F(B[k][j])
                if task == oracle.IDENTITY:
                    v = a * b
                elif task == oracle.DISCOUNT:
                    v = a * b - int(a * b > t) * a * b * F(dis[j])
                elif task == oracle.BOOST:
                    v = a * b + int(a * b > t) * (a * b - t)
                else:
                    v = Fraction(int(a * b > t))
                acc += v
                sab += abs(v)
            # products have <= 42 significant bits, terms <= 45, sums <= 49: exact in fp64
            assert F(R[i, j]) == acc and F(ab[i, j]) == sab, (i, j)


def test_f64_identity_is_integer_matmul_and_more_precise_than_fp64_dot():
    g = np.random.Generator(np.random.PCG64(41))
    A = g.integers(-2 ** 25, 2 ** 25, (7, 40)).astype(np.float64)
    B = g.integers(-2 ** 25, 2 ** 25, (40, 5)).astype(np.float64)
    R, _, _ = oracle.mmlike_f64_general(oracle.IDENTITY, A, B)
    exact = [[sum(int(A[i, k]) * int(B[k, j]) for k in range(40)) for j in range(5)] for i in range(7)]
    assert np.array_equal(R, np.array(exact, dtype=np.float64))   # correctly rounded exact sums
    # random data: agrees with numpy's fp64 matmul to fp64 round-off, against sum |term|
    A = g.standard_normal((20, 300)); B = g.standard_normal((300, 15))
    R, ab, _ = oracle.mmlike_f64_general(oracle.IDENTITY, A, B)
    assert np.all(np.abs(R - A @ B) <= 300 * 2.0 ** -53 * ab)


def test_f64_predicate_uses_the_fp64_rounded_product():
    a = 1 + 2.0 ** -27                       # a*a = 1 + 2^-26 + 2^-54 exactly; fp64 drops the 2^-54
    p = a * a
    assert p == 1 + 2.0 ** -26 and Fraction(a) * Fraction(a) > Fraction(p)
    A = np.array([[a]]); B = np.array([[a]])
    R, _, _ = oracle.mmlike_f64_general(oracle.COUNT_GT, A, B, [p])
    assert R[0, 0] == 0.0                    # rounded product equals thres: not triggered
    R, _, _ = oracle.mmlike_f64_general(oracle.COUNT_GT, A, B, [np.nextafter(p, 0.0)])
    assert R[0, 0] == 1.0
    R, _, _ = oracle.mmlike_f64_general(oracle.DISCOUNT, A, B, [p], [0.5])
    assert R[0, 0] == p


def test_f64_invariants():
    g = np.random.Generator(np.random.PCG64(43))
    A = g.standard_normal((6, 50)); B = g.standard_normal((50, 7)); R_in = g.standard_normal((6, 7))
    inf = np.full(7, np.inf)
    Ri, abi, _ = oracle.mmlike_f64_general(oracle.IDENTITY, A, B, R_in=R_in)
    for task in (oracle.DISCOUNT, oracle.BOOST):
        R, ab, _ = oracle.mmlike_f64_general(task, A, B, inf, g.uniform(0, 1, 7), R_in)
        assert np.array_equal(R, Ri) and np.array_equal(ab, abi)
    R, ab, _ = oracle.mmlike_f64_general(oracle.DISCOUNT, A, B, -inf, np.ones(7), R_in)
    assert np.array_equal(R, R_in) and not ab.any()
    # fp32 inputs widened to fp64: the fp64 oracle's identity equals the exact sum of exact
    # products, which the fp32 oracle (products rounded to fp32) only approximates
    A32 = A.astype(np.float32); B32 = B.astype(np.float32)
    R64, _, _ = oracle.mmlike_f64_general(oracle.IDENTITY, A32.astype(np.float64), B32.astype(np.float64))
    R32, ab32, _ = oracle.mmlike_f32(oracle.IDENTITY, A32, B32, None)
    assert np.all(np.abs(R32 - R64) <= 2.0 ** -23 * ab32)
    # row/column duality of boost in fp64
    th = g.standard_normal(6)
    Rr, _, _ = oracle.mmlike_f64_general(oracle.BOOST, A, B, th, thres_form=oracle.THRES_ROW)
    Rc, _, _ = oracle.mmlike_f64_general(oracle.BOOST, np.ascontiguousarray(B.T), np.ascontiguousarray(A.T), th)
    assert np.array_equal(Rr, Rc.T)
