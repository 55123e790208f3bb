"""Pins for the oracle's general form: threshold operand as thres[i], constant,
thres[i][j], and operands stored transposed ("Test Queries" figure, Sec. 6.3)."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

import amulet_workloads as wl
import oracle

FORMS = [oracle.THRES_COL, oracle.THRES_ROW, oracle.THRES_CONST, oracle.THRES_ELEM]
TASKS = [oracle.DISCOUNT, oracle.BOOST, oracle.COUNT_GT]


@pytest.fixture(scope="module")
def worked(golden_dir):
    with open(os.path.join(golden_dir, "worked_3x3.json")) as f:
        base = json.load(f)
    with open(os.path.join(golden_dir, "worked_3x3_forms.json")) as f:
        forms = json.load(f)
    return base, forms


def test_worked_example_threshold_forms(worked):
    base, g = worked
    A = np.array(base["A"], np.float32)
    B = np.array(base["B"], np.float32)
    dis = np.array(base["dis"], np.float32)
    cases = [(oracle.THRES_ROW, g["thres_row"], g["row"]),
             (oracle.THRES_CONST, [g["thres_const"]], g["const"]),
             (oracle.THRES_ELEM, g["thres_elem"], g["elem"])]
    for form, th, want in cases:
        for task, key in ((oracle.DISCOUNT, "discount"), (oracle.BOOST, "boost"), (oracle.COUNT_GT, "count_gt")):
            R, _, _ = oracle.mmlike_f32_general(task, A, B, th, dis, thres_form=form)
            assert R.tolist() == want[key], (form, key)


def _thres_for(form, M, N, g):
    n = {oracle.THRES_COL: (N,), oracle.THRES_ROW: (M,), oracle.THRES_CONST: (1,), oracle.THRES_ELEM: (M, N)}[form]
    return (g.integers(-24, 25, size=n) / 2.0).astype(np.float32)


def _literal(task, form, tA, tB, A, B, th, dis, M, N, K):
    """The printed loop text in exact rationals, with A[k][i] / B[j][k] indexing when the
    operand is stored transposed and the threshold written in the given operand form."""
    F = lambda x: Fraction(float(x))
    R = [[Fraction(0)] * N for _ in range(M)]
    for i in range(M):
        for j in range(N):
            if form == oracle.THRES_COL:
                t = F(th[j])
            elif form == oracle.THRES_ROW:
                t = F(th[i])
            elif form == oracle.THRES_CONST:
                t = F(th[0])
            else:
                t = F(th[i][j])
            for k in range(K):
                a = F(A[k][i]) if tA else F(A[i][k])
                b = F(B[j][k]) if tB else F(B[k][j])
                if task == oracle.DISCOUNT:
                    R[i][j] += a * b - int(a * b > t) * a * b * F(dis[j])
                elif task == oracle.BOOST:
                    R[i][j] += a * b + int(a * b > t) * (a * b - t)
                else:
                    R[i][j] += int(a * b > t)
    return R


@pytest.mark.parametrize("task", TASKS)
@pytest.mark.parametrize("form", FORMS)
@pytest.mark.parametrize("tA,tB", [(False, False), (True, False), (False, True), (True, True)])
def test_general_form_matches_exact_rational_literal(task, form, tA, tB):
    M, N, K = 5, 4, 6
    g = np.random.Generator(np.random.PCG64(500 + 31 * task + 7 * form + 2 * tA + tB))
    A = g.integers(-8, 9, size=(K, M) if tA else (M, K)).astype(np.float32)
    B = g.integers(-8, 9, size=(N, K) if tB else (K, N)).astype(np.float32)
    th = _thres_for(form, M, N, g)
    dis = (g.integers(0, 9, size=N) / 8.0).astype(np.float32)
    R, _, _ = oracle.mmlike_f32_general(task, A, B, th, dis, thres_form=form, trans_a=tA, trans_b=tB)
    want = _literal(task, form, tA, tB, A, B, th, dis, M, N, K)
    for i in range(M):
        for j in range(N):
            assert Fraction(float(R[i, j])) == want[i][j], (i, j)


def test_identity_transposed_is_numpy_matmul():
    g = np.random.Generator(np.random.PCG64(77))
    At = g.integers(-9, 10, (11, 7)).astype(np.float32)   # K x M
    Bt = g.integers(-9, 10, (5, 11)).astype(np.float32)   # N x K
    R, _, _ = oracle.mmlike_f32_general(oracle.IDENTITY, At, Bt, trans_a=True, trans_b=True)
    assert np.array_equal(R, (At.T.astype(np.int64) @ Bt.T.astype(np.int64)).astype(np.float32))


@pytest.mark.parametrize("task", [oracle.BOOST, oracle.COUNT_GT])
def test_row_form_is_the_column_form_of_the_transposed_problem(task):
    # g has no j-indexed operand besides thres for these tasks, and fp32 multiplication commutes:
    # task(A, B, thres[i]) == task(B^T, A^T, thres[j])^T exactly.
    g = np.random.Generator(np.random.PCG64(78 + task))
    A = g.standard_normal((9, 13)).astype(np.float32)
    B = g.standard_normal((13, 6)).astype(np.float32)
    th = g.standard_normal(9).astype(np.float32)
    R_row, ab_row, _ = oracle.mmlike_f32_general(task, A, B, th, thres_form=oracle.THRES_ROW)
    R_col, ab_col, _ = oracle.mmlike_f32(task, np.ascontiguousarray(B.T), np.ascontiguousarray(A.T), th[None])
    assert np.array_equal(R_row, R_col.T) and np.array_equal(ab_row, ab_col.T)


@pytest.mark.parametrize("task", TASKS)
def test_all_forms_agree_on_a_uniform_threshold(task):
    g = np.random.Generator(np.random.PCG64(90 + task))
    M, N, K = 7, 8, 15
    A = g.standard_normal((M, K)).astype(np.float32) * 2
    B = g.standard_normal((K, N)).astype(np.float32) * 2
    dis = g.uniform(0, 1, N).astype(np.float32)
    c = np.float32(0.75)
    ref, ab, _ = oracle.mmlike_f32_general(task, A, B, [c], dis, thres_form=oracle.THRES_CONST)
    for form, th in ((oracle.THRES_COL, np.full(N, c)), (oracle.THRES_ROW, np.full(M, c)),
                     (oracle.THRES_ELEM, np.full((M, N), c))):
        R, ab2, _ = oracle.mmlike_f32_general(task, A, B, th, dis, thres_form=form)
        assert np.array_equal(R, ref) and np.array_equal(ab2, ab)
    # and the general entry point with the column form is the planar-parameter entry point
    th = g.standard_normal(N).astype(np.float32)
    P = np.stack([th, dis]) if task == oracle.DISCOUNT else th[None]
    R1, ab1, _ = oracle.mmlike_f32(task, A, B, P)
    R2, ab2, _ = oracle.mmlike_f32_general(task, A, B, th, dis)
    assert np.array_equal(R1, R2) and np.array_equal(ab1, ab2)


def test_transposed_storage_with_strides():
    g = np.random.Generator(np.random.PCG64(99))
    M, N, K = 6, 5, 9
    A = g.standard_normal((M, K)).astype(np.float32)
    B = g.standard_normal((K, N)).astype(np.float32)
    th = g.standard_normal(N).astype(np.float32)
    ref, ab, _ = oracle.mmlike_f32(oracle.BOOST, A, B, th[None])
    bigAt = np.zeros((K, M + 3), np.float32); bigAt[:, :M] = A.T
    bigBt = np.zeros((N, K + 2), np.float32); bigBt[:, :K] = B.T
    R, ab2, _ = oracle.mmlike_f32_general(oracle.BOOST, bigAt[:, :M], bigBt[:, :K], th, trans_a=True, trans_b=True)
    assert np.array_equal(R, ref) and np.array_equal(ab, ab2)
