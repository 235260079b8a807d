"""Pins for the oracle's transposed batched matmul (Section 7, listing tbmm).

Every check compares the C loop nest with something that is not the C loop
nest: exact integer arithmetic in Python, numpy's float64 einsum/matmul,
closed forms.  Shapes are non-square so that a transposed or mis-indexed
operand cannot pass.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from paper_1802_04730_amd import inputs


def _brute(X, Y):
    B, N, K = X.shape
    M = Y.shape[1]
    Z = np.zeros((B, N, M))
    for b, n, m in itertools.product(range(B), range(N), range(M)):
        z = 0.0
        for k in range(K):
            z += float(X[b, n, k]) * float(Y[b, m, k])
        Z[b, n, m] = z
    return Z


@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (2, 3, 5, 7), (3, 4, 2, 1)])
def test_brute_force(shape):
    X, Y = inputs.make_tbmm(*shape, seed=11)
    np.testing.assert_allclose(oracle.tbmm(X, Y), _brute(X, Y), rtol=1e-14, atol=1e-15)


def test_exact_on_small_integers():
    # integer-valued inputs: every product and partial sum is exact in double,
    # so the oracle must equal Python's unbounded integer arithmetic bit for bit
    r = np.random.default_rng(5)
    B, N, M, K = 3, 5, 7, 11
    Xi = r.integers(-9, 10, size=(B, N, K))
    Yi = r.integers(-9, 10, size=(B, M, K))
    want = np.zeros((B, N, M), dtype=np.int64)
    for b, n, m in itertools.product(range(B), range(N), range(M)):
        want[b, n, m] = sum(int(Xi[b, n, k]) * int(Yi[b, m, k]) for k in range(K))
    got = oracle.tbmm(Xi.astype(np.float32), Yi.astype(np.float32))
    assert np.array_equal(got, want.astype(np.float64))


@pytest.mark.parametrize("cfg", [1, 2])
def test_matches_numpy_einsum_at_benchmark_shapes(cfg, oracle_threads):
    _, (X, Y) = inputs.make_config(cfg)
    ref = np.einsum("bnk,bmk->bnm", X.astype(np.float64), Y.astype(np.float64))
    got = oracle.tbmm(X, Y)
    assert got.shape == (X.shape[0], 26, 72)
    np.testing.assert_allclose(got, ref, rtol=1e-13, atol=1e-13)


def test_paper_text_shape():
    # the paper's own naming gives output 26 x 26 with a reduction of 72
    X, Y = inputs.make_tbmm(4, 26, 26, 72, seed=3)
    ref = np.matmul(X.astype(np.float64), np.swapaxes(Y.astype(np.float64), 1, 2))
    np.testing.assert_allclose(oracle.tbmm(X, Y), ref, rtol=1e-13, atol=1e-13)


def test_single_batch_is_transposed_matmul():
    # B = 1 reduces to tmm: C(m,n) = sum_kk A(m,kk) * B(n,kk)  (Section 7, listing tmm)
    X, Y = inputs.make_tbmm(1, 6, 9, 4, seed=2)
    ref = X[0].astype(np.float64) @ Y[0].astype(np.float64).T
    np.testing.assert_allclose(oracle.tbmm(X, Y)[0], ref, rtol=1e-14, atol=1e-15)


def test_identity_operand_copies_x():
    X, _ = inputs.make_tbmm(3, 5, 8, 8, seed=4)
    Y = np.broadcast_to(np.eye(8, dtype=np.float32), (3, 8, 8)).copy()
    assert np.array_equal(oracle.tbmm(X, Y), X.astype(np.float64))


def test_all_ones_gives_k():
    X = np.ones((2, 3, 26), np.float32)
    Y = np.ones((2, 4, 26), np.float32)
    assert np.array_equal(oracle.tbmm(X, Y), np.full((2, 3, 4), 26.0))


def test_batches_are_independent_and_ordered():
    X, Y = inputs.make_tbmm(4, 3, 5, 6, seed=8)
    Z = oracle.tbmm(X, Y)
    for b in range(4):
        np.testing.assert_array_equal(Z[b], oracle.tbmm(X[b:b + 1], Y[b:b + 1])[0])
    perm = [2, 0, 3, 1]
    np.testing.assert_array_equal(oracle.tbmm(X[perm], Y[perm]), Z[perm])


def test_thread_count_does_not_change_result():
    X, Y = inputs.make_tbmm(9, 7, 5, 13, seed=1)
    oracle.set_threads(1)
    a = oracle.tbmm(X, Y)
    oracle.set_threads(3)
    b = oracle.tbmm(X, Y)
    oracle.set_threads(1)
    assert np.array_equal(a, b)


def test_float64_result_is_not_rounded_to_float():
    # 1 + 2^-30 needs more than 24 mantissa bits: a float accumulator would lose it
    X = np.array([[[1.0, 2.0 ** -15]]], np.float32)
    Y = np.array([[[1.0, 2.0 ** -15]]], np.float32)
    assert oracle.tbmm(X, Y)[0, 0, 0] == 1.0 + 2.0 ** -30


def test_empty_batch_and_bad_shapes():
    Z = oracle.tbmm(np.zeros((0, 3, 4), np.float32), np.zeros((0, 5, 4), np.float32))
    assert Z.shape == (0, 3, 5)
    with pytest.raises(ValueError):
        oracle.tbmm(np.zeros((2, 3, 4), np.float32), np.zeros((2, 5, 3), np.float32))
    with pytest.raises(ValueError):
        oracle.tbmm(np.zeros((2, 3, 0), np.float32), np.zeros((2, 5, 0), np.float32))


def test_planted_mistakes_are_caught():
    # the pins above must be able to see a dropped term, a wrong sign and a transposed operand
    X, Y = inputs.make_tbmm(2, 3, 5, 7, seed=11)
    good = _brute(X, Y)
    Xd, Yd = X.astype(np.float64), Y.astype(np.float64)
    dropped = np.einsum("bnk,bmk->bnm", Xd[:, :, :-1], Yd[:, :, :-1])
    signed = -good
    Xs, Ys = inputs.make_tbmm(2, 5, 5, 5, seed=11)
    transposed = np.einsum("bkn,bmk->bnm", Xs.astype(np.float64), Ys.astype(np.float64))
    assert not np.allclose(dropped, good, rtol=1e-9)
    assert not np.allclose(signed, good, rtol=1e-9)
    assert not np.allclose(transposed, _brute(Xs, Ys), rtol=1e-9)


def test_paper_workload_flops():
    path = os.path.join(os.path.dirname(__file__), "golden", "workload_sizes.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        name, rest = line.split(None, 1)
        nums = rest.split('"')[0].split()
        ext, flops = [int(v) for v in nums[:-1]], int(nums[-1])
        if name == "tbmm_paper":
            assert inputs.flops_tbmm(*ext) == flops
            assert inputs.flops_tbmm(**{k: v for k, v in inputs.CONFIGS[2].items() if k != "op"}) == flops
        else:
            m, k, n = ext  # tmm = tbmm with one batch element
            assert inputs.flops_tbmm(1, m, n, k) == flops
