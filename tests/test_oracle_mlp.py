"""Pins for the oracle's fcrelu chain (Section 3 listing fcrelu; appendix MLP1 / MLP3)."""
import itertools

import numpy as np
import pytest
import torch

import oracle
from paper_1802_04730_amd import inputs


def _brute(I, Ws, bs):
    outs, cur = [], [[float(v) for v in row] for row in I]
    for W, b in zip(Ws, bs):
        nxt = []
        for row in cur:
            o_row = []
            for n in range(W.shape[0]):
                o = float(b[n])
                for m in range(W.shape[1]):
                    o += row[m] * float(W[n, m])
                o_row.append(o if o > 0 else 0.0)
            nxt.append(o_row)
        outs.append(np.array(nxt))
        cur = nxt
    return outs


def test_brute_force_three_layers():
    I, Ws, bs = inputs.make_mlp(2, (3, 4, 2, 1), seed=7, w_std=0.7, b_std=0.3)
    got = oracle.mlp_fcrelu(I, Ws, bs)
    for g, w in zip(got, _brute(I, Ws, bs)):
        np.testing.assert_allclose(g, w, rtol=1e-14, atol=1e-16)


def test_exact_on_small_integers():
    r = np.random.default_rng(9)
    I = r.integers(-4, 5, size=(3, 6))
    W0 = r.integers(-3, 4, size=(5, 6))
    b0 = r.integers(-5, 6, size=(5,))
    W1 = r.integers(-3, 4, size=(4, 5))
    b1 = r.integers(-5, 6, size=(4,))
    o0 = [[max(0, int(b0[n]) + sum(int(I[b, m]) * int(W0[n, m]) for m in range(6)))
           for n in range(5)] for b in range(3)]
    o1 = [[max(0, int(b1[n]) + sum(o0[b][m] * int(W1[n, m]) for m in range(5)))
           for n in range(4)] for b in range(3)]
    f = lambda a: a.astype(np.float32)
    got = oracle.mlp_fcrelu(f(I), [f(W0), f(W1)], [f(b0), f(b1)])
    assert np.array_equal(got[0], np.array(o0, dtype=np.float64))
    assert np.array_equal(got[1], np.array(o1, dtype=np.float64))


def test_matches_numpy_and_torch_at_benchmark_shape(oracle_threads):
    _, (I, Ws, bs) = inputs.make_config(3)
    got = oracle.mlp_fcrelu(I, Ws, bs)
    x = I.astype(np.float64)
    xt = torch.from_numpy(I).double()
    for l, (W, b) in enumerate(zip(Ws, bs)):
        x = np.maximum(x @ W.astype(np.float64).T + b.astype(np.float64), 0.0)
        xt = torch.relu(torch.nn.functional.linear(xt, torch.from_numpy(W).double(),
                                                   torch.from_numpy(b).double()))
        assert got[l].shape == (128, inputs.CONFIGS[3]["dims"][l + 1])
        np.testing.assert_allclose(got[l], x, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(got[l], xt.numpy(), rtol=1e-12, atol=1e-13)
        assert np.all(got[l] >= 0.0)
        zeros = float(np.mean(got[l] == 0.0))
        assert 0.35 < zeros < 0.65, zeros  # ReLU of a roughly centred pre-activation


def test_zero_weights_leave_clamped_bias():
    I, Ws, bs = inputs.make_mlp(4, (5, 6, 3), seed=1, b_std=1.0)
    Ws = [np.zeros_like(w) for w in Ws]
    got = oracle.mlp_fcrelu(I, Ws, bs)
    for l in range(2):
        want = np.broadcast_to(np.maximum(bs[l].astype(np.float64), 0.0), got[l].shape)
        assert np.array_equal(got[l], want)


def test_one_layer_is_fcrelu_and_prefix_of_chain():
    I, Ws, bs = inputs.make_mlp(5, (7, 4, 3), seed=2, w_std=0.5, b_std=0.5)
    one = oracle.mlp_fcrelu(I, Ws[:1], bs[:1])[0]
    want = np.maximum(I.astype(np.float64) @ Ws[0].astype(np.float64).T + bs[0], 0.0)
    np.testing.assert_allclose(one, want, rtol=1e-14, atol=1e-16)
    assert np.array_equal(oracle.mlp_fcrelu(I, Ws, bs)[0], one)


def test_identity_layer_passes_positive_rows_and_clamps_negative():
    I = np.array([[1.5, -2.0, 0.25], [-1.0, 3.0, -0.5]], np.float32)
    got = oracle.mlp_fcrelu(I, [np.eye(3, dtype=np.float32)], [np.zeros(3, np.float32)])[0]
    assert np.array_equal(got, np.maximum(I.astype(np.float64), 0.0))


def test_chain_is_carried_in_double_and_rounded_variant_differs():
    I, Ws, bs = inputs.make_mlp(8, (64, 48, 32, 16), seed=3, w_std=0.2, b_std=0.1)
    plain = oracle.mlp_fcrelu(I, Ws, bs)
    rounded = oracle.mlp_fcrelu(I, Ws, bs, round_intermediates=True)
    assert np.array_equal(plain[0], rounded[0])  # the first layer sees no intermediate
    # the rounded variant equals a chain restarted from float32 copies of each output
    step = oracle.mlp_fcrelu(plain[0].astype(np.float32), Ws[1:2], bs[1:2])[0]
    np.testing.assert_array_equal(rounded[1], step)
    assert not np.array_equal(plain[1], rounded[1])
    np.testing.assert_allclose(plain[2], rounded[2], rtol=1e-4, atol=1e-6)


def test_relu_corner_cases():
    # pre-activation exactly zero and negative zero both come out as +0
    I = np.array([[1.0, -1.0]], np.float32)
    W = np.array([[1.0, 1.0], [-1.0, -1.0]], np.float32)
    got = oracle.mlp_fcrelu(I, [W], [np.zeros(2, np.float32)])[0]
    assert np.array_equal(got, np.zeros((1, 2)))
    assert not np.any(np.signbit(got))


def test_bad_shapes():
    I, Ws, bs = inputs.make_mlp(2, (3, 4, 2), seed=1)
    with pytest.raises(ValueError):
        oracle.mlp_fcrelu(I, Ws[::-1], bs[::-1])
    with pytest.raises(ValueError):
        oracle.mlp_fcrelu(I, Ws, bs[:1])
    assert oracle.mlp_fcrelu(I[:0], Ws, bs)[1].shape == (0, 2)


def test_planted_mistakes_are_caught():
    I, Ws, bs = inputs.make_mlp(3, (5, 4, 3), seed=4, w_std=0.8, b_std=0.8)
    good = _brute(I, Ws, bs)
    x = I.astype(np.float64)
    no_bias = np.maximum(x @ Ws[0].astype(np.float64).T, 0.0)
    no_relu = x @ Ws[0].astype(np.float64).T + bs[0]
    assert not np.allclose(no_bias, good[0], rtol=1e-9)
    assert not np.allclose(no_relu, good[0], rtol=1e-9)
    got = oracle.mlp_fcrelu(I, Ws, bs)
    np.testing.assert_allclose(got[0], good[0], rtol=1e-14, atol=1e-16)
