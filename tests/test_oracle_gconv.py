"""Pins for the oracle's grouped convolution (Section 7, listing gconv; Section 3.1 ranges)."""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle
from paper_1802_04730_amd import inputs


def _brute(I, W1, bias):
    N, G, C, H, W = I.shape
    _, F, _, KH, KW = W1.shape
    OH, OW = H - KH + 1, W - KW + 1
    O = np.zeros((N, G, F, OH, OW))
    for n, g, o, h, w in itertools.product(range(N), range(G), range(F), range(OH), range(OW)):
        s = 0.0
        for i, kh, kw in itertools.product(range(C), range(KH), range(KW)):
            s += float(I[n, g, i, h + kh, w + kw]) * float(W1[g, o, i, kh, kw])
        O[n, g, o, h, w] = s + (float(bias[g * F + o]) if bias is not None else 0.0)
    return O


def _torch_conv(I, W1, bias):
    N, G, C, H, W = I.shape
    _, F, _, KH, KW = W1.shape
    x = torch.from_numpy(I).double().reshape(N, G * C, H, W)
    w = torch.from_numpy(W1).double().reshape(G * F, C, KH, KW)
    b = torch.from_numpy(bias).double() if bias is not None else None
    y = torch.nn.functional.conv2d(x, w, b, groups=G)
    return y.reshape(N, G, F, H - KH + 1, W - KW + 1).numpy()


def test_brute_force_small():
    I, W1, bias = inputs.make_gconv(1, 2, 2, 3, 5, 6, 3, 2, seed=1, w_std=0.5, b_std=0.5)
    np.testing.assert_allclose(oracle.group_conv(I, W1, bias), _brute(I, W1, bias),
                               rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(oracle.group_conv(I, W1, None), _brute(I, W1, None),
                               rtol=1e-14, atol=1e-15)


def test_exact_on_small_integers():
    r = np.random.default_rng(3)
    I = r.integers(-5, 6, size=(2, 2, 3, 6, 5)).astype(np.float32)
    W1 = r.integers(-4, 5, size=(2, 2, 3, 3, 3)).astype(np.float32)
    b = r.integers(-7, 8, size=(4,)).astype(np.float32)
    want = _brute(I, W1, b)  # integer-valued doubles: exact
    assert np.array_equal(oracle.group_conv(I, W1, b), want)
    assert np.array_equal(want, np.round(want))


@pytest.mark.parametrize("shape", [(2, 4, 16, 16, 12, 11, 3, 3), (1, 3, 5, 7, 9, 8, 2, 4),
                                   (2, 2, 4, 4, 7, 7, 3, 3)])
def test_matches_torch_grouped_conv2d(shape, oracle_threads):
    I, W1, bias = inputs.make_gconv(*shape, seed=5)
    np.testing.assert_allclose(oracle.group_conv(I, W1, bias), _torch_conv(I, W1, bias),
                               rtol=1e-12, atol=1e-13)


def test_benchmark_shape_slice_matches_torch(oracle_threads):
    c = dict(inputs.CONFIGS[4]); c.pop("op"); c["N"] = 1; c["G"] = 4
    I, W1, bias = inputs.make_gconv(seed=inputs.SEED_BASE + 4, **c)
    got = oracle.group_conv(I, W1, bias)
    assert got.shape == (1, 4, 16, 56, 56)
    np.testing.assert_allclose(got, _torch_conv(I, W1, bias), rtol=1e-12, atol=1e-13)


def test_one_group_is_ordinary_convolution_plus_bias():
    # G = 1: the listing reduces to conv2d (Section 3) followed by the bias statement
    I, W1, bias = inputs.make_gconv(2, 1, 3, 4, 8, 7, 3, 3, seed=6, w_std=0.3)
    x = torch.from_numpy(I[:, 0]).double()
    w = torch.from_numpy(W1[0]).double()
    y = torch.nn.functional.conv2d(x, w) + torch.from_numpy(bias).double().view(1, -1, 1, 1)
    np.testing.assert_allclose(oracle.group_conv(I, W1, bias)[:, 0], y.numpy(),
                               rtol=1e-12, atol=1e-13)


def test_groups_do_not_mix():
    I, W1, bias = inputs.make_gconv(1, 3, 2, 2, 6, 6, 3, 3, seed=7, w_std=0.3)
    full = oracle.group_conv(I, W1, bias)
    for g in range(3):
        one = oracle.group_conv(I[:, g:g + 1], W1[g:g + 1], bias[2 * g:2 * g + 2])
        np.testing.assert_array_equal(full[:, g], one[:, 0])


def test_pointwise_filter_is_per_group_matmul():
    I, W1, bias = inputs.make_gconv(2, 3, 4, 5, 6, 7, 1, 1, seed=8, w_std=0.3)
    want = np.einsum("ngchw,gfc->ngfhw", I.astype(np.float64), W1[..., 0, 0].astype(np.float64))
    want += bias.astype(np.float64).reshape(1, 3, 5, 1, 1)
    np.testing.assert_allclose(oracle.group_conv(I, W1, bias), want, rtol=1e-13, atol=1e-14)


def test_delta_filter_copies_a_shifted_channel():
    I, _, _ = inputs.make_gconv(1, 2, 3, 2, 7, 8, 3, 3, seed=9)
    W1 = np.zeros((2, 2, 3, 3, 3), np.float32)
    W1[0, 1, 2, 1, 2] = 1.0  # group 0, output 1 <- channel 2 shifted by (1,2)
    W1[1, 0, 0, 2, 0] = 1.0  # group 1, output 0 <- channel 0 shifted by (2,0)
    O = oracle.group_conv(I, W1, None)
    assert np.array_equal(O[0, 0, 1], I[0, 0, 2, 1:6, 2:8].astype(np.float64))
    assert np.array_equal(O[0, 1, 0], I[0, 1, 0, 2:7, 0:6].astype(np.float64))
    assert np.all(O[0, 0, 0] == 0) and np.all(O[0, 1, 1] == 0)


def test_bias_index_is_output_channel():
    I = np.zeros((1, 2, 1, 3, 3), np.float32)
    W1 = np.zeros((2, 3, 1, 3, 3), np.float32)
    bias = np.arange(6, dtype=np.float32)
    O = oracle.group_conv(I, W1, bias)
    assert np.array_equal(O[0, :, :, 0, 0], np.arange(6.0).reshape(2, 3))


def test_output_extents_from_paper():
    path = os.path.join(os.path.dirname(__file__), "golden", "range_inference.txt")
    seen = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        _, n_in, n_f, n_out = line.split('"')[0].split()
        n_in, n_f, n_out = int(n_in), int(n_f), int(n_out)
        assert oracle.group_conv_infer(n_in, n_in, n_f, n_f) == (n_out, n_out)
        I = np.zeros((1, 1, 1, n_in, n_in + 1), np.float32)
        W1 = np.zeros((1, 1, 1, n_f, n_f), np.float32)
        assert oracle.group_conv(I, W1).shape == (1, 1, 1, n_out, n_out + 1)
        seen += 1
    assert seen >= 5


def test_filter_larger_than_input_is_rejected():
    with pytest.raises(ValueError):
        oracle.group_conv_infer(2, 5, 3, 3)
    with pytest.raises(ValueError):
        oracle.group_conv(np.zeros((1, 1, 1, 2, 5), np.float32), np.zeros((1, 1, 1, 3, 3), np.float32))


def test_planted_mistakes_are_caught():
    I, W1, bias = inputs.make_gconv(1, 2, 2, 3, 5, 6, 3, 2, seed=1, w_std=0.5, b_std=0.5)
    good = _brute(I, W1, bias)
    flipped = _brute(I, W1[..., ::-1, ::-1].copy(), bias)           # correlation vs true convolution
    swapped = _brute(I, W1, bias[::-1].copy())                      # wrong bias index
    mixed = _brute(I[:, ::-1].copy(), W1, bias)                     # groups crossed
    for bad in (flipped, swapped, mixed):
        assert not np.allclose(bad, good, rtol=1e-9)
