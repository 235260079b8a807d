"""The numerical scheme of the int8 grouped convolution, emulated in numpy and held against the float64 oracle.

Not the kernel (that is tests/test_gpu_parity.py): this pins the error budget the kernel's tolerance is derived from.
Operands are scaled per block (filter row / band of 10 input rows) by a power of two to 31-bit fixed point, cut
into four signed 8-bit digits, the digit products with k + l >= 2 are summed exactly in integers, and the sum is
scaled back.  The emulation follows that description with integer numpy arrays and nothing else.
"""
import numpy as np
import pytest

import oracle
from paper_1802_04730_amd import inputs
from paper_1802_04730_amd.metric import PARITY_BAR, parity_error


def digits(v):
    """Four signed base-256 digits of an integer array, |v| <= 2^30, least significant first."""
    vp = v + 0x00808080
    d = [((vp >> (8 * k)) & 0xFF) - 128 for k in range(3)] + [vp >> 24]
    assert all(np.all((x >= -128) & (x <= 127)) for x in d)
    assert np.all(sum(d[k].astype(np.int64) << (8 * k) for k in range(4)) == v)
    return d


def exponent_above(m):
    """Smallest e with m < 2^e (m > 0)."""
    return np.frexp(m)[1]


def emulate(I, W1, bias, min_diagonal, rows=8):
    N, G, C, H, W = I.shape
    F, KH, KW = W1.shape[1], W1.shape[3], W1.shape[4]
    OH, OW = H - KH + 1, W - KW + 1
    out = np.zeros((N, G, F, OH, OW))
    worst_partial = 0
    for n in range(N):
        for g in range(G):
            wf = W1[g].reshape(F, -1).astype(np.float64)
            ea = exponent_above(np.abs(wf).max(axis=1))
            da = digits(np.rint(np.ldexp(wf, (30 - ea)[:, None])).astype(np.int64))
            for h0 in range(0, OH, rows):
                band = I[n, g, :, h0:h0 + rows + KH - 1, :].astype(np.float64)
                eb = exponent_above(np.abs(band).max())
                db = digits(np.rint(np.ldexp(band, 30 - eb)).astype(np.int64))
                total = np.zeros((F, band.shape[1] - KH + 1, OW), dtype=object)  # exact python integers
                for k in range(4):
                    wk = da[k].reshape(F, C, KH, KW)
                    for l in range(4):
                        if k + l < min_diagonal:
                            continue
                        acc = np.zeros(total.shape, dtype=np.int64)
                        for kh in range(KH):
                            for kw in range(KW):
                                acc += np.einsum("fc,chw->fhw", wk[:, :, kh, kw], db[l][:, kh:kh + total.shape[1], kw:kw + OW])
                        worst_partial = max(worst_partial, int(np.abs(acc).max()))
                        total = total + acc.astype(object) * (256 ** (k + l))
                val = np.ldexp(total.astype(np.float64), (ea + eb - 60)[:, None, None].astype(np.int32))
                out[n, g, :, h0:h0 + total.shape[1], :] = val + bias.reshape(G, F)[g][:, None, None]
    return out.astype(np.float32).astype(np.float64), worst_partial


@pytest.fixture(scope="module")
def case():
    I, W1, bias = inputs.make_gconv(1, 3, 16, 16, 26, 58, 3, 3, seed=inputs.SEED_BASE + 4)
    return I, W1, bias, oracle.group_conv(I, W1, bias)


def test_thirteen_digit_products_stay_far_below_the_bar(case):
    I, W1, bias, ref = case
    got, worst = emulate(I, W1, bias, min_diagonal=2)
    err = parity_error(got, ref)
    assert err <= 2e-6 and err <= PARITY_BAR / 10, err
    assert 4 * worst < 2 ** 31, "a diagonal of up to four digit pairs must fit an int32 accumulator"


def test_ten_digit_products_would_not_leave_a_margin(case):
    """Dropping the diagonal k + l = 2 as well costs 2^8 in accuracy: about half the bar, no margin to speak of."""
    I, W1, bias, ref = case
    got, _ = emulate(I, W1, bias, min_diagonal=3)
    assert parity_error(got, ref) > PARITY_BAR / 10


def test_digit_decomposition_round_trips():
    rng = np.random.default_rng(1)
    v = rng.integers(-(2 ** 30), 2 ** 30, size=100000, dtype=np.int64)
    v[:4] = [2 ** 30, -(2 ** 30), 0, -1]
    d = digits(v)
    assert np.abs(d[3]).max() <= 64
