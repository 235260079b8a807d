"""GPU parity of the strided convolution and the lookup-table sums (through the C ABI) against the float64 oracle.

Same bar and same tight bound as the other fp64 kernels: one fp32 rounding of the exact result.  Strided
convolutions with a multiple of 32 filters and at least 256 taps (a multiple of 4) run on the int8 matrix core
(tc355_last_path says "sconv:i8"); their bound is the int8 scheme's (tests/test_i8_scheme.py derives the budget).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_1802_04730_amd import inputs
from paper_1802_04730_amd.metric import PARITY_BAR, parity_error

pytestmark = pytest.mark.gpu

TIGHT = 2.5e-7
TIGHT_I8 = 4e-6


@pytest.fixture(scope="module")
def tc():
    from paper_1802_04730_amd import tc355
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    tc355.lib()
    return tc355


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check(gpu_tensor, ref, what, tight=TIGHT):
    torch.cuda.synchronize()
    got = gpu_tensor.cpu().numpy().astype(np.float64)
    err = parity_error(got, ref)
    print("%s: parity error %.3e" % (what, err), flush=True)
    assert err <= PARITY_BAR, "%s: %.3e exceeds the parity bar" % (what, err)
    assert err <= tight, "%s: %.3e exceeds the error this kernel's arithmetic allows (%.1e)" % (what, err, tight)


# ---------------------------------------------------------------- sconv2d
# (N, C, F, H, W, KH, KW, sh, sw)
SCONV_SHAPES = [
    (2, 16, 24, 23, 21, 3, 3, 2, 2),     # reduction 144: four whole chunks and a half; ragged filter and pixel tiles
    (1, 5, 7, 19, 30, 4, 2, 3, 2),       # reduction 40: one whole chunk and a ragged one of 8 taps
    (3, 3, 70, 12, 13, 3, 3, 1, 1),      # reduction 27: scalar filter loads; two filter tiles, the second ragged
    (2, 8, 8, 15, 15, 1, 1, 2, 2),       # 1 x 1 filter: pure subsampling plus channel mixing, one short chunk
    (1, 3, 4, 12, 12, 7, 7, 2, 2),       # 7 x 7 stride 2 (the first layer of residual networks), reduction 147
    (1, 1, 1, 3, 3, 3, 3, 5, 5),         # a single output element
    (4, 64, 80, 20, 20, 3, 3, 2, 2),     # many chunks (reduction 576), 64 x 64 blocks, the second filter block a quarter full
    (2, 28, 128, 20, 20, 3, 3, 1, 1),    # 128 filters but only 252 taps: below the int8 kernel's two blocks
    (1, 2048, 128, 4, 3, 3, 3, 1, 1),    # 18432 taps: the int8 kernel's table of tap offsets would not fit LDS
    (2, 6, 10, 9, 40, 2, 5, 1, 4),       # wide stride along w only
]


@pytest.mark.parametrize("shape", SCONV_SHAPES)
def test_sconv2d(tc, shape, oracle_threads):
    N, C, F, H, W, KH, KW, sh, sw = shape
    I, Wt, bias = inputs.make_sconv2d(N, C, F, H, W, KH, KW)
    ref = oracle.sconv2d(I, Wt, bias, sh, sw)
    O = torch.full(ref.shape, float("nan"), device="cuda")
    tc.tc_sconv2d(dev(I), dev(Wt), dev(bias), O, sh, sw)
    assert tc.last_path() == "sconv:tile"  # (every entry point names its kernel family, not only the step's)
    check(O, ref, "sconv2d %s" % (shape,))


# Shapes of the int8 kernel: 128 (or 64) filters x 16 NT pixels per workgroup, NT chosen from the number of pixel tiles
# per compute unit; reduction in blocks of 128 taps.  (N, C, F, H, W, KH, KW, sh, sw)
SCONV_I8_SHAPES = [
    (2, 64, 128, 31, 29, 3, 3, 2, 2),     # reduction 576: four blocks and a half one (a single MFMA step); 420 pixels: NT = 1, ragged
    (3, 32, 128, 20, 23, 3, 3, 1, 1),     # reduction 288: two blocks and 32 taps; 1134 pixels
    (1, 128, 256, 17, 17, 3, 3, 2, 2),    # two blocks of filters; reduction 1152: nine whole blocks; 64 pixels
    (2, 36, 128, 40, 41, 3, 3, 3, 2),     # reduction 324 (not a multiple of 16); strides 3 and 2
    (3, 32, 256, 34, 34, 3, 3, 1, 1),     # 3072 pixels for 128 compute units per filter block: NT = 2
    (5, 32, 256, 34, 35, 3, 3, 1, 1),     # 5280 pixels: NT = 3, the last workgroup ragged
    (7, 32, 256, 34, 34, 3, 3, 1, 1),     # 7168 pixels: NT = 4
    (1, 32, 128, 3, 3, 3, 3, 1, 1),       # one output pixel per filter
    (2, 256, 128, 9, 11, 1, 1, 2, 1),     # 1 x 1 filters: channel mixing and subsampling, two whole blocks
    (1, 12, 128, 21, 20, 7, 7, 2, 2),     # 7 x 7 stride 2: reduction 588
    (2, 20, 128, 14, 19, 5, 3, 1, 2),     # 5 x 3 filters: reduction 300
    (2, 64, 64, 20, 21, 3, 3, 1, 1),      # 64 filters: workgroups of 64 filters x 32 pixels (NT = 2), four and a half blocks
    (8, 32, 64, 40, 40, 3, 3, 1, 1),      # 64 filters, 11552 pixels: NT = 4
    (6, 32, 192, 34, 34, 3, 3, 1, 1),     # 192 filters = three blocks of 64, 85 compute units each: NT = 6
    (20, 32, 64, 40, 40, 3, 3, 1, 1),     # 64 filters, 28880 pixels: NT = 8, the last workgroup ragged
    (1, 72, 320, 9, 9, 2, 2, 1, 2),       # 320 filters = five blocks of 64; 2 x 2 filters
    (2, 32, 32, 20, 21, 3, 3, 1, 1),      # 32 filters: workgroups of 32 filters x 64 pixels, four wavefronts stage the filters
    (6, 32, 96, 30, 30, 3, 3, 2, 1),      # 96 filters = three blocks of 32; 5880 pixels: NT = 8
    (1, 1900, 128, 3, 4, 3, 3, 1, 1),     # 17100 taps: 134 blocks, the longest reduction the kernel takes at 128 filters
]


@pytest.mark.parametrize("shape", SCONV_I8_SHAPES)
def test_sconv2d_int8_kernel(tc, shape, oracle_threads):
    N, C, F, H, W, KH, KW, sh, sw = shape
    I, Wt, bias = inputs.make_sconv2d(N, C, F, H, W, KH, KW, seed=inputs.SEED_BASE + 60 + C)
    ref = oracle.sconv2d(I, Wt, bias, sh, sw)
    n = ref.size
    buf = torch.full((n + 512,), 7.0, device="cuda")
    O = buf[256:256 + n].view(ref.shape)
    tc.tc_sconv2d(dev(I), dev(Wt), dev(bias), O, sh, sw)
    assert tc.last_path() == "sconv:i8"
    check(O, ref, "sconv2d int8 %s" % (shape,), TIGHT_I8)
    assert torch.all(buf[:256] == 7.0) and torch.all(buf[256 + n:] == 7.0)
    # without a bias; the fp64 kernel by option; ten digit products by option
    ref0 = oracle.sconv2d(I, Wt, None, sh, sw)
    O0 = torch.full(ref.shape, float("nan"), device="cuda")
    tc.tc_sconv2d(dev(I), dev(Wt), None, O0, sh, sw)
    check(O0, ref0, "sconv2d int8 %s, no bias" % (shape,), TIGHT_I8)
    with tc.option(tc.TC_OPT_INT8, tc.TC_INT8_OFF):
        tc.tc_sconv2d(dev(I), dev(Wt), dev(bias), O0, sh, sw)
        assert tc.last_path() == "sconv:tile"
    check(O0, ref, "sconv2d %s, fp64 kernel by option" % (shape,))
    with tc.option(tc.TC_OPT_INT8, tc.TC_INT8_TEN):
        tc.tc_sconv2d(dev(I), dev(Wt), dev(bias), O0, sh, sw)
        assert tc.last_path() == "sconv:i8"
    check(O0, ref, "sconv2d int8 %s, 10 products" % (shape,), TIGHT_I8)


@pytest.mark.parametrize("kind", ["lognormal", "student3", "sparse"])
def test_sconv2d_int8_heavy_tailed_operands_stay_a_quarter_of_the_bar(tc, oracle_threads, kind):
    """A few large elements in every block of taps of the filters AND of the pixels: the default (13 digit products)
    keeps a quarter of the bar over four seeds."""
    for seed in range(4):
        I, Wt, bias = inputs.make_sconv2d(2, 64, 128, 25, 27, 3, 3, seed=70 + seed)
        rng = np.random.default_rng(9 + seed)
        if kind == "lognormal":
            mag = lambda a: np.exp(rng.normal(size=a.shape) * 1.5)
        elif kind == "student3":
            mag = lambda a: np.abs(rng.standard_t(3, size=a.shape))
        else:
            mag = lambda a: np.where(rng.random(a.shape) < 0.01, 300.0, 1.0)
        I, Wt = (I * mag(I)).astype(np.float32), (Wt * mag(Wt)).astype(np.float32)
        ref = oracle.sconv2d(I, Wt, bias, 2, 1)
        O = torch.full(ref.shape, float("nan"), device="cuda")
        tc.tc_sconv2d(dev(I), dev(Wt), dev(bias), O, 2, 1)
        assert tc.last_path() == "sconv:i8"
        torch.cuda.synchronize()
        err = parity_error(O.cpu().numpy().astype(np.float64), ref)
        print("sconv2d int8, %s magnitudes, seed %d: parity error %.3e" % (kind, seed, err), flush=True)
        assert err <= PARITY_BAR / 4


def test_sconv2d_int8_nan_stays_in_the_outputs_that_read_it(tc, oracle_threads):
    """A NaN in one input element: exactly the outputs whose windows hold it are NaN (all filters), the others keep
    their values.  A NaN in one filter: all outputs of that filter, and no other."""
    N, C, F, H, W = 2, 32, 128, 15, 17
    I, Wt, bias = inputs.make_sconv2d(N, C, F, H, W, 3, 3, seed=81)
    ref = oracle.sconv2d(I, Wt, bias, 2, 2)
    In = I.copy()
    In[1, 5, 6, 8] = np.nan                       # rows 6 = 2*2 + 2 = 2*3 + 0, columns 8 = 2*3 + 2 = 2*4 + 0
    O = torch.full(ref.shape, 0.0, device="cuda")
    tc.tc_sconv2d(dev(In), dev(Wt), dev(bias), O, 2, 2)
    assert tc.last_path() == "sconv:i8"
    got = O.cpu().numpy().astype(np.float64)
    hit = np.zeros(ref.shape, dtype=bool)
    hit[1, :, 2:4, 3:5] = True
    assert np.isnan(got[hit]).all() and not np.isnan(got[~hit]).any()
    assert parity_error(np.where(hit, ref, got), ref) <= TIGHT_I8
    Wn = Wt.copy()
    Wn[77, 3, 1, 2] = np.nan
    tc.tc_sconv2d(dev(I), dev(Wn), dev(bias), O, 2, 2)
    got = O.cpu().numpy().astype(np.float64)
    hit = np.zeros(ref.shape, dtype=bool)
    hit[:, 77] = True
    assert np.isnan(got[hit]).all() and not np.isnan(got[~hit]).any()
    assert parity_error(np.where(hit, ref, got), ref) <= TIGHT_I8


def test_sconv2d_without_bias_and_unit_strides_match_group_conv(tc, oracle_threads):
    I, Wt, _ = inputs.make_sconv2d(2, 16, 16, 18, 20, 3, 3)
    ref = oracle.sconv2d(I, Wt, None, 1, 1)
    O = torch.full(ref.shape, float("nan"), device="cuda")
    tc.tc_sconv2d(dev(I), dev(Wt), None, O, 1, 1)
    check(O, ref, "sconv2d no bias, unit strides")
    O2 = torch.full((2, 1, 16, 16, 18), float("nan"), device="cuda")
    tc.tc_group_conv(dev(I[:, None]), dev(Wt[None]), None, O2)
    torch.cuda.synchronize()
    assert torch.equal(O2[:, 0], O)  # both round the exact fp64 sum once


def test_sconv2d_resnext_like_full_size_sampled(tc, oracle_threads):
    # a down-sampling layer of the size class the paper's grouped convolutions come from: 64 -> 128 channels,
    # 56 x 56 -> 27 x 27, batch 32; the oracle evaluates two images
    N, C, F, H, W = 32, 64, 128, 56, 56
    I, Wt, bias = inputs.make_sconv2d(N, C, F, H, W, 3, 3)
    O = torch.full((N, F, 27, 27), float("nan"), device="cuda")
    tc.tc_sconv2d(dev(I), dev(Wt), dev(bias), O, 2, 2)
    assert tc.last_path() == "sconv:i8"
    torch.cuda.synchronize()
    assert not torch.isnan(O).any()
    for n in (0, 31):
        check(O[n:n + 1], oracle.sconv2d(I[n:n + 1], Wt, bias, 2, 2), "sconv2d full size, image %d" % n, TIGHT_I8)
    # every workgroup's output: the whole result against the fp64 kernel's, which the same two images pin to the oracle
    O64 = torch.full((N, F, 27, 27), float("nan"), device="cuda")
    with tc.option(tc.TC_OPT_INT8, tc.TC_INT8_OFF):
        tc.tc_sconv2d(dev(I), dev(Wt), dev(bias), O64, 2, 2)
        assert tc.last_path() == "sconv:tile"
    for n in (0, 31):
        check(O64[n:n + 1], oracle.sconv2d(I[n:n + 1], Wt, bias, 2, 2), "sconv2d full size, fp64 kernel, image %d" % n)
    check(O, O64.cpu().numpy().astype(np.float64), "sconv2d full size, int8 against fp64 kernel, all images", TIGHT_I8)


def test_sconv2d_stays_inside_its_output(tc, oracle_threads):
    N, C, F, H, W = 3, 5, 9, 11, 13
    I, Wt, bias = inputs.make_sconv2d(N, C, F, H, W, 3, 3)
    ref = oracle.sconv2d(I, Wt, bias, 2, 3)
    n = ref.size
    buf = torch.full((n + 512,), 7.0, device="cuda")
    O = buf[256:256 + n].view(ref.shape)
    tc.tc_sconv2d(dev(I), dev(Wt), dev(bias), O, 2, 3)
    check(O, ref, "sconv2d guard band")
    assert torch.all(buf[:256] == 7.0) and torch.all(buf[256 + n:] == 7.0)


# ---------------------------------------------------------------- lookup tables
# (E, D, B, L)
LUT_SHAPES = [
    (1000, 64, 128, 50),     # the paper's D, B, L on a small table: many repeated rows
    (5000, 64, 3, 1),        # one lookup per row: a gather
    (777, 20, 9, 13),        # D = 20: five 16-byte units, slots beyond the lookups
    (300, 7, 11, 70),        # D not a multiple of 4: scalar loads; more lookups than one round holds
    (50, 1, 5, 3),           # a single column
    (4000, 1100, 4, 9),      # D beyond one block of 256 units: two column blocks per row
    (100000, 256, 17, 129),  # several rounds per thread
]


@pytest.mark.parametrize("shape", LUT_SHAPES)
def test_lut_one_table(tc, shape, oracle_threads):
    E, D, B, L = shape
    LUT, Idx = inputs.make_lut(E, D, B, L)
    ref = oracle.lut(LUT, Idx)
    O = torch.full((B, D), float("nan"), device="cuda")
    tc.tc_lut([dev(LUT)], [dev(Idx)], [O])
    assert tc.last_path() == "lut:sum"
    check(O, ref, "lut %s" % (shape,))


def test_lut_two_tables_one_launch(tc, oracle_threads):
    # listing 2LUT: two tables of different heights and lookup counts, one output width and batch
    LUT1, Idx1 = inputs.make_lut(30000, 64, 128, 50, seed=inputs.SEED_BASE + 7)
    LUT2, Idx2 = inputs.make_lut(1234, 64, 128, 31, seed=inputs.SEED_BASE + 8)
    O1 = torch.full((128, 64), float("nan"), device="cuda")
    O2 = torch.full((128, 64), float("nan"), device="cuda")
    tc.tc_lut([dev(LUT1), dev(LUT2)], [dev(Idx1), dev(Idx2)], [O1, O2])
    check(O1, oracle.lut(LUT1, Idx1), "2LUT first table")
    check(O2, oracle.lut(LUT2, Idx2), "2LUT second table")


def test_lut_paper_size(tc, oracle_threads):
    # (E, D, L) = (10^7, 64, 50), B = 128 (Section 7, production models): a 2.56 GB table.  The second table is the
    # negated first one (a second 2.56 GB draw would only cost host time); its indices are drawn separately.
    E, D, B, L = 10**7, 64, 128, 50
    LUT, Idx1 = inputs.make_lut(E, D, B, L)
    Idx2 = inputs.make_lut_indices(E, B, L, seed=inputs.SEED_BASE + 8)
    T1 = dev(LUT)
    T2 = -T1
    O1 = torch.full((B, D), float("nan"), device="cuda")
    O2 = torch.full((B, D), float("nan"), device="cuda")
    tc.tc_lut([T1, T2], [dev(Idx1), dev(Idx2)], [O1, O2])
    check(O1, oracle.lut(LUT, Idx1), "2LUT paper size, first table")
    check(O2, -oracle.lut(LUT, Idx2), "2LUT paper size, second table")


def test_lut_index_outside_the_table_gives_nan_rows_only(tc, oracle_threads):
    E, D, B, L = 500, 64, 6, 10
    LUT, Idx = inputs.make_lut(E, D, B, L)
    ref = oracle.lut(LUT, Idx)
    bad = Idx.copy()
    bad[1, 3] = E          # one past the end
    bad[4, 0] = -1
    O = torch.full((B, D), 3.0, device="cuda")
    tc.tc_lut([dev(LUT)], [dev(bad)], [O])
    torch.cuda.synchronize()
    got = O.cpu().numpy()
    assert np.all(np.isnan(got[[1, 4]]))
    keep = [0, 2, 3, 5]
    assert parity_error(got[keep].astype(np.float64), ref[keep]) <= TIGHT


def test_lut_stays_inside_its_output(tc, oracle_threads):
    E, D, B, L = 300, 12, 7, 5
    LUT, Idx = inputs.make_lut(E, D, B, L)
    buf = torch.full((B * D + 512,), 7.0, device="cuda")
    O = buf[256:256 + B * D].view(B, D)
    tc.tc_lut([dev(LUT)], [dev(Idx)], [O])
    check(O, oracle.lut(LUT, Idx), "lut guard band")
    assert torch.all(buf[:256] == 7.0) and torch.all(buf[256 + B * D:] == 7.0)


# ---------------------------------------------------------------- both operators from a HIP graph
def test_sconv2d_and_lut_replay_from_a_hip_graph(tc, oracle_threads):
    # Both entry points enqueue one kernel and nothing else, so they can be captured and replayed; replays are
    # interleaved with eager work and every one is checked.
    I, Wt, bias = inputs.make_sconv2d(2, 16, 24, 23, 21, 3, 3, seed=31)
    LUT1, Idx1 = inputs.make_lut(3000, 64, 32, 50, seed=32)
    LUT2, Idx2 = inputs.make_lut(500, 64, 32, 7, seed=33)
    ref_s = oracle.sconv2d(I, Wt, bias, 2, 2)
    ref_1, ref_2 = oracle.lut(LUT1, Idx1), oracle.lut(LUT2, Idx2)
    Id, Wd, bd = dev(I), dev(Wt), dev(bias)
    T = [dev(LUT1), dev(LUT2)]
    J = [dev(Idx1), dev(Idx2)]
    Os = torch.empty(ref_s.shape, device="cuda")
    O1, O2 = torch.empty((32, 64), device="cuda"), torch.empty((32, 64), device="cuda")

    I8, W8, b8 = inputs.make_sconv2d(2, 32, 128, 14, 15, 3, 3, seed=34)  # the int8 kernel
    ref_8 = oracle.sconv2d(I8, W8, b8, 1, 2)
    I8d, W8d, b8d = dev(I8), dev(W8), dev(b8)
    O8 = torch.empty(ref_8.shape, device="cuda")

    def step():
        tc.tc_sconv2d(Id, Wd, bd, Os, 2, 2)
        tc.tc_sconv2d(I8d, W8d, b8d, O8, 1, 2)
        tc.tc_lut(T, J, [O1, O2])

    step()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep in range(3):
        for t in (Os, O8, O1, O2):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        scratch = torch.randn(1 << 20, device="cuda").sum()  # eager work between replays
        torch.cuda.synchronize()
        check(Os, ref_s, "graph replay %d sconv2d" % rep)
        check(O8, ref_8, "graph replay %d sconv2d, int8 kernel" % rep, TIGHT_I8)
        check(O1, ref_1, "graph replay %d lut 1" % rep)
        check(O2, ref_2, "graph replay %d lut 2" % rep)
        del scratch


# ---------------------------------------------------------------- every entry point, seeded random shapes
def test_seeded_random_shapes_through_every_entry_point(tc, oracle_threads):
    """A seeded draw of shapes for all six entry points (ragged extents, shapes on both sides of every dispatch rule),
    each checked element by element against the oracle, with a guard band around every output.  The bound is the one
    of the arithmetic that ran (tc355_last_path): a quarter of the bar on the int8 paths, one fp32 rounding elsewhere."""
    rng = np.random.default_rng(413)
    ri = lambda a, b: int(rng.integers(a, b + 1))
    pick = lambda xs: xs[int(rng.integers(0, len(xs)))]
    f32 = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    GUARD = 64

    def guarded(shape):
        n = int(np.prod(shape))
        buf = torch.full((n + 2 * GUARD,), 777.0, device="cuda")
        return buf, buf[GUARD:GUARD + n].view(shape)

    def verify(buf, out, ref, what):
        tight = PARITY_BAR / 4 if ":i8" in tc.last_path() else TIGHT
        check(out, ref, "%s on %s" % (what, tc.last_path()), tight=tight)
        n = out.numel()
        assert bool((buf[:GUARD] == 777.0).all()) and bool((buf[GUARD + n:] == 777.0).all()), what + ": wrote outside its output"

    paths = set()
    for it in range(10):
        # transposed batched matmul: small per-batch matrices, mid-sized ones, long reductions
        B, N, M, K = [(ri(1, 300), ri(1, 40), ri(1, 90), pick([4, 12, 26, 28, 64, 100])), (ri(1, 3), ri(1, 150), ri(1, 200), ri(1, 200)),
                      (1, 128, 64 * ri(1, 12), 128 * ri(1, 4))][it % 3]
        X, Y = f32(rng.standard_normal((B, N, K))), f32(rng.standard_normal((B, M, K)))
        buf, Z = guarded((B, N, M))
        tc.tc_tbmm(dev(X), dev(Y), Z)
        paths.add(tc.last_path())
        verify(buf, Z, oracle.tbmm(X, Y), "tbmm %s" % ((B, N, M, K),))
        # Kronecker layer: the LDS kernel's factors of 64 with a ragged I, and anything else
        Bk, Ik, Kk, Jk, Lk = (ri(1, 40), ri(1, 130), 64, 64, 64) if it % 2 == 0 else (ri(1, 12), ri(1, 40), ri(1, 40), ri(1, 40), ri(1, 40))
        W1, W2, Xk = f32(rng.standard_normal((Ik, Kk)) / 8), f32(rng.standard_normal((Jk, Lk)) / 8), f32(rng.standard_normal((Bk, Kk, Lk)))
        buf, Yk = guarded((Bk, Ik, Jk))
        tc.tc_kron(dev(W1), dev(W2), dev(Xk), Yk)
        paths.add(tc.last_path())
        verify(buf, Yk, oracle.kron(W1, W2, Xk), "kron %s" % ((Bk, Ik, Kk, Jk, Lk),))
        # grouped convolution: the three int8 geometries, the small-channel ones, anything else
        gk = it % 5
        if gk == 0: shp = (ri(1, 2), ri(1, 3), 16, 16, 8 * ri(1, 4) + 2, 58, 3, 3)
        elif gk == 1: shp = (4, ri(1, 3), 16, 16, 14, 14, 3, 3)
        elif gk == 2: shp = (4, ri(1, 3), 32, 32, 7, 7, 3, 3)
        elif gk == 3: shp = (ri(1, 3), ri(1, 3)) + pick([(4, 4, 56, 56), (8, 8, 28, 28)]) + (3, 3)
        else: shp = (ri(1, 3), ri(1, 4), ri(1, 20), ri(1, 20), ri(3, 24), ri(3, 24), ri(1, 3), ri(1, 3))
        N_, G, C, F, H, W, KH, KW = shp
        I, Wg, bg = inputs.make_gconv(N_, G, C, F, H, W, KH, KW, seed=1000 + it)
        buf, Og = guarded((N_, G, F, H - KH + 1, W - KW + 1))
        tc.tc_group_conv(dev(I), dev(Wg), dev(bg), Og)
        paths.add(tc.last_path())
        verify(buf, Og, oracle.group_conv(I, Wg, bg), "gconv %s" % (shp,))
        # strided convolution
        if it % 2 == 0: shp = (ri(1, 3), ri(1, 30), ri(1, 100), ri(5, 30), ri(5, 30), ri(1, 4), ri(1, 4), ri(1, 3), ri(1, 3))
        else: shp = (ri(1, 3), 4 * ri(8, 24), 32 * ri(1, 6), ri(5, 30), ri(5, 30), ri(3, 4), ri(3, 4), ri(1, 3), ri(1, 3))  # the int8 kernel's range
        N_, C, F, H, W, KH, KW, sh, sw = shp
        Is, Wt, bs_ = inputs.make_sconv2d(N_, C, F, H, W, KH, KW, seed=2000 + it)
        ref = oracle.sconv2d(Is, Wt, bs_, sh, sw)
        buf, Os = guarded(ref.shape)
        tc.tc_sconv2d(dev(Is), dev(Wt), dev(bs_), Os, sh, sw)
        paths.add(tc.last_path())
        verify(buf, Os, ref, "sconv2d %s" % (shp,))
        # lookup-table sums, up to four tables in one launch
        nt, Bl, D = ri(1, 4), ri(1, 150), pick([4, 16, 33, 64, 100])
        tabs = [inputs.make_lut(ri(1, 4000), D, Bl, ri(1, 50), seed=3000 + 10 * it + t) for t in range(nt)]
        Ol = [torch.full((Bl, D), float("nan"), device="cuda") for _ in range(nt)]
        tc.tc_lut([dev(t[0]) for t in tabs], [dev(t[1]) for t in tabs], Ol)
        for t in range(nt):
            check(Ol[t], oracle.lut(*tabs[t]), "lut draw %d table %d" % (it, t))
    assert {"tbmm:lds", "tbmm:wave", "kron:lds", "kron:wave", "gconv:i8", "gconv:i8_small", "gconv:i8_c32", "gconv:quad",
            "gconv:wave", "sconv:tile", "sconv:i8"} <= paths, paths
