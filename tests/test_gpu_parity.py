"""GPU parity: libtc355 (through its C ABI) against the float64 oracle, element by element.

Bar: max |gpu - ref| / (|ref| + 1e-3 max|ref|) <= 2e-5 on the same seeded inputs.
The fp64 kernels accumulate exact fp32 x fp32 products in fp64 and round each output
once, so the error they can actually show is one fp32 rounding (2^-24 ~ 6e-8 relative);
TIGHT asserts that as well, to catch a silent loss of precision long before the bar.
The int8 grouped convolution (width 58, 16 channels, 3 x 3) sums exactly but quantises
its operands to 2^-32 of their block maximum and drops the digit products below that:
TIGHT_I8 bounds both (measured 1e-6; tests/test_i8_scheme.py derives the budget).
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


def tight_for_last_call(tc):
    """The tolerance that the arithmetic of the kernel that just ran allows (asked of the library, not re-derived)."""
    path = tc.last_path()
    return TIGHT_I8 if path.split(":")[1].startswith("i8") else TIGHT


# ---------------------------------------------------------------- tbmm
TBMM_SHAPES = [
    (8, 26, 72, 26),      # configuration 1
    (500, 26, 72, 26),    # configuration 2
    (500, 26, 26, 72),    # the paper's own naming: output 26 x 26, reduction 72
    (1, 1, 1, 1),
    (3, 17, 33, 7),       # odd K: scalar loads, ragged tiles
    (2, 16, 16, 4),       # exact tiles
    (5, 40, 200, 30),     # several strips per row tile, K even but not a multiple of 4
    (1, 128, 256, 32),    # transposed matmul of Section 7 (B = 1)
    (7, 5, 81, 64),
    (40, 100, 130, 68),   # LDS-tiled kernel (>= 128 blocks): ragged 64x64 blocks, reduction not a multiple of the chunk
    (1, 128, 1024, 1024), # the paper's medium transposed matmul (M,K,N) = (128,1024,1024): split-reduction kernel
    (1, 100, 200, 260),   # split-reduction kernel: ragged 16x16 tiles, reduction tail of 4 past two chunks
    (1, 128, 4096, 96),   # LDS-tiled kernel, one batch element, three chunks
    (130, 64, 64, 4),     # LDS-tiled kernel: a single short chunk
    (1, 128, 8192, 256),  # int8 matrix-core kernel (128 rows, >= 128 blocks of 64 columns): two reduction blocks of 128
    (2, 128, 4096, 384),  # the same, two batch elements, three reduction blocks
    (3, 128, 3072, 640),
    (1, 128, 8192, 320),  # reduction not a multiple of 128: stays on the fp64 kernels
    (2, 384, 1408, 256),  # int8 kernel, three row blocks of 128 per batch element
]


@pytest.mark.parametrize("shape", TBMM_SHAPES)
def test_tbmm(tc, shape, oracle_threads):
    B, N, M, K = shape
    X, Y = inputs.make_tbmm(B, N, M, K, seed=inputs.SEED_BASE + (1 if B == 8 else 2))
    ref = oracle.tbmm(X, Y)
    Z = torch.full((B, N, M), float("nan"), device="cuda")
    tc.tc_tbmm(dev(X), dev(Y), Z)
    print("path", tc.last_path(), flush=True)
    check(Z, ref, "tbmm %s" % (shape,), tight_for_last_call(tc))


def test_tbmm_i8_blocks_of_any_magnitude_zero_rows_and_nonfinite_rows(tc, oracle_threads):
    """The int8 kernel scales every 128-element block of every row on its own: magnitudes that differ by 2^40 between
    blocks, all-zero blocks and rows, and an Inf / a NaN that must poison exactly their own output row / column."""
    B, N, M, K = 1, 128, 8192, 256
    X, Y = inputs.make_tbmm(B, N, M, K, seed=31)
    rng = np.random.default_rng(4)
    X = (X * np.exp2(rng.integers(-20, 21, size=(B, N, K // 128)).repeat(128, axis=2))).astype(np.float32)
    Y = (Y * np.exp2(rng.integers(-20, 21, size=(B, M, K // 128)).repeat(128, axis=2))).astype(np.float32)
    X[0, 5] = 0.0
    X[0, 6, 128:256] = 0.0
    Y[0, 77] = 0.0
    ref = oracle.tbmm(X, Y)
    Z = torch.full((B, N, M), float("nan"), device="cuda")
    tc.tc_tbmm(dev(X), dev(Y), Z)
    torch.cuda.synchronize()
    got = Z.cpu().numpy().astype(np.float64)
    assert np.all(got[0, 5] == 0.0) and np.all(got[0, :, 77] == 0.0)
    worst = max(parity_error(got[0, n], ref[0, n]) for n in range(N))
    print("tbmm int8, block magnitudes over 40 binades: worst output row %.3e" % worst, flush=True)
    assert worst <= PARITY_BAR / 2
    Xb, Yb = X.copy(), Y.copy()
    Xb[0, 9, 100] = np.inf
    Yb[0, 4000, 3] = np.nan
    Z2 = torch.zeros((B, N, M), device="cuda")
    tc.tc_tbmm(dev(Xb), dev(Yb), Z2)
    torch.cuda.synchronize()
    got2 = Z2.cpu().numpy()
    assert np.isnan(got2[0, 9]).all() and np.isnan(got2[0, :, 4000]).all()
    keep = np.ones((N, M), dtype=bool); keep[9] = False; keep[:, 4000] = False
    assert np.array_equal(got2[0][keep], got.astype(np.float32)[0][keep])


@pytest.mark.parametrize("shape", [(1, 128, 8192, 300), (2, 256, 4096, 1000), (1, 128, 8192, 2116)])
def test_tbmm_int8_reduction_that_is_no_multiple_of_128(tc, shape, oracle_threads):
    """The int8 kernel fills the last block of 128 with zeros: K = 300 (two blocks and 44), 1000 (seven and 104), 2116
    (sixteen and 68: long enough for the workspace form, whose slicing kernel fills the same zeros)."""
    B, N, M, K = shape
    X, Y = inputs.make_tbmm(*shape, seed=13)
    ref = oracle.tbmm(X, Y)
    Xd, Yd = dev(X), dev(Y)
    n = ref.size
    buf = torch.full((n + 512,), 7.0, device="cuda")
    Z = buf[256:256 + n].view(ref.shape)
    tc.tc_tbmm(Xd, Yd, Z)
    assert tc.last_path() == "tbmm:i8"
    check(Z, ref, "tbmm %s, int8 path" % (shape,), TIGHT_I8)
    assert torch.all(buf[:256] == 7.0) and torch.all(buf[256 + n:] == 7.0)
    need = tc.tc_tbmm_workspace_bytes(*shape)
    if need:
        assert need == B * (N // 128) * ((K + 127) // 128) * (65536 + 1024)
        ws = torch.randint(0, 255, (need + 64,), dtype=torch.uint8, device="cuda")
        ws[need:] = 77
        Zw = torch.full(ref.shape, float("nan"), device="cuda")
        tc.tc_tbmm_ws(Xd, Yd, Zw, ws[:need])
        assert tc.last_path() == "tbmm:i8_presliced" and torch.equal(Z, Zw)
        assert bool((ws[need:] == 77).all()), "the workspace is not overrun"
    with tc.option(tc.TC_OPT_INT8, tc.TC_INT8_OFF):
        Z64 = torch.full(ref.shape, float("nan"), device="cuda")
        tc.tc_tbmm(Xd, Yd, Z64)
        assert ":i8" not in tc.last_path()
    check(Z64, ref, "tbmm %s, fp64 path" % (shape,), TIGHT)


def test_tbmm_int8_option_off_keeps_the_fp64_kernels(tc, oracle_threads):
    """TC_OPT_INT8 = TC_INT8_OFF: the same shape on the fp64 matrix core, to one fp32 rounding; TEN and the default
    (13 digit products) on the int8 matrix core."""
    shape = (1, 128, 8192, 256)
    X, Y = inputs.make_tbmm(*shape, seed=12)
    ref = oracle.tbmm(X, Y)
    Xd, Yd = dev(X), dev(Y)
    Z = torch.full((1, 128, 8192), float("nan"), device="cuda")
    with tc.option(tc.TC_OPT_INT8, tc.TC_INT8_OFF):
        tc.tc_tbmm(Xd, Yd, Z)
        assert tc.last_path().startswith("tbmm:") and tc.last_path() != "tbmm:i8"
    check(Z, ref, "tbmm %s, fp64 path by option" % (shape,), TIGHT)
    Z13 = torch.full((1, 128, 8192), float("nan"), device="cuda")
    tc.tc_tbmm(Xd, Yd, Z13)
    assert tc.last_path() == "tbmm:i8"
    check(Z13, ref, "tbmm %s, int8 path, 13 products (default)" % (shape,), TIGHT_I8)
    Z10 = torch.full((1, 128, 8192), float("nan"), device="cuda")
    with tc.option(tc.TC_OPT_INT8, tc.TC_INT8_TEN):
        tc.tc_tbmm(Xd, Yd, Z10)
    check(Z10, ref, "tbmm %s, int8 path, 10 products" % (shape,), TIGHT_I8)
    assert not torch.equal(Z, Z13) and not torch.equal(Z13, Z10), "the option selects different kernels"
    assert tc.get_option(tc.TC_OPT_INT8) == tc.TC_INT8_AUTO


def test_tbmm_int8_heavy_tailed_operands_stay_a_quarter_of_the_bar(tc, oracle_threads):
    """Log-normal magnitudes (sigma 2 on both operands: single cases of the 10-product scheme came within a factor
    of two of the bar) on the default path, four seeds."""
    for seed in range(4):
        rng = np.random.default_rng(100 + seed)
        X = (rng.standard_normal((1, 128, 512)) * np.exp(rng.normal(size=(1, 128, 512)) * 2.0)).astype(np.float32)
        Y = (rng.standard_normal((1, 8192, 512)) * np.exp(rng.normal(size=(1, 8192, 512)) * 2.0)).astype(np.float32)
        Z = torch.full((1, 128, 8192), float("nan"), device="cuda")
        tc.tc_tbmm(dev(X), dev(Y), Z)
        assert tc.last_path() == "tbmm:i8"
        torch.cuda.synchronize()
        err = parity_error(Z.cpu().numpy().astype(np.float64), oracle.tbmm(X, Y))
        print("tbmm int8, heavy-tailed operands, seed %d: %.3e" % (seed, err), flush=True)
        assert err <= PARITY_BAR / 4


# ---------------------------------------------------------------- mlp
@pytest.fixture
def mlp_option(tc):
    """Set options of this thread for one test; they are put back afterwards."""
    saved = []

    def set_(key, value):
        saved.append((key, tc.set_option(key, value)))

    yield set_
    for key, old in reversed(saved):
        tc.set_option(key, old)


def run_mlp(tc, I, Ws, bs, keep=None):
    batch = I.shape[0]
    dims = [I.shape[1]] + [w.shape[0] for w in Ws]
    n = len(Ws)
    keep = keep if keep is not None else [True] * n
    O = [torch.full((batch, dims[l + 1]), float("nan"), device="cuda") if keep[l] else None for l in range(n)]
    nbytes = tc.tc_mlp_fcrelu_workspace_bytes(batch, dims)
    ws = torch.empty(max(nbytes, 1), dtype=torch.uint8, device="cuda") if nbytes else None
    tc.tc_mlp_fcrelu(dev(I), [dev(w) for w in Ws], [dev(b) for b in bs], O, ws)
    return O


MLP_SHAPES = [
    (128, (1024, 1024, 512, 256)),  # configuration 3
    (5, (7, 9, 3)),
    (1, (33, 17)),                  # one layer = fcrelu / MLP1, odd widths
    (16, (64, 48, 32, 16)),
    (37, (130, 70, 50, 10, 4)),
    (128, (1024, 1000)),            # odd output extent 1000 (the C3 weight of Section 7)
    (48, (256, 336, 80)),           # 63 and 15 tiles: an odd number of four-wavefront teams, the last workgroup half empty
    (2048, (64, 128, 64)),          # 1024 and 512 tiles on 512 teams: two tiles per team, then one
    # the row kernel (reductions of 128, 256, 512 or 1024, at most two tiles per workgroup and layer); the 32 workgroups
    # of an XCD take single (column tile, row tile) jobs of their eighth of the columns, or pairs of row tiles:
    (100, (512, 256, 1000)),        # 7 row tiles, the last with 4 rows: 14 single jobs, then pairs with a lone last row tile and a ragged last column tile
    (16, (128, 128, 128)),          # one row tile: one job per XCD, most workgroups without any
    (200, (1024, 512, 40)),         # 13 row tiles: 28 pairs per XCD (the last one half empty), then 13 jobs in 3 XCDs only
    (64, (1024, 512)),              # a single layer with one tile per workgroup
    (128, (256, 1024, 128, 512, 256, 128)),  # five layers
    (128, (1024, 1024, 1024)),      # pairs of row tiles in a later layer too (activations of two row tiles against one weight tile)
    (512, (128, 128, 128)),         # 32 row tiles: every workgroup of an XCD on the same column tile
    (1024, (128, 128)),             # 64 row tiles, the most the kernel takes: pairs
]


@pytest.mark.parametrize("shape", MLP_SHAPES)
def test_mlp(tc, shape, oracle_threads):
    batch, dims = shape
    I, Ws, bs = inputs.make_mlp(batch, dims, seed=inputs.SEED_BASE + 3)
    ref = oracle.mlp_fcrelu(I, Ws, bs)
    O = run_mlp(tc, I, Ws, bs)
    for l in range(len(Ws)):
        check(O[l], ref[l], "mlp %s layer %d" % (shape, l))
        assert float(O[l].min()) >= 0.0


def test_mlp_shapes_that_the_row_kernel_takes(tc):
    # which kernel a chain runs on is decided by the host from the shape alone (batch <= 1024, reductions of 128, 256,
    # 512 or 1024, at most two tiles per workgroup in every layer)
    cases = [((128, (1024, 1024, 512, 256)), "mlp:rows"), ((128, (1024, 1024, 1024)), "mlp:rows"),
             ((1024, (128, 128)), "mlp:rows"), ((128, (1024, 1000)), "mlp:rows"), ((100, (512, 256, 1000)), "mlp:rows"),
             ((1024, (128, 256)), "mlp:tiles"),    # 2 column tiles per XCD x 32 pairs of row tiles: more than 32 workgroups
             ((256, (1024, 1024)), "mlp:tiles"), ((2048, (128, 128)), "mlp:tiles"), ((128, (384, 128)), "mlp:tiles")]
    for (batch, dims), path in cases:
        I, Ws, bs = inputs.make_mlp(batch, dims, seed=5)
        run_mlp(tc, I, Ws, bs)
        assert tc.last_path() == path, (batch, dims, tc.last_path())


def test_mlp_seeded_random_chains_in_the_row_kernels_range(tc, oracle_threads):
    # a seeded draw of chains whose reductions are all 128, 256, 512 or 1024: whatever deal of tiles the host picks
    # (single jobs, pairs of row tiles, or the tile-stream kernel when neither fits), every layer must agree with the
    # oracle; ragged batches and ragged last widths included
    rng = np.random.default_rng(20273)  # a draw with 9 chains for the row kernel (4 with pairs in later layers) and 3 for the other
    took = set()
    for case in range(12):
        n = int(rng.integers(1, 5))
        dims = [int(rng.choice([128, 256, 512, 1024])) for _ in range(n)] + [int(rng.integers(1, 1100))]
        batch = int(rng.choice([1, 16, 17, 50, 96, 128, 130, 200, 256, 512]))
        I, Ws, bs = inputs.make_mlp(batch, dims, seed=100 + case, w_std=1.0 / np.sqrt(max(dims[:-1])))
        ref = oracle.mlp_fcrelu(I, Ws, bs)
        O = run_mlp(tc, I, Ws, bs)
        took.add(tc.last_path())
        for l in range(n):
            check(O[l], ref[l], "mlp case %d batch %d dims %s layer %d (%s)" % (case, batch, dims, l, tc.last_path()))
    assert took == {"mlp:rows", "mlp:tiles"}


def test_mlp_tile_stream_kernel_by_option(tc, oracle_threads, mlp_option):
    # TC_OPT_MLP_KERNEL = TC_MLP_TILES: the benchmark chain on the persistent tile-stream kernel (what shapes outside
    # the row kernel's range take), with a workspace full of garbage
    mlp_option(tc.TC_OPT_MLP_KERNEL, tc.TC_MLP_TILES)
    batch, dims = 128, (1024, 1024, 512, 256)
    I, Ws, bs = inputs.make_mlp(batch, dims, seed=inputs.SEED_BASE + 3)
    ref = oracle.mlp_fcrelu(I, Ws, bs)
    O = [torch.full((batch, d), float("nan"), device="cuda") for d in dims[1:]]
    ws = torch.full((tc.tc_mlp_fcrelu_workspace_bytes(batch, dims),), 0xCD, dtype=torch.uint8, device="cuda")
    Id, Wd, bd = dev(I), [dev(w) for w in Ws], [dev(b) for b in bs]
    for _ in range(2):
        tc.tc_mlp_fcrelu(Id, Wd, bd, O, ws)
        assert tc.last_path() == "mlp:tiles"
    for l in range(3):
        check(O[l], ref[l], "mlp tile-stream kernel, layer %d" % l)
    assert int(ws[:256].view(torch.int32)[33]) == 0


def test_mlp_per_layer_launch_path(tc, oracle_threads, mlp_option):
    # the same chain through one launch per layer (the path taken when a width is not a multiple of 4)
    mlp_option(tc.TC_OPT_MLP_KERNEL, tc.TC_MLP_PER_LAYER)
    batch, dims = 128, (1024, 1024, 512, 256)
    I, Ws, bs = inputs.make_mlp(batch, dims, seed=inputs.SEED_BASE + 3)
    ref = oracle.mlp_fcrelu(I, Ws, bs)
    O = run_mlp(tc, I, Ws, bs)
    for l in range(3):
        check(O[l], ref[l], "mlp per-layer launches, layer %d" % l)


@pytest.mark.parametrize("kernel", ["rows", "tiles"])
def test_mlp_bounded_wait_gives_up_and_recovers(tc, oracle_threads, mlp_option, kernel):
    # A spin limit of 0 makes every wait for another workgroup give up without looking (with a limit of 1 the row
    # kernel's first poll often finds all flags set already: its workgroups reach their polls in step).  The kernel
    # must still drain, flag the workspace, and the next ordinary call must be correct again.
    batch, dims = 128, (1024, 1024, 512, 256)
    I, Ws, bs = inputs.make_mlp(batch, dims, seed=inputs.SEED_BASE + 3)
    Id, Wd, bd = dev(I), [dev(w) for w in Ws], [dev(b) for b in bs]
    O = [torch.empty((batch, d), device="cuda") for d in dims[1:]]
    ws = torch.zeros(tc.tc_mlp_fcrelu_workspace_bytes(batch, dims), dtype=torch.uint8, device="cuda")
    mlp_option(tc.TC_OPT_MLP_KERNEL, tc.TC_MLP_ROWS if kernel == "rows" else tc.TC_MLP_TILES)
    old = tc.set_option(tc.TC_OPT_MLP_SPIN_LIMIT, 0)
    try:
        tc.tc_mlp_fcrelu(Id, Wd, bd, O, ws)
        assert tc.last_path() == "mlp:" + kernel
        torch.cuda.synchronize()
        assert int(ws[:256].view(torch.int32)[33]) == 1
    finally:
        tc.set_option(tc.TC_OPT_MLP_SPIN_LIMIT, old)
    tc.tc_mlp_fcrelu(Id, Wd, bd, O, ws)
    torch.cuda.synchronize()
    assert int(ws[:256].view(torch.int32)[33]) == 0
    ref = oracle.mlp_fcrelu(I, Ws, bs)
    for l in range(3):
        check(O[l], ref[l], "mlp after a timed-out call, layer %d" % l)


def test_mlp_workspace_may_hold_garbage(tc, oracle_threads):
    batch, dims = 64, (256, 128, 64)
    I, Ws, bs = inputs.make_mlp(batch, dims, seed=12, w_std=0.05)
    ref = oracle.mlp_fcrelu(I, Ws, bs)
    O = [torch.empty((batch, d), device="cuda") for d in dims[1:]]
    ws = torch.full((tc.tc_mlp_fcrelu_workspace_bytes(batch, dims),), 0xAB, dtype=torch.uint8, device="cuda")
    Id, Wd, bd = dev(I), [dev(w) for w in Ws], [dev(b) for b in bs]
    for _ in range(3):
        tc.tc_mlp_fcrelu(Id, Wd, bd, O, ws)
    for l in range(2):
        check(O[l], ref[l], "mlp garbage workspace, layer %d" % l)


def test_mlp_intermediates_may_be_skipped(tc, oracle_threads):
    I, Ws, bs = inputs.make_mlp(24, (96, 80, 40, 24), seed=4, w_std=0.1, b_std=0.1)
    ref = oracle.mlp_fcrelu(I, Ws, bs)
    O = run_mlp(tc, I, Ws, bs, keep=[False, False, True])
    check(O[2], ref[2], "mlp last layer only")


def test_mlp_large_weights_exercise_the_clamp(tc, oracle_threads):
    I, Ws, bs = inputs.make_mlp(20, (50, 60, 30), seed=8, w_std=1.0, b_std=1.0)
    ref = oracle.mlp_fcrelu(I, Ws, bs)
    O = run_mlp(tc, I, Ws, bs)
    for l in range(2):
        check(O[l], ref[l], "mlp big weights layer %d" % l)
        assert np.array_equal(O[l].cpu().numpy() == 0.0, ref[l] == 0.0) or parity_error(O[l].cpu().numpy(), ref[l]) <= TIGHT


# ---------------------------------------------------------------- gconv
GCONV_SHAPES = [
    (2, 4, 16, 16, 58, 58, 3, 3),   # configuration 4 geometry, fewer images/groups
    (1, 2, 2, 3, 5, 6, 3, 2),       # ragged everything
    (2, 1, 3, 4, 8, 7, 3, 3),       # G = 1: ordinary convolution
    (2, 3, 4, 5, 6, 7, 1, 1),       # pointwise filter
    (1, 2, 4, 4, 3, 3, 3, 3),       # a single output pixel
    (2, 4, 32, 32, 7, 7, 3, 3),     # paper table shape (32,32,32,32,7,7), fewer images/groups (bank-stationary kernel)
    (5, 3, 32, 32, 7, 7, 3, 3),     # bank-stationary kernel: odd image count, ragged last chunk
    (1, 2, 32, 32, 7, 7, 3, 3),     # bank-stationary kernel: a single image per group
    (2, 4, 4, 4, 56, 56, 3, 3),     # paper table shape (32,32,4,4,56,56), fewer images/groups
    (1, 2, 5, 20, 9, 11, 2, 4),     # two channel tiles, odd reduction length
    (1, 2, 16, 16, 21, 58, 3, 3),   # width-58 kernels: odd height (unaligned planes), ragged last band
    (2, 1, 16, 16, 12, 58, 3, 3),   # width-58 kernels: two bands, second one partial
    (1, 1, 16, 16, 3, 58, 3, 3),    # width-58 kernels: a single output row
    (3, 5, 16, 16, 18, 58, 3, 3),   # int8 kernel: 15 (image, group) pairs, two bands
    (1, 3, 16, 16, 10, 58, 3, 3),   # int8 kernel: a single band
    (37, 29, 16, 16, 26, 58, 3, 3), # int8 kernel: 1073 pairs on 512 persistent workgroups (2 or 3 images each)
    (1, 3, 16, 16, 20, 30, 3, 3),   # 16x16 channels, other width: runtime-width LDS kernel
    (2, 3, 16, 16, 14, 14, 3, 3),   # width-14 band kernel (paper table shape), whole image = one band
    (4, 3, 32, 32, 7, 7, 3, 3),     # int8 kernel for 32-channel small images: three iterations of four images
    (12, 5, 32, 32, 7, 7, 3, 3),    # 15 iterations: runs that cross a group boundary
    (4, 3, 16, 16, 14, 14, 3, 3),   # int8 kernel for small images: three iterations of four images
    (12, 5, 16, 16, 14, 14, 3, 3),  # 15 iterations: runs that cross a group boundary
    (2052, 1, 16, 16, 14, 14, 3, 3),  # 513 iterations on 512 workgroups: one run of two
    (1, 2, 16, 16, 17, 14, 3, 3),   # width-14 band kernel: odd height, two bands, unaligned planes
    (2, 3, 4, 4, 56, 56, 3, 3),     # 4x4x4-block kernel (paper table shape): four bands, last one ragged
    (1, 2, 4, 4, 5, 56, 3, 3),      # 4x4x4-block kernel: one short band
    (2, 3, 8, 8, 28, 28, 3, 3),     # 4x4x4-block kernel, 8 channels (paper table shape)
    (1, 2, 8, 8, 31, 28, 3, 3),     # 4x4x4-block kernel, 8 channels: two bands, ragged tiles
    (4, 3, 16, 16, 16, 16, 3, 3),   # int8 kernel for small images at 16 x 16 (the table shape with a border): 13 tiles, the last a quarter full
    (8, 5, 16, 16, 16, 16, 3, 3),   # the same, runs that cross a group boundary
    (2, 3, 4, 4, 58, 58, 3, 3),     # 4x4x4-block kernel at width 58 (the table shape with a border): 8-byte staging loads
    (1, 2, 4, 4, 21, 58, 3, 3),     # the same, odd height: two bands, the second ragged
    (2, 3, 8, 8, 30, 30, 3, 3),     # 4x4x4-block kernel, 8 channels at width 30: the whole image one band
    (1, 2, 8, 8, 17, 30, 3, 3),     # the same, a short image
    (2, 2, 32, 64, 12, 13, 3, 3),   # big groups (64 filters, 288 taps): the int8 kernel over gathered taps, one grid plane per group
    (1, 1, 64, 128, 20, 20, 3, 3),  # G = 1 at 64 -> 128 channels: the plain convolution of Section 3 on that kernel
    (3, 3, 36, 64, 9, 9, 3, 3),     # three groups, 324 taps, 147 pixels
    (2, 2, 16, 128, 10, 11, 4, 4),  # 4 x 4 filters: 256 taps exactly
    (3, 4, 32, 32, 14, 14, 3, 3),   # 32 filters per group of 288 taps: workgroups of 32 filters x 64 pixels (NT = 4 .. 12)
    (16, 2, 32, 32, 30, 30, 3, 3),  # the same with 12544 pixels per group: NT = 12
    (2, 3, 40, 96, 11, 12, 3, 3),   # 96 filters = three blocks of 32
    (2, 1, 12, 70, 15, 17, 3, 3),   # G = 1 with 70 filters of 108 taps: the strided convolution's fp64 kernel (stride 1)
]


@pytest.mark.parametrize("shape", GCONV_SHAPES)
def test_gconv(tc, shape, oracle_threads):
    N, G, C, F, H, W, KH, KW = shape
    I, W1, bias = inputs.make_gconv(*shape, seed=inputs.SEED_BASE + 4)
    ref = oracle.group_conv(I, W1, bias)
    O = torch.full(ref.shape, float("nan"), device="cuda")
    tc.tc_group_conv(dev(I), dev(W1), dev(bias), O)
    if F % 32 == 0 and C * KH * KW >= 256 and (H, W) != (7, 7):
        assert tc.last_path() == "gconv:i8_taps"
    check(O, ref, "gconv %s" % (shape,), tight_for_last_call(tc))


@pytest.mark.parametrize("shape", GCONV_SHAPES)
def test_gconv_with_int8_off_runs_the_fp64_kernels(tc, shape, oracle_threads):
    """TC_OPT_INT8 = TC_INT8_OFF: every shape on an fp64 kernel, to one fp32 rounding.  Where the default is an int8
    kernel, the whole output of the default path is also compared with the whole output of the fp64 path."""
    I, W1, bias = inputs.make_gconv(*shape, seed=inputs.SEED_BASE + 4)
    ref = oracle.group_conv(I, W1, bias)
    Id, Wd, bd = dev(I), dev(W1), dev(bias)
    O = torch.full(ref.shape, float("nan"), device="cuda")
    with tc.option(tc.TC_OPT_INT8, tc.TC_INT8_OFF):
        tc.tc_group_conv(Id, Wd, bd, O)
        assert ":i8" not in tc.last_path()
    check(O, ref, "gconv fp64 path %s" % (shape,))
    Od = torch.full(ref.shape, float("nan"), device="cuda")
    tc.tc_group_conv(Id, Wd, bd, Od)
    if ":i8" in tc.last_path():
        torch.cuda.synchronize()
        err = parity_error(Od.cpu().numpy().astype(np.float64), O.cpu().numpy().astype(np.float64))
        print("gconv %s: %s against the fp64 kernel, whole output: %.3e" % (shape, tc.last_path(), err), flush=True)
        assert err <= TIGHT_I8


def test_gconv_i8_wide_dynamic_range_and_nonfinite(tc, oracle_threads):
    """Per-band / per-filter scaling: magnitudes spread over many binades, an all-zero band, and Inf/NaN poisoning a band."""
    shape = (1, 2, 16, 16, 26, 58, 3, 3)   # three bands of the int8 kernel
    I, W1, bias = inputs.make_gconv(*shape, seed=77)
    rng = np.random.default_rng(5)
    I = (I * np.exp2(rng.integers(-12, 12, size=I.shape))).astype(np.float32)      # 24 binades inside every band
    I[0, 0, :, 8:18, :] = 0.0                                                      # image 0, group 0: band 1 is all zeros
    W1 = (W1 * np.exp2(rng.integers(-20, 20, size=(2, 16, 1, 1, 1)))).astype(np.float32)  # filter rows of very different scale
    ref = oracle.group_conv(I, W1, bias)
    O = torch.full(ref.shape, float("nan"), device="cuda")
    tc.tc_group_conv(dev(I), dev(W1), dev(bias), O)
    torch.cuda.synchronize()
    got = O.cpu().numpy().astype(np.float64)
    # filter rows differ by 2^40 in scale: compare every filter's plane on its own scale
    worst = max(parity_error(got[:, g, f], ref[:, g, f]) for g in range(2) for f in range(16))
    print("gconv int8, 24 binades inside every band: worst filter plane %.3e" % worst, flush=True)
    for g in range(2):
        for f in range(16):
            err = parity_error(got[:, g, f], ref[:, g, f])
            # the quantisation error is up to 2^-32 of the band maximum whatever the spread inside the band;
            # with 24 binades of spread most terms sit far below it: a quarter of the bar is the limit here
            assert err <= PARITY_BAR / 4, "group %d filter %d: %.3e" % (g, f, err)
    Ibad = I.copy()
    Ibad[0, 1, 3, 20, 7] = np.inf                                                   # rows 16..25 are band 2 (+ halo of band 1)
    O2 = torch.zeros(ref.shape, device="cuda")
    tc.tc_group_conv(dev(Ibad), dev(W1), dev(bias), O2)
    torch.cuda.synchronize()
    got2 = O2.cpu().numpy()
    assert np.isnan(got2[0, 1, :, 18:21, 5:8]).all(), "outputs that read the Inf must not be finite"
    assert np.array_equal(got2[0, 0], got[0, 0].astype(np.float32)), "the other group is untouched by it"
    assert np.isfinite(got2[0, 1, :, 0:8]).all(), "bands that never read the Inf stay finite"


@pytest.mark.parametrize("in_exp,w_exp", [(-100, 60), (100, 20), (-140, 100), (0, -120)])
def test_gconv_i8_extreme_magnitudes(tc, oracle_threads, in_exp, w_exp):
    """Block scaling must follow the operands through the whole fp32 exponent range (denormal inputs included)."""
    shape = (1, 2, 16, 16, 18, 58, 3, 3)
    I, W1, _ = inputs.make_gconv(*shape, seed=91)
    I = np.ldexp(I, in_exp).astype(np.float32)
    W1 = np.ldexp(W1, w_exp).astype(np.float32)
    ref = oracle.group_conv(I, W1, None)
    assert np.isfinite(ref).all() and np.abs(ref).max() > 0
    O = torch.full(ref.shape, float("nan"), device="cuda")
    tc.tc_group_conv(dev(I), dev(W1), None, O)
    torch.cuda.synchronize()
    got = O.cpu().numpy().astype(np.float64)
    small = np.abs(ref) < 2.0 ** -120   # outputs in the denormal range of fp32 round on a coarser grid
    err = parity_error(np.where(small, ref, got), ref)
    print("gconv extreme 2^%d x 2^%d: parity error %.3e" % (in_exp, w_exp, err), flush=True)
    assert err <= TIGHT_I8 * (4 if in_exp < -126 else 1)   # denormal inputs carry fewer bits themselves


def heavy_tailed(kind, rng, a):
    """Multiply a by magnitudes with a heavy tail (the cases in which the digit products with k + l = 2 matter)."""
    if kind == "lognormal":
        return (a * np.exp(rng.normal(size=a.shape) * 1.5)).astype(np.float32)
    if kind == "student3":
        return (a * np.abs(rng.standard_t(3, size=a.shape))).astype(np.float32)
    if kind == "sparse":
        return (a * np.where(rng.random(a.shape) < 0.01, 300.0, 1.0)).astype(np.float32)
    raise ValueError(kind)


@pytest.mark.parametrize("kind", ["lognormal", "student3", "sparse"])
@pytest.mark.parametrize("shape", [(2, 3, 16, 16, 26, 58, 3, 3), (8, 3, 16, 16, 14, 14, 3, 3), (8, 3, 32, 32, 7, 7, 3, 3)])
def test_gconv_i8_heavy_tailed_operands_stay_a_quarter_of_the_bar(tc, oracle_threads, shape, kind):
    """A few large elements in every band AND every filter row: the digit products with k + l = 2 then weigh most
    against the largest output.  The default path (no option set) keeps them where the operands call for it: a
    quarter of the bar over four seeds, on each of the three int8 kernels."""
    for seed in range(4):
        I, W1, bias = inputs.make_gconv(*shape, seed=11 + seed)
        rng = np.random.default_rng(5 + seed)
        I = heavy_tailed(kind, rng, I)
        W1 = heavy_tailed(kind, rng, W1)
        ref = oracle.group_conv(I, W1, bias)
        O = torch.full(ref.shape, float("nan"), device="cuda")
        tc.tc_group_conv(dev(I), dev(W1), dev(bias), O)
        assert ":i8" in tc.last_path()
        torch.cuda.synchronize()
        err = parity_error(O.cpu().numpy().astype(np.float64), ref)
        print("gconv %s %s, %s magnitudes, seed %d: parity error %.3e" % (tc.last_path(), shape, kind, seed, err), flush=True)
        assert err <= PARITY_BAR / 4


def test_gconv_i8_ten_thirteen_and_the_default(tc, oracle_threads):
    """TC_INT8_TEN drops the digit products with k + l = 2 whatever the operands, TC_INT8_THIRTEEN keeps them whatever
    the operands, the default decides per thread from its band and filter rows: on log-normal operands the default
    must match THIRTEEN's accuracy, on the benchmark's Gaussian operands it must be bit-equal to TEN (no extra work)."""
    shape = (2, 3, 16, 16, 26, 58, 3, 3)
    I, W1, bias = inputs.make_gconv(*shape, seed=11)
    ref_g = oracle.group_conv(I, W1, bias)
    rng = np.random.default_rng(5)
    Ih, Wh = heavy_tailed("lognormal", rng, I), heavy_tailed("lognormal", rng, W1)
    ref_h = oracle.group_conv(Ih, Wh, bias)

    def run(Ia, Wa, mode):
        O = torch.full(ref_g.shape, float("nan"), device="cuda")
        if mode is None:
            tc.tc_group_conv(dev(Ia), dev(Wa), dev(bias), O)
        else:
            with tc.option(tc.TC_OPT_INT8, mode):
                tc.tc_group_conv(dev(Ia), dev(Wa), dev(bias), O)
        assert tc.last_path() == "gconv:i8"
        torch.cuda.synchronize()
        return O.cpu().numpy()

    g = {m: run(I, W1, m) for m in (None, tc.TC_INT8_TEN, tc.TC_INT8_THIRTEEN)}
    h = {m: run(Ih, Wh, m) for m in (None, tc.TC_INT8_TEN, tc.TC_INT8_THIRTEEN)}
    eg = {m: parity_error(v.astype(np.float64), ref_g) for m, v in g.items()}
    eh = {m: parity_error(v.astype(np.float64), ref_h) for m, v in h.items()}
    print("gconv int8 Gaussian: default %.2e, ten %.2e, thirteen %.2e" % (eg[None], eg[tc.TC_INT8_TEN], eg[tc.TC_INT8_THIRTEEN]), flush=True)
    print("gconv int8 log-normal: default %.2e, ten %.2e, thirteen %.2e" % (eh[None], eh[tc.TC_INT8_TEN], eh[tc.TC_INT8_THIRTEEN]), flush=True)
    assert np.array_equal(g[None], g[tc.TC_INT8_TEN]), "Gaussian operands: the default adds no sweeps"
    assert eg[tc.TC_INT8_THIRTEEN] <= 1e-6 and eh[tc.TC_INT8_THIRTEEN] <= 2e-6
    assert eh[None] <= PARITY_BAR / 4 and eh[None] <= 4 * eh[tc.TC_INT8_THIRTEEN] + 1e-7
    assert eh[tc.TC_INT8_TEN] <= PARITY_BAR, "ten products on request: inside the bar here, by a smaller margin"
    assert eh[tc.TC_INT8_TEN] > eh[None]


@pytest.mark.parametrize("shape", [(3, 5, 16, 16, 18, 58, 3, 3), (37, 29, 16, 16, 26, 58, 3, 3)])
def test_gconv_i8_with_thirteen_digit_products(tc, shape, oracle_threads):
    I, W1, bias = inputs.make_gconv(*shape, seed=inputs.SEED_BASE + 4)
    ref = oracle.group_conv(I, W1, bias)
    O = torch.full(ref.shape, float("nan"), device="cuda")
    with tc.option(tc.TC_OPT_INT8, tc.TC_INT8_THIRTEEN):
        tc.tc_group_conv(dev(I), dev(W1), dev(bias), O)
        assert tc.last_path() == "gconv:i8"
    check(O, ref, "gconv int8 with 13 products %s" % (shape,), 1e-6)


@pytest.mark.parametrize("shape", [(8, 3, 16, 16, 14, 14, 3, 3), (8, 3, 32, 32, 7, 7, 3, 3)])
def test_gconv_i8_small_images_wide_range_and_nonfinite(tc, shape, oracle_threads):
    """The small-image int8 kernels: block scaling per whole image, magnitudes spread over binades, an all-zero image,
    and an Inf that must poison exactly the image block that holds it."""
    N, G, C, F, H, W, KH, KW = shape
    I, W1, bias = inputs.make_gconv(*shape, seed=123)
    rng = np.random.default_rng(9)
    I = (I * np.exp2(rng.integers(-8, 8, size=I.shape))).astype(np.float32)
    I[2, 1] = 0.0
    W1 = (W1 * np.exp2(rng.integers(-20, 20, size=(G, F, 1, 1, 1)))).astype(np.float32)
    ref = oracle.group_conv(I, W1, bias)
    O = torch.full(ref.shape, float("nan"), device="cuda")
    tc.tc_group_conv(dev(I), dev(W1), dev(bias), O)
    torch.cuda.synchronize()
    got = O.cpu().numpy().astype(np.float64)
    worst = max(parity_error(got[:, g, f], ref[:, g, f]) for g in range(G) for f in range(F))
    print("gconv int8 small images %s, 16 binades inside every image: worst filter plane %.3e" % (shape, worst), flush=True)
    assert worst <= PARITY_BAR / 4
    assert np.array_equal(got[2, 1], np.broadcast_to(bias.reshape(G, F)[1][:, None, None], got[2, 1].shape).astype(np.float32))
    Ibad = I.copy()
    Ibad[5, 2, 3, 4, 4] = np.inf
    O2 = torch.zeros(ref.shape, device="cuda")
    tc.tc_group_conv(dev(Ibad), dev(W1), dev(bias), O2)
    torch.cuda.synchronize()
    got2 = O2.cpu().numpy()
    assert np.isnan(got2[5, 2]).all(), "the block that holds the Inf"
    mask = np.ones((N, G), dtype=bool); mask[5, 2] = False
    assert np.array_equal(got2[mask], got.astype(np.float32)[mask]), "every other block is untouched"


def test_gconv_without_bias(tc, oracle_threads):
    I, W1, _ = inputs.make_gconv(1, 3, 4, 6, 10, 9, 3, 3, seed=2)
    ref = oracle.group_conv(I, W1, None)
    O = torch.full(ref.shape, float("nan"), device="cuda")
    tc.tc_group_conv(dev(I), dev(W1), None, O)
    check(O, ref, "gconv no bias")


def test_gconv_full_configuration_4(tc, oracle_threads):
    _, (I, W1, bias) = inputs.make_config(4)
    O = torch.full((32, 32, 16, 56, 56), float("nan"), device="cuda")
    tc.tc_group_conv(dev(I), dev(W1), dev(bias), O)
    torch.cuda.synchronize()
    ref = oracle.group_conv(I, W1, bias)
    check(O, ref, "gconv configuration 4", TIGHT_I8)


# ---------------------------------------------------------------- kron
KRON_SHAPES = [
    (256, 64, 64, 64, 64),  # configuration 5
    (1, 2, 3, 2, 3),
    (3, 5, 7, 3, 9),        # ragged
    (2, 20, 6, 70, 33),     # two column blocks, ragged l blocks
    (4, 16, 16, 16, 16),
    (2, 64, 32, 128, 48),
    (3, 40, 64, 64, 64),    # the 64 x 64 x 64 kernel with a ragged I: one block of 40 rows (clamped W1 rows, masked stores)
    (2, 70, 64, 64, 64),    # the same with two blocks per batch element, the second with 6 rows
    (1, 129, 64, 64, 64),   # three blocks, the last with a single row
]


@pytest.mark.parametrize("shape", KRON_SHAPES)
def test_kron(tc, shape, oracle_threads):
    B, I, K, J, L = shape
    W1, W2, X = inputs.make_kron(B, I, K, J, L, seed=inputs.SEED_BASE + 5)
    ref = oracle.kron(W1, W2, X)
    # Y sits between two guard bands: a write past I (or before the first row) would show
    buf = torch.full((B * I * J + 1024,), 777.0, device="cuda")
    buf[512:512 + B * I * J] = float("nan")
    Y = buf[512:512 + B * I * J].view(B, I, J)
    tc.tc_kron(dev(W1), dev(W2), dev(X), Y)
    check(Y, ref, "kron %s" % (shape,))
    assert torch.all(buf[:512] == 777.0) and torch.all(buf[512 + B * I * J:] == 777.0)


def test_outputs_need_no_zeroing_and_calls_repeat(tc, oracle_threads):
    W1, W2, X = inputs.make_kron(4, 16, 16, 16, 16, seed=1)
    ref = oracle.kron(W1, W2, X)
    Y = torch.full((4, 16, 16), 1e30, device="cuda")
    a, b, c = dev(W1), dev(W2), dev(X)
    for _ in range(3):
        tc.tc_kron(a, b, c, Y)
    check(Y, ref, "kron repeated")


# ---------------------------------------------------------------- HIP graph capture
def test_mlp_replays_when_most_workgroups_have_nothing_to_do(tc, oracle_threads):
    """Batch 16 through widths of 128: 8 of the row kernel's 256 workgroups have a tile, the others leave at
    once.  None of them may count itself out before workgroup 0 has zeroed the exit counter, or the call's token
    outlives the launch and a replay (same token) trusts flags that are about to be zeroed.  Twenty replays of a graph
    of several launches, into a workspace that starts as garbage; every replay checked; the error word stays clear."""
    batch, dims = 16, (128, 128, 128, 128)
    I, Ws, bs = inputs.make_mlp(batch, dims, seed=61, w_std=0.1)
    ref = oracle.mlp_fcrelu(I, Ws, bs)
    Id, Wd, bd = dev(I), [dev(w) for w in Ws], [dev(b) for b in bs]
    O = [torch.empty((batch, d), device="cuda") for d in dims[1:]]
    ws = torch.randint(0, 255, (tc.tc_mlp_fcrelu_workspace_bytes(batch, dims),), dtype=torch.uint8, device="cuda")
    tc.tc_mlp_fcrelu(Id, Wd, bd, O, ws)
    assert tc.last_path() == "mlp:rows"
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(4):
            tc.tc_mlp_fcrelu(Id, Wd, bd, O, ws)
    for rep in range(20):
        for o in O:
            o.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert int(ws[:256].view(torch.int32)[33]) == 0, "a bounded wait gave up in replay %d" % rep
        for l in range(3):
            assert parity_error(O[l].cpu().numpy().astype(np.float64), ref[l]) <= TIGHT, (rep, l)


def test_all_entry_points_replay_from_a_hip_graph(tc, oracle_threads):
    # The library enqueues kernels only (no memset, no allocation), so a step can be captured once and
    # replayed.  Replays are interleaved with eager work and synchronisations, and every replay is
    # checked (the fused MLP re-runs with the same barrier token on every replay).
    X, Y = inputs.make_tbmm(64, 26, 72, 26, seed=21)
    I, Ws, bs = inputs.make_mlp(128, (256, 256, 128, 64), seed=22, w_std=0.05)
    Ig, W1, bias = inputs.make_gconv(2, 4, 16, 16, 58, 58, 3, 3, seed=23)
    K1, K2, Xk = inputs.make_kron(16, 64, 64, 64, 64, seed=24)
    ref = {"tbmm": oracle.tbmm(X, Y), "mlp": oracle.mlp_fcrelu(I, Ws, bs),
           "gconv": oracle.group_conv(Ig, W1, bias), "kron": oracle.kron(K1, K2, Xk)}
    Xd, Yd, Id, Wd, bd = dev(X), dev(Y), dev(I), [dev(w) for w in Ws], [dev(b) for b in bs]
    Igd, W1d, biasd, K1d, K2d, Xkd = dev(Ig), dev(W1), dev(bias), dev(K1), dev(K2), dev(Xk)
    Z = torch.empty((64, 26, 72), device="cuda")
    O = [torch.empty((128, w.shape[0]), device="cuda") for w in Ws]
    ws = torch.empty(tc.tc_mlp_fcrelu_workspace_bytes(128, (256, 256, 128, 64)), dtype=torch.uint8, device="cuda")
    Og = torch.empty(ref["gconv"].shape, device="cuda")
    Yk = torch.empty((16, 64, 64), device="cuda")

    def step():
        tc.tc_tbmm(Xd, Yd, Z)
        tc.tc_mlp_fcrelu(Id, Wd, bd, O, ws)
        tc.tc_group_conv(Igd, W1d, biasd, Og)
        tc.tc_kron(K1d, K2d, Xkd, Yk)

    step()  # eager once: first-call set-up (LDS limits) happens outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep in range(3):
        for t in [Z, Og, Yk] + O:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        scratch = torch.randn(1 << 20, device="cuda").sum()  # eager work between replays
        torch.cuda.synchronize()
        check(Z, ref["tbmm"], "graph replay %d tbmm" % rep)
        for l in range(3):
            check(O[l], ref["mlp"][l], "graph replay %d mlp layer %d" % (rep, l))
        check(Og, ref["gconv"], "graph replay %d gconv" % rep, TIGHT_I8)
        check(Yk, ref["kron"], "graph replay %d kron" % rep)
        assert int(ws[:256].view(torch.int32)[33]) == 0
        del scratch


# ---------------------------------------------------------------- large sizes, sampled
def test_tbmm_large_batch_sampled(tc, oracle_threads):
    # 40x the benchmark batch; the oracle evaluates a sample of batch elements
    B, N, M, K = 20000, 26, 72, 26
    X, Y = inputs.make_tbmm(B, N, M, K, seed=31)
    Z = torch.full((B, N, M), float("nan"), device="cuda")
    tc.tc_tbmm(dev(X), dev(Y), Z)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(Z).all())
    pick = np.random.default_rng(0).choice(B, size=64, replace=False)
    pick = np.concatenate([pick, [0, B - 1]])
    check(Z[torch.from_numpy(pick).cuda()], oracle.tbmm(X[pick], Y[pick]), "tbmm B=20000, sampled batches")


@pytest.mark.parametrize("fused", ["default", "tiles"])
def test_mlp_large_batch_sampled(tc, oracle_threads, mlp_option, fused):
    """Batch 8192: by default one LDS-tiled launch per layer, with TC_OPT_MLP_KERNEL = TC_MLP_TILES the fused
    tile-stream kernel; sampled rows in the oracle."""
    if fused != "default":
        mlp_option(tc.TC_OPT_MLP_KERNEL, tc.TC_MLP_TILES)
    batch, dims = 8192, (1024, 1024, 512, 256)
    I, Ws, bs = inputs.make_mlp(batch, dims, seed=71)
    O = run_mlp(tc, I, Ws, bs)
    torch.cuda.synchronize()
    rng = np.random.default_rng(3)
    pick = np.sort(rng.choice(batch, size=48, replace=False))
    pick[:3] = [0, 63, 64]
    pick[-1] = batch - 1
    ref = oracle.mlp_fcrelu(np.ascontiguousarray(I[pick]), Ws, bs)
    sel = torch.from_numpy(pick).cuda()
    for l in range(3):
        assert not torch.isnan(O[l]).any()
        check(O[l][sel], ref[l], "mlp batch 8192 (fused=%s), layer %d, sampled rows" % (fused, l))


def test_tbmm_ws_slices_x_once_and_agrees_bit_for_bit(tc, oracle_threads):
    """tc_tbmm_ws: with a workspace the int8 transposed matmul reads X's digits from it (same digits, same sums: the
    result is bit-identical to tc_tbmm's); without one, with too small a one, or for a shape that has no use for it,
    it is tc_tbmm.  A reduced instance of the paper's largest tmm (Section 7), compared with the oracle in full."""
    B, N, M, K = 1, 128, 8192, 2048
    X, Y = inputs.make_tbmm(B, N, M, K, seed=41)
    ref = oracle.tbmm(X, Y)
    Xd, Yd = dev(X), dev(Y)
    need = tc.tc_tbmm_workspace_bytes(B, N, M, K)
    assert need == (K // 128) * (N // 128) * (65536 + 1024)
    Z0 = torch.full((B, N, M), float("nan"), device="cuda")
    tc.tc_tbmm(Xd, Yd, Z0)
    assert tc.last_path() == "tbmm:i8"
    check(Z0, ref, "tmm 128x2048x8192, X sliced by every workgroup", TIGHT_I8)
    ws = torch.randint(0, 255, (need + 64,), dtype=torch.uint8, device="cuda")   # garbage, and a guard band behind it
    ws[need:] = 77
    for _ in range(2):
        Z1 = torch.full((B, N, M), float("nan"), device="cuda")
        tc.tc_tbmm_ws(Xd, Yd, Z1, ws[:need])
        assert tc.last_path() == "tbmm:i8_presliced"
        assert torch.equal(Z0, Z1)
    assert bool((ws[need:] == 77).all()), "the workspace is not overrun"
    for w in (None, ws[:need - 16]):
        Z2 = torch.full((B, N, M), float("nan"), device="cuda")
        tc.tc_tbmm_ws(Xd, Yd, Z2, w)
        assert tc.last_path() == "tbmm:i8" and torch.equal(Z0, Z2)
    with tc.option(tc.TC_OPT_INT8, tc.TC_INT8_TEN):
        Z3 = torch.full((B, N, M), float("nan"), device="cuda")
        Z4 = torch.full((B, N, M), float("nan"), device="cuda")
        tc.tc_tbmm(Xd, Yd, Z3)
        tc.tc_tbmm_ws(Xd, Yd, Z4, ws[:need])
        assert tc.last_path() == "tbmm:i8_presliced" and torch.equal(Z3, Z4) and not torch.equal(Z3, Z0)
    # a shape with no use for a workspace: the argument is ignored
    assert tc.tc_tbmm_workspace_bytes(500, 26, 72, 26) == 0 and tc.tc_tbmm_workspace_bytes(2, 256, 4096, 512) == 0
    Xs, Ys = inputs.make_tbmm(8, 26, 72, 26, seed=1)
    Zs = torch.full((8, 26, 72), float("nan"), device="cuda")
    tc.tc_tbmm_ws(dev(Xs), dev(Ys), Zs, ws[:need])
    assert tc.last_path() == "tbmm:lds"
    check(Zs, oracle.tbmm(Xs, Ys), "tc_tbmm_ws on configuration 1")


def test_tbmm_ws_with_several_blocks_of_rows_and_batches(tc, oracle_threads):
    """The pre-sliced path with B = 2 and N = 256: four blocks of 128 rows of X, each with its own digit records and
    inverse scales in the workspace.  Bit-identical to tc_tbmm; sampled columns against the oracle."""
    B, N, M, K = 2, 256, 8192, 2048
    rng = np.random.default_rng(52)
    X = rng.standard_normal((B, N, K)).astype(np.float32)
    Y = rng.standard_normal((B, M, K)).astype(np.float32)
    X[1, 130] *= 1e6      # rows of very different scale in different blocks
    X[0, 7, 256:384] = 0  # an all-zero (row, k block)
    Xd, Yd = dev(X), dev(Y)
    need = tc.tc_tbmm_workspace_bytes(B, N, M, K)
    assert need == 2 * 2 * 16 * (65536 + 1024)
    ws = torch.randint(0, 255, (need,), dtype=torch.uint8, device="cuda")
    Z0 = torch.full((B, N, M), float("nan"), device="cuda")
    Z1 = torch.full((B, N, M), float("nan"), device="cuda")
    tc.tc_tbmm(Xd, Yd, Z0)
    assert tc.last_path() == "tbmm:i8"
    tc.tc_tbmm_ws(Xd, Yd, Z1, ws)
    assert tc.last_path() == "tbmm:i8_presliced"
    assert torch.equal(Z0, Z1)
    pick = np.sort(rng.choice(M, size=48, replace=False))
    pick[:3] = [0, 63, 64]
    pick[-1] = M - 1
    ref = oracle.tbmm(X, np.ascontiguousarray(Y[:, pick]))
    got = Z1[:, :, torch.from_numpy(pick).cuda()].cpu().numpy().astype(np.float64)
    # row 130 of batch 1 is 10^6 times the others: every row on its own scale
    worst = max(parity_error(got[b, n], ref[b, n]) for b in range(B) for n in range(N))
    print("tbmm_ws (2,256,8192,2048), 48 sampled columns, worst row: %.3e" % worst, flush=True)
    assert worst <= TIGHT_I8


def test_tmm_largest_paper_shape_sampled(tc, oracle_threads):
    """Section 7, tmm (M,K,N) = (128,4096,16384) through tc_tbmm with B = 1: full size on the GPU, sampled columns in the oracle."""
    rng = np.random.default_rng(77)
    X = rng.standard_normal((1, 128, 4096)).astype(np.float32)
    Y = rng.standard_normal((1, 16384, 4096)).astype(np.float32)
    Z = torch.full((1, 128, 16384), float("nan"), device="cuda")
    tc.tc_tbmm(dev(X), dev(Y), Z)
    torch.cuda.synchronize()
    assert not torch.isnan(Z).any()
    pick = np.sort(rng.choice(16384, size=96, replace=False))
    pick[:4] = [0, 63, 64, 16383]
    ref = oracle.tbmm(X, np.ascontiguousarray(Y[:, pick]))
    assert tc.last_path() == "tbmm:i8"
    check(Z[:, :, torch.from_numpy(pick).cuda()], ref, "tmm 128x4096x16384, 96 sampled columns", TIGHT_I8)
    # every workgroup's output: the whole result against the whole result of the fp64 kernels (which the sampled
    # columns pin to the oracle as well)
    Z64 = torch.full((1, 128, 16384), float("nan"), device="cuda")
    with tc.option(tc.TC_OPT_INT8, tc.TC_INT8_OFF):
        tc.tc_tbmm(dev(X), dev(Y), Z64)
        assert tc.last_path() != "tbmm:i8"
    check(Z64[:, :, torch.from_numpy(pick).cuda()], ref, "tmm 128x4096x16384 on the fp64 path, 96 sampled columns")
    torch.cuda.synchronize()
    err = parity_error(Z.cpu().numpy().astype(np.float64), Z64.cpu().numpy().astype(np.float64))
    print("tmm 128x4096x16384: int8 path against fp64 path, whole output: %.3e" % err, flush=True)
    assert err <= TIGHT_I8
    # with X sliced once into a workspace: the same digits and sums, bit for bit
    ws = torch.empty(tc.tc_tbmm_workspace_bytes(1, 128, 16384, 4096), dtype=torch.uint8, device="cuda")
    Zw = torch.full((1, 128, 16384), float("nan"), device="cuda")
    tc.tc_tbmm_ws(dev(X), dev(Y), Zw, ws)
    assert tc.last_path() == "tbmm:i8_presliced" and torch.equal(Z, Zw)


@pytest.mark.parametrize("shape", [
    (32, 32, 16, 16, 14, 14, 3, 3),
    (32, 32, 32, 32, 7, 7, 3, 3),
    (32, 32, 4, 4, 56, 56, 3, 3),
    (32, 32, 8, 8, 28, 28, 3, 3),
])
def test_gconv_paper_table_shapes_full_size_sampled(tc, oracle_threads, shape):
    """Section 7, grouped-convolution table: full size on the GPU, four sampled images in the oracle."""
    N, G, C, F, H, W, KH, KW = shape
    I, W1, bias = inputs.make_gconv(*shape, seed=55)
    O = torch.full((N, G, F, H - KH + 1, W - KW + 1), float("nan"), device="cuda")
    tc.tc_group_conv(dev(I), dev(W1), dev(bias), O)
    torch.cuda.synchronize()
    assert not torch.isnan(O).any()
    pick = np.array([0, 13, 14, 31])
    ref = oracle.group_conv(np.ascontiguousarray(I[pick]), W1, bias)
    path = tc.last_path()
    check(O[torch.from_numpy(pick).cuda()], ref, "gconv %s, images %s" % (shape, pick.tolist()),
          tight_for_last_call(tc))
    # every workgroup's output: where the default is an int8 kernel, its whole result against the whole result of
    # the fp64 kernel (which the sampled images pin to the oracle as well)
    if ":i8" in path:
        O64 = torch.full(O.shape, float("nan"), device="cuda")
        with tc.option(tc.TC_OPT_INT8, tc.TC_INT8_OFF):
            tc.tc_group_conv(dev(I), dev(W1), dev(bias), O64)
            assert ":i8" not in tc.last_path()
        check(O64[torch.from_numpy(pick).cuda()], ref, "gconv %s on the fp64 path, images %s" % (shape, pick.tolist()))
        torch.cuda.synchronize()
        err = parity_error(O.cpu().numpy().astype(np.float64), O64.cpu().numpy().astype(np.float64))
        print("gconv %s: %s against the fp64 kernel, whole output: %.3e" % (shape, path, err), flush=True)
        assert err <= TIGHT_I8


def test_kron_and_gconv_stay_inside_their_outputs(tc, oracle_threads):
    # canaries on both sides of the outputs survive
    W1, W2, X = inputs.make_kron(5, 40, 64, 64, 64, seed=32)  # 40 rows: the tuned kernel with a ragged row block
    buf = torch.full((5 * 40 * 64 + 512,), 777.0, device="cuda")
    Yv = buf[256:256 + 5 * 40 * 64].view(5, 40, 64)
    tc.tc_kron(dev(W1), dev(W2), dev(X), Yv)
    check(Yv, oracle.kron(W1, W2, X), "kron guard band")
    assert torch.all(buf[:256] == 777.0) and torch.all(buf[256 + 5 * 40 * 64:] == 777.0)

    for H in (21, 26):  # fp64 band kernel with a ragged last band; int8 kernel, three whole bands
        Ig, Wg, bias = inputs.make_gconv(1, 2, 16, 16, H, 58, 3, 3, seed=33)
        n = 1 * 2 * 16 * (H - 2) * 56
        buf = torch.full((n + 512,), 777.0, device="cuda")
        Ov = buf[256:256 + n].view(1, 2, 16, H - 2, 56)
        tc.tc_group_conv(dev(Ig), dev(Wg), dev(bias), Ov)
        check(Ov, oracle.group_conv(Ig, Wg, bias), "gconv guard band H=%d" % H, TIGHT_I8)
        assert torch.all(buf[:256] == 777.0) and torch.all(buf[256 + n:] == 777.0)
