"""tc_mlp_fcrelu_static: the MLP chain on the library's static scratch array, for callers that cannot allocate.

Through the raw C ABI, two calls in a row, the second with a smaller input: each must give exactly what
tc_mlp_fcrelu gives with a caller-supplied workspace (same kernels, same arithmetic), which in turn is held to the
parity bar against the float64 oracle.  A chain that needs more than the static array is refused before any launch.
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_1802_04730_amd import inputs
from paper_1802_04730_amd.metric import PARITY_BAR, parity_error

pytestmark = pytest.mark.gpu


def _raw_args(I, Ws, bs, Os):
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    n = len(Ws)
    dims = [I.shape[1]] + [w.shape[0] for w in Ws]
    return (I.data_ptr(), I.shape[0], n, (i64 * (n + 1))(*dims), (vp * n)(*[w.data_ptr() for w in Ws]),
            (vp * n)(*[b.data_ptr() for b in bs]), (vp * n)(*[o.data_ptr() for o in Os]))


def _run_both(tc, batch, dims, seed):
    L = tc.lib()
    I, Ws, bs = inputs.make_mlp(batch, dims, seed=seed)
    dI = torch.from_numpy(I).cuda()
    dW = [torch.from_numpy(w).cuda() for w in Ws]
    db = [torch.from_numpy(b).cuda() for b in bs]
    stream = torch.cuda.current_stream().cuda_stream
    # the existing entry point, caller-supplied workspace
    O_ws = [torch.full((batch, w.shape[0]), float("nan"), device="cuda") for w in Ws]
    nbytes = tc.tc_mlp_fcrelu_workspace_bytes(batch, dims)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    a = _raw_args(dI, dW, db, O_ws)
    assert L.tc_mlp_fcrelu(*a, ws.data_ptr(), ws.numel(), stream) == 0
    # the entry point that allocates nothing
    O_st = [torch.full((batch, w.shape[0]), float("nan"), device="cuda") for w in Ws]
    a = _raw_args(dI, dW, db, O_st)
    before = torch.cuda.memory_allocated()
    assert L.tc_mlp_fcrelu_static(*a, stream) == 0
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    ref = oracle.mlp_fcrelu(I, Ws, bs)
    for l in range(len(Ws)):
        got = O_st[l].cpu().numpy()
        assert np.array_equal(got, O_ws[l].cpu().numpy()), "layer %d differs from tc_mlp_fcrelu" % l
        err = parity_error(got.astype(np.float64), ref[l])
        print("static-scratch MLP batch %d dims %s layer %d: parity error %.3e" % (batch, dims, l, err), flush=True)
        assert err <= PARITY_BAR


def test_mlp_static_scratch_two_calls_second_smaller(oracle_threads):
    from paper_1802_04730_amd import tc355 as tc
    assert torch.cuda.is_available()
    _run_both(tc, 128, (1024, 1024, 512, 256), seed=inputs.SEED_BASE + 3)   # benchmark configuration 3
    _run_both(tc, 24, (96, 200, 64), seed=77)                               # smaller, ragged tiles, two layers
    _run_both(tc, 5, (30, 50, 7), seed=78)                                  # reduction not a multiple of 4: per-layer kernels


def test_mlp_static_scratch_limit_is_refused_before_any_launch():
    from paper_1802_04730_amd import tc355 as tc
    L = tc.lib()
    batch, dims = 2048, (64, 1024, 64)          # 2048 x 1024 fp64 activations = 16 MiB > 8 MiB
    assert tc.tc_mlp_fcrelu_workspace_bytes(batch, dims) > tc.TC_MLP_STATIC_SCRATCH_BYTES
    I = torch.zeros((batch, dims[0]), device="cuda")
    Ws = [torch.zeros((dims[l + 1], dims[l]), device="cuda") for l in range(2)]
    bs = [torch.zeros((dims[l + 1],), device="cuda") for l in range(2)]
    Os = [torch.full((batch, dims[l + 1]), 7.0, device="cuda") for l in range(2)]
    st = L.tc_mlp_fcrelu_static(*_raw_args(I, Ws, bs, Os), torch.cuda.current_stream().cuda_stream)
    assert st == 8 and b"SCRATCH" in L.tc_status_string(st)
    torch.cuda.synchronize()
    assert all(bool((o == 7.0).all()) for o in Os), "nothing may be written on error"
