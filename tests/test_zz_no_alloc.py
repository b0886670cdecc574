"""The allocation-free forward entry point (static device scratch inside the library) against
the ordinary one and against the oracle: two calls in a row, the second on a smaller problem, so
that stale contents of the shared array from the first call would show."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
from gpu_util import DEV, check_product, say, to_dev
from paper_2511_00874_amd import lib as L
from paper_2511_00874_amd import synth

pytestmark = pytest.mark.gpu


def _case(M, N, K, seed, kind):
    A, W, _ = synth.single_layer(M, N, K, seed=seed)
    tA, tW = to_dev(A), to_dev(W)
    sA, sW = oracle.absmax_scale(A, kind), oracle.absmax_scale(W, kind)
    qA = L.Quant(kind, sA, seed=seed, counter_offset=5)
    qW = L.Quant(kind, sW, seed=seed, counter_offset=5 + (M * K + 7) // 8)
    oqA = oracle.Quant(kind, sA, seed, 5)
    oqW = oracle.Quant(kind, sW, seed, 5 + (M * K + 7) // 8)
    return (A, W, tA, tW, qA, qW, oqA, oqW)


def _raw_static(out, tA, tW, qA, qW, M, N, K):
    """Straight through the C symbol: no workspace argument exists."""
    return L.raw.sr_linear_fwd_static(out.data_ptr(), tA.data_ptr(), L.F32, tW.data_ptr(), L.F32, M, N, K,
                                      C.byref(qA.c()), C.byref(qW.c()), torch.cuda.current_stream().cuda_stream)


@pytest.mark.parametrize("kind", [L.INT8, L.E5M2])
def test_static_scratch_forward_twice_second_smaller(kind):
    # first call: several tiles, ragged edges, and a contraction long enough to be cut in slices
    # (partials in the scratch); second call: a smaller problem over the same array
    for (M, N, K) in ((272, 208, 4096), (64, 128, 128)):
        say("static-scratch forward", L.KIND_NAMES[kind], M, N, K)
        A, W, tA, tW, qA, qW, oqA, oqW = _case(M, N, K, 11, kind)
        want = L.sr_linear_fwd(tA, tW, qA, qW)
        got = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
        assert _raw_static(got, tA, tW, qA, qW, M, N, K) == L.OK
        torch.cuda.synchronize()
        assert torch.equal(got, want)                      # same kernels, same arithmetic
        ref, ref_abs = oracle.linear_fwd(A, W, oqA, oqW, want_abs=True)
        check_product(got.cpu().numpy(), ref, ref_abs, "Y static")
        if kind == L.INT8:  # integer path: exact accumulators, one rounding
            assert np.array_equal(got.cpu().numpy(), ref)


def test_static_scratch_limit_is_an_error_not_a_launch():
    limit = L.raw.sr_linear_fwd_static_limit()
    assert limit == 32 << 20
    M, N, K = 8192, 8192, 4096   # 64 MiB of codes
    assert L.sr_linear_workspace_bytes(L.OP_FWD, M, N, K) > limit
    q = L.Quant(L.INT8, 1.0)
    # the size check comes first: the (tiny, wrong-size) tensors are never touched
    t = torch.zeros(16, dtype=torch.float32, device=DEV)
    st = L.raw.sr_linear_fwd_static(t.data_ptr(), t.data_ptr(), L.F32, t.data_ptr(), L.F32, M, N, K,
                                    C.byref(q.c()), C.byref(q.c()), None)
    assert st == -8 and "static" in L.status_string(st)
