"""The C-ABI library loads and exports what include/srq.h declares; host-side argument checks.

No GPU here: every call below is rejected by validation before anything is launched.
"""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2511_00874_amd import build
    if build.stale():
        build.build()
    from paper_2511_00874_amd import lib as L
    return L


def _declared():
    text = open(os.path.join(ROOT, "include", "srq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sr_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert len(names) >= 14
    for n in names:
        assert hasattr(lib.raw, n), n
    assert sorted(lib.EXPORTS) == names


def test_struct_layout_matches_header(lib):
    assert C.sizeof(lib.srq_quant) == 40
    assert lib.srq_quant.scale_dev.offset == 16
    assert lib.srq_quant.seed.offset == 24
    assert lib.srq_quant.counter_offset.offset == 32


def test_status_strings(lib):
    seen = {lib.status_string(s) for s in range(0, -9, -1)}
    assert len(seen) == 9 and "ok" in seen
    assert lib.status_string(-99) == "unknown status"


def _q(lib, kind=1, rnd=0, scale=1.0, flags=0):
    q = lib.srq_quant()
    q.kind, q.round, q.scale, q.flags, q.scale_dev, q.seed, q.counter_offset = kind, rnd, scale, flags, None, 0, 0
    return q


def test_quantize_argument_checks(lib):
    r = lib.raw
    buf = 0x1000  # never dereferenced: validation fails first
    assert r.sr_quantize(buf, buf, 0, 4, 8, 0, None, None) == -1
    assert r.sr_quantize(None, buf, 0, 4, 8, 0, C.byref(_q(lib)), None) == -1
    assert r.sr_quantize(buf, buf, 0, 4, 8, 0, C.byref(_q(lib, kind=9)), None) == -3
    assert r.sr_quantize(buf, buf, 0, 4, 8, 0, C.byref(_q(lib, kind=0)), None) == -6
    assert r.sr_quantize(buf, buf, 0, 4, 8, 0, C.byref(_q(lib, rnd=5)), None) == -3
    assert r.sr_quantize(buf, buf, 7, 4, 8, 0, C.byref(_q(lib)), None) == -3
    for bad in (0.0, -1.0, float("inf"), float("nan"), 1e-45):
        assert r.sr_quantize(buf, buf, 0, 4, 8, 0, C.byref(_q(lib, scale=bad)), None) == -3
    assert r.sr_quantize(buf, buf, 0, 4, 8, 0, C.byref(_q(lib, flags=8)), None) == -3
    assert r.sr_quantize(buf, buf, 0, 4, 8, 0, C.byref(_q(lib, flags=2)), None) == -4    # device counter: NULL address
    assert r.sr_quantize(buf, buf + 4, 0, 4, 8, 0, C.byref(_q(lib)), None) == -4
    assert r.sr_quantize(buf, buf, 0, 4, 12, 1, C.byref(_q(lib)), None) == -4       # cols % 8
    assert r.sr_quantize(buf, buf, 0, 3, 5, 0, C.byref(_q(lib, kind=2)), None) == -4  # odd int4 count
    assert r.sr_quantize(buf, buf, 0, 3, 8, 1, C.byref(_q(lib, kind=2)), None) == -4  # odd rows, int4^T
    assert r.sr_quantize(buf, buf, 0, 2**40, 2**40, 0, C.byref(_q(lib)), None) == -2
    # empty input is a no-op, pointers not needed
    assert r.sr_quantize(None, None, 0, 0, 8, 0, C.byref(_q(lib)), None) == 0


def test_update_argument_checks(lib):
    import ctypes as C
    raw = lib.raw
    assert raw.sr_update_bf16(None, None, 0.1, 0, lib.SR, 0, 0, None) == 0          # empty: no-op
    assert raw.sr_update_bf16(None, C.c_void_p(256), 0.1, 8, lib.SR, 0, 0, None) == -1
    assert raw.sr_update_bf16(C.c_void_p(256), C.c_void_p(512), 0.1, 8, 7, 0, 0, None) == -3
    assert raw.sr_update_bf16(C.c_void_p(256), C.c_void_p(512), float("nan"), 8, lib.SR, 0, 0, None) == -3
    assert raw.sr_update_bf16(C.c_void_p(258), C.c_void_p(512), 0.1, 8, lib.SR, 0, 0, None) == -4


def test_linear_argument_checks(lib):
    r = lib.raw
    buf = 0x1000
    q8, qf = _q(lib, 1), _q(lib, 3)
    ws = 1 << 30
    args = (buf, buf, 0, buf, 0)
    assert r.sr_linear_fwd(*args, 64, 128, 128, C.byref(q8), C.byref(q8), None, 0, None) == -5
    assert r.sr_linear_fwd(*args, 64, 128, 128, C.byref(q8), C.byref(q8), buf, 16, None) == -5
    assert r.sr_linear_fwd(*args, 64, 128, 120, C.byref(q8), C.byref(q8), buf, ws, None) == -4
    assert r.sr_linear_fwd(*args, 0, 128, 128, C.byref(q8), C.byref(q8), buf, ws, None) == -2
    assert r.sr_linear_fwd(*args, 64, 128, 128, C.byref(q8), C.byref(qf), buf, ws, None) == -6
    # the two operands must agree on the matrix pipeline for 8-bit floats
    assert r.sr_linear_fwd(*args, 64, 128, 128, C.byref(qf), C.byref(_q(lib, 4, flags=1)), buf, ws, None) == -6
    assert r.sr_linear_fwd(None, buf, 0, buf, 0, 64, 128, 128, C.byref(q8), C.byref(q8), buf, ws, None) == -1
    assert r.sr_linear_bwd_weight(*args, 64, 128, 128, C.byref(q8), C.byref(q8), 0.5, buf, ws, None) == -6
    # int32 accumulation bound: contraction longer than 2^31 / 127^2
    assert r.sr_linear_bwd_weight(*args, 133168, 16, 16, C.byref(q8), C.byref(q8), 0.0, buf, 1 << 40, None) == -6
    # an operand matrix of 2 GiB or more (32-bit buffer offsets inside the product kernel)
    assert r.sr_linear_fwd(*args, 1 << 20, 128, 4096, C.byref(q8), C.byref(q8), buf, 1 << 40, None) == -6
    q52 = _q(lib, 4)
    assert r.sr_linear_bwd(buf, buf, buf, 0, buf, 0, buf, 0, 1 << 20, 2048, 128, C.byref(q52), C.byref(q52), C.byref(q52),
                           0.0, buf, 1 << 40, None) == -6
    # the stash pair: integer forward formats only; a missing stash is a workspace error
    assert r.sr_linear_fwd_stash(*args, 64, 128, 128, C.byref(qf), C.byref(qf), C.byref(q52), C.byref(q52), buf, ws, buf, ws,
                                 None) == -6
    assert r.sr_linear_fwd_stash(*args, 64, 128, 128, C.byref(q8), C.byref(q8), C.byref(q52), C.byref(q52), None, 0, buf, ws,
                                 None) == -5
    assert lib.sr_linear_stash_bytes(64, 128, 128) >= 2 * 128 * (64 + 128)
    # the same pair in halves: an unknown phase is refused before anything else is looked at
    assert r.sr_linear_fwd_stash_phase(*args, 64, 128, 128, C.byref(q8), C.byref(q8), C.byref(q52), C.byref(q52), buf, ws, buf,
                                       ws, 4, None) == -3
    assert r.sr_linear_fwd_stash_phase(*args, 64, 128, 128, C.byref(qf), C.byref(qf), C.byref(q52), C.byref(q52), buf, ws, buf,
                                       ws, 1, None) == -6
    assert r.sr_linear_bwd_stashed_phase(buf, buf, buf, 0, 64, 128, 128, C.byref(q52), C.byref(q52), C.byref(q52), buf, ws,
                                         0.0, buf, ws, 0, None) == -3
    assert r.sr_linear_bwd_stashed_phase(buf, buf, buf, 0, 64, 128, 128, C.byref(q52), C.byref(q52), C.byref(q52), None, 0,
                                         0.0, buf, 1 << 30, 2, None) == -5
    # the identity quantizer: row operand of the forward and input-gradient products only
    q0 = _q(lib, 0)
    assert r.sr_linear_fwd(*args, 64, 128, 128, C.byref(q8), C.byref(q0), buf, ws, None) == -6
    assert r.sr_linear_bwd_weight(*args, 64, 128, 128, C.byref(q0), C.byref(q8), 0.0, buf, ws, None) == -6
    assert r.sr_linear_fwd(*args, 64, 128, 128, C.byref(q0), C.byref(q8), buf, 16, None) == -5
    assert r.sr_linear_fwd(*args, 64, 128, 120, C.byref(q0), C.byref(q8), buf, ws, None) == -4
    assert r.sr_linear_bwd_data(None, buf, 0, buf, 0, 64, 128, 128, C.byref(q0), C.byref(q8), buf, ws, None) == -1
    # the forward product with the quantizers inside it: integer pairs or E5M2 pairs, no workspace
    assert r.sr_linear_fwd_fused(*args, 64, 128, 128, C.byref(qf), C.byref(qf), None) == -6
    assert r.sr_linear_fwd_fused(*args, 64, 128, 128, C.byref(q8), C.byref(q52), None) == -6
    assert r.sr_linear_fwd_fused(*args, 64, 128, 128, C.byref(q0), C.byref(q8), None) == -6
    assert r.sr_linear_fwd_fused(*args, 64, 128, 120, C.byref(q8), C.byref(q8), None) == -4
    assert r.sr_linear_fwd_fused(None, buf, 0, buf, 0, 64, 128, 128, C.byref(q8), C.byref(q8), None) == -1
    assert r.sr_linear_fwd_fused(*args, 1 << 31, 1 << 31, 16, C.byref(q8), C.byref(q8), None) == -6
    # SRQ_FLAG_QUANTIZE_ONCE is a known flag
    assert r.sr_linear_fwd(*args, 64, 128, 128, C.byref(_q(lib, 1, flags=4)), C.byref(q8), None, 0, None) == -5
    assert r.sr_gemm_codes(buf, buf, 1, buf, 3, 16, 16, 16, 1.0, 0.0, None, 0, None) == -6
    assert r.sr_gemm_codes(buf, buf, 1, buf, 1, 16, 16, 24, 1.0, 0.0, None, 0, None) == -4


def test_workspace_sizes(lib):
    M, N, K = 8192, 3072, 768
    fwd = lib.sr_linear_workspace_bytes(lib.OP_FWD, M, N, K)
    assert fwd >= M * K + N * K
    assert lib.sr_linear_workspace_bytes(lib.OP_BWD_DATA, M, N, K) >= M * N + N * K
    assert lib.sr_linear_workspace_bytes(lib.OP_BWD_WEIGHT, M, N, K) >= M * N + M * K
    assert lib.sr_linear_workspace_bytes(99, M, N, K) == 0
    # weight-only products: three bfloat16 planes of the row operand, W as codes and as bfloat16
    assert lib.sr_linear_workspace_bytes(lib.OP_FWD_WEIGHT_ONLY, M, N, K) >= 6 * M * K + 3 * N * K
    assert lib.sr_linear_workspace_bytes(lib.OP_BWD_DATA_WEIGHT_ONLY, M, N, K) >= 6 * M * N + 3 * N * K
    assert lib.sr_linear_workspace_bytes(lib.OP_FWD, 0, N, K) == 0
    assert lib.sr_gemm_workspace_bytes(4096, 4096, 4096) == 0          # enough tiles: no split
    assert lib.sr_gemm_workspace_bytes(256, 256, 65536) > 0            # few tiles, long contraction


def test_compute_calls_need_device_tensors(lib):
    import torch
    x = torch.zeros(16)
    with pytest.raises(RuntimeError):
        lib.sr_quantize(x, lib.Quant(lib.INT8, 1.0))
