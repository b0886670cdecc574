"""Helpers for the GPU parity tests: oracle <-> library glue (no arithmetic of the method)."""
import numpy as np
import torch

import oracle
from paper_2511_00874_amd import lib as L

DEV = "cuda:0"
KINDS = [L.INT8, L.INT4, L.E4M3, L.E5M2, L.E4M2, L.E4M1, L.E4M0]


def say(*a):
    print(*a, flush=True)


def to_dev(x_np, bf16=False):
    t = torch.from_numpy(np.ascontiguousarray(x_np)).to(DEV)
    return t.to(torch.bfloat16) if bf16 else t


def host_src(t):
    """numpy view the oracle accepts: float32, or uint16 bit patterns for bfloat16."""
    if t.dtype == torch.bfloat16:
        return t.cpu().view(torch.int16).numpy().view(np.uint16)
    return t.cpu().numpy()


def oracle_codes(t, kind, scale, seed, off, mode=oracle.SR, transpose=False, packed=True):
    """What sr_quantize must return for tensor t (bytes, packed for int4)."""
    src = host_src(t)
    codes = oracle.quantize(src, kind, scale, seed, off, mode)
    if transpose:
        codes = np.ascontiguousarray(codes.T)
    flat = codes.reshape(-1)
    return oracle.pack_int4(flat) if (kind == L.INT4 and packed) else flat


def check_product(got, ref, ref_abs, what=""):
    """The parity bar for products: fp32 accumulation over identical quantized operands."""
    got = got.astype(np.float64).reshape(-1)
    ref = ref.astype(np.float64).reshape(-1)
    bound = 1e-5 * ref_abs.astype(np.float64).reshape(-1)
    err = np.abs(got - ref)
    worst = int(np.argmax(err - bound))
    assert np.all(err <= bound + 1e-30), (what, worst, got[worst], ref[worst], bound[worst])
    assert err.max() <= 1e-5 * max(np.abs(ref).max(), 1e-30), what


def check_product_f8_pipeline(got, ref, group_max_sum, ref_abs, what=""):
    """Bar for the fp8 matrix pipeline, derived from its arithmetic: the products of each run
    of 8 consecutive contraction indices are aligned to the largest and truncated to 14 bits,
    so each of the other 7 loses less than 2^-13 of the group's largest |product|."""
    got = got.astype(np.float64).reshape(-1)
    ref = ref.astype(np.float64).reshape(-1)
    bound = 7 * 2.0**-13 * group_max_sum.reshape(-1) + 1e-6 * ref_abs.astype(np.float64).reshape(-1)
    err = np.abs(got - ref)
    worst = int(np.argmax(err - bound))
    assert np.all(err <= bound + 1e-30), (what, worst, got[worst], ref[worst], bound[worst])


def group_max_sum(Xv, Zv, scale):
    """sum over groups of 8 consecutive r of max_r |X[p][r] Z[q][r]|, for all (p, q)."""
    P, R = Xv.shape
    Q = Zv.shape[0]
    pad = (-R) % 8
    Xg = np.pad(np.abs(Xv), ((0, 0), (0, pad))).reshape(P, -1, 8)
    Zg = np.pad(np.abs(Zv), ((0, 0), (0, pad))).reshape(Q, -1, 8)
    out = np.zeros((P, Q))
    for g in range(Xg.shape[1]):
        out += (Xg[:, None, g, :] * Zg[None, :, g, :]).max(axis=2)
    return out * scale
