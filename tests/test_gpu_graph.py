"""The entry points under HIP graph capture, and stream positions held on the device: a step
recorded once must give, on every replay, what the same calls give when launched directly, and
with device-resident counters a replay after advancing them must give the codes of the new
positions."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import DEV, host_src, oracle_codes, say
from paper_2511_00874_amd import lib as L
from paper_2511_00874_amd import synth

pytestmark = pytest.mark.gpu


def test_device_counter_gives_the_codes_of_the_same_host_offset():
    x = torch.from_numpy(synth.gaussian((300, 200), 2.0, 3)).to(DEV)
    for off in (0, 77, (1 << 40) + 5):
        ctr = torch.tensor([off], dtype=torch.int64, device=DEV)
        for kind in (L.INT8, L.INT4, L.E5M2):
            for tr in (False, True):
                a = L.sr_quantize(x, L.Quant(kind, 0.05, seed=9, counter_offset=ctr), transpose_out=tr)
                b = L.sr_quantize(x, L.Quant(kind, 0.05, seed=9, counter_offset=off), transpose_out=tr)
                assert torch.equal(a, b), (off, kind, tr)
    ragged = torch.from_numpy(synth.gaussian((4099,), 1.0, 4)).to(DEV)
    ctr = torch.tensor([12345], dtype=torch.int64, device=DEV)
    got = L.sr_quantize(ragged, L.Quant(L.E4M3, 0.1, seed=2, counter_offset=ctr)).cpu().numpy()
    assert np.array_equal(got, oracle_codes(ragged, L.E4M3, 0.1, 2, 12345))


def _layer_state(M, N, K, seed):
    A, W, dY = synth.single_layer(M, N, K, seed, std_dy=1e-3)
    t = {"A": torch.from_numpy(A).to(DEV), "W": torch.from_numpy(W).to(DEV), "dY": torch.from_numpy(dY).to(DEV)}
    kinds = {"A_fwd": L.INT8, "W_fwd": L.INT8, "A_bwd": L.E5M2, "W_bwd": L.E5M2, "dY_bwd": L.E5M2}
    scales = torch.empty(5, device=DEV)
    counters = torch.zeros(5, dtype=torch.int64, device=DEV)
    base = [0, 1 << 20, 2 << 20, 3 << 20, 4 << 20]
    counters.copy_(torch.tensor(base, dtype=torch.int64))
    q = {n: L.Quant(k, scales[i:i + 1], seed=seed, counter_offset=counters[i:i + 1]) for i, (n, k) in enumerate(kinds.items())}
    absmax = L.AbsmaxBatch([(t[n.split("_")[0]], k, scales[i:i + 1]) for i, (n, k) in enumerate(kinds.items())])
    out = {"Y": torch.zeros((M, N), device=DEV), "dA": torch.zeros((M, K), device=DEV), "dW": torch.zeros((N, K), device=DEV)}
    ws = torch.empty(max(L.sr_linear_workspace_bytes(op, M, N, K) for op in (L.OP_FWD, L.OP_BWD)), dtype=torch.uint8, device=DEV)

    def step():
        absmax.run()
        L.sr_linear_fwd(t["A"], t["W"], q["A_fwd"], q["W_fwd"], out=out["Y"], workspace=ws)
        L.sr_linear_bwd(t["dY"], t["W"], t["A"], q["dY_bwd"], q["W_bwd"], q["A_bwd"], out_dA=out["dA"], out_dW=out["dW"],
                        workspace=ws)
    return t, kinds, scales, counters, base, out, step


def test_captured_step_replays_like_direct_launches_and_follows_device_counters():
    say("graph replay")
    M, N, K, seed = 272, 144, 208, 6
    t, kinds, scales, counters, base, out, step = _layer_state(M, N, K, seed)
    step()
    torch.cuda.synchronize()
    eager0 = {k: v.clone() for k, v in out.items()}
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        step()                      # warm up on the capture stream (first-use attribute calls)
        torch.cuda.synchronize()
        g.capture_begin()
        step()
        g.capture_end()
    torch.cuda.synchronize()
    for rep in range(3):
        # replay at the recorded positions, with direct work and synchronisation in between
        for v in out.values():
            v.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(out[k], eager0[k]) for k in out), rep
        # advance the device counters as a training loop would, replay, compare with direct
        # launches at the same positions
        counters.add_(7 + rep)
        g.replay()
        torch.cuda.synchronize()
        replayed = {k: v.clone() for k, v in out.items()}
        for v in out.values():
            v.zero_()
        step()
        torch.cuda.synchronize()
        assert all(torch.equal(out[k], replayed[k]) for k in out), rep
        assert not torch.equal(replayed["dW"], eager0["dW"])
        counters.copy_(torch.tensor(base, dtype=torch.int64))
    # and the advanced positions are the ones the oracle would use: forward product of the last shift
    shift = 7 + 2
    counters.add_(shift)
    g.replay()
    torch.cuda.synchronize()
    hA, hW = host_src(t["A"]), host_src(t["W"])
    sc = scales.cpu().numpy()
    assert float(sc[0]) == oracle.absmax_scale(hA, oracle.INT8)
    ref, ab = oracle.linear_fwd(hA, hW, oracle.Quant(oracle.INT8, float(sc[0]), seed, base[0] + shift),
                                oracle.Quant(oracle.INT8, float(sc[1]), seed, base[1] + shift), want_abs=True)
    assert np.all(np.abs(out["Y"].cpu().numpy().astype(np.float64) - ref) <= 1e-5 * ab + 1e-30)
