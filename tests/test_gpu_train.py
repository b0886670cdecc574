"""The autograd face (Alg. 1 / Alg. 2 through torch.autograd) and the training step with the
bfloat16 weight update of Eq. 10, against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import DEV, check_product, host_src, say
from paper_2511_00874_amd import lib as L
from paper_2511_00874_amd import train

pytestmark = pytest.mark.gpu


def oracle_layer_pass(a, w_bits, dy, seed, kinds=(oracle.INT8, oracle.E5M2)):
    """What one forward + backward of a fresh SRLinear must produce: the stream positions are
    W_fwd, A_fwd, A_bwd, W_bwd, dY_bwd in that order, each tensor ceil(n / 8) blocks."""
    fk, bk = kinds
    M, K = a.shape
    N = w_bits.shape[0]
    ab, wb = (M * K + 7) // 8, (N * K + 7) // 8
    pos = {"W_fwd": 0, "A_fwd": wb, "A_bwd": wb + ab, "W_bwd": wb + 2 * ab, "dY_bwd": 2 * wb + 2 * ab}

    def q(x, kind, name):
        return oracle.Quant(kind, oracle.absmax_scale(x, kind), seed, pos[name])

    y, y_abs = oracle.linear_fwd(a, w_bits, q(a, fk, "A_fwd"), q(w_bits, fk, "W_fwd"), want_abs=True)
    da, da_abs = oracle.linear_bwd_data(dy, w_bits, q(dy, bk, "dY_bwd"), q(w_bits, bk, "W_bwd"), want_abs=True)
    dw, dw_abs = oracle.linear_bwd_weight(dy, a, q(dy, bk, "dY_bwd"), q(a, bk, "A_bwd"), want_abs=True)
    return (y, y_abs), (da, da_abs), (dw, dw_abs), pos["dY_bwd"] + (M * N + 7) // 8


@pytest.mark.parametrize("chunk", [None, 32])
def test_autograd_linear_matches_oracle(chunk, monkeypatch):
    say("autograd linear", chunk)
    if chunk:
        monkeypatch.setattr(train, "MAX_ROWS", chunk)
    M, K, N, seed = 80, 64, 48, 21
    layer = train.SRLinear(K, N, seed, device=DEV)
    g = torch.Generator(device=DEV).manual_seed(4)
    x = torch.randn((5, 16, K), device=DEV, generator=g).requires_grad_()
    dy = torch.randn((5, 16, N), device=DEV, generator=g) * 1e-3
    y = layer(x)
    y.backward(dy)
    torch.cuda.synchronize()
    w_bits = host_src(layer.weight)
    (yr, ya), (dar, daa), (dwr, dwa), end = oracle_layer_pass(x.detach().reshape(M, K).cpu().numpy(), w_bits,
                                                                dy.reshape(M, N).cpu().numpy(), seed)
    check_product(y.detach().cpu().numpy(), yr, ya, "Y")
    check_product(x.grad.cpu().numpy(), dar, daa, "dA")
    check_product(layer.dW.cpu().numpy(), dwr, dwa, "dW")
    assert layer.position == end and layer.have_grad
    # the update of Eq. 10 consumes the accumulated gradient at the next stream position
    grad = layer.dW.cpu().numpy().reshape(-1).copy()
    layer.update(0.5)
    torch.cuda.synchronize()
    assert np.array_equal(host_src(layer.weight).reshape(-1), oracle.update_bf16(w_bits.reshape(-1), grad, 0.5, seed, end))
    assert not layer.have_grad


def test_chunked_rows_give_the_same_codes_as_one_call(monkeypatch):
    # Y and dA rows are independent of the chunking (same codes, same sums): bit-for-bit equal
    M, K, N = 96, 64, 32
    g = torch.Generator(device=DEV).manual_seed(8)
    x0 = torch.randn((M, K), device=DEV, generator=g)
    dy = torch.randn((M, N), device=DEV, generator=g) * 1e-2
    outs = []
    for chunk in (train.MAX_ROWS, 32):
        monkeypatch.setattr(train, "MAX_ROWS", chunk)
        layer = train.SRLinear(K, N, 5, device=DEV)
        x = x0.clone().requires_grad_()
        y = layer(x)
        y.backward(dy)
        torch.cuda.synchronize()
        outs.append((y.detach().clone(), x.grad.clone(), layer.dW.clone()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    assert torch.allclose(outs[0][2], outs[1][2], rtol=1e-5, atol=1e-7 * float(outs[0][2].abs().max()))


def test_micro_batches_accumulate_the_weight_gradient():
    K, N = 64, 32
    layer = train.SRLinear(K, N, 2, device=DEV)
    g = torch.Generator(device=DEV).manual_seed(1)
    parts = []
    for _ in range(2):
        x = torch.randn((32, K), device=DEV, generator=g).requires_grad_()
        layer(x).backward(torch.randn((32, N), device=DEV, generator=g))
        torch.cuda.synchronize()
        parts.append(layer.dW.clone())
    single = train.SRLinear(K, N, 2, device=DEV)
    assert torch.equal(single.weight, layer.weight)
    assert float((parts[1] - parts[0]).abs().max()) > 0  # the second call added to the first


def test_training_step_of_a_small_decoder_reduces_the_loss():
    say("decoder step")
    torch.manual_seed(0)
    model = train.Decoder(vocab=512, d=64, heads=4, layers=2, seq=32, seed=3, device=DEV)
    ids = torch.randint(0, 512, (8, 32), device=DEV)
    tgt = torch.roll(ids, -1, dims=1)
    w0 = model.head.weight.clone()
    losses = [float(train.train_step(model, ids, tgt, lr=0.05, micro_batches=2)) for _ in range(12)]
    say("losses", [round(v, 3) for v in losses])
    assert all(np.isfinite(losses))
    assert losses[-1] < losses[0] - 0.05
    assert not torch.equal(w0, model.head.weight)
    assert train.flops_per_token(model) == 6.0 * (2 * (64 * 192 + 64 * 64 + 2 * 64 * 256) + 64 * 512)


def test_weight_only_objective_through_autograd():
    # Sec. 3.2: one quantized copy of W per forward call, the same in its backward pass;
    # activations and gradients unquantized; dW is then the plain product dY^T A
    say("weight-only autograd linear")
    M, K, N, seed = 80, 64, 48, 31
    layer = train.SRLinear(K, N, seed, device=DEV, weight_only=True)
    g = torch.Generator(device=DEV).manual_seed(6)
    x = torch.randn((M, K), device=DEV, generator=g).requires_grad_()
    dy = torch.randn((M, N), device=DEV, generator=g) * 1e-3
    for rep in range(2):  # the second pass accumulates dW and draws a fresh copy of W
        if x.grad is not None:
            x.grad = None
        start = layer.position
        y = layer(x)
        y.backward(dy)
        torch.cuda.synchronize()
        w_bits = host_src(layer.weight)
        oq = oracle.Quant(oracle.INT8, oracle.absmax_scale(w_bits, oracle.INT8), seed, start)
        yr, ya = oracle.linear_fwd_weight_only(x.detach().cpu().numpy(), w_bits, oq, want_abs=True)
        dar, daa = oracle.linear_bwd_data_weight_only(dy.cpu().numpy(), w_bits, oq, want_abs=True)
        check_product(y.detach().cpu().numpy(), yr, ya, "Y")
        check_product(x.grad.cpu().numpy(), dar, daa, "dA")
        dw = (rep + 1) * (dy.double().t() @ x.detach().double())
        assert torch.allclose(layer.dW.double(), dw, rtol=1e-4, atol=1e-6 * float(dw.abs().max()))
        assert layer.position == start + (N * K + 7) // 8


def test_weight_only_training_step_reduces_the_loss():
    torch.manual_seed(0)
    model = train.Decoder(vocab=512, d=64, heads=4, layers=2, seq=32, seed=3, device=DEV, weight_only=True)
    ids = torch.randint(0, 512, (8, 32), device=DEV)
    tgt = torch.roll(ids, -1, dims=1)
    losses = [float(train.train_step(model, ids, tgt, lr=0.05, micro_batches=2)) for _ in range(12)]
    say("weight-only losses", [round(v, 3) for v in losses])
    assert all(np.isfinite(losses)) and losses[-1] < losses[0] - 0.05
