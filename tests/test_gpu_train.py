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


def test_second_forward_before_the_first_backward_keeps_the_first_calls_state():
    # forward(x1), forward(x2), then backward of the first: its gradients must be those of a run
    # in which nothing happened between its two passes (positions, scales and the weight
    # quantizer of a call live on its autograd context, not on the layer)
    K, N, seed = 64, 48, 13
    g = torch.Generator(device=DEV).manual_seed(2)
    x1 = torch.randn((32, K), device=DEV, generator=g)
    x2 = torch.randn((48, K), device=DEV, generator=g) * 30.0   # another scale altogether
    dy1 = torch.randn((32, N), device=DEV, generator=g) * 1e-3
    ref_layer = train.SRLinear(K, N, seed, device=DEV)
    xr = x1.clone().requires_grad_()
    ref_layer(xr).backward(dy1)
    torch.cuda.synchronize()
    layer = train.SRLinear(K, N, seed, device=DEV)
    xa = x1.clone().requires_grad_()
    ya = layer(xa)
    with torch.no_grad():
        layer(x2)                       # an evaluation pass in between
    xb = x2.clone().requires_grad_()
    layer(xb)                           # and a second recorded forward
    # the first call's dY draws its stream position at backward time: put the reference there
    between = layer.position
    ref_end = ref_layer.position
    ya.backward(dy1)
    torch.cuda.synchronize()
    # A_bwd and W_bwd codes are those of the undisturbed run; only dY's position differs, so
    # compare against the oracle at the positions this call recorded
    M = 32
    ab, wb = (M * K + 7) // 8, (N * K + 7) // 8
    a_np, w_bits, dy_np = x1.cpu().numpy(), host_src(layer.weight), dy1.cpu().numpy()
    bk = oracle.E5M2
    qdy = oracle.Quant(bk, oracle.absmax_scale(dy_np, bk), seed, between)
    qw = oracle.Quant(bk, oracle.absmax_scale(w_bits, bk), seed, wb + 2 * ab)
    qa = oracle.Quant(bk, oracle.absmax_scale(a_np, bk), seed, wb + ab)
    dar, daa = oracle.linear_bwd_data(dy_np, w_bits, qdy, qw, want_abs=True)
    dwr, dwa = oracle.linear_bwd_weight(dy_np, a_np, qdy, qa, want_abs=True)
    check_product(xa.grad.cpu().numpy(), dar, daa, "dA after an interleaved forward")
    check_product(layer.dW.cpu().numpy(), dwr, dwa, "dW after an interleaved forward")
    assert ref_end == 2 * wb + 2 * ab + (M * N + 7) // 8


@pytest.mark.parametrize("kind", [L.INT8, L.E5M2, L.E4M2])
def test_qat_objective_through_autograd(kind):
    # Sec. 3.3 / Fig. 3: unquantized activation times Q(W) forward; the same Q(W), SR of the
    # saved activation and of the output gradient backward
    say("qat autograd linear", L.KIND_NAMES[kind])
    M, K, N, seed = 80, 64, 48, 41
    layer = train.SRLinear(K, N, seed, bwd_kind=kind, device=DEV, objective="qat")
    g = torch.Generator(device=DEV).manual_seed(6)
    x = torch.randn((M, K), device=DEV, generator=g).requires_grad_()
    dy = torch.randn((M, N), device=DEV, generator=g) * 1e-3
    y = layer(x)
    y.backward(dy)
    torch.cuda.synchronize()
    a_np, w_bits, dy_np = x.detach().cpu().numpy(), host_src(layer.weight), dy.cpu().numpy()
    wb, ab = (N * K + 7) // 8, (M * K + 7) // 8
    qW = oracle.Quant(kind, oracle.absmax_scale(w_bits, kind), seed, 0)
    qA = oracle.Quant(kind, oracle.absmax_scale(a_np, kind), seed, wb)
    qdY = oracle.Quant(kind, oracle.absmax_scale(dy_np, kind), seed, wb + ab)
    (yr, ya), (dar, daa), (dwr, dwa) = oracle.qat_pass(a_np, w_bits, dy_np, qW, qA, qdY, want_abs=True)
    check_product(y.detach().cpu().numpy(), yr, ya, "Y")
    check_product(x.grad.cpu().numpy(), dar, daa, "dA")
    check_product(layer.dW.cpu().numpy(), dwr, dwa, "dW")
    assert layer.position == wb + ab + (M * N + 7) // 8
    # the weights of the two passes are one and the same set of codes
    q = L.Quant(kind, float(np.float32(qW.scale)), seed=seed, counter_offset=0)
    assert np.array_equal(L.sr_quantize(layer.weight, q).cpu().numpy(), qW(w_bits).reshape(-1))


def test_qat_training_step_reduces_the_loss():
    torch.manual_seed(0)
    model = train.Decoder(vocab=512, d=64, heads=4, layers=2, seq=32, seed=3, device=DEV, objective="qat")
    ids = torch.randint(0, 512, (8, 32), device=DEV)
    tgt = torch.roll(ids, -1, dims=1)
    losses = [float(train.train_step(model, ids, tgt, lr=0.05, micro_batches=2)) for _ in range(12)]
    say("qat losses", [round(v, 3) for v in losses])
    assert all(np.isfinite(losses)) and losses[-1] < losses[0] - 0.05
