"""Training with the SR-quantized linear layer: an autograd face of Alg. 1 / Alg. 2 and the
weight update of Eq. 10, plus a small decoder whose linears all go through it.

Only the linears and the weight update are this library's; embedding, layer norm, attention,
GELU and the loss are plain PyTorch operators (they are not quantized in the paper's method,
Sec. 3.1: the quantization sites are the inputs of the matrix products).
"""
import torch
import torch.nn.functional as F

from . import lib as L

# Rows per call: keeps every operand matrix of the products below the library's 2 GiB limit for
# the widest layer used here (32000 outputs in the two-byte form).  Token chunks are independent
# in Y and dA; dW accumulates over them (beta = 1), which is also how micro-batches accumulate.
MAX_ROWS = 16384
NOQ = L.Quant(L.NONE, 1.0)  # the identity quantizer of the weight-only objective


class SRLinearFn(torch.autograd.Function):
    """Everything the backward pass of ONE forward call needs travels on the autograd context:
    the saved activation -- as the codes of its backward quantizer when the forward pass can write
    them (the stash of sr_linear_fwd_stash: integer forward formats), else in binary32 -- the
    stream positions drawn for the backward quantizers of A and W, the scales found for them and (objectives that share one quantized weight copy between the
    passes) the weight quantizer itself.  A second forward of the same layer before the first
    backward therefore cannot disturb the first one's gradients."""

    @staticmethod
    def forward(ctx, x, layer):
        ctx.layer = layer
        ctx.shape = x.shape
        a = x.reshape(-1, x.shape[-1]).contiguous().float()
        y, ctx.saved = layer._forward(a)
        if "stash" not in ctx.saved:  # the backward pass quantizes (or multiplies) the activation itself
            ctx.save_for_backward(a)
        return y.reshape(*x.shape[:-1], layer.out_features)

    @staticmethod
    def backward(ctx, dy):
        a = ctx.saved_tensors[0] if ctx.saved_tensors else None
        layer = ctx.layer
        da = layer._backward(dy.reshape(-1, layer.out_features).contiguous().float(), a, ctx.saved)
        return da.reshape(ctx.shape), None


OBJECTIVES = ("five", "weight_only", "qat")


class SRLinear(torch.nn.Module):
    """y = Q(x) Q(W)^T with the five quantizers of Alg. 1 / Alg. 2 (per-tensor absmax scales,
    fresh stream positions every call); W is held in bfloat16 and updated by Eq. 10.

    The weight gradient is kept by the layer (`self.dW`, float32, accumulated over backward
    calls until `update`), not handed to autograd: the update consumes it in place.

    objective:
      "five"         all five quantizers independent (Alg. 1 / Alg. 2 in general form): A and W
                     to `fwd_kind` in the forward pass, A, W and dY to `bwd_kind` in the backward.
      "weight_only"  Sec. 3.2: only the weights are quantized (to `fwd_kind`, one quantized copy
                     per forward call, used again in its backward pass); activations and
                     gradients stay in binary32, so the weight gradient dY^T A has no quantized
                     operand and is a plain matrix product.
      "qat"          Sec. 3.3 (Fig. 3), the estimator whose expectation is the gradient of the
                     quantization-aware objective (Eq. 6-7): the forward pass multiplies the
                     unquantized activation by Q(W); the backward pass uses the SAME quantized
                     weights (same thresholds: one copy per mini-batch) and stochastically
                     rounds the saved activation and the output gradient.  One format
                     (`bwd_kind`) for all four quantizers, as in the paper (one Delta).
    weight_only=True is kept as a synonym of objective="weight_only"."""

    def __init__(self, in_features, out_features, seed, fwd_kind=L.INT8, bwd_kind=L.E5M2, device="cuda:0",
                 init_std=0.02, round_mode=L.SR, weight_only=False, objective=None):
        super().__init__()
        self.in_features, self.out_features = in_features, out_features
        g = torch.Generator(device=device).manual_seed(seed)
        w = torch.randn((out_features, in_features), device=device, generator=g) * init_std
        self.weight = w.to(torch.bfloat16)           # not an nn.Parameter: autograd never sees it
        self.dW = torch.zeros((out_features, in_features), dtype=torch.float32, device=device)
        self.have_grad = False
        self.objective = objective or ("weight_only" if weight_only else "five")
        assert self.objective in OBJECTIVES
        self.weight_only = self.objective == "weight_only"
        if self.objective == "qat":
            fwd_kind = bwd_kind  # one Delta: the weights are quantized once, for both passes
        self.kinds = {"A_fwd": fwd_kind, "W_fwd": fwd_kind, "A_bwd": bwd_kind, "W_bwd": bwd_kind, "dY_bwd": bwd_kind}
        self.seed, self.position, self.round_mode = seed, 0, round_mode
        self.ws = None

    def _q(self, name, scale, position):
        return L.Quant(self.kinds[name], scale, seed=self.seed, counter_offset=position, round_mode=self.round_mode)

    def _scales(self, n):
        return torch.empty(n, dtype=torch.float32, device=self.weight.device)

    def _workspace(self, op, M):
        need = L.sr_linear_workspace_bytes(op, M, self.out_features, self.in_features)
        if self.ws is None or self.ws.numel() < need:
            self.ws = torch.empty(need, dtype=torch.uint8, device=self.weight.device)
        return self.ws

    # -- objectives that multiply an unquantized activation by Q(W) in the forward pass ---------
    def _forward_unquantized_a(self, a):
        M, K = a.shape
        N = self.out_features
        w = self.weight
        qat = self.objective == "qat"
        sc = self._scales(2)                          # W, and (qat) A for the backward pass
        reqs = [(w, self.kinds["W_fwd"], sc[0:1])]
        if qat:
            reqs.append((a, self.kinds["A_bwd"], sc[1:2]))
        L.sr_absmax_scales(reqs)
        saved = {"qw": self._q("W_fwd", sc[0:1], self.position)}  # the same copy serves the backward pass
        self.position += (N * K + 7) // 8
        if qat:
            saved["sA"], saved["pos_a"] = sc[1:2], self.position
            self.position += (M * K + 7) // 8
        y = torch.empty((M, N), dtype=torch.float32, device=a.device)
        for r0 in range(0, M, MAX_ROWS):
            r1 = min(M, r0 + MAX_ROWS)
            L.sr_linear_fwd(a[r0:r1], w, NOQ, saved["qw"], out=y[r0:r1],
                            workspace=self._workspace(L.OP_FWD_WEIGHT_ONLY, r1 - r0))
        return y, saved

    def _backward_weight_only(self, dy, a, saved):
        M, N = dy.shape
        da = torch.empty((M, self.in_features), dtype=torch.float32, device=dy.device)
        for r0 in range(0, M, MAX_ROWS):
            r1 = min(M, r0 + MAX_ROWS)
            L.sr_linear_bwd_data(dy[r0:r1], self.weight, NOQ, saved["qw"], out=da[r0:r1],
                                 workspace=self._workspace(L.OP_BWD_DATA_WEIGHT_ONLY, r1 - r0))
        if self.have_grad:
            self.dW.addmm_(dy.t(), a)
        else:
            torch.mm(dy.t(), a, out=self.dW)
        self.have_grad = True
        return da

    def _forward(self, a):
        if self.objective != "five":
            return self._forward_unquantized_a(a)
        M, K = a.shape
        N = self.out_features
        w = self.weight
        sc = self._scales(4)
        L.sr_absmax_scales([(a, self.kinds["A_fwd"], sc[0:1]), (w, self.kinds["W_fwd"], sc[1:2]),
                            (a, self.kinds["A_bwd"], sc[2:3]), (w, self.kinds["W_bwd"], sc[3:4])])
        # every tensor gets its own stretch of the stream (in blocks of 8 elements); a chunk that
        # starts at row r0 continues where the rows before it would have drawn, so the codes do
        # not depend on the chunking.  The backward quantizers of A and W get theirs now.
        a_blocks, w_blocks = (M * K + 7) // 8, (N * K + 7) // 8
        pos_w, pos_a = self.position, self.position + w_blocks
        saved = {"sA": sc[2:3], "pos_a": pos_a + a_blocks,
                 "qw": self._q("W_bwd", sc[3:4], pos_a + 2 * a_blocks)}
        self.position = pos_a + 2 * a_blocks + w_blocks
        y = torch.empty((M, N), dtype=torch.float32, device=a.device)
        qw = self._q("W_fwd", sc[1:2], pos_w)
        # integer forward formats: the same pass over A and W also writes the codes of their backward
        # quantizers (one stash per chunk of rows), and the activation itself need not be kept
        stash = self.kinds["A_fwd"] in (L.INT8, L.INT4)
        if stash:
            saved["stash"] = []
        for r0 in range(0, M, MAX_ROWS):
            r1 = min(M, r0 + MAX_ROWS)
            qa = self._q("A_fwd", sc[0:1], pos_a + (r0 * K) // 8)
            if stash:
                qa_bwd = self._q("A_bwd", saved["sA"], saved["pos_a"] + (r0 * K) // 8)
                _, st = L.sr_linear_fwd_stash(a[r0:r1], w, qa, qw, qa_bwd, saved["qw"], out=y[r0:r1],
                                              workspace=self._workspace(L.OP_FWD_STASH, r1 - r0))
                saved["stash"].append(st)
            else:
                L.sr_linear_fwd(a[r0:r1], w, qa, qw, out=y[r0:r1], workspace=self._workspace(L.OP_FWD, r1 - r0))
        return y, saved

    def _backward(self, dy, a, saved):
        if self.weight_only:
            return self._backward_weight_only(dy, a, saved)
        # "five" and "qat" differ only in where the weight quantizer comes from: its own draw, or
        # the forward pass's (Fig. 3: W_hat is shared by the two passes)
        M, N = dy.shape
        K = self.in_features
        w = self.weight
        sdy = self._scales(1)
        L.sr_absmax_scales([(dy, self.kinds["dY_bwd"], sdy)])
        da = torch.empty((M, K), dtype=torch.float32, device=dy.device)
        pos_dy = self.position
        self.position += (M * N + 7) // 8
        for i, r0 in enumerate(range(0, M, MAX_ROWS)):
            r1 = min(M, r0 + MAX_ROWS)
            qdy = self._q("dY_bwd", sdy, pos_dy + (r0 * N) // 8)
            qa = self._q("A_bwd", saved["sA"], saved["pos_a"] + (r0 * K) // 8)
            beta = 1.0 if self.have_grad else 0.0
            if "stash" in saved:
                L.sr_linear_bwd_stashed(dy[r0:r1], saved["stash"][i], K, qdy, saved["qw"], qa, out_dA=da[r0:r1],
                                        out_dW=self.dW, beta=beta, workspace=self._workspace(L.OP_BWD_STASHED, r1 - r0))
            else:
                L.sr_linear_bwd(dy[r0:r1], w, a[r0:r1], qdy, saved["qw"], qa, out_dA=da[r0:r1], out_dW=self.dW,
                                beta=beta, workspace=self._workspace(L.OP_BWD, r1 - r0))
            self.have_grad = True
        return da

    def forward(self, x):
        return SRLinearFn.apply(x, self)

    def update(self, lr):
        """Eq. 10: W <- Q_SR(W - lr * dW) on the bfloat16 grid; clears the accumulated gradient."""
        if self.have_grad:
            L.sr_update_bf16(self.weight.view(-1), self.dW.view(-1), lr, seed=self.seed, counter_offset=self.position,
                             round_mode=self.round_mode)
            self.position += (self.weight.numel() + 7) // 8
            self.have_grad = False


class Block(torch.nn.Module):
    def __init__(self, d, heads, seed, device, objective="five"):
        super().__init__()
        self.heads = heads
        self.ln1 = torch.nn.LayerNorm(d, device=device)
        self.ln2 = torch.nn.LayerNorm(d, device=device)
        self.qkv = SRLinear(d, 3 * d, seed, device=device, objective=objective)
        self.proj = SRLinear(d, d, seed + 1, device=device, objective=objective)
        self.fc1 = SRLinear(d, 4 * d, seed + 2, device=device, objective=objective)
        self.fc2 = SRLinear(4 * d, d, seed + 3, device=device, objective=objective)

    def forward(self, x):
        B, T, d = x.shape
        q, k, v = self.qkv(self.ln1(x)).view(B, T, 3, self.heads, d // self.heads).permute(2, 0, 3, 1, 4)
        att = F.scaled_dot_product_attention(q.bfloat16(), k.bfloat16(), v.bfloat16(), is_causal=True).float()
        x = x + self.proj(att.transpose(1, 2).reshape(B, T, d))
        return x + self.fc2(F.gelu(self.fc1(self.ln2(x))))


class Decoder(torch.nn.Module):
    """Pre-norm decoder: token + position embedding, `layers` blocks, final norm, output head."""

    def __init__(self, vocab=32000, d=768, heads=12, layers=12, seq=1024, seed=1, device="cuda:0", weight_only=False,
                 objective=None):
        super().__init__()
        objective = objective or ("weight_only" if weight_only else "five")
        self.tok = torch.nn.Embedding(vocab, d, device=device)
        self.pos = torch.nn.Embedding(seq, d, device=device)
        torch.nn.init.normal_(self.tok.weight, std=0.02)
        torch.nn.init.normal_(self.pos.weight, std=0.02)
        self.blocks = torch.nn.ModuleList([Block(d, heads, seed + 10 * i, device, objective) for i in range(layers)])
        self.ln = torch.nn.LayerNorm(d, device=device)
        self.head = SRLinear(d, vocab, seed + 10 * layers, device=device, objective=objective)

    def sr_linears(self):
        return [m for m in self.modules() if isinstance(m, SRLinear)]

    def forward(self, ids):
        B, T = ids.shape
        x = self.tok(ids) + self.pos(torch.arange(T, device=ids.device))
        for blk in self.blocks:
            x = blk(x)
        return self.head(self.ln(x))


def train_step(model, ids, targets, lr, micro_batches=1):
    """One mini-batch step: forward and backward over `micro_batches` slices of the batch (weight
    gradients accumulate inside the SR linears, the others in .grad), then the updates: Eq. 10 for
    the SR linears, plain SGD for the float32 parameters.  Returns the mean loss (device tensor)."""
    total = None
    for ids_mb, tgt_mb in zip(ids.chunk(micro_batches), targets.chunk(micro_batches)):
        logits = model(ids_mb)
        loss = F.cross_entropy(logits.view(-1, logits.shape[-1]), tgt_mb.reshape(-1)) / micro_batches
        loss.backward()
        total = loss.detach() if total is None else total + loss.detach()
    for m in model.sr_linears():
        m.update(lr)
    with torch.no_grad():
        for p in model.parameters():
            if p.grad is not None:
                p.add_(p.grad, alpha=-lr)
                p.grad = None
    return total


def flops_per_token(model):
    """6 x (parameters of the SR linears): forward + the two backward products."""
    return 6.0 * sum(m.in_features * m.out_features for m in model.sr_linears())


__all__ = ["SRLinear", "Decoder", "train_step", "flops_per_token", "MAX_ROWS"]
