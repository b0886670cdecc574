"""Seeded synthetic inputs shared by the GPU tests, the oracle tests and bench.py.

Nothing here is part of the method: no rounding, no scaling, no RNG of the
quantizer.  Only tensors with the shapes and value distributions of the
workloads (transformer-shaped Gaussian activations, weights and gradients).
The second parameter of N(.,.) is a standard deviation.
"""
import numpy as np


def gaussian(shape, std, seed):
    """float32 ~ N(0, std), numpy generator, reproducible anywhere."""
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)


def single_layer(M=64, N=128, K=128, seed=0, std_a=1.0, std_w=0.02, std_dy=1.0):
    """A (M,K), W (N,K), dY (M,N): the small CPU-checkable layer."""
    return (gaussian((M, K), std_a, seed), gaussian((N, K), std_w, seed + 1),
            gaussian((M, N), std_dy, seed + 2))


def outlier_tensor_np(n, seed, outlier_frac=0.01, outlier_std=50.0):
    """N(0,1) with an independent Bernoulli(outlier_frac) mask replaced by N(0, outlier_std)."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(n, dtype=np.float32)
    mask = rng.random(n, dtype=np.float32) < outlier_frac
    big = rng.standard_normal(n, dtype=np.float32) * np.float32(outlier_std)
    return np.where(mask, big, x).astype(np.float32)


def outlier_tensor_torch(n, seed, device, outlier_frac=0.01, outlier_std=50.0):
    """Same recipe generated on `device` with torch (for tensors too large to ship)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    x = torch.randn(n, generator=g, device=device, dtype=torch.float32)
    mask = torch.rand(n, generator=g, device=device, dtype=torch.float32) < outlier_frac
    x[mask] = torch.randn(int(mask.sum().item()), generator=g, device=device,
                          dtype=torch.float32) * outlier_std
    return x


def gaussian_torch(shape, std, seed, device, dtype=None):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std
    return x if dtype is None else x.to(dtype)


def to_bf16_bits(x):
    """float32 numpy array -> uint16 array of bfloat16 bit patterns (round to nearest even)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


# (name, N = out features, K = in features)
GPT2_SMALL_MLP = [("fc1", 3072, 768), ("fc2", 768, 3072)]
LLAMA_1B_LINEARS = [("q", 2048, 2048), ("k", 2048, 2048), ("v", 2048, 2048), ("o", 2048, 2048),
                    ("gate", 5632, 2048), ("up", 5632, 2048), ("down", 2048, 5632)]
