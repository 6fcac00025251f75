"""Seeded synthetic inputs for the MXFP4 linear-layer path.

This module holds input generators and workload shapes only -- none of the
method's arithmetic -- so that the CPU oracle's tests and the HIP path's tests
and benchmark draw the same tensors.  The tensors stand in for the activations,
weights and output gradients of DeiT/ViT linear layers (the paper trains on
ImageNet-1K, which is not available here): activations are N(0,1) with a few
outlier channels scaled x20, weights N(0, 0.02^2), output gradients heavy-tailed
Student-t(3) x 1e-3.
"""
import numpy as np

# (name, D_in -> C_out) of the four linear layers of one transformer block
_BLOCK = lambda d, mlp: [("qkv", d, 3 * d), ("proj", d, d), ("fc1", d, mlp), ("fc2", mlp, d)]

CONFIGS = {
    # single small layer: the case the oracle finishes in well under a second
    "c1_single": {"N": 256, "layers": [("fc1", 192, 768)], "dtype": "f32", "outliers": 4},
    "vit_tiny_b64": {"N": 64 * 197, "layers": _BLOCK(192, 768), "dtype": "bf16", "outliers": 4},
    "vit_small_b128": {"N": 128 * 197, "layers": _BLOCK(384, 1536), "dtype": "bf16", "outliers": None},
    "vit_base_b256": {"N": 256 * 197, "layers": _BLOCK(768, 3072), "dtype": "bf16", "outliers": None},
    "vit_large_b256": {"N": 256 * 197, "layers": _BLOCK(1024, 4096), "dtype": "bf16", "outliers": None},
}


def round_to_bf16(a):
    """Round an FP32 array to the nearest bf16 value (ties to even); result stays FP32."""
    a = np.ascontiguousarray(a, np.float32)
    u = a.view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    out = ((u + r) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return out.view(np.float32)


def bf16_bits(a):
    """uint16 bit patterns of an FP32 array whose values are already bf16-representable."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "values are not bf16-representable"
    return (u >> np.uint32(16)).astype(np.uint16)


def _n_outliers(D, outliers):
    if outliers is None:                      # 1 % of the channels, at least one
        return max(1, int(np.ceil(0.01 * D)))
    return min(int(outliers), D)


def activations(N, D, seed, outliers=None, dtype="f32"):
    rng = np.random.default_rng([seed, 1, N, D])
    x = rng.standard_normal((N, D), dtype=np.float32)
    cols = rng.choice(D, size=_n_outliers(D, outliers), replace=False)
    x[:, cols] *= np.float32(20.0)
    return round_to_bf16(x) if dtype == "bf16" else x


def weights(C, D, seed, dtype="f32"):
    rng = np.random.default_rng([seed, 2, C, D])
    w = rng.standard_normal((C, D), dtype=np.float32) * np.float32(0.02)
    return round_to_bf16(w) if dtype == "bf16" else w


def out_grads(N, C, seed, dtype="f32"):
    """Student-t with 3 degrees of freedom, scaled by 1e-3: z / sqrt(chi2_3 / 3)."""
    rng = np.random.default_rng([seed, 3, N, C])
    z = rng.standard_normal((N, C), dtype=np.float32)
    chi = np.zeros((N, C), np.float32)
    for _ in range(3):
        g = rng.standard_normal((N, C), dtype=np.float32)
        chi += g * g
    t = z / np.sqrt(chi / np.float32(3.0))
    t *= np.float32(1e-3)
    return round_to_bf16(t) if dtype == "bf16" else t


def weight_walk(C, D, seed, steps, sigma=1e-4):
    """Master-weight trajectory for the Q-EMA workload: W0 ~ N(0, 0.02^2), then
    `steps` updates W <- W + N(0, sigma^2).  Yields FP32 matrices W0, W1, ..."""
    rng = np.random.default_rng([seed, 4, C, D])
    w = rng.standard_normal((C, D), dtype=np.float32) * np.float32(0.02)
    yield w.copy()
    for _ in range(steps):
        w += rng.standard_normal((C, D), dtype=np.float32) * np.float32(sigma)
        yield w.copy()


def linear_layer(N, D, C, seed=0, dtype="f32", outliers=None):
    """(X[N,D], W[C,D], dY[N,C]) for one linear layer."""
    return (activations(N, D, seed, outliers, dtype),
            weights(C, D, seed, dtype),
            out_grads(N, C, seed, dtype))


def config_layers(name, n_tokens=None):
    """[(layer name, N, D, C)] of a named configuration; n_tokens overrides N."""
    cfg = CONFIGS[name]
    N = cfg["N"] if n_tokens is None else n_tokens
    return [(ln, N, d, c) for (ln, d, c) in cfg["layers"]]


# ---- the same laws drawn directly in device memory (for the benchmark's large tensors) ----

def device_linear_layer(N, D, C, seed=0, dtype="bf16", outliers=None, device="cuda"):
    """(X[N,D], W[C,D], dY[N,C]) as torch tensors on `device`, same distributions as
    linear_layer() but drawn with torch's generator (a different stream of numbers)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) * 1000003 + N * 31 + D * 17 + C)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    x = torch.randn((N, D), generator=g, device=device, dtype=torch.float32)
    cols = torch.randperm(D, generator=g, device=device)[:_n_outliers(D, outliers)]
    x[:, cols] *= 20.0
    w = torch.randn((C, D), generator=g, device=device, dtype=torch.float32) * 0.02
    z = torch.randn((N, C), generator=g, device=device, dtype=torch.float32)
    chi = torch.zeros((N, C), device=device, dtype=torch.float32)
    for _ in range(3):
        t = torch.randn((N, C), generator=g, device=device, dtype=torch.float32)
        chi += t * t
        del t
    dy = z / torch.sqrt(chi / 3.0) * 1e-3
    del z, chi
    return x.to(tdt), w.to(tdt), dy.to(tdt)
