"""Seeded synthetic workloads (numpy only, no arithmetic of the method itself).

The paper trains GPT-2 / ViT models on OpenWebText / ImageNet-1K, neither of
which is available; these tensors stand in for them.  They copy the shapes of
the linear layers of a Transformer block and the outlier statistics the paper
reports: "normal" activations of order 1-10, "extreme" outliers above 1000
(Sec. 1), baseline peaks of several hundred to tens of thousands (Tables 1
and 2) and the outlier-free regime |a| <= 20 of TWEO-trained models (Table 2).

All tensors are bf16, carried as uint16 bit patterns so that the CPU oracle and
the GPU library see identical bits.  Random numbers come from numpy's
counter-based Philox generator, keyed by (config, tensor).
"""
from dataclasses import dataclass

import numpy as np

BASE_SEED = 20251123


def f32_to_bf16_bits(a):
    """float32 array -> bf16 bit patterns (round to nearest even; inputs are finite)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(
        np.uint16)


def bf16_bits_to_f32(h):
    return (np.asarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(cfg, tensor_index):
    return np.random.Generator(np.random.Philox(key=BASE_SEED + 1000 * cfg + tensor_index))


def normal(shape, std, rng):
    out = np.empty(shape, np.float32)
    flat = out.reshape(-1)
    step = 1 << 24
    for i in range(0, flat.size, step):
        n = min(step, flat.size - i)
        flat[i:i + n] = rng.standard_normal(n, dtype=np.float32) * np.float32(std)
    return out


def inject_sparse_outliers(x, frac, lo, hi, rng):
    """Replace round(frac*size) entries (uniform, without replacement) by +-U(lo,hi)."""
    flat = x.reshape(-1)
    k = int(round(frac * flat.size))
    if k == 0:
        return x
    # k distinct positions, uniform: draw with a little slack, drop repeats, keep the first k
    pos = np.empty(0, np.int64)
    while pos.size < k:
        draw = rng.integers(0, flat.size, size=k + k // 8 + 16)
        _, first = np.unique(np.concatenate([pos, draw]), return_index=True)
        pos = np.concatenate([pos, draw])[np.sort(first)]
    pos = pos[:k]
    mag = rng.uniform(lo, hi, size=k).astype(np.float32)
    sgn = np.where(rng.integers(0, 2, size=k) == 0, np.float32(-1), np.float32(1))
    flat[pos] = mag * sgn
    return x


def inject_channel_outliers(x, n_channels, factor, rng):
    """Multiply n_channels seed-chosen columns (same for every token) by factor."""
    cols = rng.choice(x.shape[1], size=n_channels, replace=False)
    x[:, cols] *= np.float32(factor)
    return x


@dataclass(frozen=True)
class Gemm:
    name: str
    M: int
    K: int
    N: int


# The five workload families.  cfg 0 is the small parity/latency case, cfg 1-3
# are block-shaped training workloads, cfg 4 is W8A8 inference.
CONFIGS = {
    0: dict(name="single-linear-256x512x512", gemms=[Gemm("linear", 256, 512, 512)],
            outliers=("sparse", 1e-3, 1000.0, 10000.0)),
    1: dict(name="gpt2-small-block-8192tok",
            gemms=[Gemm("qkv", 8192, 768, 2304), Gemm("proj", 8192, 768, 768),
                   Gemm("fc1", 8192, 768, 3072), Gemm("fc2", 8192, 3072, 768)],
            outliers=("sparse", 1e-4, 1000.0, 5000.0)),
    2: dict(name="vit-b16-block-256x197tok",
            gemms=[Gemm("qkv", 50432, 768, 2304), Gemm("fc1", 50432, 768, 3072),
                   Gemm("fc2", 50432, 3072, 768)],
            outliers=("channel", 3, 2000.0)),
    3: dict(name="llama1b-swiglu-block-16384tok",
            gemms=[Gemm("qkv", 16384, 2048, 6144), Gemm("o", 16384, 2048, 2048),
                   Gemm("gate", 16384, 2048, 5632), Gemm("up", 16384, 2048, 5632),
                   Gemm("down", 16384, 5632, 2048)],
            outliers=("sparse", 1e-4, 1000.0, 10000.0)),
    4: dict(name="w8a8-7b-inference",
            gemms=[Gemm("qkv", 0, 4096, 12288), Gemm("gate", 0, 4096, 11008),
                   Gemm("up", 0, 4096, 11008), Gemm("down", 0, 11008, 4096)],
            m_values=(1, 16, 64, 4096), clip=20.0),
}


def fp8_linear_inputs(cfg, gemm_index, M=None, K=None, N=None):
    """bf16 bit patterns (X[M,K], W[N,K], dY[M,N]) of one linear layer of a training config.

    M/K/N override the shape (used by reduced-size parity cases that keep the
    value distribution of the config).
    """
    c = CONFIGS[cfg]
    g = c["gemms"][gemm_index]
    M, K, N = M or g.M, K or g.K, N or g.N
    base = 10 * gemm_index
    rx, rw, rdy, ro = (_rng(cfg, base + i) for i in range(4))
    x = normal((M, K), 1.0, rx)
    kind = c["outliers"]
    if kind[0] == "sparse":
        inject_sparse_outliers(x, kind[1], kind[2], kind[3], ro)
    else:
        inject_channel_outliers(x, kind[1], kind[2], ro)
    w = normal((N, K), 0.02, rw)
    dy = normal((M, N), 1.0, rdy)
    return f32_to_bf16_bits(x), f32_to_bf16_bits(w), f32_to_bf16_bits(dy)


def residual_input(cfg, gemm_index, M, N):
    """bf16 residual stream R[M,N] ~ N(0,1) for the block-output form y = x + f(x) (Sec. 3.3)."""
    return f32_to_bf16_bits(normal((M, N), 1.0, _rng(cfg, 10 * gemm_index + 7)))


def w8a8_inputs(gemm_index, M, K=None, N=None, with_w=True):
    """bf16 X[M,K] ~ N(0,1) clipped to |x|<20 and bf16 W[N,K] ~ N(0,0.02) for the INT8 config
    (with_w=False: W is None; it does not depend on M, so a caller that has it need not regenerate it)."""
    c = CONFIGS[4]
    g = c["gemms"][gemm_index]
    K, N = K or g.K, N or g.N
    rx, rw = _rng(4, 10 * gemm_index + 100 * (M % 97)), _rng(4, 10 * gemm_index + 1)
    x = np.clip(normal((M, K), 1.0, rx), -c["clip"], c["clip"])
    w = normal((N, K), 0.02, rw) if with_w else None
    return f32_to_bf16_bits(x), (f32_to_bf16_bits(w) if with_w else None)


def gemm_flops(M, N, K):
    return 2.0 * M * N * K
