"""Seeded synthetic inputs for the LoRDO hot path.

This module only *generates inputs*: weight matrices, gradients, Gaussian test
matrices for the range finder and an averaged pseudo-gradient.  It holds none of
the method's arithmetic, so both the float64 oracle's tests and the HIP path's
tests may draw from it without sharing any code of the method.

The gradients stand in for those of the peri-LN transformers the paper trains
(App. C, Table "model architectures": 125M = 12 blocks, d = 768, FFN ratio 4),
which need a dataset that is not available: a low-rank "spike" (the informative
subspace a projection should find) on top of dense noise (the stochastic part).

Everything on the host comes from numpy's PCG64 with the seed scheme of
`seed_for`; bf16 inputs are rounded once here (round-to-nearest-even) so that
every consumer sees the identical value.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 260204396


def seed_for(config: int, matrix: int, step: int | None = None) -> int:
    """One documented seed per (config, matrix[, step])."""
    s = BASE_SEED + 1000 * config + matrix
    if step is not None:
        s = s * 4096 + step
    return s


# ----------------------------------------------------------------------------
# bf16 helpers (input preparation only)
# ----------------------------------------------------------------------------
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit pattern (uint16), round-to-nearest-even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    out = ((u + rounding) >> 16).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = 0x7FC0
    return out


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round to bf16 and return the rounded values as float32."""
    return bf16_to_f32(bf16_bits(x))


# ----------------------------------------------------------------------------
# shapes of the benchmark configurations: lists of (p, q, r)
# ----------------------------------------------------------------------------
def _layers(n_layers, per_layer, r):
    out = []
    for _ in range(n_layers):
        for (p, q, cnt) in per_layer:
            out += [(p, q, r)] * cnt
    return out


def config_shapes(name: str, rank: int | None = None):
    name = name.lower()
    if name == "c1":
        return [(256, 256, rank or 16)]
    if name == "c2":
        return _layers(12, [(768, 768, 4), (768, 3072, 1), (3072, 768, 1)], rank or 128)
    if name == "c3":
        return _layers(24, [(2048, 2048, 4), (2048, 5632, 2), (5632, 2048, 1)], rank or 256)
    if name == "c4":
        return _layers(32, [(4096, 4096, 4), (4096, 11008, 2), (11008, 4096, 1)], rank or 512)
    if name == "c5":
        return [(8192, 28672, rank or 256)]
    raise ValueError(f"unknown config {name!r}")


CONFIG_DEFAULTS = {
    # name: (n_spike, noise kind, refresh period, outer period H, power iters)
    "c1": dict(n_spike=8, noise="gauss", refresh_every=0, outer_every=10, power_iters=2),
    "c2": dict(n_spike=32, noise="gauss", refresh_every=200, outer_every=32, power_iters=2),
    "c3": dict(n_spike=64, noise="student", refresh_every=64, outer_every=64, power_iters=1),
    "c4": dict(n_spike=64, noise="gauss", refresh_every=0, outer_every=0, power_iters=1),
    "c5": dict(n_spike=64, noise="gauss", refresh_every=0, outer_every=0, power_iters=1),
}


# ----------------------------------------------------------------------------
# host generators
# ----------------------------------------------------------------------------
def orthonormal(rng: np.random.Generator, n: int, k: int) -> np.ndarray:
    """n x k matrix with orthonormal columns (QR of a Gaussian)."""
    q, _ = np.linalg.qr(rng.standard_normal((n, k)))
    return q


def weights(rng: np.random.Generator, p: int, q: int) -> np.ndarray:
    """W_0 ~ N(0, 0.02^2), float32."""
    return (0.02 * rng.standard_normal((p, q))).astype(np.float32)


def omega(rng: np.random.Generator, q: int, r: int) -> np.ndarray:
    """Gaussian start block of the range finder, q x r float32."""
    return rng.standard_normal((q, r)).astype(np.float32)


def c1_signal(rng: np.random.Generator, p: int = 256, q: int = 256, k: int = 8) -> np.ndarray:
    """Rank-k signal with singular values 10..1 (linearly spaced)."""
    a = orthonormal(rng, p, k)
    b = orthonormal(rng, q, k)
    s = np.linspace(10.0, 1.0, k)
    return (a * s) @ b.T


def c1_gradient(signal: np.ndarray, rng: np.random.Generator, noise: float = 0.01) -> np.ndarray:
    """fp32 gradient of config 1: signal + N(0, noise^2)."""
    return (signal + noise * rng.standard_normal(signal.shape)).astype(np.float32)


class SpikedGradient:
    """G_t = sigma * Z_t + sum_k s_k a_k b_k^T for one p x q matrix.

    sigma = 1e-3; Z_t is Gaussian or Student-t(nu = 4); the spike is fixed per
    matrix with s_k = e * 20 * 10^{-(k-1)/(K-1)}, e = sigma (sqrt p + sqrt q)
    the edge of the noise spectrum, so the spike spans 20x .. 2x that edge.
    """

    def __init__(self, p, q, n_spike, seed, noise="gauss", sigma=1e-3, bf16=True):
        self.p, self.q, self.sigma, self.noise, self.bf16 = p, q, sigma, noise, bf16
        rng = np.random.default_rng(seed)
        k = min(n_spike, p, q)
        self.a = orthonormal(rng, p, k)
        self.b = orthonormal(rng, q, k)
        edge = sigma * (np.sqrt(p) + np.sqrt(q))
        expo = np.arange(k) / max(k - 1, 1)
        self.s = edge * 20.0 * 10.0 ** (-expo)
        self.spike = (self.a * self.s) @ self.b.T
        self.seed = seed

    def draw(self, step: int) -> np.ndarray:
        """float32 array holding the (bf16-representable if bf16=True) gradient of `step`."""
        rng = np.random.default_rng(self.seed * 4096 + step)
        z = rng.standard_normal((self.p, self.q))
        if self.noise == "student":
            chi = rng.chisquare(4, size=(self.p, self.q)) / 4.0
            z = z / np.sqrt(chi)
        g = (self.sigma * z + self.spike).astype(np.float32)
        return bf16_round(g) if self.bf16 else g


def avg_pseudograd(own_delta: np.ndarray, other: np.ndarray, workers: int = 4) -> np.ndarray:
    """Stand-in for the cross-worker mean: (own + (M-1) * other) / M, float32."""
    return ((own_delta + (workers - 1) * other) / workers).astype(np.float32)


# ----------------------------------------------------------------------------
# device generators for the full-size benchmark sets (torch is only the RNG and
# the allocator here; same recipe as SpikedGradient)
# ----------------------------------------------------------------------------
def device_spiked_gradient(torch, p, q, n_spike, seed, noise="gauss", sigma=1e-3,
                           dtype=None, device="cuda"):
    """Returns (draw(step) -> tensor of `dtype`, spike factors) on `device`."""
    dtype = dtype or torch.bfloat16
    k = min(n_spike, p, q)
    rng = np.random.default_rng(seed)          # the thin spike factors are built on the host
    a = torch.tensor(orthonormal(rng, p, k), dtype=torch.float32, device=device)
    b = torch.tensor(orthonormal(rng, q, k), dtype=torch.float32, device=device)
    edge = sigma * (p ** 0.5 + q ** 0.5)
    expo = torch.arange(k, device=device, dtype=torch.float32) / max(k - 1, 1)
    s = edge * 20.0 * 10.0 ** (-expo)
    a_s = a * s

    def draw(step: int):
        g = torch.Generator(device=device)
        g.manual_seed(seed * 4096 + step)
        z = torch.randn(p, q, generator=g, device=device)
        if noise == "student":
            chi = torch.zeros(p, q, device=device)
            for _ in range(4):
                chi += torch.randn(p, q, generator=g, device=device) ** 2
            z = z / torch.sqrt(chi / 4.0)
        out = torch.addmm(sigma * z, a_s, b.T)
        return out.to(dtype).contiguous()

    return draw
