"""Seeded synthetic inputs shaped like the paper's workloads.

This module holds no arithmetic of the method: it only draws random numbers.  It serves
the oracle's tests and the GPU tests alike and imports neither of them.  The paper trains
detection models on an image dataset (Sec. VI); none of that is available here, so the
partial gradients are synthetic tensors with the sizes of those models (25.6 M coordinates
for the ResNet-50-sized case) and the value distributions listed per configuration.

Every generator is a pure function of its integer seed.
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

PHILOX_SEED_BASE = 0x260515890


@dataclass
class Config:
    """One named workload: sizes, laws of the random inputs, iteration count."""
    index: int
    name: str
    n: int                      # workers
    k: int                      # partitions
    s: int                      # cyclic replication factor
    d: int                      # coordinates
    law: str                    # "normal" | "layered" | "student_t3" | "least_squares"
    p_law: tuple                # ("fixed", [..]) | ("uniform", lo, hi)
    bits_law: tuple             # ("fixed", [..]) | ("alloc", mean_bits) | ("uniform", lo, hi)
    iters: int
    allow_1bit: bool = False
    extra: dict = field(default_factory=dict)

    @property
    def torch_seed(self) -> int:
        return 15890 + self.index

    @property
    def philox_seed(self) -> int:
        return PHILOX_SEED_BASE + self.index


CONFIGS = {
    "tiny": Config(1, "tiny", 4, 4, 2, 4096, "normal", ("fixed", [0.1, 0.2, 0.3, 0.4]),
                   ("fixed", [8, 6, 4, 2]), 1000),
    "n16_d1m": Config(2, "n16_d1m", 16, 16, 3, 1 << 20, "normal", ("uniform", 0.05, 0.5),
                      ("alloc", 4), 200),
    "resnet18": Config(3, "resnet18", 32, 32, 4, 11_700_000, "layered", ("uniform", 0.05, 0.6),
                       ("uniform", 1, 8), 20, allow_1bit=True,
                       extra={"blocks": 60, "log10_sigma": (-4.0, -1.0)}),
    "resnet50": Config(4, "resnet50", 64, 64, 4, 25_600_000, "student_t3", ("uniform", 0.05, 0.6),
                       ("alloc", 3), 100, extra={"scale": 1e-3}),
    # end-to-end gradient descent on synthetic least squares; d is the feature dimension and the
    # partial gradients come from least_squares_* below
    "lsq": Config(5, "lsq", 32, 32, 3, 4096, "least_squares", ("uniform", 0.05, 0.5), ("alloc", 4), 500,
                  extra={"n_rows": 1 << 20}),
}


def straggler_probs(cfg: Config) -> np.ndarray:
    if cfg.p_law[0] == "fixed":
        return np.asarray(cfg.p_law[1], dtype=np.float64)
    rng = np.random.default_rng(1000 + cfg.index)
    return rng.uniform(cfg.p_law[1], cfg.p_law[2], size=cfg.n)


def random_bits(cfg: Config) -> Optional[np.ndarray]:
    """Bit-widths for the laws that are plain random draws; None when the configuration
    takes them from the bit allocator (a routine of the method, not of this module)."""
    if cfg.bits_law[0] == "fixed":
        return np.asarray(cfg.bits_law[1], dtype=np.uint8)
    if cfg.bits_law[0] == "uniform":
        rng = np.random.default_rng(2000 + cfg.index)
        return rng.integers(cfg.bits_law[1], cfg.bits_law[2] + 1, size=cfg.n).astype(np.uint8)
    return None


def arrival_mask(cfg: Config, p: np.ndarray, iteration: int) -> np.ndarray:
    """Independent Bernoulli arrivals: mask[i] = 1 with probability 1 - p_i."""
    rng = np.random.default_rng([cfg.index, iteration])
    return (rng.random(cfg.n) >= p).astype(np.uint8)


def layer_sigmas(cfg: Config, d: int):
    """Per-coordinate standard deviation of the "layered" law: contiguous blocks of
    near-equal length, block l scaled by 10^U[lo,hi]; the same for every partition."""
    nb = cfg.extra["blocks"]
    lo, hi = cfg.extra["log10_sigma"]
    rng = np.random.default_rng(3000 + cfg.index)
    sig = 10.0 ** rng.uniform(lo, hi, size=nb)
    edges = np.linspace(0, d, nb + 1).astype(np.int64)
    return sig, edges


def layer_ends(cfg: Config, d: Optional[int] = None):
    """Ends of the layers of a "layered" configuration for layer-wise scales: the law's own block
    edges moved down to multiples of 256 (a 256-coordinate block lies in one layer), duplicates
    dropped, the last one d itself."""
    d = cfg.d if d is None else d
    _, edges = layer_sigmas(cfg, d)
    ends = sorted({int(e) // 256 * 256 for e in edges[1:-1]} - {0})
    return np.array([e for e in ends if e < d] + [d], dtype=np.int64)


def partial_gradients_numpy(cfg: Config, d: Optional[int] = None, seed_offset: int = 0) -> np.ndarray:
    """k x d float32 partial gradients on the host (for sizes the CPU handles)."""
    d = cfg.d if d is None else d
    rng = np.random.default_rng(cfg.torch_seed + 7919 * seed_offset)
    if cfg.law == "normal":
        return rng.standard_normal((cfg.k, d), dtype=np.float32)
    if cfg.law == "layered":
        G = rng.standard_normal((cfg.k, d), dtype=np.float32)
        sig, edges = layer_sigmas(cfg, d)
        for l in range(len(sig)):
            G[:, edges[l]:edges[l + 1]] *= np.float32(sig[l])
        return G
    if cfg.law == "student_t3":
        z = rng.standard_normal((cfg.k, d), dtype=np.float32)
        chi = np.zeros((cfg.k, d), dtype=np.float32)
        for _ in range(3):
            chi += rng.standard_normal((cfg.k, d), dtype=np.float32) ** 2
        return (np.float32(cfg.extra["scale"]) * z / np.sqrt(chi / np.float32(3.0))).astype(np.float32)
    raise ValueError(cfg.law)


def partial_gradients_torch(cfg: Config, device, d: Optional[int] = None, seed_offset: int = 0):
    """k x d float32 partial gradients generated on `device` with torch's generator, row by
    row so that the largest configuration never needs more than one extra row of scratch."""
    import torch
    d = cfg.d if d is None else d
    gen = torch.Generator(device=device)
    gen.manual_seed(cfg.torch_seed + 7919 * seed_offset)
    G = torch.empty((cfg.k, d), dtype=torch.float32, device=device)
    if cfg.law == "layered":
        sig, edges = layer_sigmas(cfg, d)
        sig_vec = torch.empty(d, dtype=torch.float32, device=device)
        for l in range(len(sig)):
            sig_vec[int(edges[l]):int(edges[l + 1])] = float(sig[l])
    for j in range(cfg.k):
        row = G[j]
        row.normal_(generator=gen)
        if cfg.law == "layered":
            row.mul_(sig_vec)
        elif cfg.law == "student_t3":
            chi = torch.zeros(d, dtype=torch.float32, device=device)
            tmp = torch.empty(d, dtype=torch.float32, device=device)
            for _ in range(3):
                tmp.normal_(generator=gen)
                chi.addcmul_(tmp, tmp)
            row.div_(torch.sqrt(chi / 3.0)).mul_(cfg.extra["scale"])
            del chi, tmp
    return G


# ----------------------------------------------------------------------------------------
# least-squares problem of the end-to-end loop: X ~ N(0, 1/F) stored as bfloat16,
# y = X w* + 0.01 * noise (the paper's own experiments train detection models; this synthetic
# regression only supplies partial gradients that come from an actual loss)
# ----------------------------------------------------------------------------------------
def least_squares_numpy(n_rows: int, n_feat: int, seed: int = 5):
    """Returns (X as uint16 bfloat16 bit patterns, y float32, w_star float32)."""
    rng = np.random.default_rng(15890 + seed)
    X = (rng.standard_normal((n_rows, n_feat), dtype=np.float32) / np.float32(np.sqrt(n_feat)))
    u = X.view(np.uint32).astype(np.uint64)
    X_bits = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)     # round to nearest even
    Xb = (X_bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    w_star = rng.standard_normal(n_feat, dtype=np.float32)
    y = (Xb.astype(np.float64) @ w_star.astype(np.float64)
         + 0.01 * rng.standard_normal(n_rows)).astype(np.float32)
    return X_bits, y, w_star


def least_squares_torch(n_rows: int, n_feat: int, device, seed: int = 5):
    """Same law generated on the device, slab by slab (X is 8 GiB at the full configuration).
    Returns (X torch.bfloat16, y float32, w_star float32)."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(15890 + seed)
    w_star = torch.randn(n_feat, generator=gen, device=device, dtype=torch.float32)
    X = torch.empty((n_rows, n_feat), dtype=torch.bfloat16, device=device)
    y = torch.empty(n_rows, dtype=torch.float32, device=device)
    slab = 1 << 15
    for r0 in range(0, n_rows, slab):
        r1 = min(n_rows, r0 + slab)
        xs = torch.randn((r1 - r0, n_feat), generator=gen, device=device, dtype=torch.float32) / (n_feat ** 0.5)
        X[r0:r1] = xs.to(torch.bfloat16)
        y[r0:r1] = X[r0:r1].to(torch.float32) @ w_star + 0.01 * torch.randn(r1 - r0, generator=gen, device=device)
    return X, y, w_star
