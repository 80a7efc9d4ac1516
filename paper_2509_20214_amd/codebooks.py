"""Code books fitted on the device (Appendix C.1 / C.2 / C.3.1, "Codebook construction").

Seeded standard Gaussian samples are drawn with torch (input generation); the fitting itself -
Lloyd's algorithm - runs in the library's kernels (qp_kmeans).  The paper does not say how its
k-means runs were started; here the first k samples are the start (sorted for scalar tables, which
keeps the levels in ascending order throughout)."""
from __future__ import annotations

from .binding import qp_kmeans


def _fit(samples, k, max_iter, tol):
    import torch
    d = 1 if samples.dim() == 1 else samples.shape[1]
    init = samples[:k].clone()
    if d == 1:
        init = torch.sort(init).values.contiguous()
    out16 = torch.empty(init.shape, dtype=torch.float16, device=samples.device)
    stats = torch.zeros(3, dtype=torch.float64, device=samples.device)
    qp_kmeans(samples, init, max_iter, tol, centres_f16=out16, stats=stats)
    return out16, stats


def train_scalar(bits: int, n_samples: int = 10_000_000, seed: int = 0, max_iter: int = 300, tol: float = 1e-6,
                 device="cuda"):
    """2^bits fp16 levels, ascending (the paper fits 10^8 samples)."""
    import torch
    g = torch.Generator(device=device).manual_seed(seed)
    x = torch.randn(n_samples, generator=g, device=device, dtype=torch.float32)
    return _fit(x, 1 << bits, max_iter, tol)[0]


def train_vector(code_bits: int, n_samples: int = 10_000_000, seed: int = 0, max_iter: int = 300,
                 tol: float = 1e-6, device="cuda"):
    """2^code_bits fp16 points of the plane, [2^code_bits, 2]."""
    import torch
    g = torch.Generator(device=device).manual_seed(seed)
    x = torch.randn((n_samples, 2), generator=g, device=device, dtype=torch.float32)
    return _fit(x, 1 << code_bits, max_iter, tol)[0]


def train_tlut(tlut_bits: int = 9, n_samples: int = 1 << 20, seed: int = 0, scale: float = 0.8, max_iter: int = 300,
               tol: float = 1e-6, device="cuda"):
    """The small table of the trellis quantizer's hybrid code book: 2^tlut_bits pairs fitted to
    2^20 Gaussian pairs.  The paper scales the samples by a factor it does not state; measured at
    2 bits per weight, the distortion of N(0,1) weights is least for a factor of 0.75 .. 0.8
    (0.0706; 0.0799 unscaled; the paper's own figure, 0.07101, lies between the results for 0.8 and
    0.85), hence the default."""
    import torch
    g = torch.Generator(device=device).manual_seed(seed)
    x = torch.randn((n_samples, 2), generator=g, device=device, dtype=torch.float32) * scale
    return _fit(x, 1 << tlut_bits, max_iter, tol)[0]
