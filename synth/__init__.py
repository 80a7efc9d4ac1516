"""Seeded synthetic inputs for the quantized-linear hot path.

This module only *draws* arrays (packed code bytes, lookup tables, scales,
activations, sign vectors).  It holds none of the arithmetic of the method:
no bit unpacking, no decode, no Hadamard transform, no matmul.  Both the CPU
oracle's tests and the GPU library's tests consume what it returns; neither
side generates inputs of its own.

Recipe (one generator for everything):
    numpy.random.Generator(PCG64(SeedSequence([cfg, layer, tensor])))
with cfg = 1..5 the benchmark configuration, layer a small integer naming the
projection, tensor one of the TENSOR_* constants below.

Why uniform random bytes stand in for real packed codes: after the rotation
and per-output-channel scaling the weights are close to N(0,1) per column
(Section 3.3 "Reducing rotation overhead"), the codebooks are fitted to
N(0,1), so the codes of a well-designed quantizer are close to uniform; the
row length in bytes is a whole number for every benchmark shape, so uniform
bytes ARE uniform codes (a vector-quantized row whose 5- or 7-bit codes end inside
a byte gets that byte whole; its spare bits belong to no code).  Byte traffic and lookup pattern are those of a real
layer.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

TENSOR_CODES, TENSOR_LUT, TENSOR_SCALES, TENSOR_X, TENSOR_SIGNS = 0, 1, 2, 3, 4

SQ, VQ, TCQ, TCQH = 0, 1, 2, 3   # TCQH: trellis (V=2) with the hybrid computed code book
TCQHH = 4                        # half-TCQ: TCQH with code_bits per step on the first N/2 input channels,
                                 # code_bits + 1 on the rest, one small table (that of code_bits + 1)
SCHEME_NAMES = {SQ: "sq", VQ: "vq", TCQ: "tcq", TCQH: "tcqh", TCQHH: "tcqhh"}


def rng(cfg: int, layer: int, tensor: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([cfg, layer, tensor])))


# --------------------------------------------------------------------------
# Codebooks
# --------------------------------------------------------------------------
def _phi(t):
    return math.exp(-0.5 * t * t) / math.sqrt(2.0 * math.pi)


def _Phi(t):
    return 0.5 * math.erfc(-t / math.sqrt(2.0))


def lloyd_max_gaussian(levels: int, tol: float = 1e-13, max_iter: int = 200000) -> np.ndarray:
    """Fixed point of Lloyd's iteration on the *analytic* N(0,1) density.

    The paper fits its scalar codebooks by 1-D k-means on 1e8 Gaussian samples
    (Appendix C.1, "Codebook construction"); k-means on samples converges to
    this fixed point as the sample grows.  Thresholds are midpoints of
    neighbouring levels; each level is the conditional mean of its cell,
        c = (phi(a) - phi(b)) / (Phi(b) - Phi(a))   on the cell (a, b).
    Returns the levels in ascending order, float64.
    """
    # start from equal-probability cell medians (any strictly increasing start works)
    from statistics import NormalDist
    nd = NormalDist()
    c = np.array([nd.inv_cdf((i + 0.5) / levels) for i in range(levels)], dtype=np.float64)
    for _ in range(max_iter):
        t = np.concatenate(([-np.inf], 0.5 * (c[:-1] + c[1:]), [np.inf]))
        new = np.empty_like(c)
        for i in range(levels):
            a, b = t[i], t[i + 1]
            pa = 0.0 if a == -np.inf else _phi(a)
            pb = 0.0 if b == np.inf else _phi(b)
            Pa = 0.0 if a == -np.inf else _Phi(a)
            Pb = 1.0 if b == np.inf else _Phi(b)
            new[i] = (pa - pb) / (Pb - Pa)
        done = np.max(np.abs(new - c)) < tol
        c = new
        if done:
            break
    return np.sort(c)


def sq_lut(bits: int) -> np.ndarray:
    """2^bits Lloyd-Max levels for N(0,1), ascending, rounded to fp16."""
    return lloyd_max_gaussian(1 << bits).astype(np.float16)


def vq_lut(cfg: int, layer: int, code_bits: int) -> np.ndarray:
    """[2^code_bits, 2] fp16 points drawn N(0,1)."""
    return rng(cfg, layer, TENSOR_LUT).standard_normal((1 << code_bits, 2)).astype(np.float16)


def tcqh_tlut(cfg: int, layer: int, tlut_bits: int = 9) -> np.ndarray:
    """[2^tlut_bits, 2] fp16 points drawn N(0,1): the small table from which the hybrid
    code book is computed (the paper fits it by k-means on 2-D Gaussian samples,
    Appendix C.3.1; seeded Gaussian points stand in for it)."""
    return rng(cfg, layer, TENSOR_LUT).standard_normal((1 << tlut_bits, 2)).astype(np.float16)


def tcq_lut(cfg: int, layer: int, L: int = 16, V: int = 1) -> np.ndarray:
    """[2^L * V] fp16 values drawn N(0,1): the state -> value table."""
    return rng(cfg, layer, TENSOR_LUT).standard_normal((1 << L) * V).astype(np.float16)


# --------------------------------------------------------------------------
# Layers
# --------------------------------------------------------------------------
@dataclass
class Layer:
    """One quantized linear layer in the canonical (row-major bitstream) layout."""
    scheme: int
    M: int                 # out_features = rows of W^
    N: int                 # in_features  = columns
    code_bits: int         # SQ: bits/weight; VQ: bits per 2-vector; TCQ: k bits shifted per step
    vec: int               # V
    window_bits: int       # TCQ: L, else 0
    tile: int              # TCQ: T, else 0
    codes: np.ndarray      # uint8 [M, row_bytes]
    lut: np.ndarray        # float16, flat
    scales: np.ndarray     # float16 [M]
    name: str = ""
    tlut_bits: int = 0     # TCQH: log2 of the small table's entries, else 0
    meta: dict = field(default_factory=dict)

    @property
    def row_bytes(self) -> int:
        return self.codes.shape[1]

    @property
    def bits_per_weight(self) -> float:
        return self.row_bytes * 8 / self.N

    @property
    def code_bytes(self) -> int:
        return self.M * self.row_bytes


def row_bytes_for(scheme: int, N: int, code_bits: int, vec: int) -> int:
    if scheme == TCQHH:
        if N % 512:
            raise ValueError("each half must be whole 256-weight tiles")
        return row_bytes_for(TCQH, N // 2, code_bits, vec) + row_bytes_for(TCQH, N // 2, code_bits + 1, vec)
    bits = N // vec * code_bits
    if bits % 8 and scheme != VQ:
        raise ValueError("row is not a whole number of bytes")
    return (bits + 7) // 8   # a row of 5- or 7-bit codes may end inside its last byte (the spare bits are never read)


def make_layer(cfg: int, layer: int, scheme: int, M: int, N: int, code_bits: int,
               *, vec: int | None = None, window_bits: int = 16, tile: int = 256,
               lut: np.ndarray | None = None, name: str = "", tlut_bits: int | None = None) -> Layer:
    if vec is None:
        vec = 2 if scheme in (VQ, TCQH, TCQHH) else 1
    if tlut_bits is None:   # table size by bitwidth, as in the paper (App. C.3.1; half-TCQ takes
        # the table of its higher bitwidth, App. C.3.2)
        top = code_bits + (1 if scheme == TCQHH else 0)
        tlut_bits = 9 if top <= 8 else 10 if top == 9 else 11
    rb = row_bytes_for(scheme, N, code_bits, vec)
    codes = rng(cfg, layer, TENSOR_CODES).integers(0, 256, size=(M, rb), dtype=np.uint8)
    scales = rng(cfg, layer, TENSOR_SCALES).uniform(0.5, 1.5, size=M).astype(np.float16)
    if lut is None:
        if scheme == SQ:
            lut = sq_lut(code_bits)
        elif scheme == VQ:
            lut = vq_lut(cfg, layer, code_bits).reshape(-1)
        elif scheme in (TCQH, TCQHH):
            lut = tcqh_tlut(cfg, layer, tlut_bits).reshape(-1)
        else:
            lut = tcq_lut(cfg, layer, window_bits, vec)
    trellis = scheme in (TCQ, TCQH, TCQHH)
    return Layer(scheme=scheme, M=M, N=N, code_bits=code_bits, vec=vec,
                 window_bits=window_bits if trellis else 0,
                 tile=tile if trellis else 0,
                 codes=codes, lut=np.ascontiguousarray(lut, dtype=np.float16).reshape(-1),
                 scales=scales, name=name or f"cfg{cfg}.L{layer}",
                 tlut_bits=tlut_bits if scheme in (TCQH, TCQHH) else 0)


def make_x(cfg: int, layer: int, B: int, N: int) -> np.ndarray:
    """Activations fp16 [B, N] ~ N(0,1)."""
    return rng(cfg, layer, TENSOR_X).standard_normal((B, N)).astype(np.float16)


def make_signs(cfg: int, layer: int, n: int) -> np.ndarray:
    """Random sign vector, int8 in {-1,+1}, length n."""
    return (rng(cfg, layer, TENSOR_SIGNS).integers(0, 2, size=n, dtype=np.int8) * 2 - 1).astype(np.int8)


def hadamard_block(N: int) -> int:
    """Block length of the block-diagonal rotation: N itself when it is a power
    of two, else 1024 (14336 = 14 x 1024, 28672 = 28 x 1024) where that divides N,
    else the largest power of two that does (11008 = 43 x 256, 13824 = 27 x 512)."""
    if N & (N - 1) == 0:
        return N
    return 1024 if N % 1024 == 0 else N & -N


# --------------------------------------------------------------------------
# The five benchmark configurations
# --------------------------------------------------------------------------
def config_layers(cfg: int, *, small: bool = False):
    """Descriptions (not arrays) of the layers of configuration cfg:
    list of dict(layer, name, scheme, M, N, code_bits).  `small` shrinks M so
    the oracle finishes in seconds while still spanning several row blocks."""
    def d(layer, name, scheme, M, N, cb):
        return dict(cfg=cfg, layer=layer, name=name, scheme=scheme,
                    M=(min(M, 80) if small else M), N=N, code_bits=cb)
    if cfg == 1:
        return [d(0, "sq4_1024x1024", SQ, 1024, 1024, 4)]
    if cfg == 2:
        return [d(0, "tcq2_q_proj_4096x4096", TCQ, 4096, 4096, 2)]
    if cfg == 3:
        return [d(0, "vq2.5_down_4096x14336", VQ, 4096, 14336, 5)]
    if cfg == 4:
        return [d(0, "tcq3_qkv_6144x4096", TCQ, 6144, 4096, 3),
                d(1, "tcq3_o_4096x4096", TCQ, 4096, 4096, 3),
                d(2, "tcq3_gateup_28672x4096", TCQ, 28672, 4096, 3),
                d(3, "tcq3_down_4096x14336", TCQ, 4096, 14336, 3)]
    if cfg == 5:
        # Llama-3-70B-shaped decoder layer; one scheme per fused group, drawn from seed.
        pal = [(SQ, 4), (VQ, 5), (VQ, 7), (TCQ, 2), (TCQ, 3), (TCQ, 4)]
        g = rng(5, 0, 99)
        shapes = [("qkv", 10240, 8192), ("o", 8192, 8192), ("gateup", 57344, 8192), ("down", 8192, 28672)]
        out = []
        for i, (nm, M, N) in enumerate(shapes):
            s, cb = pal[int(g.integers(0, len(pal)))]
            out.append(d(i, f"{SCHEME_NAMES[s]}{cb}_{nm}_{M}x{N}", s, M, N, cb))
        return out
    if cfg == 6:
        # beyond the five benchmark configurations: the paper's own trellis quantizer (V = 2, hybrid
        # computed code book) on the Llama-3-8B down projection at 2 .. 5 bits per weight
        return [d(0, "tcqh2_down_4096x14336", TCQH, 4096, 14336, 4),
                d(1, "tcqh2.5_down_4096x14336", TCQH, 4096, 14336, 5),
                d(2, "tcqh3_down_4096x14336", TCQH, 4096, 14336, 6),
                d(3, "tcqh2_q_proj_4096x4096", TCQH, 4096, 4096, 4),
                d(4, "tcqh4_down_4096x14336", TCQH, 4096, 14336, 8),
                d(5, "tcqh4.5_down_4096x14336", TCQH, 4096, 14336, 9),
                d(6, "tcqh5_down_4096x14336", TCQH, 4096, 14336, 10),
                # half-TCQ: 2 / 2.5 bits and 3 / 3.5 bits on the two halves of the input channels
                d(7, "tcqhh2.25_down_4096x14336", TCQHH, 4096, 14336, 4),
                d(8, "tcqhh3.25_down_4096x14336", TCQHH, 4096, 14336, 6),
                d(9, "tcqhh3.25_gateup_28672x4096", TCQHH, 28672, 4096, 6),
                # down projections of the 7B- and 13B-shaped models: 11008 = 43 x 256 and 13824 = 54 x 256
                # input channels, not multiples of 1024
                d(10, "vq2.5_down_4096x11008", VQ, 4096, 11008, 5),
                d(11, "tcqh3_down_5120x13824", TCQH, 5120, 13824, 6),
                # the 70B-shaped down projection at 2.5 bits: 56 units of 16 x 1024 per workgroup
                d(12, "vq2.5_down_8192x28672", VQ, 8192, 28672, 5)]
    raise ValueError(cfg)


def config5_model(n_layers: int = 80):
    """Llama-3-70B-shaped model of configuration 5: for every decoder layer the four
    (fused) projections, each with a quantizer drawn from the seed among SQ 4, VQ 2.5 / 3.5
    and TCQ 2 / 3 / 4 bits.  Returns descriptions only (list of lists)."""
    pal = [(SQ, 4), (VQ, 5), (VQ, 7), (TCQ, 2), (TCQ, 3), (TCQ, 4)]
    shapes = [("qkv", 10240, 8192), ("o", 8192, 8192), ("gateup", 57344, 8192), ("down", 8192, 28672)]
    g = rng(5, 1, 99)
    model = []
    for L in range(n_layers):
        row = []
        for i, (nm, M, N) in enumerate(shapes):
            s, cb = pal[int(g.integers(0, len(pal)))]
            row.append(dict(cfg=5, layer=1000 + 4 * L + i, name=f"L{L}.{SCHEME_NAMES[s]}{cb}_{nm}", scheme=s,
                            M=M, N=N, code_bits=cb))
        model.append(row)
    return model


def model_8b(scheme: int, code_bits: int, n_layers: int = 32):
    """Llama-3-8B-shaped model (configuration 4's four fused projections per decoder layer) with one
    quantizer for every projection.  Returns descriptions only (list of lists)."""
    shapes = [("qkv", 6144, 4096), ("o", 4096, 4096), ("gateup", 28672, 4096), ("down", 4096, 14336)]
    return [[dict(cfg=4, layer=2000 + 4 * L + i, name=f"L{L}.{SCHEME_NAMES[scheme]}{code_bits}_{nm}", scheme=scheme,
                  M=M, N=N, code_bits=code_bits) for i, (nm, M, N) in enumerate(shapes)] for L in range(n_layers)]


def model_7b(scheme: int, code_bits: int, n_layers: int = 32):
    """Llama-2-7B-shaped model with one quantizer for every projection: 4096 hidden and 11008
    intermediate channels - the down projection's 11008 = 43 x 256 input channels are not a multiple of
    1024 (its rotation runs in blocks of 256).  Returns descriptions only (list of lists)."""
    shapes = [("qkv", 12288, 4096), ("o", 4096, 4096), ("gateup", 22016, 4096), ("down", 4096, 11008)]
    return [[dict(cfg=7, layer=3000 + 4 * L + i, name=f"L{L}.{SCHEME_NAMES[scheme]}{code_bits}_{nm}", scheme=scheme,
                  M=M, N=N, code_bits=code_bits) for i, (nm, M, N) in enumerate(shapes)] for L in range(n_layers)]


def build(desc: dict) -> Layer:
    return make_layer(desc["cfg"], desc["layer"], desc["scheme"], desc["M"], desc["N"],
                      desc["code_bits"], name=desc["name"])
