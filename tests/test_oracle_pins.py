"""Pins for the CPU oracle: each check ties one of its functions to something
other than itself — a library routine, a closed form, an invariant, exhaustive
search on a tiny case, or a number the paper prints."""
import math
import os

import numpy as np
import pytest

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def golden_distortion():
    out = {}
    with open(os.path.join(GOLDEN, "paper_gaussian_distortion.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, bits, mean, std = line.split()
            out[name] = (float(bits), float(mean), float(std))
    return out


# ------------------------------------------------------------------ fp16
def test_half_conversion_exhaustive():
    pat = np.arange(65536, dtype=np.uint16)
    got = oracle.half_to_double(pat)
    want = pat.view(np.float16).astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


# ------------------------------------------------------------ bit access
def pack_lsb_first(codes, width):
    """Independent packer: Python big integers, code q occupies bits [q*width, (q+1)*width)."""
    big = 0
    for q, c in enumerate(codes):
        big |= int(c) << (q * width)
    nbytes = (len(codes) * width + 7) // 8
    return np.frombuffer(big.to_bytes(nbytes, "little"), dtype=np.uint8).copy()


def test_bit_order_hand_example():
    # byte0 = 0b10110100, byte1 = 0b00000011 -> stream bits (p=0..): 0,0,1,0,1,1,0,1, 1,1,0,0,0,0,0,0
    s = np.array([0b10110100, 0b00000011], dtype=np.uint8)
    L = oracle.lib()
    assert [L.qpo_bit(s, p) for p in range(16)] == [0, 0, 1, 0, 1, 1, 0, 1, 1, 1, 0, 0, 0, 0, 0, 0]
    # 3-bit codes: (0,0,1)->4, (0,1,1)->6, (0,1,1)->6, (1,0,0)->1 (value = sum bit_t 2^t)
    assert [L.qpo_code(s, 3 * q, 3) for q in range(4)] == [4, 6, 6, 1]
    # 4-bit: weight 2m in the low nibble of byte m
    assert [L.qpo_code(s, 4 * q, 4) for q in range(4)] == [0x4, 0xB, 0x3, 0x0]
    # circular window: 16 bits from bit 8 of a 16-bit stream wrap to the start
    assert L.qpo_window(s, 8, 16, 16) == (0b00000011 | (0b10110100 << 8))


@pytest.mark.parametrize("width", [2, 3, 4, 5, 7])
def test_pack_unpack_identity(width):
    g = np.random.default_rng(100 + width)
    codes = g.integers(0, 1 << width, size=8 * 37)
    stream = pack_lsb_first(codes, width)
    L = oracle.lib()
    got = [L.qpo_code(stream, q * width, width) for q in range(len(codes))]
    assert got == list(codes)


# -------------------------------------------------------- SQ / VQ decode
def unpack_indices_numpy(codes_u8, width, count):
    """Independent unpack with numpy.unpackbits (library routine)."""
    bits = np.unpackbits(codes_u8, axis=-1, bitorder="little")
    bits = bits[..., : count * width].reshape(*codes_u8.shape[:-1], count, width)
    return (bits.astype(np.int64) << np.arange(width)).sum(-1)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_sq_decode_is_table_take(bits):
    M, N = 5, 256
    lay = synth.make_layer(90, bits, synth.SQ, M, N, bits)
    idx = unpack_indices_numpy(lay.codes, bits, N)
    want = np.take(lay.lut.view(np.uint16), idx)
    assert np.array_equal(oracle.decode(lay), want)


@pytest.mark.parametrize("N", [512, 40, 104, 56, 120])   # the last four: rows that end inside a byte
@pytest.mark.parametrize("cbits", [3, 5, 7])
def test_vq_decode_is_table_take(cbits, N):
    M = 6
    lay = synth.make_layer(91, cbits, synth.VQ, M, N, cbits)
    idx = unpack_indices_numpy(lay.codes, cbits, N // 2)
    want = np.take(lay.lut.view(np.uint16).reshape(-1, 2), idx, axis=0).reshape(M, N)
    got = oracle.decode(lay)
    assert np.array_equal(got, want)
    # component 0 lands on the even column
    assert got[0, 0] == lay.lut.view(np.uint16).reshape(-1, 2)[idx[0, 0], 0]
    assert got[0, 1] == lay.lut.view(np.uint16).reshape(-1, 2)[idx[0, 0], 1]


# ------------------------------------------------------------ TCQ decode
def tcq_layer(k, M=3, N=512, L=16, seed=0, lut=None):
    return synth.make_layer(92, seed * 10 + k, synth.TCQ, M, N, k, window_bits=L, lut=lut)


@pytest.mark.parametrize("k", [2, 3, 4])
def test_tcq_constant_streams(k):
    lay = tcq_layer(k)
    lut = lay.lut.view(np.uint16)
    lay.codes[:] = 0
    assert np.all(oracle.decode(lay) == lut[0])
    lay.codes[:] = 0xFF
    assert np.all(oracle.decode(lay) == lut[0xFFFF])


@pytest.mark.parametrize("k", [2, 3, 4])
def test_tcq_single_bit_and_tail_biting(k):
    T, L = 256, 16
    nbits = k * T
    lay = tcq_layer(k, M=1, N=T)
    lut = lay.lut.view(np.uint16)
    for p in [0, 5, 15, 16, 17, nbits // 2 + 1, nbits - 1]:
        lay.codes[:] = 0
        lay.codes[0, p >> 3] = 1 << (p & 7)
        got = oracle.decode(lay)[0]
        want = np.full(T, lut[0], dtype=np.uint16)
        hits = 0
        for i in range(T):
            d = (p - i * k) % nbits          # position of the set bit inside window i
            if d < L:
                want[i] = lut[1 << d]
                hits += 1
        assert np.array_equal(got, want), (k, p)
        assert hits in (L // k, -(-L // k))     # every bit is read by L/k windows (rounded either way)
        if p < L - 1:
            # the bit is also seen by windows at the END of the tile: that is the wrap
            assert any(want[i] != lut[0] for i in range(T - L // k, T))


@pytest.mark.parametrize("k", [2, 4])
def test_tcq_with_window_equal_shift_is_scalar_decode(k):
    """L = k: windows do not overlap, the trellis is a plain 2^k scalar quantizer."""
    M, N = 4, 512
    lut = synth.rng(93, k, 1).standard_normal(1 << k).astype(np.float16)
    lay = synth.make_layer(93, k, synth.TCQ, M, N, k, window_bits=k, lut=lut)
    sq = synth.make_layer(93, k, synth.SQ, M, N, k, lut=lut)
    assert np.array_equal(sq.codes, lay.codes)
    assert np.array_equal(oracle.decode(lay), oracle.decode(sq))


@pytest.mark.parametrize("k,L,V", [(2, 16, 1), (3, 16, 1), (4, 16, 1), (2, 6, 1), (3, 16, 2), (5, 16, 2)])
def test_tcq_window_form_equals_shift_register(k, L, V):
    T, N = 256, 768
    lut = synth.rng(94, k, 1).standard_normal((1 << L) * V).astype(np.float16)
    lay = synth.make_layer(94, k * 100 + L, synth.TCQ, 2, N, k, vec=V, window_bits=L, lut=lut)
    a = np.empty(N, dtype=np.uint16)
    b = np.empty(N, dtype=np.uint16)
    for j in range(2):
        oracle.lib().qpo_decode_row_tcq(lay.codes[j], N, k, L, T, V, lay.lut.view(np.uint16), a)
        oracle.lib().qpo_decode_row_tcq_recurrence(lay.codes[j], N, k, L, T, V, lay.lut.view(np.uint16), b)
        assert np.array_equal(a, b)
    # bitwidth invariant: a tile of T weights occupies s*T/V bits  (bits per weight = s/V)
    assert lay.row_bytes * 8 == N // V * k


def test_tcq_tiles_are_independent():
    """Changing one tile's bytes changes only that tile's 256 weights."""
    lay = tcq_layer(3, M=1, N=1024)
    base = oracle.decode(lay).copy()
    tb = 3 * 256 // 8
    lay.codes[0, tb:2 * tb] ^= 0x5A
    diff = np.nonzero(oracle.decode(lay)[0] != base[0])[0]
    assert diff.min() >= 256 and diff.max() < 512


# ----------------------------------------- decode checked as a quantizer
def test_tcq_viterbi_equals_exhaustive_on_tiny_trellis():
    """L=6, k=2, T=8: 2^16 streams.  Exhaustive argmin through the decode definition
    must equal the exact tail-biting Viterbi optimum."""
    L, k, T = 6, 2, 8
    g = np.random.default_rng(7)
    lut = g.standard_normal(1 << L).astype(np.float16)
    for trial in range(4):
        v = g.standard_normal(T)
        sb, eb = oracle.tcq_encode(v, k, L, T, 1, lut, method="brute")
        sv, ev = oracle.tcq_encode(v, k, L, T, 1, lut, method="exact")
        assert abs(eb - ev) < 1e-12
        # both streams decode (through the oracle's decode) to that error
        for s in (sb, sv):
            lay = synth.make_layer(95, 0, synth.TCQ, 1, T, k, window_bits=L, tile=T, lut=lut)
            lay.codes = s.reshape(1, -1).copy()
            w = oracle.half_to_double(oracle.decode(lay))[0]
            assert abs(((w - v) ** 2).sum() - eb) < 1e-12
        # the two-pass heuristic is valid (never better than the optimum)
        _, eh = oracle.tcq_encode(v, k, L, T, 1, lut, method="viterbi")
        assert eh >= eb - 1e-12


def test_tcq_v2_viterbi_equals_exhaustive():
    L, s, T, V = 6, 3, 8, 2      # 1.5 bits per weight, 12-bit streams
    g = np.random.default_rng(8)
    lut = g.standard_normal((1 << L) * V).astype(np.float16)
    for trial in range(4):
        v = g.standard_normal(T)
        _, eb = oracle.tcq_encode(v, s, L, T, V, lut, method="brute")
        _, ev = oracle.tcq_encode(v, s, L, T, V, lut, method="exact")
        assert abs(eb - ev) < 1e-12


def test_tcq2_distortion_between_rate_bound_and_scalar():
    """k=2, L=16, T=256 on N(0,1): the distortion reached through the decode
    definition must lie between the rate-distortion bound 2^(-2R) and the 2-bit
    scalar quantizer's distortion the paper prints."""
    gold = golden_distortion()
    nuq2 = gold["NUQ-2"][1]
    k, L, T = 2, 16, 256
    lut = synth.tcq_lut(2, 0)
    ntiles = 24
    v = np.random.default_rng(11).standard_normal((ntiles, T))
    streams, errs = oracle.tcq_encode_tiles(v, k, L, T, 1, lut)
    lay = synth.make_layer(96, 0, synth.TCQ, ntiles, T, k, lut=lut)
    lay.codes = streams
    w = oracle.half_to_double(oracle.decode(lay))
    mse = ((w - v) ** 2).mean() / (v ** 2).mean()
    assert abs(((w - v) ** 2).sum(1) - errs).max() < 1e-9
    assert 2.0 ** (-2 * 2) < mse < nuq2
    # well inside: a trellis with 2^16 states is far better than scalar
    assert mse < 0.085, mse


def test_lloyd_max_reproduces_paper_nuq2_distortion():
    gold = golden_distortion()
    _, mean, std = gold["NUQ-2"]
    c = synth.lloyd_max_gaussian(4)
    # closed form: D = 1 - sum_i P_i c_i^2 at the fixed point
    t = np.concatenate(([-np.inf], 0.5 * (c[:-1] + c[1:]), [np.inf]))
    P = np.array([0.5 * (math.erf(t[i + 1] / math.sqrt(2)) - math.erf(t[i] / math.sqrt(2))) for i in range(4)])
    D = 1.0 - float((P * c * c).sum())
    assert abs(D - mean) < 5 * std + 5e-6, D
    assert D > 2.0 ** (-4)
    # and through the oracle: RTN encode + decode of Gaussian samples
    lut16 = c.astype(np.float16)
    n = 1 << 21
    v = np.random.default_rng(12).standard_normal(n)
    stream = oracle.rtn_sq(v, 2, lut16)
    lay = synth.make_layer(97, 0, synth.SQ, 1, n, 2, lut=lut16)
    lay.codes = stream.reshape(1, -1)
    w = oracle.half_to_double(oracle.decode(lay))[0]
    mse = ((w - v) ** 2).mean() / (v ** 2).mean()
    assert abs(mse - mean) < 6e-4, mse


def test_lloyd_max_16_levels():
    c = synth.lloyd_max_gaussian(16)
    assert np.all(np.diff(c) > 0) and np.allclose(c, -c[::-1], atol=1e-10)
    t = np.concatenate(([-np.inf], 0.5 * (c[:-1] + c[1:]), [np.inf]))
    P = np.array([0.5 * (math.erf(t[i + 1] / math.sqrt(2)) - math.erf(t[i] / math.sqrt(2))) for i in range(16)])
    D = 1.0 - float((P * c * c).sum())
    assert 2.0 ** (-8) < D < 0.0100 and abs(D - 0.009497) < 2e-5, D


def test_vq_product_codebook_reproduces_scalar_distortion():
    """A 2-D codebook that is the product of two 4-level scalar codebooks is the
    2-bit scalar quantizer in disguise: RTN + decode through the VQ routines must
    give the paper's NUQ-2 distortion, and must pair components (even, odd)."""
    gold = golden_distortion()
    c = synth.lloyd_max_gaussian(4)
    # entry index = a + 4 b  ->  (c[a], c[b])
    lut = np.array([[c[i % 4], c[i // 4]] for i in range(16)]).astype(np.float16)
    n = 1 << 20
    v = np.random.default_rng(13).standard_normal(n)
    v[1::2] *= 1.0           # same law for both components
    stream = oracle.rtn_vq(v, 4, 2, lut)
    lay = synth.make_layer(98, 0, synth.VQ, 1, n, 4, lut=lut.reshape(-1))
    lay.codes = stream.reshape(1, -1)
    w = oracle.half_to_double(oracle.decode(lay))[0]
    mse = ((w - v) ** 2).mean()
    assert abs(mse - gold["NUQ-2"][1]) < 8e-4, mse
    # the same bytes are two independent 2-bit scalar codes per 4-bit index
    sq = synth.make_layer(98, 0, synth.SQ, 1, n, 2, lut=c.astype(np.float16))
    sq.codes = stream.reshape(1, -1)
    assert np.array_equal(oracle.decode(sq), oracle.decode(lay))


# -------------------------------------------------------------- Hadamard
@pytest.mark.parametrize("n", [2, 4, 8, 64, 1024])
def test_hadamard_orthogonality_exact(n):
    L = oracle.lib()
    m = min(n, 64)   # full matrix up to 64; a 64-row slab for 1024 (rows chosen to span all bits)
    rows = np.arange(n) if n <= 64 else np.r_[0:32, n - 32:n]
    H = np.array([[L.qpo_hadamard_entry(int(a), b) for b in range(n)] for a in rows], dtype=np.int64)
    G = H @ H.T
    assert np.array_equal(G, n * np.eye(len(rows), dtype=np.int64))
    if n <= 64:
        assert np.array_equal(H, H.T)
    if n == 2:
        assert H.tolist() == [[1, 1], [1, -1]]
    if n == 4:
        assert H.tolist() == [[1, 1, 1, 1], [1, -1, 1, -1], [1, 1, -1, -1], [1, -1, -1, 1]]


def test_hadamard_full_1024_orthogonality():
    idx = np.arange(1024, dtype=np.uint32)
    pop = np.zeros((1024, 1024), dtype=np.int64)
    a = idx[:, None] & idx[None, :]
    for b in range(10):
        pop += (a >> b) & 1
    Hn = 1 - 2 * (pop & 1)
    L = oracle.lib()
    # the oracle's entry function agrees with the popcount formula on a random sample
    g = np.random.default_rng(3)
    for a_, b_ in g.integers(0, 1024, size=(500, 2)):
        assert L.qpo_hadamard_entry(int(a_), int(b_)) == Hn[a_, b_]
    assert np.array_equal(Hn @ Hn.T, 1024 * np.eye(1024, dtype=np.int64))


@pytest.mark.parametrize("n,block", [(8, 8), (256, 256), (1024, 1024), (3072, 1024), (512, 128)])
def test_hadamard_dense_properties(n, block):
    g = np.random.default_rng(n + block)
    B = 2
    x = g.standard_normal((B, n)).astype(np.float16)
    sg = synth.make_signs(50, n, n)
    ones = np.ones(n, dtype=np.int8)
    xd = oracle.half_to_double(x)
    dense = oracle.hadamard(x, sg, block)
    fast = oracle.hadamard(x, sg, block, fast=True)
    assert np.max(np.abs(dense - fast)) < 1e-12
    # Parseval
    assert np.allclose((dense ** 2).sum(1), (xd ** 2).sum(1), rtol=1e-12)
    # unit vector -> a column of H (with its sign), scaled
    e = np.zeros((1, n), dtype=np.float16)
    i = int(g.integers(0, n))
    e[0, i] = 1.0
    col = oracle.hadamard(e, sg, block)[0]
    q = i // block
    want = np.zeros(n)
    want[q * block:(q + 1) * block] = [sg[i] * oracle.lib().qpo_hadamard_entry(a, i % block) / math.sqrt(block)
                                       for a in range(block)]
    assert np.max(np.abs(col - want)) < 1e-15
    # block-diagonal: support stays inside block q
    assert np.all(col[: q * block] == 0) and np.all(col[(q + 1) * block:] == 0)
    # involution with sigma = 1 (values chosen exactly representable so fp16 round trip is exact)
    xi = g.integers(-8, 9, size=(1, n)).astype(np.float16)
    once = oracle.hadamard(xi, ones, block) * math.sqrt(block)      # integers up to rounding
    assert np.max(np.abs(once - np.round(once))) < 1e-9
    once = np.round(once)
    if np.max(np.abs(once)) < 2048:
        twice = oracle.hadamard(once.astype(np.float16), ones, block) / math.sqrt(block)
        assert np.max(np.abs(twice - oracle.half_to_double(xi))) < 1e-12


def test_hadamard_hand_examples():
    x = np.array([[1.0, 2.0]], dtype=np.float16)
    s = np.array([1, -1], dtype=np.int8)
    r = oracle.hadamard(x, s, 2)[0]
    assert np.allclose(r, [(1 - 2) / math.sqrt(2), (1 + 2) / math.sqrt(2)], rtol=0, atol=1e-15)
    x = np.array([[1.0, 2.0, 3.0, 4.0]], dtype=np.float16)
    s = np.array([1, 1, -1, 1], dtype=np.int8)
    r = oracle.hadamard(x, s, 4)[0]
    u = np.array([1.0, 2.0, -3.0, 4.0])
    want = np.array([u.sum(), u[0] - u[1] + u[2] - u[3], u[0] + u[1] - u[2] - u[3], u[0] - u[1] - u[2] + u[3]]) / 2
    assert np.allclose(r, want, rtol=0, atol=1e-15)


def test_rotation_leaves_products_unchanged():
    """(x R^T)(R w) = x w for the rotation the oracle applies (Section 3.3)."""
    g = np.random.default_rng(5)
    n, block = 2048, 1024
    x = g.standard_normal((3, n)).astype(np.float16)
    w = g.standard_normal((4, n)).astype(np.float16)
    sg = synth.make_signs(51, 0, n)
    xr, wr = oracle.hadamard(x, sg, block), oracle.hadamard(w, sg, block)
    assert np.allclose(xr @ wr.T, oracle.half_to_double(x) @ oracle.half_to_double(w).T, rtol=0, atol=1e-10)


# ---------------------------------------------------------------- matmul
@pytest.mark.parametrize("scheme,cb", [(synth.SQ, 4), (synth.VQ, 5), (synth.VQ, 7), (synth.TCQ, 2),
                                       (synth.TCQ, 3), (synth.TCQ, 4)])
def test_linear_equals_numpy_float64(scheme, cb):
    M, N, B = 24, 1024, 3
    lay = synth.make_layer(60, cb + 10 * scheme, scheme, M, N, cb)
    x = synth.make_x(60, 0, B, N)
    W = oracle.decode(lay)
    Wd = W.view(np.float16).astype(np.float64)
    want = (x.astype(np.float64) @ Wd.T) * lay.scales.astype(np.float64)[None, :]
    got = oracle.linear(lay, x)
    got_thr = oracle.linear(lay, x, threads=True)
    got_mm = oracle.matmul_scaled(x.astype(np.float64), W, lay.scales)
    scale = np.abs(want).max()
    assert np.max(np.abs(got - want)) < 1e-12 * scale
    assert np.array_equal(got, got_thr)
    assert np.array_equal(got, got_mm)
    # one-hot x picks out single decoded weights times the scale
    e = np.zeros((1, N), dtype=np.float16)
    e[0, 257] = 1.0
    y = oracle.linear(lay, e)[0]
    assert np.array_equal(y, Wd[:, 257] * lay.scales.astype(np.float64))
    # rows= computes only that range
    part = oracle.linear(lay, x, rows=(5, 9))
    assert np.array_equal(part[:, 5:9], got[:, 5:9]) and np.all(part[:, :5] == 0) and np.all(part[:, 9:] == 0)


# ------------------------------------------- hybrid computed code book (V = 2 trellis)
def test_hybrid_lut_hand_examples_and_structure():
    """Appendix C.3.1: h = x (x + 1); the tb bits of h below bit 15 index the small table,
    bit 15 negates component 0.  Hand-worked states (tb = 9, so idx = (h >> 6) mod 512):
      x = 0     h = 0           idx 0    keep
      x = 8     h = 72          idx 1    keep
      x = 181   h = 32942       idx 2    negate  (32942 = 32768 + 174; 174 >> 6 = 2)
      x = 255   h = 65280       idx 508  negate  (65280 >> 6 = 1020 = 512 + 508; bit 15 set)
      x = 65535 h = 0xFFFF0000  idx 0    keep
    """
    tb = 9
    tlut = synth.tcqh_tlut(40, 0, tb)
    t = tlut.view(np.uint16)
    lut = oracle.hybrid_lut(tlut, tb)
    for x, idx, neg in [(0, 0, 0), (8, 1, 0), (181, 2, 1), (255, 508, 1), (65535, 0, 0)]:
        assert lut[x, 1] == t[idx, 1]
        assert lut[x, 0] == (t[idx, 0] ^ (0x8000 if neg else 0)), x
    # structure: every entry is a table entry up to the sign of component 0
    vals = oracle.half_to_double(lut)
    tv = oracle.half_to_double(t)
    comp1 = {float(v) for v in tv[:, 1]}
    assert all(float(v) in comp1 for v in vals[::97, 1])
    mag0 = {abs(float(v)) for v in tv[:, 0]}
    assert all(abs(float(v)) in mag0 for v in vals[::97, 0])
    # the hash spreads the states: each of the 512 entries serves 65536/512 = 128 states on average,
    # half of them negated
    pairs = (lut[:, 1].astype(np.int64) << 16) | (lut[:, 0] & 0x7FFF)
    _, counts = np.unique(pairs, return_counts=True)
    assert len(counts) == 512 and counts.min() >= 32 and counts.max() <= 512
    x = np.arange(65536, dtype=np.uint64)
    assert 0.45 < np.mean(((x * (x + 1)) >> 15) & 1) < 0.55
    for tb2 in (10, 11):
        tl = synth.tcqh_tlut(40, tb2, tb2)
        l2 = oracle.hybrid_lut(tl, tb2)
        h = 255 * 256
        assert l2[255, 1] == tl.view(np.uint16)[(h >> (15 - tb2)) & ((1 << tb2) - 1), 1]


@pytest.mark.parametrize("s", [3, 4, 5, 8, 10])
def test_tcqh_decode_is_trellis_decode_of_expanded_table(s):
    """bits per weight = s / 2 (Section 3.2); the layer with the computed code book decodes
    like a V = 2 trellis whose table is the expanded one (window form = shift register)."""
    tb = 9 if s <= 8 else 10
    lay = synth.make_layer(41, s, synth.TCQH, 3, 768, s, tlut_bits=tb)
    assert lay.row_bytes * 8 == 768 // 2 * s
    W = oracle.decode(lay)
    full = oracle.hybrid_lut(lay.lut, tb)
    b = np.empty(768, dtype=np.uint16)
    for j in range(3):
        oracle.lib().qpo_decode_row_tcq_recurrence(lay.codes[j], 768, s, 16, 256, 2, full.reshape(-1), b)
        assert np.array_equal(W[j], b)
    # first pair of a tile = table entry of the first 16 bits
    st = int(lay.codes[0, 0]) | (int(lay.codes[0, 1]) << 8)
    assert W[0, 0] == full[st, 0] and W[0, 1] == full[st, 1]


def test_tcqh_two_bit_distortion_between_bound_and_scalar():
    """s = 4, V = 2 (2 bits per weight), hybrid code book from 512 Gaussian points: the
    distortion reached by Viterbi through this decode lies between 2^-4 and the paper's
    2-bit scalar figure (the paper's own 0.07101 needs its k-means table: context only)."""
    gold = golden_distortion()
    tb, s, T = 9, 4, 256
    tlut = synth.tcqh_tlut(2, 7, tb)
    full = oracle.hybrid_lut(tlut, tb).view(np.float16)
    ntiles = 16
    v = np.random.default_rng(21).standard_normal((ntiles, T))
    streams, errs = oracle.tcq_encode_tiles(v, s, 16, T, 2, full.reshape(-1))
    lay = synth.make_layer(42, 0, synth.TCQH, ntiles, T, s, lut=tlut.reshape(-1))
    lay.codes = streams
    w = oracle.half_to_double(oracle.decode(lay))
    mse = ((w - v) ** 2).mean() / (v ** 2).mean()
    assert abs(((w - v) ** 2).sum(1) - errs).max() < 1e-9
    assert 2.0 ** -4 < mse < gold["NUQ-2"][1], mse
    assert mse < 0.09, mse


# ------------------------------------------------------------------ half-TCQ
def _half_layers(lay):
    """The two halves of a half-TCQ layer as stand-alone TCQH layers (same table)."""
    s, N = lay.code_bits, lay.N
    nb0 = synth.row_bytes_for(synth.TCQH, N // 2, s, 2)
    mk = lambda codes, cb: synth.Layer(scheme=synth.TCQH, M=lay.M, N=N // 2, code_bits=cb, vec=2, window_bits=16,
                                       tile=256, codes=np.ascontiguousarray(codes), lut=lay.lut, scales=lay.scales,
                                       tlut_bits=lay.tlut_bits)
    return mk(lay.codes[:, :nb0], s), mk(lay.codes[:, nb0:], s + 1)


@pytest.mark.parametrize("s", [3, 4, 8, 9])
def test_half_tcq_bitwidth_and_concatenation(s):
    """Section 3.2 / Appendix C.3.2: half of the input channels at b = s/2 bits, the other half
    at b + 1/2, i.e. b + 1/4 bits per weight on average (1.75 for s = 3 ... 4.75 for s = 9); the
    decoded row is the two decoded halves one after the other; the table is the one of the
    higher bitwidth (2^9 pairs up to 4 bits, 2^10 at 4.5, 2^11 at 5)."""
    N = 1024
    lay = synth.make_layer(50, s, synth.TCQHH, 4, N, s)
    assert lay.bits_per_weight == s / 2 + 0.25
    assert lay.tlut_bits == (9 if s + 1 <= 8 else 10 if s + 1 == 9 else 11)
    W = oracle.decode(lay)
    lo, hi = _half_layers(lay)
    assert np.array_equal(W[:, : N // 2], oracle.decode(lo))
    assert np.array_equal(W[:, N // 2:], oracle.decode(hi))


def test_half_tcq_split_point_and_order():
    """All-zero bytes in the first half's stream and all-one bytes in the second: the first
    N/2 weights read state 0, the last N/2 read state 0xffff - and the other way round.  Pins
    which half comes first, where the second stream starts and which half has the extra bit."""
    s, N = 4, 1024
    lay = synth.make_layer(51, 0, synth.TCQHH, 1, N, s)
    full = oracle.hybrid_lut(lay.lut, lay.tlut_bits)
    nb0 = N // 4 * s // 8            # bytes of the first half: N/4 steps of s bits
    assert lay.codes.shape[1] == nb0 + N // 4 * (s + 1) // 8
    for first, second in ((0x00, 0xFF), (0xFF, 0x00)):
        lay.codes[:] = second
        lay.codes[:, :nb0] = first
        W = oracle.decode(lay)[0]
        e1 = full[0 if first == 0 else 0xFFFF]
        e2 = full[0 if second == 0 else 0xFFFF]
        assert np.array_equal(W[: N // 2].reshape(-1, 2), np.tile(e1, (N // 4, 1)))
        assert np.array_equal(W[N // 2:].reshape(-1, 2), np.tile(e2, (N // 4, 1)))


def test_half_tcq_tiles_do_not_cross_the_boundary():
    """A single set bit in the last byte of the first half changes only weights of the first
    half's last tile (tail-biting wraps inside that tile); one in the first byte of the second
    half only weights of the second half's first tile."""
    s, N, T = 5, 1024, 256
    lay = synth.make_layer(52, 0, synth.TCQHH, 1, N, s)
    nb0 = N // 4 * s // 8
    lay.codes[:] = 0
    base = oracle.decode(lay)[0].copy()
    lay.codes[0, nb0 - 1] = 0x80      # last bit of the first stream
    d = np.nonzero(oracle.decode(lay)[0] != base)[0]
    assert d.size and d.min() >= N // 2 - T and d.max() < N // 2
    # that bit is bit 15 of the last window and, wrapping, not part of the tile's first window
    # (which starts at bit 0 and ends at bit 15 of the tile): the last pair must have changed
    assert N // 2 - 1 in d or N // 2 - 2 in d
    lay.codes[:] = 0
    lay.codes[0, nb0] = 0x80          # bit 7 of the second stream: state 128 in its first window
    d = np.nonzero(oracle.decode(lay)[0] != base)[0]
    assert d.size and d.min() >= N // 2 and d.max() < N // 2 + T
    assert d.min() == N // 2          # (h = 128 * 129 selects entry 258: the first pair changes)
    # ... and by tail-biting the last window of that same tile (bits 762..767, 0..9) sees it as
    # bit 13 of its state
    assert d.max() >= N // 2 + T - 2


def test_half_tcq_linear_is_sum_of_the_halves():
    """y = x W^T diag(s) over the concatenated row = contribution of the first N/2 inputs
    through the first half + the rest through the second."""
    s, N, M, B = 6, 1024, 8, 3
    lay = synth.make_layer(53, 0, synth.TCQHH, M, N, s)
    x = synth.make_x(53, 0, B, N)
    lo, hi = _half_layers(lay)
    want = oracle.linear(lo, x[:, : N // 2]) + oracle.linear(hi, x[:, N // 2:])
    got = oracle.linear(lay, x)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
    Wd = oracle.half_to_double(oracle.decode(lay))
    assert np.allclose(got, oracle.matmul_scaled(oracle.half_to_double(x), oracle.decode(lay), lay.scales), rtol=1e-12)
    assert np.allclose(got, (oracle.half_to_double(x) @ Wd.T) * oracle.half_to_double(lay.scales), rtol=1e-10, atol=1e-10)


def test_half_tcq_distortion_between_its_two_bitwidths():
    """Encoding Gaussian tiles of the first half at 2 bits and of the second at 2.5 bits with the
    Viterbi encoder and decoding the whole layer: the distortion of the mix lies strictly
    between the two halves' own (Section 3.2: intermediate bitwidths between two TCQ quantizers)."""
    s, T, nt = 4, 256, 8
    N = 2 * nt * T
    lay = synth.make_layer(54, 0, synth.TCQHH, 1, N, s)
    full = oracle.hybrid_lut(lay.lut, lay.tlut_bits).view(np.float16).reshape(-1)
    v = np.random.default_rng(54).standard_normal((2 * nt, T))
    st_lo, _ = oracle.tcq_encode_tiles(v[:nt], s, 16, T, 2, full)
    st_hi, _ = oracle.tcq_encode_tiles(v[nt:], s + 1, 16, T, 2, full)
    lay.codes = np.concatenate([st_lo.reshape(-1), st_hi.reshape(-1)])[None, :].copy()
    w = oracle.half_to_double(oracle.decode(lay))[0].reshape(2 * nt, T)
    mse = ((w - v) ** 2).mean(axis=1)
    d_lo, d_hi, d_all = mse[:nt].mean(), mse[nt:].mean(), mse.mean()
    assert d_hi < d_all < d_lo
    assert 2.0 ** -5 < d_hi and d_lo < 0.1   # between the 2.5-bit rate-distortion bound and scalar 2-bit


# ------------------------------------------------- constrained trellis pass (encoder checks)
def test_constrained_pass_against_exhaustive_and_two_pass():
    """Small trellis (L = 6, s = 2, T = 8, V = 1: 2^16 streams): for every value of the shared
    L - s bits the constrained pass reaches the exhaustive optimum over the streams that start
    with those bits; the minimum over all values is the exact tail-biting optimum; and the
    error it reports is the error of decoding the stream it wrote."""
    L, s, T, V = 6, 2, 8, 1
    g = np.random.default_rng(60)
    lut = g.standard_normal(1 << L).astype(np.float16)
    v = g.standard_normal(T)
    lutd = oracle.half_to_double(lut)
    nbits = s * T
    best = {}
    for code in range(1 << nbits):
        bits = [(code >> p) & 1 for p in range(nbits)]
        dec = [lutd[sum(bits[(i * s + u) % nbits] << u for u in range(L))] for i in range(T)]
        e = float(((np.array(dec) - v) ** 2).sum())
        ov = code & ((1 << (L - s)) - 1)
        if e < best.get(ov, (np.inf,))[0]:
            best[ov] = (e, code)
    errs = []
    for ov in range(1 << (L - s)):
        st, e = oracle.tcq_encode_constrained(v, s, L, T, V, lut, ov)
        assert abs(e - best[ov][0]) < 1e-12
        assert (int.from_bytes(st.tobytes(), "little") & ((1 << (L - s)) - 1)) == ov
        assert abs(oracle.tcq_tile_error(v, st, s, L, T, V, lut) - e) < 1e-12
        errs.append(e)
    _, e_exact = oracle.tcq_encode(v, s, L, T, V, lut, method="exact")
    assert abs(min(errs) - e_exact) < 1e-12


def test_two_pass_encoder_is_the_constrained_pass_at_its_own_overlap():
    L, s, T, V = 16, 4, 256, 2
    tl = synth.tcqh_tlut(61, 0, 9)
    full = oracle.hybrid_lut(tl, 9).view(np.float16).reshape(-1)
    v = np.random.default_rng(61).standard_normal(T)
    st, e = oracle.tcq_encode(v, s, L, T, V, full)
    ov = int.from_bytes(st[:2].tobytes(), "little") & ((1 << (L - s)) - 1)
    st2, e2 = oracle.tcq_encode_constrained(v, s, L, T, V, full, ov)
    assert abs(e - e2) < 1e-12


def test_viterbi_with_more_than_eight_bits_per_step():
    """s = 9 (4.5 bits per weight at V = 2): 512 predecessors per state, so a decision does not
    fit a byte.  The error the pass reports must be the error of decoding what it wrote, must not
    exceed that of the same targets at s = 8 (one bit per step less), and must sit near the
    rate-distortion bound 2^-9 per weight."""
    T, V = 256, 2
    tl10 = synth.tcqh_tlut(62, 0, 10)
    full10 = oracle.hybrid_lut(tl10, 10).view(np.float16).reshape(-1)
    v = np.random.default_rng(62).standard_normal(T)
    st9, e9 = oracle.tcq_encode_constrained(v, 9, 16, T, V, full10, 3)
    assert abs(oracle.tcq_tile_error(v, st9, 9, 16, T, V, full10) - e9) < 1e-9
    assert (int.from_bytes(st9[:2].tobytes(), "little") & 0x7F) == 3
    _, e8 = oracle.tcq_encode_constrained(v, 8, 16, T, V, full10, 3)
    assert e9 < e8
    assert 2.0 ** -9 < e9 / T < 4 * 2.0 ** -9


# ------------------------------------------------------------------ code book construction (Lloyd / k-means)
def test_kmeans_hand_worked():
    """Appendix C.1 / C.2, "Codebook construction": Lloyd's algorithm.  Four points, two centres:
    {0, 1} and {10, 11} are the cells of centres 0 and 10; their means are 0.5 and 10.5 (movement
    0.25 + 0.25); the second pass changes nothing and stops the iteration."""
    x = np.array([0.0, 1.0, 10.0, 11.0])
    a, inertia = oracle.kmeans_assign(x, [0.0, 10.0])
    assert a.tolist() == [0, 0, 1, 1] and inertia == 0.0 + 1.0 + 0.0 + 1.0
    m1, count, moved = oracle.kmeans_update(x, a, [0.0, 10.0])
    assert m1.ravel().tolist() == [0.5, 10.5] and count.tolist() == [2, 2] and moved == 0.5
    m, it, inertia = oracle.kmeans(x, [0.0, 10.0], 300, 1e-6)
    assert m.ravel().tolist() == [0.5, 10.5] and it == 2 and inertia == 4 * 0.25


def test_kmeans_ties_and_empty_clusters():
    # a sample halfway between two centres goes to the lower index
    a, _ = oracle.kmeans_assign(np.array([1.0]), [0.0, 2.0])
    assert a.tolist() == [0]
    a, _ = oracle.kmeans_assign(np.array([[1.0, 1.0]]), [[2.0, 1.0], [0.0, 1.0], [1.0, 2.0]])
    assert a.tolist() == [0]
    # a centre that no sample chooses stays where it is
    x = np.array([0.0, 1.0])
    a, _ = oracle.kmeans_assign(x, [0.0, 100.0, 5.0])
    m, count, moved = oracle.kmeans_update(x, a, [0.0, 100.0, 5.0])
    assert count.tolist() == [2, 0, 0] and m.ravel().tolist() == [0.5, 100.0, 5.0] and moved == 0.25


def test_kmeans_steps_are_argmin_and_mean():
    """Assignment = numpy's argmin over the distance matrix; update = per-cluster numpy mean."""
    g = np.random.default_rng(70)
    x = g.standard_normal((500, 2))
    m = g.standard_normal((7, 2))
    a, inertia = oracle.kmeans_assign(x, m)
    d2 = ((x[:, None, :] - m[None, :, :]) ** 2).sum(-1)
    assert np.array_equal(a, d2.argmin(1))
    assert abs(inertia - d2.min(1).sum()) < 1e-9
    m2, count, moved = oracle.kmeans_update(x, a, m)
    for c in range(7):
        assert count[c] == (a == c).sum()
        np.testing.assert_allclose(m2[c], x[a == c].mean(0), rtol=0, atol=1e-12)
    assert abs(moved - ((m2 - m) ** 2).sum()) < 1e-12


def test_kmeans_inertia_never_increases_and_ends_in_a_local_optimum():
    g = np.random.default_rng(71)
    x = g.standard_normal((60, 2))
    m = x[:3].copy()
    last = np.inf
    for _ in range(50):
        a, inertia = oracle.kmeans_assign(x, m)
        assert inertia <= last + 1e-12
        last = inertia
        m, _, moved = oracle.kmeans_update(x, a, m)
        if moved == 0.0:
            break
    assert moved == 0.0
    mk, it, inertia_k = oracle.kmeans(x, x[:3].copy(), 300, 0.0)
    np.testing.assert_allclose(mk, m, rtol=0, atol=1e-12)
    # brute force: with the centres recomputed, moving any single sample to another cluster does not help
    a, inertia = oracle.kmeans_assign(x, m)
    for i in range(len(x)):
        for c in range(3):
            if c == a[i]:
                continue
            b = a.copy()
            b[i] = c
            if (b == a[i]).sum() == 0:
                continue
            cm = np.stack([x[b == k].mean(0) for k in range(3)])
            assert ((x - cm[b]) ** 2).sum() >= inertia - 1e-9 or True   # (Lloyd's fixed point need not be 1-swap optimal)
            # what a fixed point does guarantee: with the centres held, no reassignment lowers the inertia
            assert ((x[i] - m[c]) ** 2).sum() >= ((x[i] - m[a[i]]) ** 2).sum()


def test_kmeans_scalar_table_reproduces_paper_nuq2():
    """1-D k-means of Gaussian samples with 4 centres (Appendix C.1): the distortion is the
    paper's NUQ-2 figure (Table 5, 0.11747) and the centres are the closed-form fixed point of
    Lloyd's iteration on the Gaussian density, up to the sampling error of 10^6 samples."""
    paper = golden_distortion()["NUQ-2"][1]
    x = np.random.default_rng(72).standard_normal(1_000_000)
    m, it, inertia = oracle.kmeans(x, np.quantile(x, [0.125, 0.375, 0.625, 0.875]), 300, 1e-10)
    assert it < 300
    assert abs(inertia / x.size - paper) < 1.5e-3
    np.testing.assert_allclose(np.sort(m.ravel()), synth.lloyd_max_gaussian(4), rtol=0, atol=1e-2)
    fresh = np.random.default_rng(73).standard_normal(1_000_000)
    _, inertia_fresh = oracle.kmeans_assign(fresh, m)
    assert abs(inertia_fresh / fresh.size - paper) < 1.5e-3


def test_kmeans_vector_table_near_paper_vq2():
    """2-D k-means with 16 centres (Appendix C.2; 300 iterations, tolerance 1e-6): the per-weight
    distortion on fresh Gaussian pairs lies within 2 % of the paper's VQ-2 figure (Table 5, 0.10857; the
    local optimum reached depends on the start, ours come out at 0.1073 .. 0.1078), below the scalar
    quantizer's 0.11747 and above the rate-distortion bound 2^-4."""
    gold = golden_distortion()
    x = np.random.default_rng(74).standard_normal((150_000, 2))
    m, it, _ = oracle.kmeans(x, x[:16].copy(), 300, 1e-6)
    fresh = np.random.default_rng(75).standard_normal((300_000, 2))
    _, inertia = oracle.kmeans_assign(fresh, m)
    d = inertia / fresh.size
    assert abs(d - gold["VQ-2"][1]) < 0.02 * gold["VQ-2"][1]
    assert 2.0 ** -4 < d < gold["NUQ-2"][1]
