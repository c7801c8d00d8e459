"""Pins of the MX (OCP Microscaling) oracle: value sets, round-to-nearest-even, saturation,
shared-exponent rule, wire layout, and agreement with a library cast where one exists."""
import numpy as np
import pytest
import torch

from oracle import dq_oracle as O

FMTS = [O.MXFP8, O.MXFP6, O.MXFP4]
MAXN = {O.MXFP8: 448.0, O.MXFP6: 28.0, O.MXFP4: 6.0}
EMAX = {O.MXFP8: 8, O.MXFP6: 4, O.MXFP4: 2}
MINSUB = {O.MXFP8: 2.0 ** -9, O.MXFP6: 2.0 ** -4, O.MXFP4: 0.5}


def values(fmt, e=127):
    bits = O.MX_CODE_BITS[fmt]
    return [O.mx_decode_elem(fmt, c, e) for c in range(1 << (bits - 1))]


def test_element_value_sets():
    # the FP4 E2M1 set printed in the OCP MX specification
    assert values(O.MXFP4) == [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    for fmt in FMTS:
        v = values(fmt)
        if fmt == O.MXFP8:
            v = v[:-1]  # S.1111.111 is NaN in E4M3
        assert v == sorted(v) and len(set(v)) == len(v)
        assert max(v) == MAXN[fmt] and v[1] == MINSUB[fmt]
        # negative half mirrors the positive one
        bits = O.MX_CODE_BITS[fmt]
        for c in range(1, len(v)):
            assert O.mx_decode_elem(fmt, c | (1 << (bits - 1)), 127) == -v[c]
    # E3M2: 2 mantissa bits -> normals are {1, 1.25, 1.5, 1.75} * 2^k, k = -2..4
    v6 = values(O.MXFP6)
    assert v6[4:8] == [0.25, 0.3125, 0.375, 0.4375] and v6[-4:] == [16.0, 20.0, 24.0, 28.0]


@pytest.mark.parametrize("fmt", FMTS)
def test_every_code_roundtrips_and_scales(fmt):
    bits = O.MX_CODE_BITS[fmt]
    for e in (0, 1, 100, 127, 200, 254):
        for c in range(1 << bits):
            if fmt == O.MXFP8 and (c & 0x7F) == 0x7F:
                continue
            x = O.mx_decode_elem(fmt, c, e)
            if e in (0, 254) and (not np.isfinite(x) or (x != 0 and abs(x) < 2.0 ** -149)):
                continue
            assert x == O.mx_decode_elem(fmt, c, 127) * 2.0 ** (e - 127)
            if np.float32(x) == x:
                assert O.mx_encode_elem(fmt, x, e) == c, (fmt, e, c, x)


@pytest.mark.parametrize("fmt", FMTS)
def test_round_to_nearest_even_and_saturation(fmt):
    v = values(fmt)
    if fmt == O.MXFP8:
        v = v[:-1]
    for i in range(len(v) - 1):
        lo, hi = v[i], v[i + 1]
        mid = (lo + hi) / 2
        want_tie = i if i % 2 == 0 else i + 1        # even mantissa wins a tie
        assert O.mx_encode_elem(fmt, mid, 127) == want_tie
        assert O.mx_encode_elem(fmt, np.nextafter(np.float32(mid), np.float32(0)), 127) == i
        assert O.mx_encode_elem(fmt, np.nextafter(np.float32(mid), np.float32(1e9)), 127) == i + 1
        sign = 1 << (O.MX_CODE_BITS[fmt] - 1)
        assert O.mx_encode_elem(fmt, -mid, 127) == (want_tie | sign)
    top = len(v) - 1
    for big in (MAXN[fmt] * 1.01, MAXN[fmt] * 1.25, MAXN[fmt] * 1.9):
        assert O.mx_encode_elem(fmt, big, 127) == top   # clamps to the largest normal
    assert O.mx_encode_elem(fmt, MINSUB[fmt] / 2, 127) == 0           # tie to even (zero)
    assert O.mx_encode_elem(fmt, MINSUB[fmt] * 0.51, 127) == 1


def test_fp8_agrees_with_library_cast_in_range():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.uniform(-448, 448, 4000), rng.standard_normal(4000) * 0.05,
                        rng.standard_normal(4000) * 2.0 ** -8]).astype(np.float32)
    x = x[np.abs(x) <= 448]
    ref = torch.from_numpy(x).to(torch.float8_e4m3fn).to(torch.float32).numpy()
    got = np.array([O.mx_decode_elem(O.MXFP8, O.mx_encode_elem(O.MXFP8, float(a), 127), 127) for a in x], np.float32)
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("fmt", FMTS)
def test_shared_exponent_rule(fmt):
    """E8M0 byte = floor(log2 max|v|) - emax_elem + 127, clamped to [0, 254], 0 for a zero block."""
    em = EMAX[fmt]
    for k in (-30, -1, 0, 1, 17):
        assert O.mx_block_scale(fmt, 2.0 ** k) == k - em + 127
        assert O.mx_block_scale(fmt, np.nextafter(np.float32(2.0 ** k), np.float32(0))) == k - 1 - em + 127
        assert O.mx_block_scale(fmt, 1.999 * 2.0 ** k) == k - em + 127
    assert O.mx_block_scale(fmt, 0.0) == 0
    assert O.mx_block_scale(fmt, 1e-44) == 0                     # subnormal input clamps to 0
    assert O.mx_block_scale(fmt, 3.0e38) == 127 + 127 - em
    # the block maximum always lands in the top binade of the element format
    for m in (3e-5, 0.77, 1.0, 5.5e3):
        e = O.mx_block_scale(fmt, m)
        top = abs(O.mx_decode_elem(fmt, O.mx_encode_elem(fmt, m, e), 127))
        assert 2.0 ** em <= top <= MAXN[fmt]


@pytest.mark.parametrize("fmt", FMTS)
def test_wire_layout_and_dar(fmt):
    rng = np.random.default_rng(fmt)
    n = 512
    a = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    b = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    cb = O.MX_CODE_BITS[fmt]
    packed = O.mx_compress(fmt, a)
    assert packed.size == ((n // 32) * (cb * 4 + 1) + 15) // 16 * 16
    scales = packed[(n // 32) * cb * 4:(n // 32) * cb * 4 + n // 32]
    bits = np.unpackbits(packed[:(n // 32) * cb * 4], bitorder="little").reshape(n, cb)
    codes = (bits * (1 << np.arange(cb))).sum(axis=1)
    for blk in range(n // 32):
        v = a[blk * 32:(blk + 1) * 32]
        e = O.mx_block_scale(fmt, float(np.abs(v).max()))
        assert scales[blk] == e
        assert list(codes[blk * 32:(blk + 1) * 32]) == [O.mx_encode_elem(fmt, float(x), e) for x in v]
    dec = O.mx_decompress(fmt, packed, n)
    assert np.array_equal(dec, np.array([O.mx_decode_elem(fmt, int(c), int(scales[i // 32])) for i, c in enumerate(codes)], np.float32))
    # DAR = decode + local, re-encoded; bf16 local widens exactly
    assert np.array_equal(O.mx_dar_hop(fmt, packed, b), O.mx_compress(fmt, (dec.astype(np.float64) + b).astype(np.float32)))
    h = (b.view(np.uint32) >> 16).astype(np.uint16)
    wide = (h.astype(np.uint32) << 16).view(np.float32)
    assert np.array_equal(O.mx_dar_hop(fmt, packed, h), O.mx_dar_hop(fmt, packed, wide))
    # error of one pass: half a quantum of the top binade, or the clamp when the block maximum
    # lies above the largest normal (the top binade is wider than the format can express)
    err = np.abs(dec - a).reshape(-1, 32).max(axis=1)
    X = 2.0 ** (scales.astype(np.float64) - 127)
    quantum = X * 2.0 ** (EMAX[fmt] - {8: 3, 6: 2, 4: 1}[cb])
    clamp = np.maximum(np.abs(a).reshape(-1, 32).max(axis=1) - MAXN[fmt] * X, 0.0)
    assert np.all(err <= np.maximum(quantum / 2, clamp) * (1 + 1e-6))
