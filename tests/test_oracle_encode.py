"""Pins for the oracle's encoder and bit packing (CPU only)."""
import itertools
import os

import numpy as np
import pytest

from oracle import build

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _unit(rng, n, D):
    x = rng.standard_normal((n, D))
    return x / np.linalg.norm(x, axis=1, keepdims=True)


@pytest.mark.parametrize("D,B", [(2, 2), (2, 3), (3, 2), (3, 3), (4, 2), (4, 3), (2, 4)])
def test_encoder_equals_brute_force_over_grid(D, B):
    # Eq. (3): the code is the argmax of the cosine over ALL 2^(B*D) grid points.
    rng = np.random.default_rng(10 * D + B)
    o = _unit(rng, 25, D)
    u = build.encode_unit(o, B)
    got = build.code_cosine(u, o, B)
    grid = np.array(list(itertools.product(range(1 << B), repeat=D)), dtype=np.uint8)
    for i in range(o.shape[0]):
        cos = build.code_cosine(grid, np.repeat(o[i:i + 1], grid.shape[0], 0), B)
        assert abs(got[i] - cos.max()) < 1e-12
        # the returned code is one of the maximisers
        assert np.any(np.all(grid[np.abs(cos - cos.max()) < 1e-12] == u[i], axis=1))


def test_one_bit_code_is_sign_and_closed_form_cosine():
    rng = np.random.default_rng(3)
    for D in (32, 128, 960):
        o = _unit(rng, 50, D)
        u = build.encode_unit(o, 1)
        assert np.array_equal(u, (o >= 0).astype(np.uint8))
        a = build.code_cosine(u, o, 1)
        assert np.allclose(a, np.abs(o).sum(1) / np.sqrt(D), rtol=0, atol=1e-12)
    # E|g|/sqrt(E g^2) = sqrt(2/pi) for a uniformly random direction
    o = _unit(rng, 400, 1024)
    a = build.code_cosine(build.encode_unit(o, 1), o, 1)
    assert abs(a.mean() - np.sqrt(2 / np.pi)) < 3e-3


def test_cosine_grows_with_bits_and_msb_is_sign():
    rng = np.random.default_rng(4)
    o = _unit(rng, 40, 64)
    prev = np.zeros(40)
    for B in range(1, 7):
        u = build.encode_unit(o, B)
        a = build.code_cosine(u, o, B)
        assert np.all(a >= prev - 1e-12)
        prev = a
        msb = u >> (B - 1)
        ex = u & ((1 << (B - 1)) - 1)
        assert np.array_equal(msb, (o >= 0).astype(np.uint8))              # 1-bit code = sign
        assert np.array_equal((msb.astype(int) << (B - 1)) + ex, u)          # split is lossless
    assert prev.min() > 0.995


def test_code_is_symmetric_under_negation():
    # x -> -x maps the grid onto itself (u -> 2^B-1-u), so codes of -o mirror.
    rng = np.random.default_rng(5)
    o = _unit(rng, 20, 32)
    o[np.abs(o) < 1e-9] = 0.1
    for B in (2, 4):
        u1 = build.encode_unit(o, B).astype(int)
        u2 = build.encode_unit(-o, B).astype(int)
        assert np.array_equal(u1 + u2, np.full_like(u1, (1 << B) - 1))


def test_critical_factor_count_matches_paper():
    # Section 2.2: D * 2^(B-1) critical rescaling factors (start state + events).
    with open(os.path.join(GOLD, "paper_sizes.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    want = {r[0]: r[1:] for r in rows}
    D, B, cnt = map(int, want["critical_factors"])
    L = (1 << (B - 1)) - 1
    assert D * L + D == cnt  # D*(2^(B-1)-1) level changes + the D initial levels


def test_pack_bits_fixture_and_roundtrip():
    # hand-written fixture: bit i (LSB=0) of word w <-> dimension 32w+i
    bits = np.zeros((2, 64), np.uint8)
    bits[0, [0, 1, 31, 32]] = 1
    bits[1, [5, 63]] = 1
    w = build.pack_bits(bits)
    assert w.tolist() == [[0x80000003, 0x00000001], [0x00000020, 0x80000000]]
    rng = np.random.default_rng(6)
    b = rng.integers(0, 2, (37, 96)).astype(np.uint8)
    assert np.array_equal(build.unpack_bits(build.pack_bits(b), 96), b)
    for F in (2, 4, 8):
        v = rng.integers(0, 1 << F, (11, 64)).astype(np.uint8)
        assert np.array_equal(build.unpack_fields(build.pack_fields(v, F), F, 64), v)
    # 4-bit fields: dims 0..7 in word 0, dim 0 in the low nibble
    v = np.zeros((1, 32), np.uint8); v[0, 0] = 0xA; v[0, 7] = 0x3; v[0, 8] = 0xF
    assert build.pack_fields(v, 4)[0, :2].tolist() == [0x3000000A, 0x0000000F]
    assert [build.long_field_bits(B) for B in range(2, 9)] == [2, 4, 4, 8, 8, 8, 8]
