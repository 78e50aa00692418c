"""Pins for the oracle's quantizer (the properties Corollary 2.1 asks for)."""
from fractions import Fraction
import math

import numpy as np
import pytest

from oracle import quantizer as qz
from oracle import rng

ALL_R16 = np.arange(65536, dtype=np.uint32)


@pytest.mark.parametrize("x,eps", [(0.3, 1.0), (-0.3, 1.0), (5.0 + 1 / 1024, 0.125), (-7.75, 0.5),
                                   (3.0, 1.0), (1e-3, 2.0 ** -12), (-2.718281, 0.01), (123.456, 0.1)])
def test_sr_up_probability_closed_form(x, eps):
    """Exhaustive over the 2^16 random halves: #up = ceil(frac 2^16 - 1/2)."""
    z = qz.stochastic_round(np.full(65536, x, dtype=np.float32), eps, ALL_R16)
    t = Fraction(float(np.float32(x) * (np.float32(1) / np.float32(eps))))   # the float32 product, exactly
    fl = math.floor(t)
    frac = Fraction(float(np.float32(float(t - fl))))                         # one float32 subtraction
    assert set(np.unique(z).tolist()) <= {fl, fl + 1}
    n_up = int((z == fl + 1).sum())
    assert n_up == max(0, math.ceil(frac * 65536 - Fraction(1, 2)))
    assert abs(Fraction(n_up, 65536) - frac) <= Fraction(1, 2 ** 17)          # unbiased to 2^-17


def test_sr_lattice_points_are_fixed_and_error_below_eps():
    eps = 0.25
    ints = np.arange(-50, 50)
    z = qz.stochastic_round((ints * eps).astype(np.float32), eps, np.full(ints.size, 65535))
    assert np.array_equal(z, ints)
    gen = np.random.Generator(np.random.PCG64(1))
    x = (gen.standard_normal(100000) * 10).astype(np.float32)
    z = qz.stochastic_round(x, eps, gen.integers(0, 65536, x.size))
    assert np.all(np.abs(z * eps - x.astype(np.float64)) < eps)


def test_sr_unbiased_on_averaged_trials():
    """Corollary 2.1 item 1: the mean of eps*z over independent Philox draws -> x."""
    eps, d, trials = 2.0 ** -4, 512, 4000
    gen = np.random.Generator(np.random.PCG64(2))
    x = gen.standard_normal(d).astype(np.float32)
    acc = np.zeros(d)
    for ev in range(trials):
        acc += qz.stochastic_round(x, eps, rng.sr_halves(5, 0, ev, 0, d)) * eps
    err = acc / trials - x
    assert np.abs(err).max() < 5 * (eps / 2) / math.sqrt(trials) + eps * 2 ** -16
    assert abs(err.mean()) < 5 * (eps / 2) / math.sqrt(trials * d) + eps * 2 ** -16
    # second moment: E (Q(x)-x)^2 = eps^2 frac (1 - frac) <= eps^2 / 4
    frac = x / eps - np.floor(x / eps)
    z = qz.stochastic_round(np.tile(x, 64), eps, np.random.Generator(np.random.PCG64(3)).integers(0, 65536, d * 64))
    emp = ((z * eps - np.tile(x, 64)) ** 2).mean()
    assert emp == pytest.approx((eps ** 2 * frac * (1 - frac)).mean(), rel=0.05)


@pytest.mark.parametrize("bits", [2, 4, 8, 16])
def test_decode_brute_force_window(bits):
    """z' == z  iff  z - k in [-2^(b-1), 2^(b-1)-1]; z' is always the member of
    the code's residue class inside that window around the key's cell k."""
    half = 1 << (bits - 1)
    span = 300 if bits <= 8 else 40000
    zs = np.arange(-span, span + 1, 7 if bits == 16 else 1)
    ks = np.array([-span, -257, -129, -3, -1, 0, 1, 2, 100, 255, span])
    eps = 0.5
    for k in ks:
        key = np.full(zs.size, k * eps, dtype=np.float32)          # key sits exactly on cell k
        zd = qz.decode(qz.code(zs, bits), key, eps, bits)
        ok = (zs - k >= -half) & (zs - k <= half - 1)
        assert np.array_equal(zd == zs, ok)
        assert np.all((zd - zs) % (1 << bits) == 0)
        assert np.all((zd - k >= -half) & (zd - k <= half - 1))


@pytest.mark.parametrize("bits", [4, 8])
def test_decode_radius_on_random_reals(bits):
    """|x - y| <= (2^(b-1) - 5/2) eps in every coordinate => exact recovery."""
    gen = np.random.Generator(np.random.PCG64(bits))
    eps = 2.0 ** -6
    radius = ((1 << (bits - 1)) - 2.5) * eps
    x = (gen.standard_normal(200000) * 3).astype(np.float32)
    y = (x + gen.uniform(-radius, radius, x.size)).astype(np.float32)
    y = np.where(np.abs(y.astype(np.float64) - x) <= radius, y, x)
    z = qz.stochastic_round(x, eps, gen.integers(0, 65536, x.size))
    assert np.array_equal(qz.decode(qz.code(z, bits), y, eps, bits), z)
    far = (x + 3 * (1 << bits) * eps).astype(np.float32)               # far outside: wraps
    zf = qz.decode(qz.code(z, bits), far, eps, bits)
    assert np.all(zf != z) and np.all((zf - z) % (1 << bits) == 0)


def test_key_cell_ties_to_even():
    assert qz.key_cell(np.array([0.5, 1.5, 2.5, -0.5, -1.5], dtype=np.float32), 1.0).tolist() == [0, 2, 2, 0, -2]


def test_pack_byte_images():
    assert qz.pack([1, 2, 3, 4, 5, 6, 7, 8], 4).tolist() == [0x21, 0x43, 0x65, 0x87]
    assert qz.pack([0, 1, 2, 3, 3, 2, 1, 0], 2).tolist() == [0xE4, 0x1B]
    assert qz.pack([1, 2, 3, 4, 5, 6, 7, 255], 8).tolist() == [1, 2, 3, 4, 5, 6, 7, 255]
    assert qz.pack([0x1234, 1, 2, 3, 4, 5, 6, 0xFFFF], 16).tolist()[:4] == [0x34, 0x12, 0x01, 0x00]
    gen = np.random.Generator(np.random.PCG64(0))
    for bits in (2, 4, 8, 16):
        c = gen.integers(0, 1 << bits, 256).astype(np.uint32)
        buf = qz.pack(c, bits)
        assert buf.size == 256 * bits // 8
        assert np.array_equal(qz.unpack(buf, bits, 256), c)


def test_negative_lattice_points_use_twos_complement_residues():
    assert qz.code([-1, -2, -16, -17], 4).tolist() == [15, 14, 0, 15]


def test_clamp_flag_and_bound():
    t, clamped = qz.lattice_coordinate(np.array([1e12, -1e12, 1.0], dtype=np.float32), 1e-3)
    assert clamped.tolist() == [True, True, False]
    # what is not a number is flagged too and takes the lower end of the clamp; infinities saturate
    t, clamped = qz.lattice_coordinate(np.array([np.nan, np.inf, -np.inf, 0.5], dtype=np.float32), 0.5)
    assert clamped.tolist() == [True, True, True, False]
    assert t.tolist() == [-2.0 ** 29, 2.0 ** 29, -2.0 ** 29, 1.0]
    z = qz.stochastic_round(np.array([np.nan, np.inf], dtype=np.float32), 0.5, np.zeros(2, dtype=np.uint32))
    assert z.tolist() == [-2 ** 29, 2 ** 29]
    assert abs(t[0]) == 2.0 ** 29 and abs(t[1]) == 2.0 ** 29
    z = qz.stochastic_round(np.array([1e12], dtype=np.float32), 1e-3, [7])
    assert int(z[0]) == 2 ** 29


def test_quantize_dequantize_round_trip_with_own_model_as_key():
    gen = np.random.Generator(np.random.PCG64(4))
    x = gen.standard_normal(4096).astype(np.float32)
    eps = 2.0 ** -5
    for bits in (2, 4, 8, 16):
        buf = qz.quantize(x, eps, bits, rng.sr_halves(1, 0, 0, 0, x.size))
        # key = the vector itself: z - rint(t) is in {-1, 0, 1}, inside even the 2-bit window [-2, 1]
        q = qz.dequantize(buf, x, eps, bits)
        assert np.all(np.abs(q - x) < eps)


@pytest.mark.parametrize("bits", [4, 8, 16])
def test_pair_scale_is_the_smallest_power_of_two_inside_the_radius(bits):
    """eps_ij = 2^ceil(log2(m / (2^(b-1) - 3))): a power of two, m <= (2^(b-1) - 3) eps (inside the
    decoding radius (2^(b-1) - 5/2) eps), and eps/2 would not do; with it no decode can fail."""
    gen = np.random.Generator(np.random.PCG64(bits))
    R = (1 << (bits - 1)) - 3
    for m in list(gen.uniform(1e-6, 50, 200)) + [R * 0.25, R * 0.5, float(np.float32(1e-3)), 0.0]:
        m = float(np.float32(m))
        eps = qz.pair_scale(m, bits)
        assert math.log2(eps) == int(math.log2(eps))
        if m > 2.0 ** -90:
            assert m <= R * eps and m > R * eps / 2 * (1 - 1e-6)
    x = (gen.standard_normal(20000) * 3).astype(np.float32)
    y = (x + gen.uniform(-1, 1, x.size) * 0.7).astype(np.float32)
    eps = qz.pair_scale(np.abs(x - y).max(), bits)
    z = qz.stochastic_round(x, eps, gen.integers(0, 65536, x.size))
    assert np.array_equal(qz.decode(qz.code(z, bits), y, eps, bits), z)


# ---------------------------------------------------------------- multi-resolution register
def lattice_and_key(seed, d, eps, distance):
    gen = np.random.Generator(np.random.PCG64(seed))
    x = (gen.standard_normal(d) * 3).astype(np.float32)
    z = qz.stochastic_round(x, eps, gen.integers(0, 65536, d))
    y = (x + gen.uniform(-distance, distance, d)).astype(np.float32)
    return z, y


def hashed_weights(j):
    """The two weights of position j, in plain Python integers."""
    x = ((2 * j + 1) * 0x9E3779B1) % 2 ** 32
    x ^= x >> 15
    x = (x * 0x85EBCA6B) % 2 ** 32
    x ^= x >> 13
    y = (x * 0xC2B2AE35) % 2 ** 32
    y ^= y >> 16
    return x | 1, y | 1


def test_prefix_register_image_by_hand():
    """Plane of bits 0-3 (two coordinates per byte, low nibble first), plane of bits 4-7, plane of
    bits 8-15 (one byte per coordinate), then per tile the two sums of z * weight mod 2^32."""
    z = np.array([0x1234, -1, 5, 0x0FF0, 7, 0x8000, 0x00A0, 3], dtype=np.int64)
    reg = qz.prefix_register(z)
    assert reg[:4].tolist() == [0xF4, 0x05, 0x07, 0x30]           # nibbles 4,F | 5,0 | 7,0 | 0,3
    assert reg[4:8].tolist() == [0xF3, 0xF0, 0x00, 0x0A]          # nibbles 3,F | 0,F | 0,0 | A,0
    assert reg[8:16].tolist() == [0x12, 0xFF, 0x00, 0x0F, 0x00, 0x80, 0x00, 0x00]
    want = [sum((int(v) % 2 ** 32) * hashed_weights(j)[f] for j, v in enumerate(z)) % 2 ** 32 for f in (0, 1)]
    assert reg[16:].view('<u4').tolist() == want and reg.size == 24
    w = [hashed_weights(j) for j in range(512)]
    assert all(a % 2 == 1 and b % 2 == 1 for a, b in w) and len({a for a, _ in w}) == 512 and len({b for _, b in w}) == 512
    two_tiles = qz.prefix_checksums(np.concatenate([z, np.zeros(504, dtype=np.int64), z]))
    assert np.array_equal(two_tiles[0], two_tiles[1])             # the position inside the tile sets the weight


def test_prefix_planes_are_the_fixed_width_codes():
    """The b low bits of the register are the b-bit code of the same lattice point: a reader of a
    prefix sees exactly what the fixed codec would have sent with that many bits."""
    z, _ = lattice_and_key(1, 1024, 0.25, 1.0)
    reg = qz.prefix_register(z)
    d = z.size
    assert np.array_equal(reg[:d // 2], qz.pack(qz.code(z, 4), 4))
    lo, mid = qz.unpack(reg[:d // 2], 4, d), qz.unpack(reg[d // 2:d], 4, d)
    assert np.array_equal(lo | (mid << 4), qz.code(z, 8))
    assert np.array_equal(lo | (mid << 4) | (qz.unpack(reg[d:2 * d], 8, d) << 8), qz.code(z, 16))


@pytest.mark.parametrize("cells,level", [(1.0, 0), (4.0, 0), (9.0, 1), (100.0, 1), (140.0, 2), (20000.0, 2)])
def test_prefix_read_uses_as_many_bits_as_the_distance_needs(cells, level):
    """Item 3 of Corollary 2.1: the bits needed grow with log(|x - y| / eps).  A key within
    (2^(b-1) - 5/2) cells decodes with b bits; the reader stops at the first level that does, and that
    level is the smallest whose decode equals the writer's lattice point (checked against the truth,
    not against the checksum)."""
    eps, d = 2.0 ** -4, 512 * 3 + 40
    z, y = lattice_and_key(int(cells), d, eps, cells * eps)
    zp, lev, conf = qz.prefix_read(qz.prefix_register(z), y, eps)
    assert np.array_equal(zp, z) and conf.all()
    assert lev.max() == level or cells in (4.0, 100.0)           # well inside a radius: may need fewer bits
    codes16 = qz.code(z, 16)
    for t in range(lev.size):
        sl = slice(512 * t, min(512 * (t + 1), d))
        ok = [np.array_equal(qz.decode(codes16[sl] & ((1 << b) - 1), y[sl], eps, b), z[sl]) for b in qz.PREFIX_LEVELS]
        assert lev[t] == ok.index(True)
    if cells <= 2 ** 3 - 2.5:
        assert (lev == 0).all()
    elif cells <= 2 ** 7 - 2.5:
        assert (lev <= 1).all()


def test_prefix_checksum_catches_every_single_wrapped_coordinate():
    """A decode that fails is off by a multiple of 2^b in some coordinates; with odd weights a single
    such coordinate always changes the checksum."""
    z, _ = lattice_and_key(3, 512, 0.5, 1.0)
    base = qz.prefix_checksums(z)[0]
    for k in range(0, 512, 7):
        for b in (4, 8):
            for mult in (-3, -1, 1, 2):
                w = z.copy()
                w[k] += mult * (1 << b)
                assert not np.array_equal(qz.prefix_checksums(w)[0], base)


def test_prefix_checksum_does_not_cancel_on_balanced_wraps():
    """What a failed decode looks like: many coordinates off by +2^b and as many by -2^b.  With weights
    linear in the position every pattern with equal position sums cancels; the hashed weights must not
    (all such four-coordinate patterns in a stretch of the tile, and random larger ones)."""
    z, _ = lattice_and_key(5, 512, 0.5, 1.0)
    base = qz.prefix_checksums(z)[0]
    for b in (4, 8):
        step = 1 << b
        for j1 in range(0, 40):
            for j2 in range(j1 + 1, 40):
                for j3 in range(j1 + 1, j2):
                    j4 = j1 + j2 - j3                       # j1 + j2 = j3 + j4: cancels for linear weights
                    if j4 <= j3:
                        continue
                    w = z.copy()
                    w[[j1, j2]] += step
                    w[[j3, j4]] -= step
                    assert not np.array_equal(qz.prefix_checksums(w)[0], base)
    gen = np.random.Generator(np.random.PCG64(6))
    for _ in range(2000):
        count = int(gen.integers(1, 120))
        idx = gen.choice(512, 2 * count, replace=False)
        w = z.copy()
        w[idx[:count]] += 16
        w[idx[count:]] -= 16
        assert not np.array_equal(qz.prefix_checksums(w)[0], base)


def test_prefix_read_beyond_sixteen_bits_is_reported():
    eps, d = 2.0 ** -6, 1024
    z, y = lattice_and_key(4, d, eps, 1.0)
    y[700] += 40000 * eps                                        # farther than the 16-bit radius: tile 1 only
    zp, lev, conf = qz.prefix_read(qz.prefix_register(z), y, eps)
    assert conf.tolist() == [True, False] and lev.tolist() == [lev[0], 2]
    assert np.array_equal(zp[:512], z[:512]) and zp[700] != z[700] and (zp[700] - z[700]) % 65536 == 0


# ---------------------------------------------------------------- properties over arbitrary inputs
from hypothesis import given, settings, strategies as st


@settings(max_examples=200, deadline=None)
@given(bits=st.sampled_from([2, 4, 8, 16]), e=st.integers(-12, 6), x=st.floats(-1e3, 1e3, width=32),
       offset=st.floats(-1.0, 1.0), r16=st.integers(0, 65535))
def test_decode_recovers_the_sender_inside_the_radius_for_any_input(bits, e, x, offset, r16):
    """Corollary 2.1's precondition in this instantiation: whenever |x - y| <= (2^(b-1) - 5/2) eps the
    receiver decodes exactly the sender's lattice point, whatever x, eps and the rounding draw."""
    eps = 2.0 ** e
    radius = (2 ** (bits - 1) - 2.5) * eps
    if abs(x) / eps > 2.0 ** 28 or radius <= 0:
        return
    x32 = np.float32(x)
    y32 = np.float32(float(x32) + offset * radius * 0.999)
    if abs(float(y32) - float(x32)) > radius:
        return
    z = qz.stochastic_round(np.array([x32]), eps, np.array([r16]))
    got = qz.decode(qz.code(z, bits), np.array([y32]), eps, bits)
    assert got[0] == z[0] and abs(z[0] * eps - float(x32)) < eps * (1 + 1e-6)


@settings(max_examples=100, deadline=None)
@given(seed=st.integers(0, 2 ** 32 - 1), d=st.sampled_from([8, 24, 512, 520, 1032]), spread=st.floats(0.0, 200.0))
def test_prefix_read_is_exact_whenever_sixteen_bits_reach(seed, d, spread):
    """Any key within the 16-bit radius of the writer's point decodes exactly, at the smallest level
    that does, and every tile is confirmed."""
    eps = 2.0 ** -3
    gen = np.random.Generator(np.random.PCG64(seed))
    x = (gen.standard_normal(d) * 5).astype(np.float32)
    z = qz.stochastic_round(x, eps, gen.integers(0, 65536, d))
    y = (x + gen.uniform(-spread, spread, d) * eps).astype(np.float32)
    zp, level, confirmed = qz.prefix_read(qz.prefix_register(z), y, eps)
    assert np.array_equal(zp, z) and confirmed.all()
    cells = np.abs(x.astype(np.float64) - y) / eps
    for t in range(level.size):
        worst = cells[512 * t:512 * (t + 1)].max()
        if worst <= 2 ** 3 - 2.5:
            assert level[t] == 0
        elif worst <= 2 ** 7 - 2.5:
            assert level[t] <= 1
