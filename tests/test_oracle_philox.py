"""Pins for the oracle's Philox4x32-10 and the streams derived from it."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import rng
from oracle.philox import philox4x32_10

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def vendor_philox(tmp_path_factory):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc) or not os.path.exists("/opt/rocm/include/rocrand/rocrand_philox4x32_10.h"):
        pytest.skip("vendor Philox header / hipcc not available")
    exe = str(tmp_path_factory.mktemp("vp") / "vendor_philox_host")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-O1", os.path.join(HERE, "vendor_philox_host.cpp"),
                    "-o", exe], check=True, capture_output=True)
    return exe


def test_philox_matches_vendor_engine(vendor_philox):
    """Library pin: same key and counter give the same four words as rocRAND's
    engine run on the host (counter word c1 < 2^30 so the vendor offset fits)."""
    gen = np.random.Generator(np.random.PCG64(7))
    rows = [(0, 0, 0, 0, 0), (1, 2, 3, 4, 5), (0xFFFFFFFFFFFFFFFF, 0xFFFFFFFF, 0x3FFFFFFF, 0xFFFFFFFF, 0xFFFFFFFF)]
    for _ in range(200):
        rows.append((int(gen.integers(0, 2 ** 63)) * 2 + int(gen.integers(0, 2)),
                     int(gen.integers(0, 2 ** 32)), int(gen.integers(0, 2 ** 30)),
                     int(gen.integers(0, 2 ** 32)), int(gen.integers(0, 2 ** 32))))
    text = "\n".join(" ".join(str(v) for v in r) for r in rows) + "\n"
    out = subprocess.run([vendor_philox], input=text, capture_output=True, text=True, check=True).stdout
    want = np.array([[int(v) for v in line.split()] for line in out.strip().splitlines()], dtype=np.uint64)
    assert want.shape == (len(rows), 4)
    r = np.array(rows, dtype=np.uint64)
    for idx, row in enumerate(rows):                      # scalar path
        got = philox4x32_10((row[0] & 0xFFFFFFFF, row[0] >> 32), *row[1:])
        assert [int(g) for g in got] == [int(v) for v in want[idx]]
    same_seed = rows[1][0]                                # vectorised path, one key
    got = philox4x32_10((same_seed & 0xFFFFFFFF, same_seed >> 32), r[:, 1], r[:, 2], r[:, 3], r[:, 4])
    sub = subprocess.run([vendor_philox], input="\n".join(
        " ".join(str(v) for v in (same_seed,) + tuple(row[1:])) for row in rows) + "\n",
        capture_output=True, text=True, check=True).stdout
    want2 = np.array([[int(v) for v in line.split()] for line in sub.strip().splitlines()], dtype=np.uint32)
    assert np.array_equal(np.stack(got, axis=1), want2)


def test_stream_counter_layout(vendor_philox):
    """The named streams put (index, tag|q|index_hi, id, event) in the counter."""
    seed, tag, q, ident, event, index = 0x123456789ABCDEF, rng.TAG_NOISE, 2, 17, 40000, 123456
    got = rng.stream(seed, tag, q, ident, event, np.array([index]))
    c1 = (tag << 24) | (q << 16)
    out = subprocess.run([vendor_philox], input=f"{seed} {index} {c1} {ident} {event}\n",
                         capture_output=True, text=True, check=True).stdout.split()
    assert [int(g[0]) for g in got] == [int(v) for v in out]


def test_philox_is_a_bijection_of_the_counter():
    """Distinct counters never collide (Philox is a permutation per key)."""
    c0 = np.arange(1 << 16, dtype=np.uint64)
    w = np.stack(philox4x32_10((5, 9), c0, 0, 0, 0), axis=1)
    assert len({tuple(r) for r in w.tolist()}) == c0.size


def test_words_are_equidistributed():
    w = np.stack(rng.stream(3, rng.TAG_SR, 0, 1, 2, np.arange(1 << 16)), axis=1).reshape(-1)
    counts = np.bincount(w >> np.uint32(24), minlength=256)
    expected = w.size / 256
    chi2 = ((counts - expected) ** 2 / expected).sum()
    assert chi2 < 255 + 6 * np.sqrt(2 * 255)
    bits = np.unpackbits(w.view(np.uint8))
    assert abs(bits.mean() - 0.5) < 4 * 0.5 / np.sqrt(bits.size)


def test_sr_halves_layout():
    """Coordinate 8g+m uses word m//2 of call g, low half first."""
    seed, node, ev = 11, 3, 5
    h = rng.sr_halves(seed, node, ev, 16, 48)
    w = np.stack(rng.stream(seed, rng.TAG_SR, 0, node, ev, np.arange(2, 6)), axis=1)
    for g in range(4):
        for m in range(8):
            word = int(w[g, m // 2])
            assert h[8 * g + m] == ((word >> 16) if m % 2 else (word & 0xFFFF))
    # a window is a slice of the whole row
    assert np.array_equal(rng.sr_halves(seed, node, ev, 0, 64)[16:48], h)


def test_normals_moments_and_window():
    z = rng.normals(1, 2, 3, 1, 0, 1 << 18)
    assert abs(z.mean()) < 5 / np.sqrt(z.size)
    assert abs(z.var() - 1) < 5 * np.sqrt(2 / z.size)
    assert abs((z ** 4).mean() - 3) < 0.1
    pairs = z.reshape(-1, 2)
    assert abs(np.corrcoef(pairs[:, 0], pairs[:, 1])[0, 1]) < 0.01
    assert np.array_equal(rng.normals(1, 2, 3, 1, 4096, 8192), z[4096:8192])
    assert not np.array_equal(rng.normals(1, 2, 3, 0, 0, 64), z[:64])     # q selects a fresh sample


def test_normals_box_muller_by_hand():
    """One call written out: u1=(w0>>8 +1)/2^24, u2=(w1>>8)/2^24."""
    w = [int(x[0]) for x in rng.stream(9, rng.TAG_DATA, 0, 4, 6, np.array([10]))]
    z = rng.normals(9, 4, 6, 0, 40, 44)
    import math
    for pair in range(2):
        u1 = ((w[2 * pair] >> 8) + 1) / 2 ** 24
        u2 = (w[2 * pair + 1] >> 8) / 2 ** 24
        r = math.sqrt(-2 * math.log(u1))
        assert z[2 * pair] == pytest.approx(r * math.cos(2 * math.pi * u2), abs=1e-12)
        assert z[2 * pair + 1] == pytest.approx(r * math.sin(2 * math.pi * u2), abs=1e-12)


def test_noise_normals_law_and_window():
    """The gradient noise is standard normal: moments, a Kolmogorov-Smirnov test against
    the normal CDF (scipy), no correlation inside a Box-Muller pair or between neighbours."""
    from scipy import stats
    z = rng.noise_normals(1, 2, 3, 1, 0, 1 << 18)
    assert abs(z.mean()) < 5 / np.sqrt(z.size)
    assert abs(z.var() - 1) < 5 * np.sqrt(2 / z.size)
    assert abs((z ** 3).mean()) < 0.05
    assert abs((z ** 4).mean() - 3) < 0.1
    assert stats.kstest(z, "norm").pvalue > 1e-3
    assert np.abs(z).max() <= np.sqrt(34 * np.log(2))            # 16-bit radius: u1 >= 2^-17
    pairs = z.reshape(-1, 2)
    assert abs(np.corrcoef(pairs[:, 0], pairs[:, 1])[0, 1]) < 0.01
    assert abs(np.corrcoef(z[:-1], z[1:])[0, 1]) < 0.01
    assert abs(np.corrcoef(z[:-8], z[8:])[0, 1]) < 0.01          # neighbouring generator calls
    assert np.array_equal(rng.noise_normals(1, 2, 3, 1, 4096, 8192), z[4096:8192])
    for other in (rng.noise_normals(1, 2, 3, 0, 0, 64), rng.noise_normals(1, 3, 3, 1, 0, 64),
                  rng.noise_normals(1, 2, 4, 1, 0, 64), rng.noise_normals(2, 2, 3, 1, 0, 64)):
        assert not np.array_equal(other, z[:64])                 # step, node, event and seed all matter


def test_noise_normals_by_hand():
    """One generator call written out: word p -> coordinates 8g+2p (cosine) and 8g+2p+1 (sine),
    radius from the low half, angle from the high half."""
    import math
    g = 10
    w = [int(x[0]) for x in rng.stream(9, rng.TAG_NOISE, 2, 4, 6, np.array([g]))]
    z = rng.noise_normals(9, 4, 6, 2, 8 * g, 8 * g + 8)
    for p in range(4):
        u1 = ((w[p] & 0xFFFF) + 0.5) / 65536
        u2 = (w[p] >> 16) / 65536
        r = math.sqrt(-2 * math.log(u1))
        assert z[2 * p] == pytest.approx(r * math.cos(2 * math.pi * u2), abs=1e-12)
        assert z[2 * p + 1] == pytest.approx(r * math.sin(2 * math.pi * u2), abs=1e-12)


def test_scaled_index_is_floor_u_times_m():
    words = np.array([0, 1, 2 ** 31, 2 ** 32 - 1, 12345678], dtype=np.uint64)
    for m in (1, 3, 8, 255, 1000):
        from fractions import Fraction
        want = [int(Fraction(int(w), 2 ** 32) * m) for w in words]
        assert rng.scaled_index(words, m).tolist() == want
