"""Lattice quantizer with a decoding key (instantiates Corollary 2.1).

The paper states the quantizer by its properties only: unbiased, error
proportional to eps and independent of the norm of x, and decodable from any
key y close enough to x, with more bits buying a larger distance.  This build
realises it as stochastic rounding to the lattice eps*Z^d, sending each lattice
coordinate modulo 2^b, and decoding to the representative of that residue
class nearest to the key.  Test infrastructure only.

The rounding decision and the key's lattice cell are float32 decisions (single
IEEE operations: one multiply, floor, one subtract, one compare; one multiply
and one round-to-nearest-even), identical on CPU and GPU.
"""
import numpy as np

F32 = np.float32
CLAMP = F32(2.0 ** 29)     # |x/eps| is clamped here so z_i + z_j' fits int32
SUPPORTED_BITS = (2, 4, 8, 16)


def inv_eps_of(eps):
    return F32(1.0) / F32(eps)


def lattice_coordinate(x, eps):
    """t = clamp(x * (1/eps)) in float32, and whether the clamp was active.  A coordinate that is
    not a number has no lattice point: it is flagged like an overflow and sent as the lower end of
    the clamp, so that a diverged model cannot pass for a finite one unnoticed."""
    with np.errstate(invalid="ignore", over="ignore"):
        t = np.asarray(x, dtype=F32) * inv_eps_of(eps)
        clamped = ~(np.abs(t) <= CLAMP)
    t = np.where(np.isnan(t), -CLAMP, t)
    return np.clip(t, -CLAMP, CLAMP).astype(F32), clamped


def stochastic_round(x, eps, r16):
    """z = floor(t) + [r16 + 1/2 < frac(t) * 2^16],  t = x/eps (float32).

    r16 is uniform on {0..65535}, so P(up) = ceil(frac*2^16 - 1/2) / 2^16:
    within 2^-17 of frac, which makes E[eps*z] = x up to that resolution
    (Corollary 2.1 item 1) and |eps*z - x| < eps (item 2's analogue)."""
    t, _ = lattice_coordinate(x, eps)
    f = np.floor(t)
    frac = (t - f).astype(F32)
    up = (np.asarray(r16).astype(F32) + F32(0.5)) < frac * F32(65536.0)
    return f.astype(np.int64) + up.astype(np.int64)


def code(z, bits):
    """The b low bits of the lattice coordinate: z mod 2^b."""
    return (np.asarray(z, dtype=np.int64) & ((1 << bits) - 1)).astype(np.uint32)


def key_cell(y, eps):
    """Lattice coordinate nearest to the key (ties to even)."""
    t, _ = lattice_coordinate(y, eps)
    return np.rint(t).astype(np.int64)


def decode(c, y, eps, bits):
    """The integer congruent to c (mod 2^b) in [k - 2^(b-1), k + 2^(b-1) - 1],
    k = key_cell(y).  Equals the sender's z iff z - k lies in that window,
    which holds whenever |x - y| <= (2^(b-1) - 5/2) eps in every coordinate."""
    k = key_cell(y, eps)
    m = 1 << bits
    delta = (np.asarray(c, dtype=np.int64) - k) % m       # in [0, 2^b)
    delta = np.where(delta >= m // 2, delta - m, delta)   # sign-extend
    return k + delta


def pack(c, bits):
    """Codes -> bytes, coordinate k in bits [k*b, (k+1)*b) of a little-endian
    bit stream.  len(c) must be a multiple of 8."""
    c = np.asarray(c, dtype=np.uint32)
    assert c.size % 8 == 0 and bits in SUPPORTED_BITS
    if bits == 16:
        return c.astype('<u2').view(np.uint8).copy()
    if bits == 8:
        return c.astype(np.uint8)
    per = 8 // bits
    c = c.reshape(-1, per).astype(np.uint32)
    out = np.zeros(c.shape[0], dtype=np.uint32)
    for m in range(per):
        out |= c[:, m] << np.uint32(m * bits)
    return out.astype(np.uint8)


def unpack(buf, bits, count):
    buf = np.asarray(buf, dtype=np.uint8)
    assert bits in SUPPORTED_BITS
    if bits == 16:
        return buf.view('<u2').astype(np.uint32)[:count]
    if bits == 8:
        return buf.astype(np.uint32)[:count]
    per = 8 // bits
    shifts = (np.arange(per, dtype=np.uint32) * np.uint32(bits))
    c = (buf.astype(np.uint32)[:, None] >> shifts[None, :]) & np.uint32((1 << bits) - 1)
    return c.reshape(-1)[:count]


def quantize(x, eps, bits, r16):
    """Enc: packed codes of the stochastically rounded lattice point."""
    return pack(code(stochastic_round(x, eps, r16), bits), bits)


def dequantize(buf, key, eps, bits):
    """Dec: lattice point nearest the key in the code's class, times eps (float64)."""
    key = np.asarray(key, dtype=F32)
    z = decode(unpack(buf, bits, key.size), key, eps, bits)
    return z.astype(np.float64) * float(F32(eps))


# ---- multi-resolution register: a 16-bit code read by prefixes ---------------------------------
# Proof of Corollary 2.1, second case: the writer does not know its reader's key, so it writes its
# messages for every resolution into its own register and the reader uses only a prefix; item 3 of
# the corollary: the first B bits suffice, B growing with log(|x - y| / eps).  Here the messages are
# nested: the b low bits of one 16-bit residue are the b-bit code, so the register holds the 16-bit
# code split into planes (bits 0-3, 4-7, 8-15 of every coordinate) and a reader fetches planes until
# the decode is confirmed.  The confirmation that the interactive protocol gets from the receiver's
# reply is a 64-bit checksum of the writer's lattice coordinates (two 32-bit sums with pseudo-random
# odd weights), one per tile of 512 coordinates, kept beside the planes: a reader stops at the first
# level whose decoded tile has that checksum.  A failed decode is off by multiples of 2^b in some
# coordinates, often +1 and -1 multiples in many of them at once, so weights that are linear in the
# position would cancel far too often; hashed weights make a false confirmation a 2^-(64-2b) event.
PREFIX_LEVELS = (4, 8, 16)      # bits per coordinate known after reading 1, 2, 3 planes
PREFIX_TILE = 512               # coordinates per checksum
_M32 = np.uint64(0xFFFFFFFF)


def prefix_weights(count):
    """The two odd 32-bit weights of every coordinate, by its position j inside its tile:
    x = (2j+1) 0x9E3779B1;  x ^= x >> 15;  x *= 0x85EBCA6B;  x ^= x >> 13;  w1 = x | 1;
    y = x 0xC2B2AE35;  y ^= y >> 16;  w2 = y | 1   (all modulo 2^32)."""
    j = np.arange(count, dtype=np.uint64) % np.uint64(PREFIX_TILE)
    x = ((np.uint64(2) * j + np.uint64(1)) * np.uint64(0x9E3779B1)) & _M32
    x ^= x >> np.uint64(15)
    x = (x * np.uint64(0x85EBCA6B)) & _M32
    x ^= x >> np.uint64(13)
    y = (x * np.uint64(0xC2B2AE35)) & _M32
    y ^= y >> np.uint64(16)
    return x | np.uint64(1), y | np.uint64(1)


def prefix_checksums(z):
    """(tiles, 2) uint32: sum_k (z_k mod 2^32) * w_k mod 2^32 for both weight families over every
    tile of 512 coordinates (the last may be short)."""
    z = np.asarray(z, dtype=np.int64)
    zu = (z & 0xFFFFFFFF).astype(np.uint64)
    tiles = -(-z.size // PREFIX_TILE)
    out = np.zeros((tiles, 2), dtype=np.uint64)
    for col, w in enumerate(prefix_weights(z.size)):
        np.add.at(out[:, col], np.arange(z.size) // PREFIX_TILE, (zu * w) & _M32)
    return (out & _M32).astype(np.uint32)


def prefix_register(z):
    """Register image of a lattice point: plane of bits 0-3 (d/2 bytes), plane of bits 4-7 (d/2 bytes),
    plane of bits 8-15 (d bytes), then the tile checksums (two little-endian uint32 per tile)."""
    z = np.asarray(z, dtype=np.int64)
    p0 = pack(z & 15, 4)
    p1 = pack((z >> 4) & 15, 4)
    p2 = pack((z >> 8) & 255, 8)
    return np.concatenate([p0, p1, p2, prefix_checksums(z).astype('<u4').reshape(-1).view(np.uint8)])


def prefix_read(register, key, eps):
    """Decode a register against `key`, tile by tile, from the shortest confirmed prefix.

    Returns (z', level per tile in {0, 1, 2}, confirmed per tile).  Level l uses the
    PREFIX_LEVELS[l] low bits of every coordinate; an unconfirmed tile keeps the 16-bit decode."""
    key = np.asarray(key, dtype=F32)
    d = key.size
    register = np.asarray(register, dtype=np.uint8)
    lo = unpack(register[:d // 2], 4, d)
    mid = unpack(register[d // 2:d], 4, d)
    hi = unpack(register[d:2 * d], 8, d)
    checks = register[2 * d:].view('<u4').reshape(-1, 2)
    codes = (lo, lo | (mid << np.uint32(4)), lo | (mid << np.uint32(4)) | (hi << np.uint32(8)))
    tiles = -(-d // PREFIX_TILE)
    z = np.empty(d, dtype=np.int64)
    level = np.zeros(tiles, dtype=np.int64)
    confirmed = np.zeros(tiles, dtype=bool)
    for t in range(tiles):
        k0, k1 = t * PREFIX_TILE, min((t + 1) * PREFIX_TILE, d)
        for l, bits in enumerate(PREFIX_LEVELS):
            zt = decode(codes[l][k0:k1], key[k0:k1], eps, bits)
            level[t] = l
            if np.array_equal(prefix_checksums(zt)[0], checks[t]):
                confirmed[t] = True
                break
        z[k0:k1] = zt
    return z, level, confirmed


def pair_scale(m, bits):
    """Lattice scale for a pair at max-norm distance m: the smallest power of two that is
    >= m / (2^(b-1) - 3) (and >= 2^-100), so the pair sits inside the decoding radius
    (2^(b-1) - 5/2) eps -- the case of Corollary 2.1's proof where the writer knows the distance."""
    q = max(F32(m), F32(2.0 ** -100)) / F32((1 << (bits - 1)) - 3)
    f, k = np.frexp(F32(q))                    # q = f 2^k, f in [1/2, 1)
    return float(np.ldexp(F32(1.0), int(k) - 1 if f == 0.5 else int(k)))
