"""Random draws of the swarm simulation, as named Philox streams.

Every random number the method uses is a pure function of
(seed, stream tag, local-step index q, node or edge id, event id, index), so
any column window of a round can be evaluated on its own.  The paper needs
unbiased rounding (Corollary 2.1 item 1), a uniformly random initiator and a
uniformly random neighbour (Algorithm 1, sampling lines) and fresh gradient
samples at every local step (appendix, definition of the local steps); which
generator provides them is this build's choice.  Test infrastructure only.

Counter words:  c0 = index (low 32 bits)
                c1 = tag << 24 | q << 16 | index >> 32   (16 high index bits)
                c2 = node id or edge id
                c3 = event id (gossip round r, or interaction number t)
Key words:      (seed & 0xffffffff, seed >> 32)
"""
import numpy as np

from .philox import philox4x32_10

TAG_SR = 1      # stochastic rounding, index = coordinate // 8
TAG_NOISE = 2   # gradient noise, index = coordinate // 8 (see noise_normals)
TAG_MATCH = 3   # edge priorities of the round's matching, c2 = edge id
TAG_PICK = 4    # sequential model: initiator and responder
TAG_BATCH = 5   # least squares: minibatch rows, index = draw // 4
TAG_STALE = 6   # staleness of a node's read of its partner
TAG_DATA = 7    # MLP: features of the synthetic mixture (labels use tag 8)
TAG_STEPS = 9   # geometric number of local steps: Bernoulli trials, index = trial // 4


def seed_key(seed):
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    return (seed & 0xFFFFFFFF, seed >> 32)


def stream(seed, tag, q, ident, event, index):
    """Four uint32 words per entry of `index` (array of non-negative ints)."""
    index = np.asarray(index, dtype=np.uint64)
    c0 = index & np.uint64(0xFFFFFFFF)
    c1 = (np.uint64((tag << 24) | ((q & 0xFF) << 16))
          | ((index >> np.uint64(32)) & np.uint64(0xFFFF)))
    return philox4x32_10(seed_key(seed), c0, c1, ident, int(event) & 0xFFFFFFFF)


def sr_halves(seed, node, event, k0, k1):
    """16-bit random integers for coordinates k0..k1-1 (k0, k1 multiples of 8).

    One Philox call serves 8 consecutive coordinates: coordinate 8g+m takes
    word m//2, low half when m is even, high half when m is odd."""
    assert k0 % 8 == 0 and k1 % 8 == 0
    g = np.arange(k0 // 8, k1 // 8, dtype=np.uint64)
    w = np.stack(stream(seed, TAG_SR, 0, node, event, g), axis=1)   # (groups, 4)
    lo = w & np.uint32(0xFFFF)
    hi = w >> np.uint32(16)
    halves = np.stack([lo, hi], axis=2)                             # (groups, 4, 2)
    return halves.reshape(-1).astype(np.uint32)


def normals(seed, node, event, q, k0, k1, tag=TAG_DATA):
    """Standard normal draws for coordinates k0..k1-1 (multiples of 4), float64.

    One Philox call serves 4 consecutive coordinates through two Box-Muller
    transforms: (w0, w1) -> coordinates 4g, 4g+1 and (w2, w3) -> 4g+2, 4g+3,
    with u1 = ((w >> 8) + 1) 2^-24 in (0, 1] and u2 = (w >> 8) 2^-24 in [0, 1);
    the pair is (r cos 2 pi u2, r sin 2 pi u2), r = sqrt(-2 ln u1)."""
    assert k0 % 4 == 0 and k1 % 4 == 0
    g = np.arange(k0 // 4, k1 // 4, dtype=np.uint64)
    w0, w1, w2, w3 = stream(seed, tag, q, node, event, g)
    out = np.empty((g.size, 4), dtype=np.float64)
    for col, (wa, wb) in enumerate(((w0, w1), (w2, w3))):
        u1 = ((wa >> np.uint32(8)).astype(np.float64) + 1.0) * 2.0 ** -24
        u2 = (wb >> np.uint32(8)).astype(np.float64) * 2.0 ** -24
        r = np.sqrt(-2.0 * np.log(u1))
        out[:, 2 * col] = r * np.cos(2.0 * np.pi * u2)
        out[:, 2 * col + 1] = r * np.sin(2.0 * np.pi * u2)
    return out.reshape(-1)


def noise_normals(seed, node, event, q, k0, k1):
    """Gradient-noise draws for coordinates k0..k1-1 (multiples of 8), float64.

    One Philox call (stream TAG_NOISE, index = coordinate // 8) serves 8
    consecutive coordinates: word p of the call gives the Box-Muller pair of
    coordinates 8g+2p and 8g+2p+1 from its two 16-bit halves,
        u1 = (low half + 1/2) 2^-16 in (0, 1),   u2 = high half * 2^-16 in [0, 1),
        (r cos 2 pi u2, r sin 2 pi u2),  r = sqrt(-2 ln u1).
    Sixteen-bit uniforms bound |z| by sqrt(34 ln 2) = 4.855 and halve the
    generator work per draw compared with `normals`; for simulated gradient
    noise the discretisation is far below what SGD can see."""
    assert k0 % 8 == 0 and k1 % 8 == 0
    g = np.arange(k0 // 8, k1 // 8, dtype=np.uint64)
    words = stream(seed, TAG_NOISE, q, node, event, g)
    out = np.empty((g.size, 8), dtype=np.float64)
    for p, w in enumerate(words):
        u1 = ((w & np.uint32(0xFFFF)).astype(np.float64) + 0.5) * 2.0 ** -16
        u2 = (w >> np.uint32(16)).astype(np.float64) * 2.0 ** -16
        r = np.sqrt(-2.0 * np.log(u1))
        out[:, 2 * p] = r * np.cos(2.0 * np.pi * u2)
        out[:, 2 * p + 1] = r * np.sin(2.0 * np.pi * u2)
    return out.reshape(-1)


def scaled_index(word, m):
    """floor(u * m) for u = word / 2^32, computed as (word * m) >> 32."""
    return (np.asarray(word, dtype=np.uint64) * np.uint64(m)) >> np.uint64(32)
