"""One swarm interaction, step by step (Algorithm 1 and Section 3 of the paper).

Test infrastructure only.  State (columns [k0, k1) of each):
  X     current / communicated model of every node  ("current model" register)
  W     live copy carrying the local steps that have been computed but are only
        applied after the averaging (Section 3, description of an interaction)
  Xhat  model at the node's last initiation (sequential model only)
  ring  S+1 slots of packed codes: slot r mod (S+1) holds Enc(X_r) of every node
All node models start equal (Algorithm 1, initial models), zero by default.
"""
import numpy as np

from . import quantizer as qz
from . import rng


class SwarmOracle:
    def __init__(self, n, d, edges, bits, eps, H, lr, stale_max=0, seed=0, x0=None,
                 k0=0, k1=None, state_dtype=np.float32, apply_mode="deferred", steps_law="constant", scale_policy="fixed",
                 codec="fixed"):
        self.n, self.d = int(n), int(d)
        self.k0 = int(k0)
        self.k1 = self.d if k1 is None else int(k1)
        assert self.k0 % 8 == 0 and self.k1 % 8 == 0 and self.d % 8 == 0
        self.edges = np.asarray(edges, dtype=np.int64).reshape(-1, 2)
        self.bits, self.eps = int(bits), float(np.float32(eps))
        self.H, self.lr = int(H), float(np.float32(lr))
        self.S, self.seed = int(stale_max), int(seed)
        assert self.bits in (0,) + qz.SUPPORTED_BITS and (self.bits > 0 or self.S == 0)
        # "deferred": the paper's rule (steps computed, averaged model adopted, steps added on top);
        # "inplace": the steps update the exchanged model itself before the averaging.
        assert apply_mode in ("deferred", "inplace")
        self.apply_mode = apply_mode
        # "constant": H steps (the paper's experiments); "geometric": H_i ~ geometric of mean H, the
        # paper's stand-in for activation by Poisson clocks (Section 3, "Sequential model").
        assert steps_law in ("constant", "geometric") and (steps_law == "constant" or self.H >= 1)
        self.steps_law = steps_law
        # "fixed": one eps for every exchange; "pair_linf": each matched pair uses the smallest power of
        # two that puts it inside the decoding radius (the writer knows its distance to the key).
        # "global_linf": one scale per round, set from the largest disagreement the previous round's
        # pairs saw (the writer does not know who will read its code, or when; appendix, second case
        # of the quantization discussion -- with a fixed number of bits the scale has to follow).
        assert scale_policy in ("fixed", "pair_linf", "global_linf")
        assert scale_policy != "pair_linf" or (self.bits >= 4 and self.S == 0)
        if scale_policy == "global_linf":
            # at least 8 bits: the max-norm rule makes a 4-bit lattice coarser than the typical
            # disagreement, and the rounding noise then feeds the disagreement it is sized from
            assert self.bits >= 8 and self.k0 == 0 and self.k1 == self.d
            assert np.frexp(self.eps)[0] == 0.5, "the starting scale must be a power of two"
        self.scale_policy = scale_policy
        # "fixed": every register holds and every reader fetches b bits per coordinate.  "prefix": the
        # register holds a 16-bit code in planes plus tile checksums and a reader fetches the shortest
        # prefix whose decode is confirmed (proof of Corollary 2.1, second case; its item 3).
        assert codec in ("fixed", "prefix")
        if codec == "prefix":
            assert self.bits == 16 and scale_policy == "fixed" and self.k0 % qz.PREFIX_TILE == 0
        self.codec = codec
        self.prefix_levels = np.zeros(len(qz.PREFIX_LEVELS), dtype=np.int64)   # tiles decoded at each level
        self.prefix_unconfirmed = 0                                             # tiles no level confirmed
        self.eps_ring = [np.float32(self.eps)] * (self.S + 1)   # scale of the codes in each ring slot
        self.eps_cur = np.float32(self.eps)                      # scale of the coming round
        self.max_disagreement = np.float32(0.0)                  # of the last round with pairs
        self.dtype = state_dtype
        dw = self.k1 - self.k0
        self.X = np.zeros((self.n, dw), dtype=state_dtype)
        if x0 is not None:
            self.X[:] = np.asarray(x0)[self.k0:self.k1]
        self.W = self.X.copy()
        self.Xhat = self.X.copy()
        self.pending = np.zeros(self.n, dtype=bool)      # W_i carries unapplied steps
        self.ring = [[None] * self.n for _ in range(self.S + 1)]
        self.round = 0            # gossip rounds done
        self.interactions = 0     # pairwise interactions done (the paper's unit of time)
        self.bits_communicated = 0
        self.decode_failures = 0
        self.range_clamped = False
        self.objective = None
        self.adj = [sorted(set(self.edges[self.edges[:, 0] == i, 1]) |
                           set(self.edges[self.edges[:, 1] == i, 0])) for i in range(self.n)]

    # ---- local steps: h~_i^q = g~_i(base - eta sum_{s<q} h~_i^s), fresh sample each q ----
    def steps_of(self, node, event):
        """H, or 1 + the number of failed Bernoulli(p) trials before the first success, p =
        floor(2^32 / H) / 2^32, one trial per 32-bit word of the node's STEPS stream, capped at 255.
        Mean H and second moment 2H^2 - H (appendix, properties of the local steps)."""
        if self.steps_law == "constant" or self.H == 1:
            return self.H
        threshold = (1 << 32) // self.H
        k = 1
        for call in range(64):
            for word in rng.stream(self.seed, rng.TAG_STEPS, 0, node, event, np.array([call])):
                if int(word[0]) < threshold or k >= 255:
                    return k
                k += 1
        return k

    def sample_steps(self):
        return np.array([self.steps_of(i, self.round) for i in range(self.n)], dtype=np.int64)

    def local_steps(self, nodes=None, sequential=False):
        nodes = range(self.n) if nodes is None else nodes
        event = self.interactions if sequential else self.round
        for i in nodes:
            base = self.Xhat[i] if sequential else self.X[i]
            w = base.astype(np.float64)
            for q in range(self.steps_of(i, event)):
                w = w - self.lr * self.objective.gradient(i, w, self.seed, event, q)
            if self.apply_mode == "inplace":
                assert not sequential
                self.X[i] = w
                self.W[i] = self.X[i]
            else:
                self.W[i] = w
                self.pending[i] = True

    def _delta(self, i, base):
        """Pending update -eta h~_i = W_i - base (zero if no local steps are pending)."""
        if not self.pending[i]:
            return 0.0
        return self.W[i].astype(np.float64) - base.astype(np.float64)

    # ---- pair selection -----------------------------------------------------------------
    def sample_pair(self):
        """Initiator uniform over nodes, responder uniform over its neighbours."""
        w = rng.stream(self.seed, rng.TAG_PICK, 0, 0, self.interactions, np.array([0]))
        i = int(rng.scaled_index(w[0][0], self.n))
        nb = self.adj[i]
        return i, int(nb[int(rng.scaled_index(w[1][0], len(nb)))])

    def edge_priorities(self, r=None):
        r = self.round if r is None else r
        e = np.arange(len(self.edges), dtype=np.uint64)
        w0 = rng.stream(self.seed, rng.TAG_MATCH, 0, e, r, np.zeros_like(e))[0]
        return (w0.astype(np.uint64) << np.uint64(32)) | e

    def sample_matching(self):
        """Random maximal matching: scan edges by increasing random priority and
        keep an edge when both endpoints are still free.  Pairs are listed by
        increasing edge index, each in the orientation of the edge list."""
        prio = self.edge_priorities()
        free = np.ones(self.n, dtype=bool)
        chosen = []
        for e in np.argsort(prio):
            u, v = self.edges[e]
            if free[u] and free[v]:
                free[u] = free[v] = False
                chosen.append(int(e))
        return self.edges[sorted(chosen)].copy()

    def sample_stale(self):
        """Per node: how many rounds old the partner's code it reads is,
        uniform on {0..S}, limited to the rounds that exist."""
        i = np.arange(self.n, dtype=np.uint64)
        w0 = rng.stream(self.seed, rng.TAG_STALE, 0, i, self.round, np.zeros_like(i))[0]
        return np.minimum(rng.scaled_index(w0, self.S + 1), self.round).astype(np.int64)

    # ---- quantized exchange -------------------------------------------------------------
    def _lattice_point(self, i, event, eps=None):
        eps = self.eps if eps is None else eps
        r16 = rng.sr_halves(self.seed, i, event, self.k0, self.k1)
        z = qz.stochastic_round(self.X[i], eps, r16)
        self.range_clamped |= bool(qz.lattice_coordinate(self.X[i], eps)[1].any())
        return z

    def _read(self, reader, sender, slot, z_true=None, eps=None):
        """reader decodes the sender's published code against its own model."""
        eps = self.eps if eps is None else eps
        self.range_clamped |= bool(qz.lattice_coordinate(self.X[reader], eps)[1].any())
        if self.codec == "prefix":
            z, level, confirmed = qz.prefix_read(self.ring[slot][sender], self.X[reader], eps)
            dw = self.k1 - self.k0
            widths = np.minimum(qz.PREFIX_TILE, dw - np.arange(level.size) * qz.PREFIX_TILE)   # coordinates per tile
            self.bits_communicated += int((np.array(qz.PREFIX_LEVELS)[level] * widths).sum()) + 64 * level.size
            self.prefix_levels += np.bincount(level, minlength=len(qz.PREFIX_LEVELS))
            self.prefix_unconfirmed += int((~confirmed).sum())
            if z_true is not None:
                self.decode_failures += int((z != z_true).sum())
            return z
        c = qz.unpack(self.ring[slot][sender], self.bits, self.k1 - self.k0)
        z = qz.decode(c, self.X[reader], eps, self.bits)
        self.bits_communicated += self.d * self.bits
        if z_true is not None:
            self.decode_failures += int((z != z_true).sum())
        return z

    def gossip_round(self, pairs, stale=None):
        """Round model: the matched pairs interact at once, every matched node
        acting as the initiator of its own update:
            X_i' = (Q(X_i) + Q(X_j)) / 2 - eta h~_i ,  likewise for j,
        where Q(X_j) is decoded by i from the code j published `stale[i]` rounds
        ago, with i's own model as key.  Unmatched nodes apply their own steps."""
        pairs = np.asarray(pairs, dtype=np.int64).reshape(-1, 2)
        r, dw = self.round, self.k1 - self.k0
        stale = np.zeros(self.n, dtype=np.int64) if stale is None else np.asarray(stale)
        new = {}
        matched = np.zeros(self.n, dtype=bool)
        if self.bits == 0:                                   # Q = identity (Corollary 4.2)
            for i, j in pairs:
                avg = 0.5 * (self.X[i].astype(np.float64) + self.X[j].astype(np.float64))
                new[i] = avg + self._delta(i, self.X[i])
                new[j] = avg + self._delta(j, self.X[j])
                self.bits_communicated += 2 * self.d * 32
        elif self.scale_policy == "pair_linf":               # each pair at its own scale; full rows only
            assert self.k0 == 0 and self.k1 == self.d
            for i, j in pairs:
                m = np.abs(self.X[i].astype(np.float32) - self.X[j].astype(np.float32)).max()
                eps = qz.pair_scale(m, self.bits)
                zi, zj = self._lattice_point(i, r, eps), self._lattice_point(j, r, eps)
                self.ring[0][i] = qz.pack(qz.code(zi, self.bits), self.bits)
                self.ring[0][j] = qz.pack(qz.code(zj, self.bits), self.bits)
                zj_seen = self._read(i, j, 0, zj, eps)
                zi_seen = self._read(j, i, 0, zi, eps)
                new[i] = (zi + zj_seen) * (0.5 * eps) + self._delta(i, self.X[i])
                new[j] = (zj + zi_seen) * (0.5 * eps) + self._delta(j, self.X[j])
        elif self.scale_policy == "global_linf":
            self._gossip_round_global(pairs, stale, new)
        else:
            slot = r % (self.S + 1)
            z = {}
            for i in range(self.n):                          # everyone publishes Enc(X_r^i)
                z[i] = self._lattice_point(i, r)
                self.ring[slot][i] = (qz.prefix_register(z[i]) if self.codec == "prefix"
                                      else qz.pack(qz.code(z[i], self.bits), self.bits))
            for i, j in pairs:
                si, sj = min(int(stale[i]), r), min(int(stale[j]), r)
                assert 0 <= si <= self.S and 0 <= sj <= self.S
                zj_seen = self._read(i, j, (r - si) % (self.S + 1), z[j] if si == 0 else None)
                zi_seen = self._read(j, i, (r - sj) % (self.S + 1), z[i] if sj == 0 else None)
                new[i] = (z[i] + zj_seen) * (0.5 * self.eps) + self._delta(i, self.X[i])
                new[j] = (z[j] + zi_seen) * (0.5 * self.eps) + self._delta(j, self.X[j])
        for i, j in pairs:
            assert not matched[i] and not matched[j] and i != j
            matched[i] = matched[j] = True
        for u in range(self.n):
            if matched[u]:
                self.X[u] = new[u]
            elif self.pending[u]:
                self.X[u] = self.W[u]
        self.pending[:] = False
        self.round += 1
        self.interactions += len(pairs)

    def _gossip_round_global(self, pairs, stale, new):
        """Round with one lattice scale per round.  Every node rounds to eps_r Z and publishes the
        code; a reader decodes a code of age s at the scale eps_(r-s) it was written with, against
        its own model, and averages the two lattice points each at its own scale:
            X_i' = (eps_r z_i + eps_(r-s) z_j') / 2 + delta_i .
        The round also records m = max over matched nodes and coordinates of
        |X_i - eps_(r-s) z_j'| (float32): how far the decoded partner is from the key.  The next round uses
            eps_(r+1) = max(pair_scale(2 m), eps_r / 2)        (eps_r if nobody was matched),
        i.e. the smallest power of two that puts twice the disagreement just seen inside the
        decoding radius, shrinking by at most a factor two per round.  A wrapped decode shows up
        as a disagreement near the radius, so a scale that is too small grows fourfold per round."""
        r = self.round
        eps_r = np.float32(self.eps_cur)
        slot = r % (self.S + 1)
        self.eps_ring[slot] = eps_r
        z = {}
        for i in range(self.n):
            z[i] = self._lattice_point(i, r, float(eps_r))
            self.ring[slot][i] = qz.pack(qz.code(z[i], self.bits), self.bits)
        m = np.float32(0.0)
        for i, j in pairs:
            for me, other in ((i, j), (j, i)):
                age = min(int(stale[me]), r)
                assert 0 <= age <= self.S
                src = (r - age) % (self.S + 1)
                eps_old = np.float32(self.eps_ring[src])
                z_seen = self._read(me, other, src, z[other] if age == 0 else None, float(eps_old))
                mine = z[me].astype(np.float32) * eps_r                 # float32 throughout: m decides eps
                theirs = z_seen.astype(np.float32) * eps_old
                m = max(m, np.abs(self.X[me].astype(np.float32) - theirs).max())
                new[me] = (mine.astype(np.float64) + theirs.astype(np.float64)) * 0.5 + self._delta(me, self.X[me])
        if len(pairs):
            self.max_disagreement = np.float32(m)
            self.eps_cur = np.float32(max(qz.pair_scale(np.float32(2.0) * m, self.bits), eps_r * np.float32(0.5)))

    def interact(self, i, j):
        """One step of Algorithm 1: initiator i, responder j.
            X_i' = (Q(X_i) + Q(X_j)) / 2 - eta h~_i(Xhat_i) ,  X_j' = (Q(X_i) + Q(X_j)) / 2,
        i's snapshot becomes X_i'; j's snapshot and pending steps are untouched."""
        assert self.S == 0 and j in self.adj[i] and self.scale_policy == "fixed"
        t = self.interactions
        if self.H > 0 and self.objective is not None:
            self.local_steps([i], sequential=True)
        delta = self._delta(i, self.Xhat[i])
        if self.bits == 0:
            avg = 0.5 * (self.X[i].astype(np.float64) + self.X[j].astype(np.float64))
            self.bits_communicated += 2 * self.d * 32
        else:
            zi, zj = self._lattice_point(i, t), self._lattice_point(j, t)
            if self.codec == "prefix":
                self.ring[0][i], self.ring[0][j] = qz.prefix_register(zi), qz.prefix_register(zj)
            else:
                self.ring[0][i] = qz.pack(qz.code(zi, self.bits), self.bits)
                self.ring[0][j] = qz.pack(qz.code(zj, self.bits), self.bits)
            before = self.bits_communicated
            zj_seen = self._read(i, j, 0, zj)                 # i reads j's register ...
            # ... and writes the average back: b bits, or with multi-resolution registers as many as it
            # read (it knows the distance to j's key now: first case of the proof of Corollary 2.1)
            self.bits_communicated += self.bits_communicated - before
            avg = (zi + zj_seen) * (0.5 * self.eps)
        self.X[i] = avg + delta
        self.X[j] = avg
        self.Xhat[i] = self.X[i]
        self.pending[i] = False
        self.interactions += 1

    def step_sequential(self):
        i, j = self.sample_pair()
        self.interact(i, j)
        return i, j

    # ---- potentials ---------------------------------------------------------------------
    def mean(self):
        return self.X.astype(np.float64).mean(axis=0)

    def potential(self):
        """Gamma = sum_i |X_i - mu|^2."""
        x = self.X.astype(np.float64)
        return float(((x - x.mean(axis=0)) ** 2).sum())

    def potential_hat(self):
        """Gamma-hat = sum_i |Xhat_i - mu|^2 (appendix, auxiliary potentials)."""
        mu = self.mean()
        return float(((self.Xhat.astype(np.float64) - mu) ** 2).sum())
