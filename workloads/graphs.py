"""Communication graphs G as undirected edge lists (u < v), uint32 (E, 2)."""
import numpy as np


def complete_graph(n):
    return np.array([(u, v) for u in range(n) for v in range(u + 1, n)], dtype=np.uint32)


def torus_graph(rows, cols):
    """rows x cols torus: (r, c) ~ (r+-1, c), (r, c+-1), indices wrap."""
    edges = set()
    for r in range(rows):
        for c in range(cols):
            u = r * cols + c
            for v in (((r + 1) % rows) * cols + c, r * cols + (c + 1) % cols):
                if u != v:
                    edges.add((min(u, v), max(u, v)))
    return np.array(sorted(edges), dtype=np.uint32)


def _connected(n, edges):
    parent = list(range(n))

    def find(x):
        while parent[x] != x:
            parent[x] = parent[parent[x]]
            x = parent[x]
        return x
    for u, v in edges:
        parent[find(int(u))] = find(int(v))
    return len({find(x) for x in range(n)}) == 1


def random_regular_graph(n, degree, seed):
    """Random simple connected `degree`-regular graph: stubs are paired at random, a pair
    that would make a loop or a repeated edge goes back into the pool, and the attempt
    restarts when only unusable stubs remain."""
    assert (n * degree) % 2 == 0 and degree < n
    gen = np.random.Generator(np.random.PCG64(seed))
    while True:
        edges = set()
        stubs = np.repeat(np.arange(n), degree)
        stuck = False
        while stubs.size and not stuck:
            gen.shuffle(stubs)
            left = []
            for u, v in stubs.reshape(-1, 2).tolist():
                key = (min(u, v), max(u, v))
                if u != v and key not in edges:
                    edges.add(key)
                else:
                    left += [u, v]
            stuck = len(left) == stubs.size and not any(
                u != v and (min(u, v), max(u, v)) not in edges for u in set(left) for v in set(left))
            stubs = np.array(left, dtype=np.int64)
        if stuck:
            continue
        arr = np.array(sorted(edges), dtype=np.uint32)
        if _connected(n, arr):
            return arr


def adjacency(n, edges):
    nb = [[] for _ in range(n)]
    for u, v in np.asarray(edges).tolist():
        nb[u].append(v)
        nb[v].append(u)
    return [sorted(x) for x in nb]


def laplacian_lambda2(n, edges):
    """Second-smallest Laplacian eigenvalue (the paper's spectral gap)."""
    L = np.zeros((n, n))
    for u, v in np.asarray(edges).tolist():
        L[u, u] += 1
        L[v, v] += 1
        L[u, v] -= 1
        L[v, u] -= 1
    return float(np.sort(np.linalg.eigvalsh(L))[1])
