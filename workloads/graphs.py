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
    """Pairing model with rejection until the graph is simple and connected."""
    assert (n * degree) % 2 == 0 and degree < n
    gen = np.random.Generator(np.random.PCG64(seed))
    while True:
        stubs = np.repeat(np.arange(n), degree)
        gen.shuffle(stubs)
        pairs = stubs.reshape(-1, 2)
        if (pairs[:, 0] == pairs[:, 1]).any():
            continue
        und = {(min(u, v), max(u, v)) for u, v in pairs.tolist()}
        if len(und) != len(pairs):
            continue
        edges = np.array(sorted(und), dtype=np.uint32)
        if _connected(n, edges):
            return edges


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
