"""Stochastic gradients g~_i of the three synthetic node objectives, float64.

The paper only requires E[g~_i(x)] = grad f_i(x) with bounded variance
(Section 2, "Stochastic Optimization"); the objectives themselves are the
synthetic stand-ins of this build's workloads.  Test infrastructure only.
"""
import numpy as np

from . import rng


class DiagQuadratic:
    """f_i(x) = 1/2 sum_k a_ik (x_k - c_ik)^2 ; g~ = a (x - c) + sigma N(0, I).

    a, c hold the columns [k0, k1) of the n x d data."""

    def __init__(self, a, c, sigma, k0=0):
        self.a = np.asarray(a, dtype=np.float64)
        self.c = np.asarray(c, dtype=np.float64)
        self.sigma = float(np.float32(sigma))
        self.k0 = k0

    def gradient(self, node, w, seed, event, q):
        k1 = self.k0 + w.size
        noise = rng.noise_normals(seed, node, event, q, self.k0, k1) if self.sigma != 0.0 else 0.0
        return self.a[node] * (w - self.c[node]) + self.sigma * noise


class LeastSquares:
    """f_i(x) = 1/2 |A_i x - b_i|^2 over m rows; the stochastic gradient uses
    `batch` rows drawn uniformly with replacement and is scaled by m/batch so
    that its expectation is A_i^T (A_i x - b_i)."""

    def __init__(self, A, b, batch):
        self.A = np.asarray(A, dtype=np.float64)      # (n, m, d)
        self.b = np.asarray(b, dtype=np.float64)      # (n, m)
        self.m = self.A.shape[1]
        self.batch = int(batch)
        assert self.batch % 4 == 0

    def batch_rows(self, node, seed, event, q):
        words = rng.stream(seed, rng.TAG_BATCH, q, node, event, np.arange(self.batch // 4))
        words = np.stack(words, axis=1).reshape(-1)           # draw s = word s%4 of call s//4
        return rng.scaled_index(words, self.m).astype(np.int64)

    def gradient(self, node, w, seed, event, q):
        rows = self.batch_rows(node, seed, event, q)
        Ab = self.A[node][rows]
        resid = Ab @ w - self.b[node][rows]
        return (self.m / self.batch) * (Ab.T @ resid)


class MixtureMLP:
    """Two-layer perceptron in -> hid -> out with ReLU and softmax cross-entropy
    (mean over the batch) on a synthetic Gaussian mixture: class y has mean
    class_means[y], features are mean + data_sigma N(0, I), and node i draws
    labels from its own law given as a float32 CDF row label_cdf[i].

    Flat parameter layout: W1 (hid x in, row-major), b1 (hid), W2 (out x hid), b2 (out)."""

    TAG_LABEL = 8

    def __init__(self, n_in, n_hid, n_out, class_means, label_cdf, data_sigma, batch):
        self.n_in, self.n_hid, self.n_out = n_in, n_hid, n_out
        self.means = np.asarray(class_means, dtype=np.float32)     # (out, in)
        self.cdf = np.asarray(label_cdf, dtype=np.float32)         # (n, out)
        self.data_sigma = float(np.float32(data_sigma))
        self.batch = int(batch)
        assert self.batch % 4 == 0 and n_in % 4 == 0
        self.d = n_hid * n_in + n_hid + n_out * n_hid + n_out

    def split(self, w):
        i, h, o = self.n_in, self.n_hid, self.n_out
        p = 0
        W1 = w[p:p + h * i].reshape(h, i); p += h * i
        b1 = w[p:p + h]; p += h
        W2 = w[p:p + o * h].reshape(o, h); p += o * h
        b2 = w[p:p + o]
        return W1, b1, W2, b2

    def batch_data(self, node, seed, event, q):
        words = rng.stream(seed, self.TAG_LABEL, q, node, event, np.arange(self.batch // 4))
        words = np.stack(words, axis=1).reshape(-1)
        u = (words >> np.uint32(8)).astype(np.float32) * np.float32(2.0 ** -24)   # exact in float32
        y = (self.cdf[node][None, :] <= u[:, None]).sum(axis=1)                   # inverse CDF
        y = np.minimum(y, self.n_out - 1)
        z = rng.normals(seed, node, event, q, 0, self.batch * self.n_in, tag=rng.TAG_DATA)
        x = self.means[y].astype(np.float64) + self.data_sigma * z.reshape(self.batch, self.n_in)
        return x, y

    def loss_and_gradient(self, w, x, y):
        W1, b1, W2, b2 = self.split(w)
        B = x.shape[0]
        pre = x @ W1.T + b1
        hid = np.maximum(pre, 0.0)
        logits = hid @ W2.T + b2
        logits = logits - logits.max(axis=1, keepdims=True)
        logp = logits - np.log(np.exp(logits).sum(axis=1, keepdims=True))
        loss = -logp[np.arange(B), y].mean()
        dlogits = np.exp(logp)
        dlogits[np.arange(B), y] -= 1.0
        dlogits /= B
        dW2 = dlogits.T @ hid
        db2 = dlogits.sum(axis=0)
        dpre = (dlogits @ W2) * (pre > 0.0)
        dW1 = dpre.T @ x
        db1 = dpre.sum(axis=0)
        return loss, np.concatenate([dW1.reshape(-1), db1, dW2.reshape(-1), db2])

    def gradient(self, node, w, seed, event, q):
        x, y = self.batch_data(node, seed, event, q)
        return self.loss_and_gradient(w, x, y)[1]
