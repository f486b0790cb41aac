"""Seeded synthetic inputs: topologies and state/gradient generators.

Holds none of the method's arithmetic: it only makes the inputs (mixing
matrices as CSR, initial iterates, gradient streams) that are handed, as the
same numpy arrays, to the HIP library and to the CPU oracle.  Shapes follow
the paper's workloads (Section 5: ring / torus with n in {4,...,64}, flat
parameter vectors of about 0.27 M and 28 M entries); the values are random
stand-ins because the datasets and models are not available.
"""
import numpy as np


def ring_csr(n, wdtype=np.float32):
    """Ring of n nodes, uniform weights 1/3 on self and both neighbours
    (Section 5, Table of topologies; w_ij = 1/max(deg) with the self-loop
    counted).  n = 1 and n = 2 degenerate to the complete graph."""
    rows = []
    for i in range(n):
        nb = sorted({(i - 1) % n, i, (i + 1) % n})
        rows.append(nb)
    return _uniform_rows(rows, wdtype)


def torus_csr(rows_, cols_, wdtype=np.float32):
    """2-D torus rows_ x cols_, uniform weights 1/5 (self + 4 neighbours)."""
    n = rows_ * cols_
    rows = []
    for i in range(n):
        r, c = divmod(i, cols_)
        nb = {i, ((r - 1) % rows_) * cols_ + c, ((r + 1) % rows_) * cols_ + c,
              r * cols_ + (c - 1) % cols_, r * cols_ + (c + 1) % cols_}
        rows.append(sorted(nb))
    return _uniform_rows(rows, wdtype)


def complete_csr(n, wdtype=np.float32):
    return _uniform_rows([list(range(n)) for _ in range(n)], wdtype)


def _uniform_rows(rows, wdtype=np.float32):
    """CSR (row_ptr, col_idx, w) with w_ij = 1/len(row) rounded to wdtype.  Only valid
    (symmetric, doubly stochastic) when all rows have the same length, which
    holds for the ring, the torus and the complete graph."""
    n = len(rows)
    deg = {len(r) for r in rows}
    assert len(deg) == 1, "uniform weights need a regular graph"
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    col, w = [], []
    for i, r in enumerate(rows):
        row_ptr[i + 1] = row_ptr[i] + len(r)
        col.extend(r)
        w.extend([wdtype(1.0) / wdtype(len(r))] * len(r))
    return row_ptr, np.asarray(col, dtype=np.int32), np.asarray(w, dtype=wdtype)


def metropolis_csr(adj):
    """Irregular graph given as a symmetric boolean adjacency (no self loops):
    w_ij = 1/(1 + max(deg i, deg j)) on edges, self weight = the remainder
    (Section 3: weights from local node degrees)."""
    adj = np.asarray(adj, dtype=bool)
    n = adj.shape[0]
    deg = adj.sum(1)
    W = np.zeros((n, n), dtype=np.float64)
    for i in range(n):
        for j in range(n):
            if i != j and adj[i, j]:
                W[i, j] = 1.0 / (1.0 + max(deg[i], deg[j]))
    for i in range(n):
        W[i, i] = 1.0 - W[i].sum()
    return dense_to_csr(W)


def irregular_graph(n, max_degree, seed):
    """Connected irregular graph standing in for the paper's 32-node social network
    (Section 5: maximum degree 14): a ring for connectivity plus random chords, with one
    hub raised to max_degree.  Returns a symmetric boolean adjacency without self loops."""
    rng = np.random.default_rng(seed)
    adj = np.zeros((n, n), dtype=bool)
    for i in range(n):
        adj[i, (i + 1) % n] = adj[(i + 1) % n, i] = True
    for _ in range(2 * n):
        a, b = rng.integers(0, n, size=2)
        if a != b and adj[a].sum() < max_degree - 1 and adj[b].sum() < max_degree - 1:
            adj[a, b] = adj[b, a] = True
    hub = 0
    others = [j for j in rng.permutation(n) if j != hub]
    for j in others:
        if adj[hub].sum() >= max_degree:
            break
        if adj[j].sum() < max_degree:
            adj[hub, j] = adj[j, hub] = True
    return adj


def layer_table(lengths, fraction=0.01, pad=4):
    """(start, length, k) int64 arrays for layers laid end to end, every start rounded up
    to a multiple of pad; k[l] = max(1, floor(fraction * length[l])) (the paper's floor(a d)
    applied per layer, with at least one entry so that no layer is silent)."""
    lengths = np.asarray(lengths, dtype=np.int64)
    start = np.zeros_like(lengths)
    pos = 0
    for l, ln in enumerate(lengths):
        start[l] = pos
        pos = (pos + int(ln) + pad - 1) // pad * pad
    k = np.maximum(1, np.floor(fraction * lengths).astype(np.int64))
    return start, lengths.copy(), k


def layers_dim(layers):
    """Length of the flat vector that a layer table describes."""
    start, length, _ = layers
    return int(start[-1] + length[-1])


def resnet20_like_lengths():
    """Parameter counts, layer by layer, of a 20-layer CIFAR residual network with 16/32/64
    channels, batch-norm scale and shift after every convolution and 1x1 projection
    shortcuts (272,474 parameters in all: the 0.27 M model of Section 5).  Only the
    sizes matter here: they give the mix of many small and a few 36,864-entry layers that
    per-layer compression meets."""
    out = []

    def conv(cin, cout, ksz):
        out.extend([cin * cout * ksz * ksz, cout, cout])   # weights, bn scale, bn shift

    conv(3, 16, 3)
    for stage, (cin, cout) in enumerate(((16, 16), (16, 32), (32, 64))):
        for block in range(3):
            conv(cin if block == 0 else cout, cout, 3)
            conv(cout, cout, 3)
            if block == 0 and stage > 0:
                conv(cin, cout, 1)
    out.extend([64 * 10, 10])
    return np.asarray(out, dtype=np.int64)


def lstm_like_lengths(vocab=33278, hidden=650, layers=3):
    """Parameter tensors of a word-level language model in the style of Section 5's second
    model (three LSTM layers of hidden size 650 over a tied embedding): one embedding matrix
    of tens of millions of entries, 1.69 M-entry weight matrices, 2,600-entry biases.  Only the
    mix of sizes matters here (31.8 M entries in all; the paper's own count is 28.95 M)."""
    out = [vocab * hidden]
    for _ in range(layers):
        out.extend([4 * hidden * hidden, 4 * hidden * hidden, 4 * hidden, 4 * hidden])
    out.append(vocab)
    return np.asarray(out, dtype=np.int64)


def dense_to_csr(W):
    W = np.asarray(W)
    n = W.shape[0]
    row_ptr = np.zeros(n + 1, dtype=np.int32)
    col, w = [], []
    for i in range(n):
        nz = [j for j in range(n) if W[i, j] != 0 or j == i]
        row_ptr[i + 1] = row_ptr[i] + len(nz)
        col.extend(nz)
        w.extend(np.float32(W[i, j]) for j in nz)
    return row_ptr, np.asarray(col, dtype=np.int32), np.asarray(w, dtype=np.float32)


def csr_to_dense(row_ptr, col_idx, w, dtype=np.float64):
    n = len(row_ptr) - 1
    W = np.zeros((n, n), dtype=dtype)
    for i in range(n):
        for p in range(row_ptr[i], row_ptr[i + 1]):
            W[i, col_idx[p]] = w[p]
    return W


def normal_state(n, d, seed, std=1.0, shared=False, dtype=np.float32):
    """Initial iterates: iid N(0, std^2); shared=True gives every worker the
    same row (Algorithm 1 starts all nodes from one point)."""
    rng = np.random.default_rng(seed)
    if shared:
        row = rng.standard_normal(d) * std
        X = np.repeat(row[None, :], n, axis=0)
    else:
        X = rng.standard_normal((n, d)) * std
    return np.ascontiguousarray(X, dtype=dtype)


class GradientStream:
    """Synthetic non-IID gradients g_i^t = b_i + eps: a fixed per-worker bias
    b_i ~ N(0, bias_std^2) plus fresh noise eps ~ N(0, noise_std^2) per call."""

    def __init__(self, n, d, seed, noise_std=0.01, bias_std=0.001, dtype=np.float32):
        self.n, self.d, self.dtype = n, d, dtype
        self.rng = np.random.default_rng(seed)
        self.noise_std = noise_std
        self.bias = (self.rng.standard_normal((n, d)) * bias_std) if bias_std > 0 else 0.0

    def next(self):
        g = self.rng.standard_normal((self.n, self.d)) * self.noise_std + self.bias
        return np.ascontiguousarray(g, dtype=self.dtype)


class LogisticProblem:
    """Synthetic L2-regularised logistic regression split over n workers: per worker
    `samples` feature rows ~ N(0, 1) scaled to unit norm, labels +-1 from a planted w* with a
    fraction `flip` of them flipped.  gradient(X, t) draws a fresh minibatch per worker and
    step (seeded by (seed, t, worker)) and returns the stochastic gradients at the rows of X,
    the regulariser lam * x included.  This is the objective's arithmetic, an INPUT of the
    path under test (it plays the role of the model's backward pass)."""

    def __init__(self, n, d, samples=1000, seed=0, flip=0.05, lam=1e-4, batch=32):
        rng = np.random.default_rng(seed)
        self.n, self.d, self.samples, self.seed, self.lam, self.batch = n, d, samples, seed, lam, batch
        A = rng.standard_normal((n, samples, d))
        A /= np.linalg.norm(A, axis=2, keepdims=True)
        w_star = rng.standard_normal(d)
        y = np.sign(A @ w_star)
        y[y == 0] = 1.0
        y[rng.random((n, samples)) < flip] *= -1.0
        self.A, self.y = A, y

    def gradient(self, X, t):
        X = np.asarray(X, dtype=np.float64)
        G = np.empty_like(X)
        for i in range(self.n):
            idx = np.random.default_rng([self.seed, t, i]).integers(0, self.samples, size=self.batch)
            a, y = self.A[i, idx], self.y[i, idx]
            margin = y * (a @ X[i])
            coef = -y / (1.0 + np.exp(margin))
            G[i] = (coef[:, None] * a).mean(0) + self.lam * X[i]
        return np.ascontiguousarray(G, dtype=np.float32)

    def loss(self, x):
        """Full objective at one point x (every worker's data)."""
        x = np.asarray(x, dtype=np.float64)
        margin = self.y * (self.A @ x)
        return float(np.logaddexp(0.0, -margin).mean() + 0.5 * self.lam * (x @ x))
