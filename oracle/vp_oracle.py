"""CPU oracle for the vocabulary layers of Vocabulary Parallelism (arXiv 2411.05288).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the HIP path is
checked against.  It is imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg, and by nothing else; it imports nothing from the
HIP package and shares no code with it.

Everything is NumPy in fp64 (the embedding backward also has an fp32 variant that
adds in token order, which is the order the definition implies).  Inputs arrive as
fp64 arrays holding the exact values of the stored fp32 / bf16 tensors.

Notation follows the paper: X (= H) is [N, h] with N = b*s token rows, W is [V, h]
(one row per vocabulary entry), Y = X W^T are the logits, m_i / sum_i the row maximum
and the row sum of exponentials, G the one-hot ground-truth matrix (G[i, g_i] = 1).
A shard r owns vocabulary rows [off_r, off_r + V/p).

Readings of points the paper leaves open (the paper writes no loss and no 1/N):
  * the loss is the mean over the N tokens of  -log softmax(Y_i)[g_i];  the gradients
    of section 4.2 are multiplied by ``grad_scale`` (1/N for the mean; 1 gives the
    paper's unscaled form);
  * in Algorithms 1 and 2 the factor applied to softmax' is the *rescaled* local sum
    over the global sum, sum'_i e^{m'_i - m_i} / sum_i  (the identity of section 4.3);
  * the two all-reduces of barrier C1 are a MAX (for m) and a SUM (for sum);
  * a shard that does not own g_i has an all-zero row i in its local G.

Pins (tests/test_oracle_pins.py): independence of p (p = 1 is textbook log-softmax
cross-entropy), a naive un-shifted evaluation, closed forms for W = 0 and H = 0,
the |Y| ~ 200 overflow case, vocabulary permutation invariance, rows of softmax
summing to one, column sums of dW vanishing, central finite differences for dH and
dW, Algorithm 2's input-gradient identity, dense one-hot products for the embedding.
The paper prints no worked numeric example for these layers, so no printed value
is available as a pin.
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------- #
# Output layer, unsharded definition (section 4.2)
# --------------------------------------------------------------------------- #
def logits(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Y = X W^T  (section 4.2, first equation)."""
    return X @ W.T


def row_stats(Y: np.ndarray):
    """m_i = max_k Y_ik and sum_i = sum_k exp(Y_ik - m_i)  (section 4.2)."""
    m = Y.max(axis=1)
    s = np.exp(Y - m[:, None]).sum(axis=1)
    return m, s


def softmax(Y: np.ndarray) -> np.ndarray:
    """Safe softmax of every token row (section 4.2, second equation)."""
    m, s = row_stats(Y)
    return np.exp(Y - m[:, None]) / s[:, None]


def one_hot(labels: np.ndarray, V: int, offset: int = 0) -> np.ndarray:
    """Ground-truth matrix G restricted to vocabulary rows [offset, offset+V):
    G[i, g_i - offset] = 1 when the range owns g_i, the row is zero otherwise."""
    N = labels.shape[0]
    G = np.zeros((N, V), dtype=np.float64)
    loc = labels - offset
    own = (loc >= 0) & (loc < V)
    G[np.nonzero(own)[0], loc[own]] = 1.0
    return G


def output_layer(X, W, labels, grad_scale=None):
    """Unsharded output layer: loss and the gradients of section 4.2.

    Returns dict with Y, m, sum, loss_rows [N], loss (mean), D = (softmax - G)*scale,
    dX = D W, dW = D^T X.
    """
    N = X.shape[0]
    V = W.shape[0]
    if grad_scale is None:
        grad_scale = 1.0 / N
    Y = logits(X, W)
    m, s = row_stats(Y)
    target = Y[np.arange(N), labels]
    loss_rows = m + np.log(s) - target
    P = np.exp(Y - m[:, None]) / s[:, None]
    D = (P - one_hot(labels, V)) * grad_scale
    return {
        "Y": Y, "m": m, "sum": s, "target": target,
        "loss_rows": loss_rows, "loss": loss_rows.mean(),
        "D": D, "dX": D @ W, "dW": D.T @ X,
    }


# --------------------------------------------------------------------------- #
# Algorithm 1 (two barriers), pass by pass
# --------------------------------------------------------------------------- #
def alg1_S(X, W_r, labels, offset):
    """Pass S on one shard: local logits, local max, local sum, softmax' (Algorithm 1).
    Also returns the in-shard target logit t' (0 when the shard does not own g_i)."""
    Y = X @ W_r.T
    m_loc = Y.max(axis=1)
    e = np.exp(Y - m_loc[:, None])
    sum_loc = e.sum(axis=1)
    softmax_loc = e / sum_loc[:, None]
    Vs = W_r.shape[0]
    loc = labels - offset
    own = (loc >= 0) & (loc < Vs)
    t_loc = np.zeros(X.shape[0], dtype=np.float64)
    t_loc[own] = Y[np.nonzero(own)[0], loc[own]]
    return {"Y": Y, "m_loc": m_loc, "sum_loc": sum_loc, "softmax_loc": softmax_loc, "t_loc": t_loc}


def alg1_C1(m_locs, sum_locs):
    """Barrier C1: m = AllReduce-MAX m'; sum' <- sum' e^{m' - m}; sum = AllReduce-SUM sum'.
    Inputs are [p, N]; returns m [N], the rescaled sum' [p, N] and sum [N]."""
    m_locs = np.asarray(m_locs)
    sum_locs = np.asarray(sum_locs)
    m = m_locs.max(axis=0)
    sum_resc = sum_locs * np.exp(m_locs - m[None, :])
    s = sum_resc.sum(axis=0)
    return m, sum_resc, s


def combine_stats(m_locs, sum_locs, t_locs):
    """C1 plus the loss: loss_i = m_i + ln sum_i - sum_r t'_{r,i}; mean over tokens."""
    m, _, s = alg1_C1(m_locs, sum_locs)
    t = np.asarray(t_locs).sum(axis=0)
    loss_rows = m + np.log(s) - t
    return {"m": m, "sum": s, "loss_rows": loss_rows, "loss": loss_rows.mean()}


def alg1_T(X, W_r, labels, offset, softmax_loc, sum_resc_r, s, grad_scale):
    """Pass T on one shard: softmax = softmax' * sum'/sum (rescaled sum'),
    dX' = (softmax - G) W_r, dW_r = (softmax - G)^T X."""
    sm = softmax_loc * (sum_resc_r / s)[:, None]
    D = (sm - one_hot(labels, W_r.shape[0], offset)) * grad_scale
    return {"softmax": sm, "D": D, "dX_part": D @ W_r, "dW": D.T @ X}


def output_layer_alg1(X, W_shards, labels, grad_scale=None):
    """Algorithm 1 end to end over p shards (C0 and C2 become a shared X and a sum)."""
    N = X.shape[0]
    if grad_scale is None:
        grad_scale = 1.0 / N
    offs = np.cumsum([0] + [w.shape[0] for w in W_shards])
    S = [alg1_S(X, W_r, labels, offs[r]) for r, W_r in enumerate(W_shards)]
    m, sum_resc, s = alg1_C1([q["m_loc"] for q in S], [q["sum_loc"] for q in S])
    T = [alg1_T(X, W_r, labels, offs[r], S[r]["softmax_loc"], sum_resc[r], s, grad_scale)
         for r, W_r in enumerate(W_shards)]
    dX = np.zeros_like(T[0]["dX_part"])
    for q in T:            # barrier C2: Reduce, ascending shard order
        dX = dX + q["dX_part"]
    stats = combine_stats([q["m_loc"] for q in S], [q["sum_loc"] for q in S], [q["t_loc"] for q in S])
    return {
        "m_loc": np.stack([q["m_loc"] for q in S]), "sum_loc": np.stack([q["sum_loc"] for q in S]),
        "t_loc": np.stack([q["t_loc"] for q in S]),
        "Y": [q["Y"] for q in S], "D": [q["D"] for q in T],
        "m": m, "sum": s, "loss_rows": stats["loss_rows"], "loss": stats["loss"],
        "softmax": [q["softmax"] for q in T],
        "dX": dX, "dW": [q["dW"] for q in T],
    }


# --------------------------------------------------------------------------- #
# Algorithm 2 (one barrier)
# --------------------------------------------------------------------------- #
def output_layer_alg2(X, W_shards, labels, grad_scale=None):
    """Algorithm 2: S also forms A = softmax'(Y) W_r and B = G W_r; inside C1
    dX = Reduce(A * sum'/sum - B) (section 4.4); T is only dW."""
    N = X.shape[0]
    if grad_scale is None:
        grad_scale = 1.0 / N
    offs = np.cumsum([0] + [w.shape[0] for w in W_shards])
    S, A, B = [], [], []
    for r, W_r in enumerate(W_shards):
        q = alg1_S(X, W_r, labels, offs[r])
        S.append(q)
        A.append(q["softmax_loc"] @ W_r)
        B.append(one_hot(labels, W_r.shape[0], offs[r]) @ W_r)
    m, sum_resc, s = alg1_C1([q["m_loc"] for q in S], [q["sum_loc"] for q in S])
    dX = np.zeros_like(A[0])
    for r in range(len(W_shards)):
        dX = dX + (A[r] * (sum_resc[r] / s)[:, None] - B[r]) * grad_scale
    dW = []
    for r, W_r in enumerate(W_shards):
        sm = S[r]["softmax_loc"] * (sum_resc[r] / s)[:, None]
        dW.append(((sm - one_hot(labels, W_r.shape[0], offs[r])) * grad_scale).T @ X)
    return {"m": m, "sum": s, "dX": dX, "dW": dW, "A": A, "B": B}


# --------------------------------------------------------------------------- #
# Row / column sampled evaluation of the same definitions at sizes where the full
# [N, V] matrices are too large to hold or too slow to multiply three times.
# --------------------------------------------------------------------------- #
def stats_streamed(X, W_shard_iter, labels):
    """m, sum, target over the whole vocabulary with W delivered shard by shard.
    Plain definition evaluated blockwise: the maximum over all columns is the
    maximum of block maxima; the sum is taken against that global maximum in a second
    sweep over the stored block logits."""
    N = X.shape[0]
    Ys, off = [], 0
    target = np.zeros(N, dtype=np.float64)
    m = np.full(N, -np.inf)
    for W_r in W_shard_iter:
        Y = X @ W_r.T
        m = np.maximum(m, Y.max(axis=1))
        loc = labels - off
        own = (loc >= 0) & (loc < W_r.shape[0])
        target[own] = Y[np.nonzero(own)[0], loc[own]]
        Ys.append(Y)
        off += W_r.shape[0]
    s = np.zeros(N, dtype=np.float64)
    for Y in Ys:
        s += np.exp(Y - m[:, None]).sum(axis=1)
    loss_rows = m + np.log(s) - target
    return {"m": m, "sum": s, "target": target, "loss_rows": loss_rows, "loss": loss_rows.mean(), "Y": Ys}


def D_block(Y_block, m, s, labels, offset, grad_scale):
    """(softmax - G) * scale for a block of vocabulary columns starting at ``offset``,
    given the global row statistics."""
    P = np.exp(Y_block - m[:, None]) / s[:, None]
    return (P - one_hot(labels, Y_block.shape[1], offset)) * grad_scale


# --------------------------------------------------------------------------- #
# Input layer (appendix C)
# --------------------------------------------------------------------------- #
def embed_fwd(table_shard: np.ndarray, ids: np.ndarray, offset: int) -> np.ndarray:
    """Each shard builds the full-size [N, h] output: the table row for ids it owns,
    an all-zero row otherwise (the all-reduce over shards then yields the lookup).
    Works on any dtype (bit patterns included): it only moves data."""
    Vs = table_shard.shape[0]
    out = np.zeros((ids.shape[0], table_shard.shape[1]), dtype=table_shard.dtype)
    for i in range(ids.shape[0]):
        loc = int(ids[i]) - offset
        if 0 <= loc < Vs:
            out[i] = table_shard[loc]
    return out


def embed_bwd(grad_out: np.ndarray, ids: np.ndarray, offset: int, Vs: int,
              dtable: np.ndarray) -> np.ndarray:
    """Scatter-add of the (broadcast) output gradient into the shard's table gradient:
    for tokens in increasing position, dE[id_i - off] += g_i.  ``dtable`` is the
    accumulator (fp32 or fp64); it is updated in place in its own precision."""
    for i in range(ids.shape[0]):
        loc = int(ids[i]) - offset
        if 0 <= loc < Vs:
            dtable[loc] += grad_out[i].astype(dtable.dtype)
    return dtable
