"""Oracle: SparF attention (Algorithm 1), one step after the other, fp64 numpy.

TEST INFRASTRUCTURE ONLY -- not imported by the product path, shares no code with
the HIP library.

Algorithm 1 approximates decode attention for one head from a fraction of the
cache.  In the paper's order and notation (q, v-bar in R^{d_h}; K, V in
R^{S x d_h}; r, k, l in N; m, n are the page sizes of the two-step loads):

  1   i   <- indicator of the r components of q with the largest |q|
  2-3     load those r columns of K (page-wise, then filtered inside the page)
  4   s^  <- softmax( q_[i] . K^T_[:,i] / sqrt(d_h * ||q_[i]||_1 / ||q||_1) )
  5   m   <- indicator of the l most recent positions
  6   j   <- indicator of the k positions with the largest s^ + m
  7   alpha <- sum of s^ over j
  8-9     load rows j of K and V (page-wise, then filtered inside the page)
  10  s   <- softmax( q . K^T_[j,:] / sqrt(d_h) )
  11  out <- alpha * s . V_[j,:] + (1 - alpha) * v-bar

Readings where the listing is garbled or silent:
  * step 1 writes its index range as 1..S; it ranges over the d_h components of q.
  * step 5 is printed as "1 if i > S", which would leave l unused; it is read as
    i > S - l (1-based), i.e. the l most recent positions always rank first
    (s^ <= 1, so adding 1 puts them ahead of every other position).
  * v-bar is the mean of the first S rows of V (the SparQ definition the paper
    builds on); the system keeps it up to date when rows are appended.
  * 1/sqrt(d_h) enters through the caller's `scale`, like in the dense path; the
    temperature of step 4 is then scale / sqrt(||q_[i]||_1 / ||q||_1).
  * ties in a top-k are broken towards the lower index.
  * k and l are cut off at S; r at d_h; l at k.
  * steps 2-3 and 8-9 move data and leave the selected sets unchanged
    (`pages_touched` reports what the page-wise first step would fetch).
"""
from __future__ import annotations

import numpy as np


def argtopk(x: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest entries, ties towards the lower index, ascending order."""
    order = np.argsort(-np.asarray(x, dtype=np.float64), kind="stable")[:k]
    return np.sort(order)


def softmax(x: np.ndarray) -> np.ndarray:
    e = np.exp(x - x.max())
    return e / e.sum()


def sparf_one(q, K, V, scale, r, k, l, vbar=None):
    """One head.  q [D]; K, V [S, D] (the first S rows, any float type).

    Returns a dict with out [D] and the intermediate results of every step
    (i_dims, s_hat, j_rows, alpha, s) in fp64."""
    q64 = np.asarray(q, dtype=np.float64)
    K64 = np.asarray(K, dtype=np.float64)
    V64 = np.asarray(V, dtype=np.float64)
    S, D = K64.shape
    sc = np.float64(np.float32(scale))
    r, k = min(int(r), D), min(int(k), S)
    l = min(int(l), k)
    if vbar is None:
        vbar = V64.mean(axis=0)
    # step 1
    i_dims = argtopk(np.abs(q64), r)
    # step 4
    norm1_all = np.abs(q64).sum()
    rho = np.abs(q64[i_dims]).sum() / norm1_all if norm1_all > 0 else 1.0
    logits_hat = (K64[:, i_dims] @ q64[i_dims]) * (sc / np.sqrt(rho)) if rho > 0 else np.zeros(S)
    s_hat = softmax(logits_hat)
    # step 5
    m = np.zeros(S)
    m[S - l:] = 1.0
    # step 6
    j_rows = argtopk(s_hat + m, k)
    # step 7
    alpha = s_hat[j_rows].sum()
    # step 10
    s = softmax(sc * (K64[j_rows] @ q64))
    # step 11
    out = alpha * (s @ V64[j_rows]) + (1.0 - alpha) * np.asarray(vbar, dtype=np.float64)
    return dict(out=out, i_dims=i_dims, s_hat=s_hat, logits_hat=logits_hat, j_rows=j_rows,
                alpha=alpha, s=s, vbar=np.asarray(vbar, dtype=np.float64))


def finish_from_selection(q, K, V, scale, s_hat, j_rows, vbar):
    """Steps 7, 10, 11 for a given selection j (used to check an implementation
    whose fp32 top-k legitimately differs from the fp64 one at near-ties)."""
    q64 = np.asarray(q, dtype=np.float64)
    K64 = np.asarray(K, dtype=np.float64)
    V64 = np.asarray(V, dtype=np.float64)
    sc = np.float64(np.float32(scale))
    j_rows = np.asarray(j_rows, dtype=np.int64)
    alpha = np.asarray(s_hat, dtype=np.float64)[j_rows].sum()
    s = softmax(sc * (K64[j_rows] @ q64))
    return alpha * (s @ V64[j_rows]) + (1.0 - alpha) * np.asarray(vbar, dtype=np.float64), alpha


def pages_touched(j_rows, n: int) -> np.ndarray:
    """First step of the two-step load (steps 8-9): the n-row pages that hold at
    least one selected row.  The second step filters them back to j_rows."""
    return np.unique(np.asarray(j_rows) // n)


def decode(q, k_cache, v_cache, seq_lens, scale, r, k, l):
    """Batch form over contiguous caches [B, Hkv, capacity, D]; query head h reads
    KV head h // G.  Returns (out [B, Hq, D], alpha [B, Hq], list of j_rows).
    A sequence with L_b <= 0 gives a zero row and alpha = 0."""
    B, Hq, D = q.shape
    Hkv = k_cache.shape[1]
    G = Hq // Hkv
    out = np.zeros((B, Hq, D))
    alpha = np.zeros((B, Hq))
    sel = [[None] * Hq for _ in range(B)]
    for b in range(B):
        L = min(int(seq_lens[b]), k_cache.shape[2])
        if L <= 0:
            continue
        for h in range(Hq):
            res = sparf_one(q[b, h], k_cache[b, h // G, :L], v_cache[b, h // G, :L], scale, r, k, l)
            out[b, h], alpha[b, h], sel[b][h] = res["out"], res["alpha"], res["j_rows"]
    return out, alpha, sel


def bytes_moved(S: int, D: int, r: int, k: int) -> int:
    """fp16 bytes steps 2-3 and 8-9 have to read for one head: r columns of K
    plus k rows of K and of V (the dense path reads 2*S*D*2)."""
    return 2 * (min(r, D) * S + 2 * min(k, S) * D)
