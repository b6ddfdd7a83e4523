"""Oracle: SparF attention (Algorithm 1), fp64 numpy.

TEST INFRASTRUCTURE ONLY -- not imported by the product path, shares no code with
the HIP library.

What Algorithm 1 computes for one query head, from a fraction of the cache:

  * component mask: the r components of q with the largest magnitude are kept;
  * approximate weights: every position is scored from the kept components alone,
    and the scores go through a softmax whose temperature makes up for the dropped
    components, sqrt(d_h * |q_kept|_1 / |q|_1) in place of sqrt(d_h);
  * kept rows: the k positions with the largest approximate weight, the l most
    recent positions always among them;
  * kept mass: the share of the approximate softmax that falls on the kept rows;
  * exact softmax attention over the kept rows only;
  * blend: kept mass x that attention + (1 - kept mass) x mean of V.

The loads of the algorithm (the kept columns of K, then the kept rows of K and V,
each page-wise with a filter behind it) move data and leave the kept sets
unchanged; `pages_touched` reports what the page-wise first step would fetch.

Readings where the paper's listing is garbled or silent:
  * the component mask's index range is printed as running over the positions; it
    runs over the d_h components of q.
  * the recency term is printed as "1 if i > S", which would leave l unused; it is
    read as i > S - l (1-based): the l most recent positions always rank first (a
    softmax weight is at most 1, so adding 1 puts them ahead of every other one).
  * the mean of V is taken over the first S rows (the SparQ definition the paper
    builds on); the system keeps it up to date when rows are appended.
  * 1/sqrt(d_h) enters through the caller's `scale`, like in the dense path; the
    temperature of the approximate softmax is then scale / sqrt(|q_kept|_1 / |q|_1).
  * ties in either top-k go to the lower index.
  * k and l are cut off at S; r at d_h; l at k.
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


def kept_components(q, r: int) -> np.ndarray:
    """The r components of q with the largest magnitude (ascending indices)."""
    return argtopk(np.abs(np.asarray(q, dtype=np.float64)), r)


def approximate_weights(q, K, dims, scale):
    """Softmax over all positions of the scores from the components `dims` alone, with the
    temperature correction for the dropped ones.  Returns (logits, weights)."""
    q64 = np.asarray(q, dtype=np.float64)
    K64 = np.asarray(K, dtype=np.float64)
    total = np.abs(q64).sum()
    share = np.abs(q64[dims]).sum() / total if total > 0 else 1.0       # |q_kept|_1 / |q|_1
    if share > 0:
        logits = (K64[:, dims] @ q64[dims]) * (np.float64(np.float32(scale)) / np.sqrt(share))
    else:
        logits = np.zeros(K64.shape[0])
    return logits, softmax(logits)


def kept_positions(weights, k: int, l: int) -> np.ndarray:
    """The k positions of largest weight with the l most recent forced in (ascending)."""
    S = len(weights)
    recency = np.zeros(S)
    recency[S - l:] = 1.0
    return argtopk(np.asarray(weights, dtype=np.float64) + recency, k)


def blend(q, K, V, scale, weights, rows, mean_v):
    """Exact softmax attention over `rows`, blended with mean_v by the mass the approximate
    weights put on those rows.  Returns (out, kept mass, exact weights over the rows)."""
    q64 = np.asarray(q, dtype=np.float64)
    rows = np.asarray(rows, dtype=np.int64)
    mass = np.asarray(weights, dtype=np.float64)[rows].sum()
    exact = softmax(np.float64(np.float32(scale)) * (np.asarray(K, dtype=np.float64)[rows] @ q64))
    out = mass * (exact @ np.asarray(V, dtype=np.float64)[rows]) + (1.0 - mass) * np.asarray(mean_v, dtype=np.float64)
    return out, mass, exact


def sparf_one(q, K, V, scale, r, k, l, vbar=None):
    """One head.  q [D]; K, V [S, D] (the first S rows, any float type); vbar: the mean of V
    if the caller keeps one, else it is taken here.

    Returns a dict: out [D], kept_dims, approx_logits, approx_weights, kept_rows,
    kept_mass, weights (exact, over the kept rows), mean_v; all fp64."""
    K64 = np.asarray(K, dtype=np.float64)
    V64 = np.asarray(V, dtype=np.float64)
    S, D = K64.shape
    r, k = min(int(r), D), min(int(k), S)
    l = min(int(l), k)
    mean_v = V64.mean(axis=0) if vbar is None else np.asarray(vbar, dtype=np.float64)
    dims = kept_components(q, r)
    logits, approx = approximate_weights(q, K64, dims, scale)
    rows = kept_positions(approx, k, l)
    out, mass, exact = blend(q, K64, V64, scale, approx, rows, mean_v)
    return dict(out=out, kept_dims=dims, approx_logits=logits, approx_weights=approx, kept_rows=rows,
                kept_mass=mass, weights=exact, mean_v=mean_v)


def finish_from_selection(q, K, V, scale, approx_weights, kept_rows, mean_v):
    """Kept mass, exact attention and blend for a GIVEN set of kept rows (used to check an
    implementation whose fp32 top-k legitimately differs from the fp64 one at near-ties).
    Returns (out, kept mass)."""
    out, mass, _ = blend(q, K, V, scale, approx_weights, kept_rows, mean_v)
    return out, mass


def pages_touched(kept_rows, n: int) -> np.ndarray:
    """First step of the two-step row load: the n-row pages that hold at least one kept
    row.  The second step filters them back to the kept rows."""
    return np.unique(np.asarray(kept_rows) // n)


def decode(q, k_cache, v_cache, seq_lens, scale, r, k, l):
    """Batch form over contiguous caches [B, Hkv, capacity, D]; query head h reads
    KV head h // G.  Returns (out [B, Hq, D], kept mass [B, Hq], list of kept rows).
    A sequence with L_b <= 0 gives a zero row and kept mass 0."""
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
            out[b, h], alpha[b, h], sel[b][h] = res["out"], res["kept_mass"], res["kept_rows"]
    return out, alpha, sel


def bytes_moved(S: int, D: int, r: int, k: int) -> int:
    """fp16 bytes the two loads have to read for one head: r columns of K plus k rows
    of K and of V (the dense path reads 2*S*D*2)."""
    return 2 * (min(r, D) * S + 2 * min(k, S) * D)
