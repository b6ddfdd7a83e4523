"""Oracle: decode-phase attention and KV append, written out from the definition.

TEST INFRASTRUCTURE ONLY -- slow, fp64, numpy.  Not imported by the product path
and shares no code with the HIP library.

What it computes (paper, Sec. II-A "LLM Inference Basics"): attention is
softmax(Q K^T / sqrt(d_k)) V, per head, heads independent.  In the decode phase
(Sec. II-B "KV Cache") only the new token's q, k, v exist; k and v are stored
behind the cached ones and the single query row attends over the whole cache, so
the two matrix products are matrix-vector products over the sequence.  The
storage device of Sec. IV-D receives q, k, v, keeps k, v and returns the output;
the dense variant of Algorithm 1 is its last two steps with every token
selected and alpha = 1.

Conventions of this build where the paper is silent:
  * `scale` is passed explicitly (the paper's value is 1/sqrt(d_k)); it is the
    float32 the caller hands over, widened exactly to fp64.
  * `seq_lens[b]` is the length L_b INCLUDING the token appended in this step:
    append writes position L_b - 1, decode attends positions 0 .. L_b - 1.
  * Positions >= L_b have weight exactly zero and are never looked at.
  * L_b <= 0: output row of zeros, lse = -inf.  L_b is cut off at the capacity.
  * Grouped queries: query head h reads KV head h // (Hq // Hkv).
  * Paged cache: position t of sequence b lives in pool page
    page_table[b, t // page_size] at row t % page_size (the paper's 16-token,
    4 KB "group" of Sec. IV-C with an address map in front of it).

Layouts (numpy float16):
  contiguous cache  [B, Hkv, capacity, D]
  paged pool        [num_pages, Hkv, page_size, D]   + page_table [B, max_pages] int32
  q                 [B, Hq, D];   k_new, v_new [B, Hkv, D]
"""
from __future__ import annotations

import numpy as np


def _capacity(cache: np.ndarray, page_table) -> int:
    if page_table is None:
        return int(cache.shape[2])
    return int(cache.shape[2]) * int(page_table.shape[1])


def kv_append(k_cache, v_cache, k_new, v_new, seq_lens, page_table=None) -> None:
    """Store the new token's k and v at position L_b - 1 (bit copy, in place).

    Sec. IV-C "Batch Writing Requests": the decode phase produces one new k, v per
    head and step, which is added behind the stored ones.  A length outside
    [1, capacity] leaves the caches untouched.
    """
    assert k_cache.dtype == np.float16 and v_cache.dtype == np.float16
    assert k_new.dtype == np.float16 and v_new.dtype == np.float16
    B, Hkv, D = k_new.shape
    cap = _capacity(k_cache, page_table)
    for b in range(B):
        L = int(seq_lens[b])
        if L < 1 or L > cap:
            continue
        t = L - 1
        for hk in range(Hkv):
            if page_table is None:
                k_cache[b, hk, t, :] = k_new[b, hk, :]
                v_cache[b, hk, t, :] = v_new[b, hk, :]
            else:
                ps = k_cache.shape[2]
                page = int(page_table[b, t // ps])
                k_cache[page, hk, t % ps, :] = k_new[b, hk, :]
                v_cache[page, hk, t % ps, :] = v_new[b, hk, :]


def kv_write(k_cache, v_cache, k_src, v_src, start, count, page_table=None) -> None:
    """Store a run of rows per sequence (bit copy, in place): row start[b] + i of
    every KV head receives k_src[b, :, i, :] / v_src[b, :, i, :] for i < count[b].

    This is the prefill side of Sec. IV-D: a layer's K and V for all prompt tokens
    arrive at once and are laid down behind whatever is already stored.  Rows that
    would fall outside [0, capacity) are skipped; by definition it is what
    kv_append does when called once per row."""
    assert k_src.dtype == np.float16 and v_src.dtype == np.float16
    B, Hkv, N, D = k_src.shape
    cap = _capacity(k_cache, page_table)
    for b in range(B):
        for i in range(min(int(count[b]), N)):
            t = int(start[b]) + i
            if t < 0 or t >= cap:
                continue
            for hk in range(Hkv):
                if page_table is None:
                    k_cache[b, hk, t, :] = k_src[b, hk, i, :]
                    v_cache[b, hk, t, :] = v_src[b, hk, i, :]
                else:
                    ps = k_cache.shape[2]
                    page = int(page_table[b, t // ps])
                    k_cache[page, hk, t % ps, :] = k_src[b, hk, i, :]
                    v_cache[page, hk, t % ps, :] = v_src[b, hk, i, :]


def gather_rows(cache, b: int, hk: int, L: int, page_table=None) -> np.ndarray:
    """The first L rows [L, D] (float16) of sequence b, KV head hk."""
    if page_table is None:
        return cache[b, hk, :L, :]
    ps = cache.shape[2]
    D = cache.shape[3]
    rows = np.empty((L, D), dtype=cache.dtype)
    for t in range(L):
        rows[t] = cache[int(page_table[b, t // ps]), hk, t % ps]
    return rows


def attend_one(q_row, K_rows, V_rows, scale):
    """One head: q_row [D], K_rows, V_rows [L, D] (any float type, L >= 1).

    Returns (out [D], lse, w [L]) in fp64:
        s_t = scale * sum_d q_d K_td ;  w = softmax(s) ;  out = sum_t w_t V_t
        lse = log sum_t exp(s_t)
    """
    q64 = np.asarray(q_row, dtype=np.float64)
    K64 = np.asarray(K_rows, dtype=np.float64)
    V64 = np.asarray(V_rows, dtype=np.float64)
    s = np.float64(np.float32(scale)) * (K64 @ q64)
    m = s.max()
    e = np.exp(s - m)
    Z = e.sum()
    w = e / Z
    out = w @ V64
    return out, m + np.log(Z), w


def decode(q, k_cache, v_cache, seq_lens, scale, page_table=None):
    """Decode attention for a batch: returns (out [B, Hq, D] fp64, lse [B, Hq] fp64)."""
    B, Hq, D = q.shape
    Hkv = k_cache.shape[1]
    assert Hq % Hkv == 0
    G = Hq // Hkv
    cap = _capacity(k_cache, page_table)
    out = np.zeros((B, Hq, D), dtype=np.float64)
    lse = np.full((B, Hq), -np.inf, dtype=np.float64)
    for b in range(B):
        L = min(int(seq_lens[b]), cap)
        if L <= 0:
            continue
        for hk in range(Hkv):
            K_rows = gather_rows(k_cache, b, hk, L, page_table)
            V_rows = gather_rows(v_cache, b, hk, L, page_table)
            for g in range(G):
                h = hk * G + g
                out[b, h], lse[b, h], _ = attend_one(q[b, h], K_rows, V_rows, scale)
    return out, lse


def merge_segments(outs, lses):
    """Combine attention results computed over disjoint position ranges.

    outs [n, D], lses [n]: normalised output and log-sum-exp of each range (an
    empty range has lse = -inf and is ignored).  Because
    exp(lse_i) = sum over range i of exp(s_t), the result over the union is
    sum_i exp(lse_i) out_i / sum_i exp(lse_i), with lse = log sum_i exp(lse_i).
    Returns (out [D], lse); all-empty gives (zeros, -inf).
    """
    outs = np.asarray(outs, dtype=np.float64)
    lses = np.asarray(lses, dtype=np.float64)
    M = lses.max()
    if not np.isfinite(M):
        return np.zeros(outs.shape[1]), -np.inf
    wgt = np.exp(lses - M)
    tot = wgt.sum()
    live = wgt > 0.0
    out = (wgt[live, None] * outs[live]).sum(axis=0) / tot
    return out, M + np.log(tot)


def kv_cache_bytes(batch: int, seq_len: int, layers: int, hidden: int) -> int:
    """fp16 KV footprint of Sec. III-A: 2 tensors x 2 bytes x b x s x layers x hidden.

    The paper writes 4*b*s*p and calls p the parameter size; its own worked
    sizes (13B model: 128 x 2K -> about 200 GB, 32 x 4K -> about 100 GB) only
    come out when p is layers x hidden, which is the reading used here.
    """
    return 4 * batch * seq_len * layers * hidden


def decode_kv_read_bytes(seq_lens, num_kv_heads: int, head_dim: int) -> int:
    """Bytes of K and V one decode step of one layer has to read (each row once)."""
    return int(sum(max(int(L), 0) for L in seq_lens)) * num_kv_heads * head_dim * 2 * 2
