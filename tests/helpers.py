"""Shared plumbing of the GPU parity tests: run one step through the C ABI, run the
same step through the oracle on the same bits, compare."""
from __future__ import annotations

import numpy as np
import torch

from oracle import c_oracle, decode_attention as np_oracle
from paper_2409_04992_amd import binding as B

TOL = {torch.float16: 2e-3, torch.float32: 1e-4}   # max-abs, attention output
LSE_TOL = 2e-4                                     # absolute, natural-log lse (fp32 path)
# Grouped queries with fp16 output: the MFMA kernel sums the fp16-rounded weights it feeds
# to the matrix core (the row is then an exact softmax of slightly perturbed scores), so
# the sum carries up to 2^-11 = 4.9e-4 relative error and the lse as much absolute error.
LSE_TOL_F16_WEIGHTS = 6e-4
ORACLE_THREADS = 16


def host(t):
    return None if t is None else t.detach().cpu().numpy()


def gpu_step(case, out_dtype=None, append=True, want_lse=True, max_seq_len=None, fused=False):
    """append + decode through the library (two calls, or the fused entry point);
    returns (out, lse) torch tensors."""
    wl = case.wl
    dev = case.q.device
    desc = B.kv_desc(case.k_cache, case.v_cache, case.page_table)
    if out_dtype is None:
        out_dtype = torch.float32 if wl.out_dtype == "f32" else torch.float16
    if max_seq_len is None:
        max_seq_len = min(int(case.seq_lens.max().item()), case.capacity)
        max_seq_len = max(max_seq_len, 1)
    Bn, Hq, D = case.q.shape
    # the workspace as sized by the library plus a guard band that must stay untouched
    size, guard = B.decode_workspace_size(Bn, Hq, wl.num_kv_heads, D, max_seq_len), 1 << 20
    buf = torch.empty(size + guard, dtype=torch.uint8, device=dev)
    buf.fill_(0xFF)      # NaN patterns: stale workspace contents must not leak into the result
    ws = buf[:size]
    out = torch.full((Bn, Hq, D), float("nan"), dtype=out_dtype, device=dev)
    lse = torch.full((Bn, Hq), float("nan"), dtype=torch.float32, device=dev) if want_lse else None
    if append and fused:
        B.append_decode(case.q, case.k_new, case.v_new, desc, case.seq_lens, wl.num_kv_heads,
                        case.scale, out, ws, max_seq_len, lse=lse)
    else:
        if append:
            B.kv_append(desc, case.k_new, case.v_new, case.seq_lens)
        B.decode(case.q, desc, case.seq_lens, wl.num_kv_heads, case.scale, out, ws, max_seq_len,
                 lse=lse)
    torch.cuda.synchronize()
    assert bool((buf[size:] == 0xFF).all()), "write behind the workspace"
    return out, lse


def oracle_step(case, append=True, pair_stride=1, pair_offset=0):
    """Same step on host copies (taken BEFORE the GPU step mutates the caches)."""
    q, k, v = host(case.q), host(case.k_cache).copy(), host(case.v_cache).copy()
    sl, pt = host(case.seq_lens), host(case.page_table)
    if append:
        c_oracle.kv_append(k, v, host(case.k_new), host(case.v_new), sl, pt)
    out, lse = c_oracle.decode(q, k, v, sl, case.scale, pt, pair_stride=pair_stride,
                               pair_offset=pair_offset, nthreads=ORACLE_THREADS)
    return out, lse, k, v


def oracle_rows(case, pairs, appended=True):
    """Oracle output for sampled (b, h) pairs, gathering only those rows from the
    device: returns {(b, h): (out[D], lse)}.  Used where the whole cache is too
    large to copy to the host."""
    wl = case.wl
    res = {}
    ps = case.k_cache.shape[2]
    for b, h in pairs:
        hk = h // wl.group
        L = min(int(case.seq_lens[b].item()), case.capacity)
        if case.page_table is None:
            K = case.k_cache[b, hk, :L].cpu().numpy()
            V = case.v_cache[b, hk, :L].cpu().numpy()
        else:
            pages = case.page_table[b, :(L + ps - 1) // ps].long()
            K = case.k_cache[pages, hk].reshape(-1, wl.head_dim)[:L].cpu().numpy()
            V = case.v_cache[pages, hk].reshape(-1, wl.head_dim)[:L].cpu().numpy()
        if not appended:   # caches not yet updated on the device: place the new row here
            K, V = K.copy(), V.copy()
            K[L - 1] = case.k_new[b, hk].cpu().numpy()
            V[L - 1] = case.v_new[b, hk].cpu().numpy()
        out, lse, _ = np_oracle.attend_one(case.q[b, h].cpu().numpy(), K, V, case.scale)
        res[(b, h)] = (out, lse)
    return res


def lse_tol(group, out_dtype):
    return LSE_TOL_F16_WEIGHTS if group > 1 and out_dtype == torch.float16 else LSE_TOL


def assert_close(out, lse, want_out, want_lse, what="", lse_tol=LSE_TOL):
    got = out.detach().cpu().double().numpy()
    tol = TOL[out.dtype]
    mask = ~np.isnan(want_out)
    assert np.isfinite(got[mask]).all(), "%s: non-finite output" % what
    err = np.abs(got[mask] - want_out[mask]).max() if mask.any() else 0.0
    assert err <= tol, "%s: max abs err %.3e > %.1e" % (what, err, tol)
    if lse is not None:
        gl = lse.detach().cpu().double().numpy()
        ml = ~np.isnan(want_lse)
        inf = np.isinf(want_lse) & ml
        assert np.array_equal(gl[inf], want_lse[inf]), "%s: lse of empty rows" % what
        fin = ml & ~inf
        if fin.any():
            lerr = np.abs(gl[fin] - want_lse[fin]) / (1.0 + np.abs(want_lse[fin]) * 0.01)
            assert lerr.max() <= lse_tol, "%s: lse err %.3e" % (what, lerr.max())
    return err
