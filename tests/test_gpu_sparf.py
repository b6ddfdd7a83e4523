"""GPU parity of the SparF path (Algorithm 1) against its fp64 oracle.

Both top-k of the algorithm are integer decisions taken on floating-point
numbers.  The choice of components compares exact fp16 magnitudes, so the kept
components must be identical.  The choice of rows is taken by the kernel on fp32 scores, the oracle's on fp64
ones: the two selections may differ only in rows whose score is within the fp32
rounding of the threshold, so the test checks that the kernel's selection is a
valid top-k of the oracle's scores up to that rounding, and then compares the
output with the oracle's kept mass, attention and blend evaluated on the kernel's selection."""
import numpy as np
import pytest
import torch

from oracle import decode_attention as dense
from oracle import sparf_attention as sparf
from paper_2409_04992_amd import binding as B
from paper_2409_04992_amd import workloads as W

import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
SCORE_EPS = 2e-4          # fp32 rounding of an r-term dot product of magnitude <~ 50, in natural-log units


def logical(case):
    """K and V as host arrays [B][Hkv][capacity][D] whatever the layout (positions on
    unmapped pages read 0)."""
    if case.page_table is None:
        return H.host(case.k_cache).copy(), H.host(case.v_cache).copy()
    table = case.page_table.long()
    mapped = (table >= 0)[:, :, None, None, None]
    res = []
    for cache in (case.k_cache, case.v_cache):
        g = cache[table.clamp(min=0)]                       # [B][pages][Hkv][ps][D]
        g = torch.where(mapped, g, torch.zeros_like(g))
        Bn, P, Hkv, ps, D = g.shape
        res.append(g.permute(0, 2, 1, 3, 4).reshape(Bn, Hkv, P * ps, D).cpu().numpy())
    return res


def column_copy(kt, kt_table, b, L):
    """[Hkv][D][L]: the component-major copy of sequence b as the kernels see it."""
    if kt_table is None:
        return kt[b, :, :, :L]
    P = kt.shape[3]
    pages = kt_table[b, :(L + P - 1) // P].long()
    return kt[pages].permute(1, 2, 0, 3).reshape(kt.shape[1], kt.shape[2], -1)[:, :, :L]


def setup(wl, build_lens_offset=-1, kt_page=None):
    """Caches with S_b valid rows, aux built for them; the step then appends row S_b.
    kt_page: positions per page of a paged component-major copy (None: contiguous)."""
    case = W.make_case(wl, DEV, poison=True)
    Bn, Hkv, D, cap = wl.batch, wl.num_kv_heads, wl.head_dim, case.capacity
    vsum = torch.full((Bn, Hkv, D), float("nan"), dtype=torch.float32, device=DEV)
    kt_table = None
    if kt_page is None:
        kt = torch.full((Bn, Hkv, D, (cap + 7) // 8 * 8), float("nan"), dtype=torch.float16, device=DEV)
    else:
        per_seq = (cap + kt_page - 1) // kt_page
        lens = case.seq_lens.cpu()
        need = [(max(int(L), 0) + kt_page - 1) // kt_page for L in lens]
        pool = sum(need) + 2
        kt = torch.full((pool, Hkv, D, kt_page), float("nan"), dtype=torch.float16, device=DEV)
        perm = torch.randperm(pool, generator=torch.Generator().manual_seed(wl.seed + 5)).to(torch.int32)
        kt_table = torch.full((Bn, per_seq), -1, dtype=torch.int32)
        at = 0
        for b in range(Bn):
            kt_table[b, :need[b]] = perm[at:at + need[b]]
            at += need[b]
        kt_table = kt_table.to(DEV)
    desc = B.kv_desc(case.k_cache, case.v_cache, case.page_table)
    aux = B.sparf_aux(kt, vsum, kt_table)
    case.kt_table = kt_table
    before = (case.seq_lens + build_lens_offset).contiguous()
    B.sparf_build(desc, aux, before, Hkv, D)
    torch.cuda.synchronize()
    return case, desc, aux, kt, vsum, before


def run_decode(case, desc, aux, r, k, l, out_dtype, max_len=None, fused_append=False):
    wl = case.wl
    Bn, Hq, D = case.q.shape
    max_len = max_len or max(1, int(case.seq_lens.max()))
    # the workspace as sized by the library, a guard band behind it that must stay untouched
    size, guard = B.sparf_workspace_size(Bn, Hq, D, max_len, k), 1 << 20
    buf = torch.empty(size + guard, dtype=torch.uint8, device=DEV)
    buf.fill_(0xFF)
    ws = buf[:size]
    out = torch.full((Bn, Hq, D), float("nan"), dtype=out_dtype, device=DEV)
    sel = torch.full((Bn, Hq, k), -1, dtype=torch.int32, device=DEV)
    alpha = torch.full((Bn, Hq), float("nan"), dtype=torch.float32, device=DEV)
    if fused_append:
        B.sparf_append_decode(case.q, case.k_new, case.v_new, desc, aux, case.seq_lens, wl.num_kv_heads,
                              case.scale, r, k, l, out, ws, max_len, sel_rows=sel, alpha=alpha)
    else:
        B.sparf_decode(case.q, desc, aux, case.seq_lens, wl.num_kv_heads, case.scale, r, k, l, out, ws,
                       max_len, sel_rows=sel, alpha=alpha)
    torch.cuda.synchronize()
    assert bool((buf[size:] == 0xFF).all()), "write behind the workspace"
    return out, sel, alpha


def device_rows(case, b, hk, L):
    """Rows [0, L) of K and V of one (sequence, KV head), gathered on the device: for
    caches too large to copy to the host whole."""
    if case.page_table is None:
        return case.k_cache[b, hk, :L].cpu().numpy(), case.v_cache[b, hk, :L].cpu().numpy()
    ps = case.k_cache.shape[2]
    pages = case.page_table[b, :(L + ps - 1) // ps].long()
    D = case.k_cache.shape[3]
    return (case.k_cache[pages, hk].reshape(-1, D)[:L].cpu().numpy(),
            case.v_cache[pages, hk].reshape(-1, D)[:L].cpu().numpy())


def check_against_oracle(case, out, sel, alpha, r, k, l, pairs=None, rows_of=None):
    wl = case.wl
    q = H.host(case.q)
    if rows_of is None:
        K, V = logical(case)
        rows_of = lambda b, hk, L: (K[b, hk, :L], V[b, hk, :L])
    lens = H.host(case.seq_lens)
    tol = H.TOL[out.dtype]
    Bn, Hq, D = q.shape
    pairs = pairs or [(b, h) for b in range(Bn) for h in range(Hq)]
    worst = 0.0
    for b, h in pairs:
        L = int(lens[b])
        hk = h // wl.group
        if L <= 0:
            assert torch.equal(out[b, h], torch.zeros_like(out[b, h])) and float(alpha[b, h]) == 0.0
            continue
        Kr, Vr = rows_of(b, hk, L)
        res = sparf.sparf_one(q[b, h], Kr, Vr, case.scale, r, k, l)
        keff = min(k, L)
        got_rows = sel[b, h, :keff].cpu().numpy().astype(np.int64)
        assert (np.diff(got_rows) > 0).all() and got_rows[0] >= 0 and got_rows[-1] < L
        leff = min(l, keff)
        assert set(range(L - leff, L)) <= set(got_rows)            # the most recent rows are kept
        # the kept rows: a valid top-k of the oracle's scores up to fp32 rounding
        want_rows = set(res["kept_rows"].tolist())
        lg = res["approx_logits"]
        cand = np.array(sorted(want_rows - set(range(L - leff, L))))
        if len(cand):
            thr = lg[cand].min()
            for t in set(got_rows.tolist()) - want_rows:
                assert lg[t] >= thr - SCORE_EPS, (b, h, t)
            for t in want_rows - set(got_rows.tolist()):
                assert lg[t] <= thr + SCORE_EPS, (b, h, t)
        # kept mass, attention and blend on the kernel's own selection
        want_out, want_alpha = sparf.finish_from_selection(q[b, h], Kr, Vr, case.scale, res["approx_weights"],
                                                           got_rows, res["mean_v"])
        assert abs(float(alpha[b, h]) - want_alpha) <= 2e-5
        err = np.abs(out[b, h].double().cpu().numpy() - want_out).max()
        worst = max(worst, err)
        assert err <= tol, "(%d,%d): %.3e" % (b, h, err)
    return worst


def sparf_step(wl, r, k, l, out_dtype=torch.float32, pairs=None, kt_page=None, fused_append=False):
    case, desc, aux, kt, vsum, before = setup(wl, kt_page=kt_page)
    want_k, want_v = logical(case)
    dense.kv_append(want_k, want_v, H.host(case.k_new), H.host(case.v_new), H.host(case.seq_lens))
    if not fused_append:
        B.sparf_append(desc, aux, case.k_new, case.v_new, case.seq_lens)
    out, sel, alpha = run_decode(case, desc, aux, r, k, l, out_dtype, fused_append=fused_append)
    # the append part: caches bit-exact, column copy and V sums consistent with them
    got_k, got_v = logical(case)
    assert np.array_equal(got_k.view(np.uint16), want_k.view(np.uint16))
    assert np.array_equal(got_v.view(np.uint16), want_v.view(np.uint16))
    lens = H.host(case.seq_lens)
    for b in range(case.wl.batch):
        L = int(lens[b])
        if L < 1:
            continue
        cols = column_copy(kt, case.kt_table, b, L).cpu().numpy()
        assert np.array_equal(cols.view(np.uint16),
                              np.ascontiguousarray(want_k[b, :, :L].transpose(0, 2, 1)).view(np.uint16))
        ref = want_v[b, :, :L].astype(np.float64).sum(axis=1)
        np.testing.assert_allclose(vsum[b].double().cpu().numpy(), ref, rtol=0, atol=2e-3)
    return check_against_oracle(case, out, sel, alpha, r, k, l, pairs)


# ------------------------------------------------------------------ parity
@pytest.mark.parametrize("r,k,l", [(16, 64, 8), (8, 128, 0), (128, 32, 4), (1, 16, 16), (32, 700, 3)])
@pytest.mark.parametrize("out_dtype", [torch.float32, torch.float16])
@pytest.mark.parametrize("three_launches", [False, True])
def test_sparf_mha_small(options, r, k, l, out_dtype, three_launches):
    """Both forms of the path: the one-launch kernel and the three-launch pipeline
    that long rows take (forced here through the environment)."""
    if three_launches:
        options.setenv("INSTATTN_SPARF_THREE_LAUNCHES", "1")
    wl = W.Workload("sparf_mha", 3, 4, 4, 128, 1500, seq_len_min=300, seed=401)
    sparf_step(wl, r, k, l, out_dtype)


@pytest.mark.parametrize("kv_paged,kt_page", [(True, 256), (True, 16), (True, None), (False, 64), (True, 8)])
@pytest.mark.parametrize("three_launches", [False, True])
def test_sparf_paged_layouts(options, kv_paged, kt_page, three_launches):
    """The cache in 16-row pages and/or the component-major copy in pages of its own
    size, each behind its own shuffled page table, in every combination."""
    if three_launches:
        options.setenv("INSTATTN_SPARF_THREE_LAUNCHES", "1")
    wl = W.Workload("sparf_paged", 3, 4, 2, 128, 1700, seq_len_min=200, paged=kv_paged, page_size=16,
                    seed=410)
    sparf_step(wl, 16, 120, 9, torch.float32, kt_page=kt_page)


@pytest.mark.parametrize("seq_len", [0, 1, 15, 16, 17, 255, 256, 257, 2048])
def test_sparf_paged_lengths_around_page_edges(seq_len):
    wl = W.Workload("sparf_paged_len", 2, 2, 2, 64, seq_len, paged=True, page_size=16, seed=411)
    sparf_step(wl, 8, 40, 5, torch.float16, kt_page=256)


def test_sparf_paged_long_rows():
    wl = W.Workload("sparf_paged_long", 1, 2, 2, 128, 20000, paged=True, page_size=16, seed=412)
    sparf_step(wl, 16, 1300, 32, torch.float16, kt_page=1024)


@pytest.mark.parametrize("shape", ["mha", "mha64", "gqa", "paged", "long", "three"])
def test_sparf_append_decode_in_one_call(options, shape):
    """The fused entry point against the oracle, in every form it takes: the new token
    stored by the one-launch kernel itself (one query head per KV head), or by a launch
    of its own in front (grouped queries, long rows, the three-launch pipeline)."""
    if shape == "three":
        options.setenv("INSTATTN_SPARF_THREE_LAUNCHES", "1")
    wl = {
        "mha": W.Workload("sparf_f1", 3, 4, 4, 128, 1500, seq_len_min=300, seed=420),
        "mha64": W.Workload("sparf_f2", 2, 4, 4, 64, 700, seq_len_min=1, seed=421),
        "gqa": W.Workload("sparf_f3", 2, 8, 2, 128, 900, seq_len_min=100, seed=422),
        "paged": W.Workload("sparf_f4", 3, 4, 4, 128, 1700, seq_len_min=200, paged=True, page_size=16, seed=423),
        "long": W.Workload("sparf_f5", 1, 2, 2, 128, 9000, seed=424),
        "three": W.Workload("sparf_f6", 2, 4, 4, 128, 1000, seq_len_min=300, seed=425),
    }[shape]
    sparf_step(wl, 16, 100, 7, torch.float32, kt_page=256 if shape == "paged" else None, fused_append=True)


def test_sparf_append_decode_equals_the_two_calls():
    wl = W.Workload("sparf_f7", 4, 4, 4, 128, 2500, seq_len_min=0, seed=426)
    res = []
    for fused in (False, True):
        case, desc, aux, kt, vsum, _ = setup(wl)
        if not fused:
            B.sparf_append(desc, aux, case.k_new, case.v_new, case.seq_lens)
        out = run_decode(case, desc, aux, 16, 150, 8, torch.float32, fused_append=fused)
        res.append(out + (kt.clone(), vsum.clone(), case.k_cache.clone(), case.v_cache.clone()))
    for x, y in zip(*res):
        assert torch.equal(x.view(torch.int32) if x.dtype == torch.float32 else x.view(torch.int16),
                           y.view(torch.int32) if y.dtype == torch.float32 else y.view(torch.int16))


@pytest.mark.parametrize("three_launches", [False, True])
def test_sparf_new_token_alone_in_its_unit(options, three_launches):
    """Rows of a multiple of 2048 cached positions: the appended token is the only position of
    the row's last unit of the score pass (and of a step of the one-launch kernel's column
    pass).  Same bits as appending first and decoding after, whatever the form (short rows are
    sent through the pipeline by the switch), and the oracle's result."""
    if three_launches:
        options.setenv("INSTATTN_SPARF_THREE_LAUNCHES", "1")
    lens = [2049, 4097, 10241, 2048, 1, 12289, 6145, 2050]
    wl = W.Workload("sparf_lone", len(lens), 3, 3, 128, 12288, seq_len_min=1, seed=427)
    res = []
    for fused in (False, True):
        case = W.make_case(wl, DEV, poison=True, lens=lens)
        Bn, Hkv, D, cap = wl.batch, wl.num_kv_heads, wl.head_dim, case.capacity
        vsum = torch.zeros(Bn, Hkv, D, dtype=torch.float32, device=DEV)
        kt = torch.full((Bn, Hkv, D, (cap + 7) // 8 * 8), float("nan"), dtype=torch.float16, device=DEV)
        desc, aux = B.kv_desc(case.k_cache, case.v_cache), B.sparf_aux(kt, vsum)
        B.sparf_build(desc, aux, (case.seq_lens - 1).contiguous(), Hkv, D)
        if not fused:
            B.sparf_append(desc, aux, case.k_new, case.v_new, case.seq_lens)
        out = run_decode(case, desc, aux, 16, 300, 16, torch.float32, max_len=12289, fused_append=fused)
        res.append(out + (kt.clone(), vsum.clone(), case.k_cache.clone(), case.v_cache.clone()))
    for x, y in zip(*res):
        assert torch.equal(x.view(torch.int32) if x.dtype == torch.float32 else x.view(torch.int16),
                           y.view(torch.int32) if y.dtype == torch.float32 else y.view(torch.int16))
    check_against_oracle(case, *res[1][:3], 16, 300, 16)


@pytest.mark.parametrize("seq_len,k", [(20000, 1300), (8192, 100), (32767, 3000), (32768, 600), (40000, 2500),
                                       (65534, 700), (70000, 4400), (9000, 20000)])
@pytest.mark.parametrize("distributed", ["0", "1"])
def test_sparf_long_rows_take_the_three_launch_pipeline(options, seq_len, k, distributed):
    """Rows behind the one-launch limit.  One block per head: the selection keeps the
    scores in registers up to 32768 and up to 65535 positions and passes over the
    workspace beyond.  Distributed: one block per stretch of 8192 scores, three
    launches.  The attend kernel cuts the kept rows of a head into up to 8 slices."""
    options.setenv("INSTATTN_SPARF_DISTRIBUTED", distributed)
    wl = W.Workload("sparf_long", 1, 2, 2, 128, seq_len, seed=408)
    sparf_step(wl, 16, k, 32, torch.float16)


@pytest.mark.parametrize("seq_len,k,head_dim", [(8192, 100, 128), (10000, 450, 64), (16000, 400, 128),
                                                (20000, 511, 128), (32767, 500, 64), (40000, 300, 128),
                                                (65534, 200, 128), (65534, 480, 64)])
@pytest.mark.parametrize("split_tail", ["0", "1"])
def test_sparf_long_rows_selected_and_gathered_by_one_block(options, seq_len, k, head_dim, split_tail):
    """Few kept rows per head (no slices), one block per head: that block selects and
    then gathers (two launches in all), or, forced here, the selection and the gather
    stay kernels of their own.  Every block size of the selection."""
    options.setenv("INSTATTN_SPARF_DISTRIBUTED", "0")
    options.setenv("INSTATTN_SPARF_SPLIT_TAIL", split_tail)
    wl = W.Workload("sparf_tail", 2, 3, 3, head_dim, seq_len, seq_len_min=seq_len // 2, seed=414)
    sparf_step(wl, head_dim // 8, k, 16, torch.float16)


def test_sparf_one_block_tail_equals_the_two_kernels(options):
    wl = W.Workload("sparf_tail_eq", 3, 4, 2, 128, 12000, seq_len_min=0, paged=True, page_size=16, seed=415)
    case, desc, aux, kt, vsum, _ = setup(wl, kt_page=256)
    B.sparf_append(desc, aux, case.k_new, case.v_new, case.seq_lens)
    options.setenv("INSTATTN_SPARF_DISTRIBUTED", "0")
    options.setenv("INSTATTN_SPARF_SPLIT_TAIL", "1")
    a = run_decode(case, desc, aux, 16, 300, 16, torch.float32)
    options.setenv("INSTATTN_SPARF_SPLIT_TAIL", "0")
    b = run_decode(case, desc, aux, 16, 300, 16, torch.float32)
    assert torch.equal(a[1], b[1]) and torch.equal(a[2], b[2])       # same kept rows, same alpha
    assert (a[0] - b[0]).abs().max() <= 2e-6


@pytest.mark.parametrize("seq_len,k,head_dim,paged,fused", [
    (8192, 300, 128, False, True), (8200, 600, 64, True, False), (12000, 13000, 128, True, True),
    (16384, 1024, 128, False, True), (16385, 1, 64, False, True), (18431, 2000, 128, True, False),
    (18430, 5000, 64, False, True),
    (18432, 700, 128, False, True), (25000, 26000, 64, True, True), (32768, 2048, 128, False, True),
    (36863, 100, 128, True, False), (36862, 30000, 64, False, True)])
def test_sparf_one_launch_kernel_of_512_and_1024_threads(options, seq_len, k, head_dim, paged, fused):
    """Rows between 8193 and 18432 positions in the one-launch kernel's form of 512
    threads, up to 36864 positions in that of 1024 (forced here: with few heads the host
    would pick the pipeline), with and without the append inside it, up to the longest row
    each takes; kept rows beyond the room for row ids in LDS go through in pieces."""
    options.setenv("INSTATTN_SPARF_WIDE", "1")
    wl = W.Workload("sparf_wide", 2, 3, 3, head_dim, seq_len, seq_len_min=seq_len - 9000, paged=paged,
                    page_size=16, seed=416)
    sparf_step(wl, head_dim // 8, k, 16, torch.float32, kt_page=256 if paged else None, fused_append=fused)


def test_sparf_wide_one_launch_equals_the_pipeline(options):
    wl = W.Workload("sparf_wide_eq", 2, 4, 2, 128, 15000, seq_len_min=9000, seed=417)
    case, desc, aux, kt, vsum, _ = setup(wl)
    B.sparf_append(desc, aux, case.k_new, case.v_new, case.seq_lens)
    options.setenv("INSTATTN_SPARF_WIDE", "1")
    a = run_decode(case, desc, aux, 16, 900, 16, torch.float32)
    options.setenv("INSTATTN_SPARF_WIDE", "0")
    b = run_decode(case, desc, aux, 16, 900, 16, torch.float32)
    assert torch.equal(a[1], b[1])                                   # same kept rows
    assert (a[0] - b[0]).abs().max() <= 2e-6 and (a[2] - b[2]).abs().max() <= 1e-6


@pytest.mark.parametrize("distributed", ["0", "1"])
def test_sparf_one_very_long_sequence(options, distributed):
    """A million positions per head, 65536 kept: 128 stretches per head in the
    distributed selection, the pass-over-memory selection in the one-block form, eight
    slices of 8192 kept rows each."""
    options.setenv("INSTATTN_SPARF_DISTRIBUTED", distributed)
    wl = W.Workload("sparf_1m", 1, 2, 2, 128, 1 << 20, seed=418)
    sparf_step(wl, 16, 1 << 16, 16, torch.float16)


@pytest.mark.parametrize("shape", ["short_mha", "short_gqa_fused"])
def test_sparf_short_rows_forced_through_the_distributed_selection(options, shape):
    """Rows the one-launch kernel would take, sent through the pipeline with the
    selection spread over stretches (one stretch here): every switch combination must
    stay inside the workspace the library asked for (checked behind every decode of
    these tests by a guard band)."""
    options.setenv("INSTATTN_SPARF_THREE_LAUNCHES", "1")
    options.setenv("INSTATTN_SPARF_DISTRIBUTED", "1")
    if shape == "short_mha":
        wl = W.Workload("sparf_short_dist", 3, 4, 4, 128, 1500, seq_len_min=300, seed=442)
        sparf_step(wl, 16, 100, 7, torch.float32)
    else:
        wl = W.Workload("sparf_short_dist_gqa", 2, 4, 2, 64, 5212, seq_len_min=596, paged=True, page_size=16,
                        seed=443)
        sparf_step(wl, 4, 4929, 24, torch.float16, kt_page=256, fused_append=True)


@pytest.mark.parametrize("shape", ["mha_paged", "one_pair_long", "d64_ragged"])
def test_sparf_build_with_and_without_scratch(shape):
    """instattn_sparf_build with the scratch it asks for (the V sum of a pair spread over
    blocks and folded in block order) and without (one block per pair): the same column
    copy bit for bit, the same sums to fp32 rounding, each form deterministic; a guard
    band behind the scratch stays untouched."""
    wl = {"mha_paged": W.Workload("sparf_bws1", 2, 3, 3, 128, 20000, seq_len_min=300, paged=True, page_size=16,
                                  seed=444),
          "one_pair_long": W.Workload("sparf_bws2", 1, 1, 1, 128, 300_000, seed=445),
          "d64_ragged": W.Workload("sparf_bws3", 5, 2, 2, 64, 9000, seq_len_min=0, seed=446)}[shape]
    case, desc, aux, kt, vsum, lens = setup(wl, kt_page=256 if wl.paged else None)
    Hkv, D = wl.num_kv_heads, wl.head_dim
    size = B.sparf_build_workspace_size(wl.batch, Hkv, D)
    assert size > 0
    runs = []
    for use_scratch in (True, False, True, False):
        kt.fill_(float("nan"))
        vsum.fill_(float("nan"))
        buf = torch.empty(size + 4096, dtype=torch.uint8, device=DEV)
        buf.fill_(0xFF)
        B.sparf_build(desc, aux, lens, Hkv, D, workspace=buf[:size] if use_scratch else None)
        torch.cuda.synchronize()
        assert bool((buf[size:] == 0xFF).all())
        runs.append((kt.clone(), vsum.clone()))
    for kt_i, _ in runs[1:]:
        assert torch.equal(kt_i.view(torch.int16), runs[0][0].view(torch.int16))
    assert torch.equal(runs[0][1].view(torch.int32), runs[2][1].view(torch.int32))      # deterministic
    assert torch.equal(runs[1][1].view(torch.int32), runs[3][1].view(torch.int32))
    # against the fp64 sum of the rows
    K, V = logical(case)
    for b in range(wl.batch):
        n = int(lens[b])
        want = V[b, :, :n].astype(np.float64).sum(axis=1) if n > 0 else np.zeros((Hkv, D))
        for _, vs in runs[:2]:
            got = vs[b].double().cpu().numpy()
            assert np.abs(got - want).max() <= 1e-5 * max(1.0, np.abs(V[b, :, :max(n, 1)]).astype(np.float64).sum(axis=1).max())


def test_sparf_distributed_selection_equals_one_block_per_head(options):
    """Same kept rows bit for bit, alpha and out up to the order of the mass sum; ragged
    lengths so that heads use different numbers of stretches; repeated (the gathered
    members arrive in any order)."""
    wl = W.Workload("sparf_dist", 3, 4, 2, 128, 40000, seq_len_min=8300, paged=True, page_size=16, seed=414)
    case, desc, aux, kt, vsum, _ = setup(wl, kt_page=256)
    B.sparf_append(desc, aux, case.k_new, case.v_new, case.seq_lens)
    options.setenv("INSTATTN_SPARF_DISTRIBUTED", "0")
    ref = run_decode(case, desc, aux, 16, 3000, 16, torch.float32)
    options.setenv("INSTATTN_SPARF_DISTRIBUTED", "1")
    first = None
    for rep in range(3):
        got = run_decode(case, desc, aux, 16, 3000, 16, torch.float32)
        assert torch.equal(got[1], ref[1])
        assert (got[0] - ref[0]).abs().max() <= 2e-6 and (got[2] - ref[2]).abs().max() <= 1e-6
        first = first or got
        assert all(torch.equal(x, y) for x, y in zip(got, first))       # deterministic


@pytest.mark.parametrize("distributed", ["0", "1"])
def test_sparf_long_rows_of_equal_scores(options, distributed):
    """Identical keys on a long row: every score ties, the threshold bin holds the whole
    row (more than the distributed selection ranks directly: it falls back to the block
    of stretch 0).  Kept: the first k - l and the last l positions."""
    options.setenv("INSTATTN_SPARF_DISTRIBUTED", distributed)
    wl = W.Workload("sparf_long_ties", 1, 2, 2, 128, 19999, seed=415)
    case, desc, aux, kt, vsum, _ = setup(wl)
    case.k_cache[:] = case.k_cache[:, :, :1]
    case.k_new[:] = case.k_cache[:, :, 0]
    B.sparf_build(desc, aux, (case.seq_lens - 1).contiguous(), 2, 128)
    B.sparf_append(desc, aux, case.k_new, case.v_new, case.seq_lens)
    out, sel, alpha = run_decode(case, desc, aux, 16, 1000, 10, torch.float32)
    want = torch.cat([torch.arange(990), torch.arange(19990, 20000)]).to(torch.int32)
    assert torch.equal(sel[0, 0].cpu(), want) and torch.equal(sel[0, 1].cpu(), want)
    assert (alpha - 1000 / 20000).abs().max() < 1e-6


@pytest.mark.parametrize("seq_len,k", [(300_000, 20_000), (524_288, 1000)])
def test_sparf_distributed_long_member_lists(options, seq_len, k):
    """Rows so long that the threshold bin holds more scores than go through LDS: the
    list is ranked from the workspace (finer buckets, then the one bucket directly)."""
    options.setenv("INSTATTN_SPARF_DISTRIBUTED", "1")
    wl = W.Workload("sparf_long_list", 1, 2, 1, 128, seq_len, seed=419)
    sparf_step(wl, 16, k, 16, torch.float32)


def test_sparf_distributed_long_list_of_near_ties(options):
    """A long row whose keys repeat 61 distinct rows: a few dozen distinct scores, each
    thousands of times.  The list of the threshold bin is long and its finer bucket still
    holds more than can be ranked directly: the block of stretch 0 selects the whole row.
    Ties go to the lower position either way."""
    options.setenv("INSTATTN_SPARF_DISTRIBUTED", "1")
    wl = W.Workload("sparf_near_ties", 1, 2, 2, 128, 280_000, seed=420)
    case, desc, aux, kt, vsum, _ = setup(wl)
    L = int(case.seq_lens[0])
    idx = torch.randint(0, 61, (L,), device=DEV, generator=torch.Generator(device=DEV).manual_seed(5))
    case.k_cache[:, :, :L] = case.k_cache[:, :, :61][:, :, idx]
    case.k_new[:] = case.k_cache[:, :, L - 1]
    B.sparf_build(desc, aux, (case.seq_lens - 1).contiguous(), 2, 128)
    B.sparf_append(desc, aux, case.k_new, case.v_new, case.seq_lens)
    out, sel, alpha = run_decode(case, desc, aux, 16, 30_000, 16, torch.float32)
    check_against_oracle(case, out, sel, alpha, 16, 30_000, 16)


def test_sparf_distributed_edge_lengths(options):
    """Lengths around the stretch edges, k below l, k above the length, an empty row."""
    options.setenv("INSTATTN_SPARF_DISTRIBUTED", "1")
    wl = W.Workload("sparf_dist_edges", 6, 2, 2, 64, 16500, seed=416)
    case, desc, aux, kt, vsum, _ = setup(wl)
    case.seq_lens = torch.tensor([8193, 16384, 16385, 0, 9000, 16500], dtype=torch.int32, device=DEV)
    B.sparf_build(desc, aux, (case.seq_lens - 1).clamp(min=0).contiguous(), 2, 64)
    B.sparf_append(desc, aux, case.k_new, case.v_new, case.seq_lens)
    for k, l in [(300, 8), (5, 9), (20000, 3), (8200, 0)]:
        out, sel, alpha = run_decode(case, desc, aux, 8, k, l, torch.float32, max_len=16500)
        check_against_oracle(case, out, sel, alpha, 8, k, l)


@pytest.mark.parametrize("wide", ["0", "1"])
def test_sparf_long_rows_many_heads_no_slices(options, wide):
    """1040 heads of up to 9001 positions: the pipeline (score pass, then one block per
    head that selects and gathers), or the one-launch kernel's 512-thread form (the
    host's choice for this shape)."""
    options.setenv("INSTATTN_SPARF_WIDE", wide)
    wl = W.Workload("sparf_long_many", 26, 40, 40, 64, 9000, seq_len_min=100, seed=413)
    pairs = [(0, 0), (25, 39), (13, 7), (5, 20)]
    sparf_step(wl, 8, 300, 4, torch.float16, pairs=pairs)


def test_sparf_one_launch_and_three_launches_agree(options):
    wl = W.Workload("sparf_both", 2, 4, 2, 128, 4000, seq_len_min=1000, seed=409)
    case, desc, aux, kt, vsum, _ = setup(wl)
    B.sparf_append(desc, aux, case.k_new, case.v_new, case.seq_lens)
    a = run_decode(case, desc, aux, 16, 250, 16, torch.float32)
    options.setenv("INSTATTN_SPARF_THREE_LAUNCHES", "1")
    b = run_decode(case, desc, aux, 16, 250, 16, torch.float32)
    assert torch.equal(a[1], b[1])                                   # same kept rows
    assert (a[0] - b[0]).abs().max() <= 2e-6 and (a[2] - b[2]).abs().max() <= 1e-6


@pytest.mark.parametrize("head_dim,group", [(64, 1), (64, 4), (128, 8)])
def test_sparf_head_dims_and_groups(head_dim, group):
    wl = W.Workload("sparf_g", 2, 2 * group, 2, head_dim, 900, seq_len_min=100, seed=402)
    sparf_step(wl, head_dim // 8, 96, 8)


@pytest.mark.parametrize("seq_len", [0, 1, 7, 8, 9, 63, 64, 2047, 2048, 2049, 5000])
def test_sparf_lengths_around_vector_and_block_edges(seq_len):
    wl = W.Workload("sparf_len", 2, 2, 2, 128, seq_len, seed=403)
    sparf_step(wl, 16, 40, 5)


def test_sparf_keeping_every_row_equals_dense_decode():
    wl = W.Workload("sparf_all", 2, 4, 4, 128, 800, seq_len_min=200, seed=404)
    case, desc, aux, kt, vsum, _ = setup(wl)
    B.sparf_append(desc, aux, case.k_new, case.v_new, case.seq_lens)
    out, sel, alpha = run_decode(case, desc, aux, 16, 1024, 4, torch.float32)
    ref, _ = H.gpu_step(case, out_dtype=torch.float32, append=False)
    assert (out - ref).abs().max() <= 1e-5
    assert (alpha - 1).abs().max() <= 1e-5
    for b in range(2):
        L = int(case.seq_lens[b])
        assert torch.equal(sel[b, :, :L].cpu(), torch.arange(L, dtype=torch.int32).expand(4, L))


def test_sparf_empty_and_mixed_lengths():
    wl = W.Workload("sparf_mixed", 4, 2, 2, 128, 600, seed=405)
    case, desc, aux, kt, vsum, _ = setup(wl)
    case.seq_lens = torch.tensor([0, 601, 1, -2], dtype=torch.int32, device=DEV)
    B.sparf_build(desc, aux, (case.seq_lens - 1).contiguous(), 2, 128)
    B.sparf_append(desc, aux, case.k_new, case.v_new, case.seq_lens)
    out, sel, alpha = run_decode(case, desc, aux, 16, 50, 2, torch.float32, max_len=601)
    check_against_oracle(case, out, sel, alpha, 16, 50, 2)
    assert torch.equal(out[2].view(torch.int32), case.v_new[2].float().view(torch.int32))   # L = 1


def test_sparf_13b_shape_one_eighth(options):
    """The 13B-shaped layer at the paper's 1/8 compression (r = 16 of 128 columns,
    k = 256 of 4097 rows, 16 most recent kept): sampled heads against the oracle."""
    wl = W.WORKLOADS["mha13b_4k"]
    pairs = [(0, 0), (3, 17), (15, 39), (7, 8), (11, 21), (9, 30)]
    sparf_step(wl, 16, 256, 16, torch.float16, pairs=pairs)


def sampled_full_size_step(wl, r, k, l, pairs, kt_page=None):
    """A whole layer of a bench workload through instattn_sparf_append_decode (the call
    bench.py times); sampled heads against the oracle, their rows gathered on the device."""
    case, desc, aux, kt, vsum, _ = setup(wl, kt_page=kt_page)
    out, sel, alpha = run_decode(case, desc, aux, r, k, l, torch.float16, fused_append=True)
    lens = H.host(case.seq_lens)
    for b, h in pairs:
        hk, L = h // wl.group, int(lens[b])
        Kr, Vr = device_rows(case, b, hk, L)
        # the appended row, the column copy and the V sum of this (sequence, KV head)
        assert np.array_equal(Kr[L - 1].view(np.uint16), H.host(case.k_new[b, hk]).view(np.uint16))
        assert np.array_equal(Vr[L - 1].view(np.uint16), H.host(case.v_new[b, hk]).view(np.uint16))
        cols = column_copy(kt, case.kt_table, b, L)[hk].cpu().numpy()
        assert np.array_equal(cols.view(np.uint16), np.ascontiguousarray(Kr.T).view(np.uint16))
        np.testing.assert_allclose(vsum[b, hk].double().cpu().numpy(), Vr.astype(np.float64).sum(axis=0),
                                   rtol=0, atol=4e-2)
    return check_against_oracle(case, out, sel, alpha, r, k, l, pairs,
                                rows_of=lambda b, hk, L: device_rows(case, b, hk, L))


def test_sparf_32k_shape_full_size_samples():
    """8 x 40 heads x 32K: the long-row pipeline at the size bench.py times it."""
    pairs = [(0, 0), (7, 39), (3, 17), (5, 8)]
    sampled_full_size_step(W.WORKLOADS["mha13b_32k"], 16, 2048, 16, pairs)


def test_sparf_ragged_paged_full_size_samples():
    """64 ragged sequences of 1K-16K tokens, cache in 16-token pages, column copy in
    256-token pages: the launch configuration of bench.py --workload ragged_paged --sparf."""
    wl = W.WORKLOADS["ragged_paged"]
    lens = W.draw_seq_lens(wl, "cpu")
    order = torch.argsort(lens)
    pairs = [(int(order[0]), 3), (int(order[-1]), 39), (int(order[len(order) // 2]), 20), (5, 11)]
    sampled_full_size_step(wl, 16, 1024, 16, pairs, kt_page=256)


def _drawn_configs(n, seed):
    """Seeded draw of shapes and parameters across everything the entry points accept."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        D = int(rng.choice([64, 128]))
        G = int(rng.choice([1, 1, 2, 4, 8]))
        Hkv = int(rng.choice([1, 2, 3]))
        long_row = i % 5 == 4
        S = int(rng.integers(8200, 13000)) if long_row else int(rng.integers(0, 3000))
        paged = bool(rng.integers(0, 2))
        kt_page = [None, 8, 64, 256][int(rng.integers(0, 4))]
        r = int(rng.integers(1, D + 1)) if i % 3 == 0 else int(rng.choice([D // 16, D // 8, D // 4]))
        k = int(rng.integers(1, 2 * S + 3))
        l = int(rng.integers(0, 41))
        f16 = bool(rng.integers(0, 2))
        fused = bool(rng.integers(0, 2))
        out.append((i, D, G, Hkv, S, paged, kt_page, r, k, l, f16, fused))
    return out


@pytest.mark.parametrize("cfg", _drawn_configs(20, 20240917), ids=lambda c: "cfg%d" % c[0])
def test_sparf_drawn_configurations(cfg):
    i, D, G, Hkv, S, paged, kt_page, r, k, l, f16, fused = cfg
    wl = W.Workload("sparf_drawn%d" % i, 2, G * Hkv, Hkv, D, S, seq_len_min=max(0, S // 3), paged=paged,
                    page_size=16, seed=600 + i)
    sparf_step(wl, r, k, l, torch.float16 if f16 else torch.float32, kt_page=kt_page, fused_append=fused)


def _drawn_forms(n, seed):
    """Seeded draw of shapes up to 40K positions together with a setting of every switch
    that forces a form of the decode (None: the host's own choice)."""
    rng = np.random.default_rng(seed)
    names = ("INSTATTN_SPARF_WIDE", "INSTATTN_SPARF_DISTRIBUTED", "INSTATTN_SPARF_SPLIT_TAIL",
             "INSTATTN_SPARF_THREE_LAUNCHES")
    out = []
    for i in range(n):
        D = int(rng.choice([64, 128]))
        G = int(rng.choice([1, 1, 2, 4]))
        Hkv = int(rng.choice([1, 2, 3]))
        top = int(rng.choice([3000, 8192, 13000, 18432, 30000, 40000]))
        S = int(rng.integers(top // 2, top))
        kt_page = [None, 8, 64, 256, 1024][int(rng.integers(0, 5))]
        r = int(rng.choice([D // 16, D // 8, D // 4]))
        k = int(rng.integers(1, 2 * S + 3)) if i % 3 == 0 else max(1, S // int(rng.choice([8, 16, 32])))
        env = {}
        for name in names:
            v = int(rng.integers(0, 3))
            if v < 2 and not (name == "INSTATTN_SPARF_THREE_LAUNCHES" and v == 0):
                env[name] = str(v)
        out.append((i, D, G, Hkv, S, bool(rng.integers(0, 2)), kt_page, r, k, int(rng.integers(0, 41)),
                    bool(rng.integers(0, 2)), bool(rng.integers(0, 2)), env))
    return out


@pytest.mark.parametrize("cfg", _drawn_forms(30, 20240920), ids=lambda c: "cfg%d" % c[0])
def test_sparf_drawn_configurations_in_forced_forms(options, cfg):
    i, D, G, Hkv, S, paged, kt_page, r, k, l, f16, fused, env = cfg
    for name, value in env.items():
        options.setenv(name, value)
    wl = W.Workload("sparf_form%d" % i, 2, G * Hkv, Hkv, D, S, seq_len_min=int(S * 0.4), paged=paged,
                    page_size=16, seed=700 + i)
    sparf_step(wl, r, k, l, torch.float16 if f16 else torch.float32, kt_page=kt_page, fused_append=fused)


def test_calls_on_two_streams_at_once_do_not_disturb_each_other(options):
    """The library keeps no state between calls: a dense decode and a SparF decode of long
    rows (six launches), each on a stream and a workspace of its own, issued alternately so
    that they overlap on the GPU, give the bits they give one after the other."""
    options.setenv("INSTATTN_SPARF_DISTRIBUTED", "1")
    wl_s = W.Workload("two_streams_sparf", 1, 4, 4, 128, 40000, seed=811)
    wl_d = W.Workload("two_streams_dense", 3, 16, 2, 128, 9000, seq_len_min=3000, seed=812)
    case, desc, aux, _, _, _ = setup(wl_s)
    B.sparf_append(desc, aux, case.k_new, case.v_new, case.seq_lens)
    r, k, l = 16, 2500, 16
    want_out, want_sel, want_alpha = run_decode(case, desc, aux, r, k, l, torch.float16)
    dcase = W.make_case(wl_d, DEV, poison=True)
    ddesc = B.kv_desc(dcase.k_cache, dcase.v_cache, dcase.page_table)
    B.kv_append(ddesc, dcase.k_new, dcase.v_new, dcase.seq_lens)
    dmax = int(dcase.seq_lens.max())
    dws = B.alloc_workspace(wl_d.batch, wl_d.num_q_heads, wl_d.num_kv_heads, 128, dmax, DEV)
    dout = torch.empty(wl_d.batch, wl_d.num_q_heads, 128, dtype=torch.float16, device=DEV)
    B.decode(dcase.q, ddesc, dcase.seq_lens, wl_d.num_kv_heads, dcase.scale, dout, dws, dmax)
    torch.cuda.synchronize()
    want_dense = dout.clone()
    assert torch.isfinite(want_out.float()).all(), torch.isfinite(want_out.float()).all(dim=2).tolist()
    assert torch.isfinite(want_dense.float()).all(), torch.isfinite(want_dense.float()).all(dim=2).tolist()

    smax = int(case.seq_lens.max())
    sws = torch.empty(B.sparf_workspace_size(1, 4, 128, smax, k), dtype=torch.uint8, device=DEV)
    reps = 6
    souts = torch.full((reps, 1, 4, 128), float("nan"), dtype=torch.float16, device=DEV)
    ssels = torch.full((reps, 1, 4, k), -1, dtype=torch.int32, device=DEV)
    salphas = torch.full((reps, 1, 4), float("nan"), dtype=torch.float32, device=DEV)
    douts = torch.full((reps,) + tuple(dout.shape), float("nan"), dtype=torch.float16, device=DEV)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for s_ in (s1, s2):
        s_.wait_stream(torch.cuda.current_stream())
    for i in range(reps):
        with torch.cuda.stream(s1):
            B.sparf_decode(case.q, desc, aux, case.seq_lens, wl_s.num_kv_heads, case.scale, r, k, l,
                           souts[i], sws, smax, sel_rows=ssels[i], alpha=salphas[i])
        with torch.cuda.stream(s2):
            B.decode(dcase.q, ddesc, dcase.seq_lens, wl_d.num_kv_heads, dcase.scale, douts[i], dws, dmax)
    torch.cuda.synchronize()
    for i in range(reps):
        assert torch.equal(souts[i].view(torch.int16), want_out.view(torch.int16)), i
        assert torch.equal(ssels[i], want_sel), i
        assert torch.equal(salphas[i].view(torch.int32), want_alpha.view(torch.int32)), i
        assert torch.equal(douts[i].view(torch.int16), want_dense.view(torch.int16)), i


@pytest.mark.parametrize("seq_len,k", [(3000, 200), (20000, 1500)])
def test_sparf_page_ids_outside_the_pools_are_pulled_into_them(seq_len, k):
    """Both page tables are device data: ids outside their pools are replaced by the
    pool's last page in the kernels (one-launch form and pipeline), and the step gives what it gives
    for tables with those ids replaced."""
    wl = W.Workload("sparf_bad_pages", 2, 3, 3, 128, seq_len, seq_len_min=seq_len // 2, paged=True, seed=913)
    res = {}
    for kind in ("bad", "clamped"):
        case, desc, aux, kt, vsum, _ = setup(wl, kt_page=64)
        L = int(case.seq_lens[1])
        for table, page, pool in ((case.page_table, 16, case.k_cache.shape[0]), (case.kt_table, 64, kt.shape[0])):
            used = (L + page - 1) // page
            idx = torch.randperm(used, generator=torch.Generator().manual_seed(3))[:6].to(DEV)
            table[1, idx[:2]] = -1
            table[1, idx[2:4]] = 2**31 - 1
            table[1, idx[4:]] = pool + 9
            table[1, used - 1] = -3
            if kind == "clamped":
                table[(table < 0) | (table >= pool)] = pool - 1
        out, sel, alpha = run_decode(case, desc, aux, 16, k, 16, torch.float16, fused_append=True)
        res[kind] = (out.view(torch.int16), sel, alpha.view(torch.int32), case.k_cache.view(torch.int16).clone(),
                     case.v_cache.view(torch.int16).clone(), kt.view(torch.int16).clone(), vsum.view(torch.int32).clone())
    for x, y in zip(res["bad"], res["clamped"]):
        assert torch.equal(x, y)


@pytest.mark.parametrize("seq_len,k,distributed", [(3000, 200, None), (20000, 1500, "0"), (20000, 1500, "1"),
                                                   (70000, 3000, "0"), (70000, 3000, "1")])
def test_sparf_scores_that_are_not_numbers_stay_inside_their_head(options, seq_len, k, distributed):
    """NaN and infinities in K, V or q make scores the selection cannot order sensibly.
    Every address that depends on a score is bounded all the same: nothing is written
    outside the outputs (guard band, untouched neighbours), the kept positions of the
    spoilt heads lie in the row, and the other heads give the bits of the clean run."""
    if distributed is not None:
        options.setenv("INSTATTN_SPARF_DISTRIBUTED", distributed)
    wl = W.Workload("sparf_nonfinite", 2, 4, 4, 128, seq_len, seq_len_min=seq_len - 100, seed=977)
    res = {}
    for kind in ("clean", "spoilt"):
        case, desc, aux, kt, vsum, _ = setup(wl)
        if kind == "spoilt":
            L0 = int(case.seq_lens[0])
            rows = torch.randperm(L0 - 1, generator=torch.Generator().manual_seed(9))[:60].to(DEV)
            vals = torch.tensor([float("nan"), float("inf"), -float("inf")], dtype=torch.float16, device=DEV)
            # head 0 of sequence 0: spoilt keys (both copies) and values; head 1: spoilt query
            case.k_cache[0, 0, rows, ::7] = vals[torch.arange(60, device=DEV) % 3, None]
            kt[0, 0, :, rows] = case.k_cache[0, 0, rows].t()
            case.v_cache[0, 0, rows[:5], 3] = float("nan")
            case.q[0, 1, 5] = float("nan")
            case.q[0, 1, 77] = float("inf")
        out, sel, alpha = run_decode(case, desc, aux, 16, k, 16, torch.float16, fused_append=True)
        res[kind] = (out, sel, alpha, case.seq_lens.clone())
    out, sel, alpha, lens = res["spoilt"]
    for h in (0, 1):
        L0 = int(lens[0])
        assert int(sel[0, h, :min(k, L0)].min()) >= 0 and int(sel[0, h, :min(k, L0)].max()) < L0
    clean_out, clean_sel, clean_alpha, _ = res["clean"]
    for b, h in [(0, 2), (0, 3), (1, 0), (1, 1), (1, 2), (1, 3)]:
        assert torch.equal(out[b, h].view(torch.int16), clean_out[b, h].view(torch.int16)), (b, h)
        assert torch.equal(sel[b, h], clean_sel[b, h]), (b, h)
        assert torch.equal(alpha[b, h].view(torch.int32), clean_alpha[b, h].view(torch.int32)), (b, h)


@pytest.mark.parametrize("seq_len,k", [(3000, 200), (20000, 1200)])
def test_sparf_paged_pool_with_k_and_v_of_a_page_adjacent(seq_len, k):
    wl = W.Workload("sparf_kv_adjacent", 2, 3, 3, 128, seq_len, seq_len_min=seq_len // 2, paged=True,
                    kv_adjacent=True, seed=914)
    sparf_step(wl, 16, k, 16, torch.float16, kt_page=256, fused_append=True)


def test_probe_read_columns_runs_inside_the_copy():
    """The measurement aid reads r columns of every row of a component-major copy: the
    neighbours of the copy (NaN-filled guard rows in front and behind) stay what they are
    and the call returns; its argument checks run on the host (tests/test_abi_host.py)."""
    for D, cap, positions, r in [(64, 264, 256, 8), (128, 4112, 4096, 16), (128, 2056, 8, 128), (64, 40000, 39992, 3)]:
        whole = torch.full((2 + 2, 3, D, cap), float("nan"), dtype=torch.float16, device=DEV)
        kt = whole[1:3]
        kt.normal_()
        before = whole.clone()
        sink = torch.zeros(4096, dtype=torch.int32, device=DEV)
        B.probe_read_columns(kt, r, positions, sink)
        torch.cuda.synchronize()
        assert torch.equal(whole.view(torch.int16), before.view(torch.int16))


def test_sparf_is_deterministic():
    wl = W.Workload("sparf_det", 2, 4, 4, 128, 3000, seed=406)
    case, desc, aux, kt, vsum, _ = setup(wl)
    B.sparf_append(desc, aux, case.k_new, case.v_new, case.seq_lens)
    a = run_decode(case, desc, aux, 16, 200, 8, torch.float16)
    b = run_decode(case, desc, aux, 16, 200, 8, torch.float16)
    assert all(torch.equal(x, y) for x, y in zip(a, b))


def test_sparf_ties_go_to_the_lower_position():
    """Identical keys: every score ties, so the kept rows are the first k - l and the
    last l positions, and the output is alpha * mean(V kept) + (1 - alpha) * mean(V)."""
    wl = W.Workload("sparf_ties", 1, 2, 2, 128, 299, seed=407)
    case, desc, aux, kt, vsum, _ = setup(wl)
    case.k_cache[:] = case.k_cache[:, :, :1]
    case.k_new[:] = case.k_cache[:, :, 0]
    B.sparf_build(desc, aux, (case.seq_lens - 1).contiguous(), 2, 128)
    B.sparf_append(desc, aux, case.k_new, case.v_new, case.seq_lens)
    out, sel, alpha = run_decode(case, desc, aux, 16, 40, 6, torch.float32)
    want = torch.cat([torch.arange(34), torch.arange(294, 300)]).to(torch.int32)
    assert torch.equal(sel[0, 0].cpu(), want) and torch.equal(sel[0, 1].cpu(), want)
    assert (alpha - 40 / 300).abs().max() < 1e-6
    V = case.v_cache[0, :, :300].double()
    ref = (40 / 300) * V[:, want.long()].mean(dim=1) + (1 - 40 / 300) * V.mean(dim=1)
    assert (out[0].double() - ref).abs().max() < 1e-5


# ------------------------------------------------------------------ HIP graph replay
@pytest.mark.parametrize("form", ["one_launch", "one_launch_512", "pipeline_tail", "pipeline_distributed"])
def test_sparf_decode_replayed_from_a_hip_graph(options, form):
    """The launches of a SparF decode recorded into a HIP graph, in each form the host can
    pick: every replay — workspace overwritten and unrelated eager work in between —
    gives the oracle's result and bit for bit the eager one (nothing in the path
    allocates, synchronises or depends on what the workspace held before)."""
    seq_len, k = {"one_launch": (3000, 200), "one_launch_512": (12000, 700), "pipeline_tail": (12000, 200),
                  "pipeline_distributed": (20000, 1500)}[form]
    options.setenv("INSTATTN_SPARF_WIDE", "1" if form == "one_launch_512" else "0")
    options.setenv("INSTATTN_SPARF_DISTRIBUTED", "1" if form == "pipeline_distributed" else "0")
    wl = W.Workload("sparf_graph", 2, 3, 3, 128, seq_len, seq_len_min=seq_len // 2, paged=True, page_size=16,
                    seed=440)
    case, desc, aux, kt, vsum, _ = setup(wl, kt_page=256)
    B.sparf_append(desc, aux, case.k_new, case.v_new, case.seq_lens)
    r, l = 16, 16
    Bn, Hq, D = case.q.shape
    max_len = int(case.seq_lens.max())
    ws = torch.empty(B.sparf_workspace_size(Bn, Hq, D, max_len, k), dtype=torch.uint8, device=DEV)
    out = torch.empty(Bn, Hq, D, dtype=torch.float32, device=DEV)
    sel = torch.empty(Bn, Hq, k, dtype=torch.int32, device=DEV)
    alpha = torch.empty(Bn, Hq, dtype=torch.float32, device=DEV)

    def step():
        B.sparf_decode(case.q, desc, aux, case.seq_lens, wl.num_kv_heads, case.scale, r, k, l, out, ws,
                       max_len, sel_rows=sel, alpha=alpha)

    def scrub():
        ws.fill_(0xFF)
        out.fill_(float("nan"))
        sel.fill_(-1)
        alpha.fill_(float("nan"))

    scrub()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    eager = (out.clone(), sel.clone(), alpha.clone())
    check_against_oracle(case, *eager, r, k, l)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    other = W.make_case(W.Workload("sparf_graph_other", 1, 4, 4, 64, 700, seed=441), DEV)
    for rep in range(3):
        scrub()
        H.gpu_step(other)                      # unrelated eager work between the replays
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int32), eager[0].view(torch.int32)), rep
        assert torch.equal(sel, eager[1]) and torch.equal(alpha.view(torch.int32), eager[2].view(torch.int32)), rep
