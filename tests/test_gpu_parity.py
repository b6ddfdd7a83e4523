"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Bit-exact for the appended cache rows; max-abs error
<= 2e-3 (fp16 output) / 1e-4 (fp32 output) for attention rows."""
import dataclasses
import math

import numpy as np
import pytest
import torch

from paper_2409_04992_amd import binding as B
from paper_2409_04992_amd import workloads as W

import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def small(name, **kw):
    return W.scaled_down(W.WORKLOADS[name], **kw)


def full_check(wl, poison=True, out_dtype=None, lens=None, capacity=None, fused=False):
    """Whole-tensor comparison (sizes the C oracle finishes in seconds)."""
    case = W.make_case(wl, DEV, poison=poison, capacity=capacity)
    if lens is not None:
        case.seq_lens = torch.tensor(lens, dtype=torch.int32, device=DEV)
    want_out, want_lse, want_k, want_v = H.oracle_step(case)
    out, lse = H.gpu_step(case, out_dtype=out_dtype, fused=fused)
    # appended caches: bit-exact everywhere (NaN poison included, so compare bit patterns)
    assert np.array_equal(H.host(case.k_cache).view(np.uint16), want_k.view(np.uint16))
    assert np.array_equal(H.host(case.v_cache).view(np.uint16), want_v.view(np.uint16))
    return H.assert_close(out, lse, want_out, want_lse, wl.name, lse_tol=H.lse_tol(wl.group, out.dtype))


# ------------------------------------------------------------------ the five configurations
@pytest.mark.parametrize("fused", [False, True])
def test_config1_tiny_mha_fp32_out(fused):
    err = full_check(W.WORKLOADS["tiny_mha"], fused=fused)
    assert err < 1e-4


@pytest.mark.parametrize("fused", [False, True])
def test_config2_mha13b_4k_full(fused):
    full_check(W.WORKLOADS["mha13b_4k"], fused=fused)


def sampled_check(wl, pairs, poison, layer=0, fused=False):
    case = W.make_case(wl, DEV, layer=layer, poison=poison)
    out, lse = H.gpu_step(case, fused=fused)
    rows = H.oracle_rows(case, pairs)          # caches already hold the appended row
    tol = H.TOL[out.dtype]
    worst = 0.0
    for (b, h), (want, want_lse) in rows.items():
        got = out[b, h].double().cpu().numpy()
        err = np.abs(got - want).max()
        worst = max(worst, err)
        assert err <= tol, "%s (b=%d,h=%d): %.3e" % (wl.name, b, h, err)
        assert abs(float(lse[b, h]) - want_lse) <= H.lse_tol(wl.group, out.dtype) * (1 + 0.01 * abs(want_lse))
    assert torch.isfinite(out.float()).all()
    return case, out, worst


@pytest.mark.parametrize("fused", [False, True])
def test_config3_mha13b_32k_full_size(fused):
    """8 x 40 heads x 32K at full size (5.4 GB of KV): every output row and every byte of
    the caches against the oracle, which works on host copies taken before the step."""
    full_check(W.WORKLOADS["mha13b_32k"], fused=fused)


@pytest.mark.parametrize("fused", [False, True])
def test_config4_ragged_paged_full_size(fused):
    """The ragged paged batch at full size (11.4 GB of KV in 16-token pages behind a
    shuffled table), in the launch configuration the bench times (the split pass walks the
    device-built list of units): every output row, every byte of both pools."""
    wl = W.WORKLOADS["ragged_paged"]
    lens = W.draw_seq_lens(wl)
    assert lens.min() >= 1025 and lens.max() <= 16385 and len(set(lens.tolist())) > 32
    assert B.decode_launches(wl.batch, wl.num_q_heads, wl.num_kv_heads, wl.head_dim, int(lens.max()), fused,
                             paged=True)["unit_list"]
    full_check(wl, fused=fused)


@pytest.mark.parametrize("fused", [False, True])
def test_config5_gqa_layer_full_shape(fused):
    """One layer of the 80-layer GQA step at its real shape (2.1 GB of KV): whole tensors."""
    wl = dataclasses.replace(W.WORKLOADS["gqa70b_16k"], layers=1)
    full_check(wl, fused=fused)


def test_config5_all_80_layers_resident():
    """The 80-layer step as the bench runs it: every layer's cache resident (172 GB), one
    shared length array and workspace, the fused call per layer on one stream.  Every
    layer is checked: its appended rows bit for bit, and the output rows of two
    (sequence, head) pairs, a different couple per layer, against the oracle."""
    wl = W.WORKLOADS["gqa70b_16k"]
    assert wl.layers == 80
    torch.cuda.empty_cache()
    cases = [W.make_case(wl, DEV, layer=i, poison=True) for i in range(wl.layers)]
    lens = cases[0].seq_lens
    max_len = int(lens.max().item())
    ws = B.alloc_workspace(wl.batch, wl.num_q_heads, wl.num_kv_heads, wl.head_dim, max_len, DEV)
    outs = torch.full((wl.layers, wl.batch, wl.num_q_heads, wl.head_dim), float("nan"),
                      dtype=torch.float16, device=DEV)
    lses = torch.full((wl.layers, wl.batch, wl.num_q_heads), float("nan"), dtype=torch.float32, device=DEV)
    for i, c in enumerate(cases):
        assert torch.equal(c.seq_lens, lens)
        B.append_decode(c.q, c.k_new, c.v_new, B.kv_desc(c.k_cache, c.v_cache, None), lens,
                        wl.num_kv_heads, c.scale, outs[i], ws, max_len, lse=lses[i])
    torch.cuda.synchronize()
    assert torch.isfinite(outs.float()).all() and torch.isfinite(lses).all()
    tol, ltol = H.TOL[torch.float16], H.lse_tol(wl.group, torch.float16)
    for i, c in enumerate(cases):
        L = int(lens[0])
        assert torch.equal(c.k_cache[:, :, L - 1].view(torch.int16), c.k_new.view(torch.int16)), i
        assert torch.equal(c.v_cache[:, :, L - 1].view(torch.int16), c.v_new.view(torch.int16)), i
        pairs = [((7 * i + 3) % wl.batch, (13 * i + 5) % wl.num_q_heads),
                 ((11 * i) % wl.batch, (29 * i + 63) % wl.num_q_heads)]
        for (b, h), (want, want_lse) in H.oracle_rows(c, pairs).items():
            err = np.abs(outs[i, b, h].double().cpu().numpy() - want).max()
            assert err <= tol, "layer %d (b=%d,h=%d): %.3e" % (i, b, h, err)
            assert abs(float(lses[i, b, h]) - want_lse) <= ltol * (1 + 0.01 * abs(want_lse)), (i, b, h)
    del cases, outs, lses, ws
    torch.cuda.empty_cache()


@pytest.mark.parametrize("shape", ["mha_1m", "gqa_512k_paged", "mha64_600k"])
def test_one_very_long_sequence(shape):
    """A single sequence far beyond the measured configurations: hundreds of units per
    head (the merge takes its form for many units), page tables of tens of thousands of
    entries, row offsets of hundreds of MB."""
    wl = {
        "mha_1m": W.Workload("long_mha", 1, 2, 2, 128, 1 << 20, seed=431),
        "gqa_512k_paged": W.Workload("long_gqa", 1, 8, 1, 128, (1 << 19) + 77, paged=True, page_size=16, seed=432),
        "mha64_600k": W.Workload("long_mha64", 2, 1, 1, 64, 600_000, seq_len_min=400_000, out_dtype="f32", seed=433),
    }[shape]
    pairs = [(0, 0), (wl.batch - 1, wl.num_q_heads - 1)]
    sampled_check(wl, pairs, poison=True, fused=True)


@pytest.mark.parametrize("fused", [False, True])
def test_config5_gqa_scaled_down_full_check(fused):
    full_check(small("gqa70b_16k", batch=3, seq_len=1500, layers=1), fused=fused)


# ------------------------------------------------------------------ scaled-down recipes, whole tensors
@pytest.mark.parametrize("seq_len", [1, 2, 14, 15, 16, 17, 63, 64, 65, 255, 256, 257, 1000, 3000])
def test_mha_lengths_around_tile_and_chunk_edges(seq_len):
    full_check(small("mha13b_4k", batch=2, num_q_heads=3, num_kv_heads=3, seq_len=seq_len))


@pytest.mark.parametrize("seq_len", [1, 15, 16, 17, 31, 32, 33, 500, 2049])
def test_paged_lengths_around_page_edges(seq_len):
    wl = small("ragged_paged", batch=3, num_q_heads=2, num_kv_heads=2, seq_len=seq_len,
               seq_len_min=max(1, seq_len - 40))
    full_check(wl)


@pytest.mark.parametrize("head_dim,paged", [(64, False), (64, True), (128, False), (128, True)])
@pytest.mark.parametrize("out_dtype", [torch.float16, torch.float32])
def test_head_dims_layouts_output_types(head_dim, paged, out_dtype):
    wl = W.Workload("mix", 3, 4, 4, head_dim, 700, seq_len_min=300, paged=paged, seed=77)
    full_check(wl, out_dtype=out_dtype)


@pytest.mark.parametrize("group,head_dim", [(2, 128), (4, 64), (8, 128), (8, 64), (16, 128), (5, 128),
                                            (2, 64), (16, 64), (3, 64)])
@pytest.mark.parametrize("paged", [False, True])
def test_grouped_queries(group, head_dim, paged):
    wl = W.Workload("gqa", 2, 2 * group, 2, head_dim, 900, seq_len_min=100, paged=paged, seed=88)
    full_check(wl, out_dtype=torch.float32 if group == 8 else torch.float16)


@pytest.mark.parametrize("group,head_dim", [(17, 128), (32, 128), (40, 64), (64, 128), (71, 64)])
@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("fused", [False, True])
def test_groups_of_more_than_16_query_heads(group, head_dim, paged, fused):
    """Multi-query shapes: a group beyond the 16 rows of a matrix-core tile is shared out over
    several blocks per KV head, 16 heads each and the rest (17 = 16 + 1, 71 = 4 x 16 + 7);
    the fused call stores the new token in a launch of its own then."""
    wl = W.Workload("mqa", 2, 2 * group, 2, head_dim, 2500, seq_len_min=300, paged=paged, seed=89)
    full_check(wl, out_dtype=torch.float32 if group % 2 else torch.float16, fused=fused)


def test_empty_and_mixed_lengths():
    wl = small("mha13b_4k", batch=5, num_q_heads=2, num_kv_heads=2, seq_len=600)
    case = W.make_case(wl, DEV, poison=False)
    lens = [0, 1, 601, 300, -5]
    case.seq_lens = torch.tensor(lens, dtype=torch.int32, device=DEV)
    want_out, want_lse, want_k, want_v = H.oracle_step(case)
    out, lse = H.gpu_step(case, max_seq_len=601)
    assert np.array_equal(H.host(case.k_cache).view(np.uint16), want_k.view(np.uint16))
    H.assert_close(out, lse, want_out, want_lse, "mixed")
    assert torch.equal(out[0], torch.zeros_like(out[0])) and torch.isinf(lse[0]).all()
    assert torch.equal(out[4], torch.zeros_like(out[4]))


def test_all_sequences_empty_single_split():
    wl = small("tiny_mha", seq_len=100)
    case = W.make_case(wl, DEV)
    case.seq_lens = torch.zeros(wl.batch, dtype=torch.int32, device=DEV)
    out, lse = H.gpu_step(case, max_seq_len=64, append=False)
    assert torch.equal(out, torch.zeros_like(out)) and torch.isinf(lse).all() and (lse < 0).all()


def test_length_one_returns_v_row_bit_exact():
    wl = small("mha13b_4k", batch=4, num_q_heads=4, num_kv_heads=4, seq_len=0)
    case = W.make_case(wl, DEV)
    out, _ = H.gpu_step(case)          # L = 1: the appended token attends to itself
    assert torch.equal(out.view(torch.int16), case.v_new.view(torch.int16))


def test_lengths_beyond_max_seq_len_are_clamped():
    wl = small("mha13b_4k", batch=2, num_q_heads=2, num_kv_heads=2, seq_len=511)
    case = W.make_case(wl, DEV, capacity=512)
    H.gpu_step(case)                                   # append at 511
    ref, _ = H.gpu_step(case, append=False)
    case.seq_lens = torch.tensor([512 + 4000, 512], dtype=torch.int32, device=DEV)
    out, _ = H.gpu_step(case, append=False, max_seq_len=512)
    assert torch.equal(out, ref)


def _spoil(table, row, used, num_pages, seed):
    """Entries of the used part of one sequence's page-table row set to ids outside the pool."""
    idx = torch.randperm(used, generator=torch.Generator().manual_seed(seed))[:7].to(table.device)
    table[row, idx[:3]] = -1
    table[row, idx[3:5]] = 2**31 - 1
    table[row, idx[5:]] = num_pages + 5
    table[row, used - 1] = -7                       # the page the new token goes to


@pytest.mark.parametrize("group", [1, 4])
def test_page_ids_outside_the_pool_are_pulled_into_it(group):
    """A page table is device data the host cannot check: ids outside [0, num_pages) are
    replaced by the pool's last page in the kernels, so the step stays inside the pool and gives
    exactly what it gives for the table with those ids replaced; sequences with sound rows are untouched."""
    wl = W.Workload("bad_pages", 6, 4 * group, 4, 128, 3000, seq_len_min=1000, paged=True, seed=77)
    runs = {}
    for kind in ("sound", "bad", "clamped"):
        case = W.make_case(wl, DEV, poison=False)
        num_pages = case.k_cache.shape[0]
        if kind == "sound":
            # the spoilt ids land on the pool's first and last page: their owners see the new token's row
            hit = ((case.page_table == 0) | (case.page_table == num_pages - 1)).any(dim=1).tolist()
        if kind != "sound":
            _spoil(case.page_table, 1, (int(case.seq_lens[1]) + 15) // 16, num_pages, 5)
        if kind == "clamped":
            case.page_table[(case.page_table < 0) | (case.page_table >= num_pages)] = num_pages - 1
        for fused in (False, True):
            out, lse = H.gpu_step(case, fused=fused)   # the second step stores the same row again
            runs[kind, fused] = (out, lse, case.k_cache.clone(), case.v_cache.clone())
    for fused in (False, True):
        for x, y in zip(runs["bad", fused], runs["clamped", fused]):
            assert torch.equal(x.view(torch.int16) if x.dtype == torch.float16 else x.view(torch.int32),
                               y.view(torch.int16) if y.dtype == torch.float16 else y.view(torch.int32))
        others = [b for b in range(wl.batch) if b != 1 and not hit[b]]
        assert len(others) >= 3
        for b in others:
            assert torch.equal(runs["bad", fused][0][b].view(torch.int16), runs["sound", fused][0][b].view(torch.int16))


@pytest.mark.parametrize("group,head_dim", [(1, 128), (1, 64), (8, 128), (4, 64)])
@pytest.mark.parametrize("fused", [False, True])
def test_paged_pool_with_k_and_v_of_a_page_adjacent(group, head_dim, fused):
    """One pool [num_pages][Hkv][2][16][D]: K and V of a (page, head) are one contiguous 8 KB
    piece; the descriptor expresses it through the strides and two bases."""
    wl = W.Workload("kv_adjacent", 3, 2 * group, 2, head_dim, 2500, seq_len_min=200, paged=True,
                    kv_adjacent=True, seed=91)
    case = W.make_case(wl, DEV)
    assert case.k_cache.stride() == case.v_cache.stride() and not case.k_cache.is_contiguous()
    assert case.v_cache.data_ptr() - case.k_cache.data_ptr() == 16 * head_dim * 2
    full_check(wl, fused=fused)


def test_strided_cache_views():
    """Caches that are slices of larger tensors: strides larger than the dense ones."""
    wl = small("mha13b_4k", batch=2, num_q_heads=3, num_kv_heads=3, seq_len=333)
    case = W.make_case(wl, DEV, poison=True)
    want_out, want_lse, want_k, want_v = H.oracle_step(case)
    big_k = torch.full((2, 5, 400, 160), float("nan"), dtype=torch.float16, device=DEV)
    big_v = torch.full((2, 5, 400, 160), float("nan"), dtype=torch.float16, device=DEV)
    cap = case.k_cache.shape[2]
    big_k[:, 1:4, :cap, 16:144] = case.k_cache
    big_v[:, 1:4, :cap, 16:144] = case.v_cache
    case.k_cache, case.v_cache = big_k[:, 1:4, :cap, 16:144], big_v[:, 1:4, :cap, 16:144]
    out, lse = H.gpu_step(case)
    H.assert_close(out, lse, want_out, want_lse, "strided")
    assert np.array_equal(H.host(case.k_cache.contiguous()).view(np.uint16), want_k.view(np.uint16))
    assert torch.isnan(big_k[:, 0]).all() and torch.isnan(big_k[..., :16]).all()


@pytest.mark.parametrize("chunk", [128, 256, 384, 1024, 100000])
def test_result_does_not_depend_on_the_split(options, chunk):
    wl = small("mha13b_4k", batch=2, num_q_heads=4, num_kv_heads=4, seq_len=2500)
    case = W.make_case(wl, DEV)
    want_out, want_lse, _, _ = H.oracle_step(case)
    options.setenv("INSTATTN_CHUNK", str(chunk))
    assert B.decode_plan(2, 4, 4, 128, 2501)[0] == min((chunk + 127) // 128 * 128, 2560)
    out, lse = H.gpu_step(case, out_dtype=torch.float32)
    H.assert_close(out, lse, want_out, want_lse, "chunk %d" % chunk)


def test_deterministic_and_heads_independent():
    wl = small("mha13b_4k", batch=2, num_q_heads=8, num_kv_heads=8, seq_len=1200)
    case = W.make_case(wl, DEV)
    a, la = H.gpu_step(case)
    b, lb = H.gpu_step(case, append=False)
    assert torch.equal(a, b) and torch.equal(la, lb)
    # heads 4..7 alone (head-level sharding, Sec. IV-D "Scale To CSD Array"): same rows
    half = dataclasses.replace(case, q=case.q[:, 4:].contiguous(), k_cache=case.k_cache[:, 4:],
                               v_cache=case.v_cache[:, 4:], k_new=case.k_new[:, 4:].contiguous(),
                               v_new=case.v_new[:, 4:].contiguous(),
                               wl=dataclasses.replace(wl, num_q_heads=4, num_kv_heads=4))
    c, _ = H.gpu_step(half, append=False)
    assert (a[:, 4:].float() - c.float()).abs().max() <= 1e-3


def test_head_sharded_equals_unsharded_bit_for_bit_under_one_plan(options):
    """Head-level sharding (Sec. IV-D "Scale To CSD Array"): with the same unit length on
    both sides a shard's rows are the unsharded rows bit for bit, for both kernels."""
    options.setenv("INSTATTN_CHUNK", 384)
    for hq, hkv in ((8, 8), (16, 4)):
        wl = small("mha13b_4k", batch=3, num_q_heads=hq, num_kv_heads=hkv, seq_len=1500, seq_len_min=200)
        case = W.make_case(wl, DEV)
        assert B.decode_plan(3, hq, hkv, 128, 1501) == B.decode_plan(3, hq // 2, hkv // 2, 128, 1501) == (384, 4)
        a, la = H.gpu_step(case)
        half = dataclasses.replace(case, q=case.q[:, hq // 2:].contiguous(), k_cache=case.k_cache[:, hkv // 2:],
                                   v_cache=case.v_cache[:, hkv // 2:], k_new=case.k_new[:, hkv // 2:].contiguous(),
                                   v_new=case.v_new[:, hkv // 2:].contiguous(),
                                   wl=dataclasses.replace(wl, num_q_heads=hq // 2, num_kv_heads=hkv // 2))
        c, lc = H.gpu_step(half, append=False)
        assert torch.equal(a[:, hq // 2:], c) and torch.equal(la[:, hq // 2:], lc)


@pytest.mark.parametrize("chunk", [384, 100000])
@pytest.mark.parametrize("shape", ["mha_paged", "mha_contiguous", "gqa_paged", "gqa_d64"])
def test_compacted_unit_list_equals_the_grid_bit_for_bit(options, shape, chunk):
    """A ragged batch through the device-built list of units and through the plain
    (sequence, split) grid: same plan, same arithmetic per unit, so the same bits - and
    both agree with the oracle.  Lengths include empty sequences, full units, single rows
    behind a unit boundary and the longest length the cache holds; with units of 384 rows
    and with whole sequences as units (the list then orders the sequences by length)."""
    hq, hkv, dim, paged = {"mha_paged": (5, 5, 128, True), "mha_contiguous": (3, 3, 128, False),
                           "gqa_paged": (8, 2, 128, True), "gqa_d64": (6, 3, 64, False)}[shape]
    wl = small("ragged_paged", batch=9, num_q_heads=hq, num_kv_heads=hkv, head_dim=dim, seq_len=1700,
               seq_len_min=100, paged=paged)
    lens = [0, 384, 385, 1, 1701, 768, 1152, 1153, 700]
    options.setenv("INSTATTN_CHUNK", chunk)
    res = []
    for compact in (0, 1):
        options.setenv("INSTATTN_COMPACT", compact)
        assert B.decode_launches(9, hq, hkv, dim, 1701, paged=paged) == \
            {"append": False, "unit_list": bool(compact), "split_pass": True, "merge": chunk == 384}
        for fused in (False, True):
            case = W.make_case(wl, DEV, poison=True, lens=lens)
            want_out, want_lse, want_k, want_v = H.oracle_step(case)
            out, lse = H.gpu_step(case, fused=fused, out_dtype=torch.float32, max_seq_len=1701)
            H.assert_close(out, lse, want_out, want_lse, shape)
            assert np.array_equal(H.host(case.k_cache).view(np.uint16), want_k.view(np.uint16))
            assert np.array_equal(H.host(case.v_cache).view(np.uint16), want_v.view(np.uint16))
            res.append((out, lse))
    for out, lse in res[1:]:
        assert torch.equal(out, res[0][0]) and torch.equal(lse, res[0][1])


def test_compacted_unit_list_with_a_bound_below_the_lengths(options):
    """max_seq_len below some lengths: those sequences are cut off there, the new token is
    still stored at its own position (inside the capacity), and the list holds exactly the
    units of the cut-off lengths."""
    wl = small("ragged_paged", batch=6, num_q_heads=4, num_kv_heads=4, seq_len=1500, seq_len_min=300, paged=True)
    options.setenv("INSTATTN_CHUNK", 256)
    outs = []
    for compact in (0, 1):
        options.setenv("INSTATTN_COMPACT", compact)
        case = W.make_case(wl, DEV)
        k_before = case.k_cache.clone()
        out, lse = H.gpu_step(case, fused=True, max_seq_len=900)
        outs.append((out, lse, case.k_cache.clone()))
        assert not torch.equal(case.k_cache, k_before)
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
    assert torch.equal(outs[0][2].view(torch.int16), outs[1][2].view(torch.int16))


@pytest.mark.parametrize("ring", [0, 1])
@pytest.mark.parametrize("shape", ["d128", "d64", "paged", "paged_d64", "one_long_row", "short_rows"])
def test_both_forms_of_the_vector_alu_pass(options, shape, ring):
    """The host picks the form of the vector-ALU split pass by the size of the launch (tiles
    through an LDS ring for large ones, two register tiles for small ones); here every shape
    goes through both, with the append fused in and not, against the oracle: ragged lengths,
    both layouts and head dims, a row of many units, rows shorter than one tile."""
    wl = {"d128": W.Workload("form_d128", 3, 5, 5, 128, 3000, seq_len_min=100, seed=301),
          "d64": W.Workload("form_d64", 3, 5, 5, 64, 3000, seq_len_min=100, seed=302, out_dtype="f32"),
          "paged": W.Workload("form_paged", 4, 3, 3, 128, 2500, seq_len_min=1, paged=True, seed=303),
          "paged_d64": W.Workload("form_paged64", 4, 3, 3, 64, 2500, seq_len_min=1, paged=True, page_size=32, seed=304),
          "one_long_row": W.Workload("form_long", 1, 2, 2, 128, 40000, seed=305),
          "short_rows": W.Workload("form_short", 6, 4, 4, 128, 40, seq_len_min=1, seed=306)}[shape]
    options.setenv("INSTATTN_MHA_RING", ring)
    for fused in (False, True):
        full_check(wl, fused=fused)


def test_dominant_score_large_values_fp16_rounding():
    """One key far along q: the row equals that v row (values of a few units), and
    the fp16 output is within one fp16 ulp of the oracle rounded to fp16."""
    wl = small("mha13b_4k", batch=1, num_q_heads=2, num_kv_heads=2, seq_len=700, head_scale=False)
    case = W.make_case(wl, DEV)
    j = 123
    case.k_cache[0, :, j] = (case.q[0].float() * 3.0).half()
    want_out, want_lse, _, _ = H.oracle_step(case)
    out, lse = H.gpu_step(case)
    H.assert_close(out, lse, want_out, want_lse, "dominant")
    rounded = want_out.astype(np.float16).astype(np.float64)
    assert np.abs(out.double().cpu().numpy() - rounded).max() <= 2 ** -9


def test_append_bit_patterns_and_untouched_rows():
    """Arbitrary 16-bit patterns (NaN payloads, denormals) survive the append; no
    other byte of the cache changes; out-of-range lengths store nothing."""
    g = torch.Generator().manual_seed(5)
    Bn, Hkv, cap, D = 6, 3, 48, 128
    mk = lambda *s: torch.randint(0, 65536, s, generator=g, dtype=torch.int32).to(torch.uint16) \
        .view(torch.float16).to(DEV)
    k, v, kn, vn = mk(Bn, Hkv, cap, D), mk(Bn, Hkv, cap, D), mk(Bn, Hkv, D), mk(Bn, Hkv, D)
    lens = [1, 48, 17, 0, 49, -1]
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    k0, v0 = k.clone(), v.clone()
    B.kv_append(B.kv_desc(k, v), kn, vn, sl)
    torch.cuda.synchronize()
    ek, ev = k0.clone(), v0.clone()
    for b, L in enumerate(lens):
        if 1 <= L <= cap:
            ek[b, :, L - 1], ev[b, :, L - 1] = kn[b], vn[b]
    assert torch.equal(k.view(torch.int16), ek.view(torch.int16))
    assert torch.equal(v.view(torch.int16), ev.view(torch.int16))


def test_partial_then_merge_equals_decode():
    wl = small("mha13b_4k", batch=2, num_q_heads=4, num_kv_heads=4, seq_len=3000)
    case = W.make_case(wl, DEV)
    ref, ref_lse = H.gpu_step(case)
    desc = B.kv_desc(case.k_cache, case.v_cache)
    ws = B.alloc_workspace(2, 4, 4, 128, 3001, DEV)
    out = torch.empty_like(ref)
    lse = torch.empty_like(ref_lse)
    B.decode_partial(case.q, desc, case.seq_lens, 4, case.scale, out, ws, 3001, lse=lse)
    B.decode_merge(case.seq_lens, 4, 4, case.capacity, out, ws, 3001, lse=lse)
    torch.cuda.synchronize()
    assert torch.equal(out, ref) and torch.equal(lse, ref_lse)


# ------------------------------------------------------------------ fused append + decode
FUSED_CASES = [
    W.Workload("f_mha", 3, 4, 4, 128, 2999, seq_len_min=5, seed=301),
    W.Workload("f_mha64_paged", 3, 4, 4, 64, 1000, seq_len_min=5, paged=True, seed=302),
    W.Workload("f_gqa", 2, 16, 2, 128, 6100, seq_len_min=2000, seed=303),
    W.Workload("f_gqa_paged", 2, 8, 2, 128, 777, seq_len_min=1, paged=True, seed=304),
    W.Workload("f_gqa64", 2, 8, 2, 64, 900, seq_len_min=100, seed=305),      # append launched on its own
    W.Workload("f_many_short", 16, 40, 40, 128, 300, seq_len_min=1, seed=306),  # single split
]


@pytest.mark.parametrize("wl", FUSED_CASES, ids=[w.name for w in FUSED_CASES])
def test_fused_call_equals_the_two_calls(wl):
    a = W.make_case(wl, DEV, poison=True)
    b = W.make_case(wl, DEV, poison=True)
    assert torch.equal(a.k_cache.view(torch.int16), b.k_cache.view(torch.int16))
    out_a, lse_a = H.gpu_step(a, fused=False)
    out_b, lse_b = H.gpu_step(b, fused=True)
    assert torch.equal(a.k_cache.view(torch.int16), b.k_cache.view(torch.int16))
    assert torch.equal(a.v_cache.view(torch.int16), b.v_cache.view(torch.int16))
    assert torch.equal(out_a, out_b) and torch.equal(lse_a, lse_b)
    full_check(wl, fused=True)


def test_fused_append_edge_lengths():
    """Lengths of 0, below 0, at the capacity, beyond it and beyond max_seq_len:
    the fused call stores exactly what kv_append stores."""
    wl = small("mha13b_4k", batch=6, num_q_heads=2, num_kv_heads=2, seq_len=600)
    lens = [0, -3, 608, 609, 5000, 300]
    res = []
    for fused in (False, True):
        case = W.make_case(wl, DEV, poison=False)
        assert case.capacity == 608
        case.seq_lens = torch.tensor(lens, dtype=torch.int32, device=DEV)
        out, lse = H.gpu_step(case, fused=fused, max_seq_len=400)
        res.append((case, out, lse))
    (ca, oa, la), (cb, ob, lb) = res
    assert torch.equal(ca.k_cache.view(torch.int16), cb.k_cache.view(torch.int16))
    assert torch.equal(ca.v_cache.view(torch.int16), cb.v_cache.view(torch.int16))
    assert torch.equal(oa, ob) and torch.equal(la, lb)
    assert torch.equal(cb.k_cache[2, :, 607].view(torch.int16), cb.k_new[2].view(torch.int16))


# ------------------------------------------------------------------ bulk KV write (prefill side)
@pytest.mark.parametrize("paged", [False, True, "adjacent"])
@pytest.mark.parametrize("head_dim", [64, 128])
def test_kv_write_bit_exact_against_the_oracle(paged, head_dim):
    from oracle import decode_attention as oracle
    wl = W.Workload("kvw", 5, 3, 3, head_dim, 200, paged=bool(paged), kv_adjacent=paged == "adjacent", seed=501)
    case = W.make_case(wl, DEV, poison=False)
    g = torch.Generator().manual_seed(7)
    N = 150
    mk = lambda *s: torch.randint(0, 65536, s, generator=g, dtype=torch.int32).to(torch.uint16) \
        .view(torch.float16).to(DEV)
    k_src, v_src = mk(5, 3, N, head_dim), mk(5, 3, N, head_dim)
    start = torch.tensor([0, 17, 190, 60, -5], dtype=torch.int32, device=DEV)
    count = torch.tensor([150, 0, 150, 33, 20], dtype=torch.int32, device=DEV)
    want_k, want_v = H.host(case.k_cache).copy(), H.host(case.v_cache).copy()
    oracle.kv_write(want_k, want_v, H.host(k_src), H.host(v_src), H.host(start), H.host(count),
                    H.host(case.page_table))
    B.kv_write(B.kv_desc(case.k_cache, case.v_cache, case.page_table), k_src, v_src, start, count)
    torch.cuda.synchronize()
    assert np.array_equal(H.host(case.k_cache).view(np.uint16), want_k.view(np.uint16))
    assert np.array_equal(H.host(case.v_cache).view(np.uint16), want_v.view(np.uint16))


def test_kv_write_equals_one_append_per_row_on_the_gpu():
    wl = W.Workload("kvw2", 3, 2, 2, 128, 90, paged=True, seed=502)
    a, b = W.make_case(wl, DEV), W.make_case(wl, DEV)
    N = 40
    k_src = torch.randn(3, 2, N, 128, device=DEV).half()
    v_src = torch.randn(3, 2, N, 128, device=DEV).half()
    start = torch.tensor([0, 30, 51], dtype=torch.int32, device=DEV)
    count = torch.tensor([40, 25, 40], dtype=torch.int32, device=DEV)
    B.kv_write(B.kv_desc(a.k_cache, a.v_cache, a.page_table), k_src, v_src, start, count)
    db = B.kv_desc(b.k_cache, b.v_cache, b.page_table)
    for i in range(N):
        lens = torch.where(i < count, start + i + 1, torch.zeros_like(start)).to(torch.int32)
        B.kv_append(db, k_src[:, :, i].contiguous(), v_src[:, :, i].contiguous(), lens)
    torch.cuda.synchronize()
    assert torch.equal(a.k_cache.view(torch.int16), b.k_cache.view(torch.int16))
    assert torch.equal(a.v_cache.view(torch.int16), b.v_cache.view(torch.int16))


def test_prefill_write_then_decode():
    """Prompt rows laid down with kv_write, then one decode step: same result as the
    oracle on the same rows."""
    wl = small("mha13b_4k", batch=2, num_q_heads=4, num_kv_heads=4, seq_len=777)
    case = W.make_case(wl, DEV, poison=True)
    S = 777
    k_src = torch.randn(2, 4, S, 128, device=DEV).half()
    v_src = torch.randn(2, 4, S, 128, device=DEV).half()
    zero = torch.zeros(2, dtype=torch.int32, device=DEV)
    B.kv_write(B.kv_desc(case.k_cache, case.v_cache), k_src, v_src, zero, zero + S)
    torch.cuda.synchronize()
    assert torch.equal(case.k_cache[:, :, :S].view(torch.int16), k_src.view(torch.int16))
    want_out, want_lse, _, _ = H.oracle_step(case)
    out, lse = H.gpu_step(case, fused=True)
    H.assert_close(out, lse, want_out, want_lse, "prefill+decode")


# ------------------------------------------------------------------ seeded draw of shapes
def _drawn_configs(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        D = int(rng.choice([64, 128]))
        G = int(rng.choice([1, 1, 2, 3, 4, 8, 16]))
        Hkv = int(rng.choice([1, 2, 5]))
        S = int(rng.integers(0, 9000)) if i % 4 == 3 else int(rng.integers(0, 2500))
        Bn = int(rng.integers(1, 4))
        out.append((i, Bn, D, G, Hkv, S, bool(rng.integers(0, 2)), bool(rng.integers(0, 2)), bool(rng.integers(0, 2))))
    return out


@pytest.mark.parametrize("cfg", _drawn_configs(24, 20240918), ids=lambda c: "cfg%d" % c[0])
def test_drawn_configurations(cfg):
    i, Bn, D, G, Hkv, S, paged, f32, fused = cfg
    wl = W.Workload("drawn%d" % i, Bn, G * Hkv, Hkv, D, S, seq_len_min=S // 4, paged=paged, page_size=16,
                    seed=700 + i)
    full_check(wl, out_dtype=torch.float32 if f32 else torch.float16, fused=fused)


def _drawn_wide(n, seed):
    """Drawn over more of the argument space: groups beyond 16, page sizes, both pool
    layouts, split lengths forced through the environment."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        out.append(dict(i=i, D=int(rng.choice([64, 128])), G=int(rng.choice([1, 2, 5, 8, 16, 17, 24, 33, 48])),
                        Hkv=int(rng.choice([1, 2, 3])), S=int(rng.integers(0, int(rng.choice([700, 3000, 9000])))),
                        Bn=int(rng.integers(1, 5)), paged=bool(rng.integers(0, 2)), page=int(rng.choice([16, 32, 64])),
                        adjacent=bool(rng.integers(0, 2)), f32=bool(rng.integers(0, 2)), fused=bool(rng.integers(0, 2)),
                        chunk=int(rng.choice([0, 0, 128, 384, 1152]))))
    return out


@pytest.mark.parametrize("cfg", _drawn_wide(30, 20241127), ids=lambda c: "cfg%d" % c["i"])
def test_drawn_configurations_wide(options, cfg):
    if cfg["chunk"]:
        options.setenv("INSTATTN_CHUNK", str(cfg["chunk"]))
    wl = W.Workload("wide%d" % cfg["i"], cfg["Bn"], cfg["G"] * cfg["Hkv"], cfg["Hkv"], cfg["D"], cfg["S"],
                    seq_len_min=cfg["S"] // 3, paged=cfg["paged"], page_size=cfg["page"],
                    kv_adjacent=cfg["paged"] and cfg["adjacent"], seed=900 + cfg["i"])
    full_check(wl, out_dtype=torch.float32 if cfg["f32"] else torch.float16, fused=cfg["fused"])


@pytest.mark.parametrize("cfg", _drawn_configs(12, 20240919), ids=lambda c: "cfg%d" % c[0])
def test_drawn_configurations_with_rotated_walks(options, cfg):
    """INSTATTN_ROTATE=1: every unit starts at a tile of its own and wraps round (the
    remedy for cache strides that walk the HBM channels in step); same results."""
    options.setenv("INSTATTN_ROTATE", "1")
    i, Bn, D, G, Hkv, S, paged, f32, fused = cfg
    wl = W.Workload("rot%d" % i, Bn, G * Hkv, Hkv, D, S, seq_len_min=S // 4, paged=paged, page_size=16,
                    seed=800 + i)
    full_check(wl, out_dtype=torch.float32 if f32 else torch.float16, fused=fused)


def test_rotated_walk_on_the_13b_shape(options):
    options.setenv("INSTATTN_ROTATE", "1")
    full_check(W.WORKLOADS["mha13b_4k"], fused=True)


# ------------------------------------------------------------------ HIP graph replay
@pytest.mark.parametrize("shape", ["mha_splits", "gqa_paged"])
def test_step_replayed_from_a_hip_graph(shape):
    """The launches of a step (split pass with the append fused in, merge) recorded into a
    HIP graph: every replay, with eager work and synchronisation in between, gives the
    oracle's result and bit for bit the eager one."""
    if shape == "mha_splits":
        wl = W.Workload("graph_mha", 2, 4, 4, 128, 3000, seq_len_min=500, seed=501)
    else:
        wl = W.Workload("graph_gqa", 2, 8, 2, 128, 2000, seq_len_min=300, paged=True, page_size=16, seed=502)
    case = W.make_case(wl, DEV, poison=True)
    other = W.make_case(W.Workload("graph_other", 1, 4, 4, 64, 700, seed=503), DEV)
    want_out, want_lse, want_k, want_v = H.oracle_step(case)
    desc = B.kv_desc(case.k_cache, case.v_cache, case.page_table)
    max_len = int(case.seq_lens.max())
    Bn, Hq, D = case.q.shape
    ws = B.alloc_workspace(Bn, Hq, wl.num_kv_heads, D, max_len, DEV)
    out = torch.empty(Bn, Hq, D, dtype=torch.float16, device=DEV)
    lse = torch.empty(Bn, Hq, dtype=torch.float32, device=DEV)

    def step():
        B.append_decode(case.q, case.k_new, case.v_new, desc, case.seq_lens, wl.num_kv_heads, case.scale,
                        out, ws, max_len, lse=lse)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    eager_out, eager_lse = out.clone(), lse.clone()
    H.assert_close(eager_out, eager_lse, want_out, want_lse, "eager", lse_tol=H.lse_tol(wl.group, eager_out.dtype))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        out.fill_(float("nan"))
        lse.fill_(float("nan"))
        ws.fill_(0xFF)
        H.gpu_step(other)                      # unrelated eager work between the replays
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager_out.view(torch.int16)), rep
        assert torch.equal(lse.view(torch.int32), eager_lse.view(torch.int32)), rep
    assert np.array_equal(H.host(case.k_cache).view(np.uint16), want_k.view(np.uint16))
    assert np.array_equal(H.host(case.v_cache).view(np.uint16), want_v.view(np.uint16))
