"""The allocation-free entry point against instattn_decode, through the C ABI: same
out/lse bit for bit on two calls in a row, the second with a smaller input (the
library's scratch still holds the first call's partial rows then)."""
import pytest
import torch

from paper_2409_04992_amd import binding as B
from paper_2409_04992_amd import workloads as W

import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def both(wl, seed_layer):
    case = W.make_case(wl, DEV, layer=seed_layer, poison=True)
    want, want_lse = H.gpu_step(case)                       # append + instattn_decode on a caller's workspace
    desc = B.kv_desc(case.k_cache, case.v_cache, case.page_table)
    out = torch.full_like(want, float("nan"))
    lse = torch.full_like(want_lse, float("nan"))
    max_len = max(1, min(int(case.seq_lens.max()), case.capacity))
    held_before = torch.cuda.memory_allocated()
    B.decode_static(case.q, desc, case.seq_lens, wl.num_kv_heads, case.scale, out, max_len, lse=lse)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == held_before      # the call went through no allocator of torch
    assert torch.equal(out, want) and torch.equal(lse, want_lse), wl.name
    return case, out, lse


def test_decode_static_equals_decode_on_two_calls_in_a_row():
    big = W.Workload("static_big", 6, 8, 8, 128, 5000, seq_len_min=700, paged=True, seed=31)
    small = W.Workload("static_small", 2, 8, 2, 64, 900, seq_len_min=100, seed=32, out_dtype="f32")
    assert B.decode_plan(6, 8, 8, 128, 5001)[1] > 1          # both use the scratch: several splits
    assert B.decode_plan(2, 8, 2, 64, 901)[1] > 1
    both(big, 0)
    both(small, 0)
    case, out, lse = both(big, 1)
    # and against the oracle, once
    want_out, want_lse, _, _ = H.oracle_step(case, append=False)
    H.assert_close(out, lse, want_out, want_lse, "decode_static")


def test_decode_static_rejects_what_does_not_fit():
    """A shape whose workspace exceeds the library's scratch is refused before any launch."""
    import ctypes
    wl = W.Workload("static_small", 2, 4, 4, 64, 300, seed=33)
    case = W.make_case(wl, DEV)
    desc = B.kv_desc(case.k_cache, case.v_cache, None)
    # 4096 sequences x 64 heads x 2 splits of 129 floats = 270 MB of partial rows
    assert B.decode_workspace_size(4096, 64, 64, 128, 300) > B.STATIC_SCRATCH_BYTES
    st = B.lib().instattn_decode_static(case.q.data_ptr(), ctypes.byref(desc), case.seq_lens.data_ptr(), 4096, 64, 64,
                                        128, 0.1, case.q.data_ptr(), B.F16, None, 300, None)
    assert st == B.ERR_WORKSPACE
