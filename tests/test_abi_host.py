"""C-ABI checks that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments on the host before launching anything.
Every call below is built to fail validation, so no kernel is ever launched."""
import ctypes
import os
import re

import pytest

from paper_2409_04992_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000          # aligned, non-NULL, never dereferenced on the host


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "instattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(instattn_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert {"instattn_kv_append", "instattn_decode", "instattn_decode_partial",
            "instattn_decode_merge", "instattn_decode_plan", "instattn_decode_workspace_size",
            "instattn_status_string", "instattn_version", "instattn_probe_read",
            "instattn_append_decode", "instattn_kv_write", "instattn_sparf_build", "instattn_sparf_append",
            "instattn_sparf_build_workspace_size",
            "instattn_sparf_decode", "instattn_sparf_workspace_size", "instattn_sparf_append_decode",
            "instattn_sparf_plan",
            "instattn_probe_copy", "instattn_probe_read_columns"} <= set(names)
    lib = B.lib()
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings():
    assert B.version() >= 100
    texts = {B.status_string(s) for s in range(5)}
    assert len(texts) == 5 and B.status_string(99) == "unknown status"


def desc(**kw):
    d = B.KvDesc()
    d.k, d.v = FAKE, FAKE
    d.layout = B.KV_CONTIGUOUS
    d.stride_b, d.stride_h, d.stride_t = 40 * 4112 * 128, 4112 * 128, 128
    d.capacity = 4112
    d.reserved = 0
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def paged_desc(**kw):
    base = dict(layout=B.KV_PAGED, page_size=16, max_pages_per_seq=257, num_pages=5000,
                capacity=16 * 257, stride_b=40 * 16 * 128, stride_h=16 * 128, stride_t=128,
                page_table=FAKE)
    base.update(kw)
    return desc(**base)


def decode_status(d, q=FAKE, seq=FAKE, batch=16, hq=40, hkv=40, dim=128, scale=0.088, out=FAKE,
                  out_dtype=B.F16, ws=FAKE & ~255, ws_bytes=1 << 30, max_len=4097):
    return B.lib().instattn_decode(q, ctypes.byref(d) if d is not None else None, seq, batch, hq,
                                   hkv, dim, scale, out, out_dtype, None, ws, ws_bytes, max_len, None)


@pytest.mark.parametrize("kw,want", [
    (dict(q=None), B.ERR_INVALID_ARG),
    (dict(seq=None), B.ERR_INVALID_ARG),
    (dict(out=None), B.ERR_INVALID_ARG),
    (dict(q=FAKE + 2), B.ERR_INVALID_ARG),
    (dict(batch=0), B.ERR_INVALID_ARG),
    (dict(hq=40, hkv=16), B.ERR_INVALID_ARG),          # not a multiple
    (dict(hq=0), B.ERR_INVALID_ARG),
    (dict(dim=96), B.ERR_UNSUPPORTED),
    (dict(dim=256), B.ERR_UNSUPPORTED),
    (dict(out_dtype=7), B.ERR_INVALID_ARG),
    (dict(max_len=0), B.ERR_INVALID_ARG),
    (dict(max_len=5000), B.ERR_INVALID_ARG),           # beyond the capacity
    (dict(scale=float("nan")), B.ERR_INVALID_ARG),
    (dict(ws=None), B.ERR_WORKSPACE),
    (dict(ws=(FAKE & ~255) + 16), B.ERR_WORKSPACE),
    (dict(ws_bytes=1024), B.ERR_WORKSPACE),
])
def test_decode_rejects(kw, want):
    assert decode_status(desc(), **kw) == want


@pytest.mark.parametrize("d", [
    None,
    desc(k=None), desc(v=None), desc(k=FAKE + 8),
    desc(layout=5), desc(stride_t=64), desc(stride_t=129), desc(stride_h=0), desc(stride_b=-8),
    desc(capacity=0), desc(reserved=1), desc(page_table=FAKE),
    paged_desc(page_table=None), paged_desc(page_size=8), paged_desc(page_size=24),
    paged_desc(max_pages_per_seq=0), paged_desc(num_pages=0), paged_desc(capacity=4000),
])
def test_bad_kv_descriptor_rejected_by_decode_and_append(d):
    assert decode_status(d) == B.ERR_INVALID_ARG
    ptr = ctypes.byref(d) if d is not None else None
    assert B.lib().instattn_kv_append(ptr, FAKE, FAKE, FAKE, 16, 40, 128, None) == B.ERR_INVALID_ARG


@pytest.mark.parametrize("args", [
    (None, FAKE, FAKE, 16, 40, 128), (FAKE, None, FAKE, 16, 40, 128), (FAKE, FAKE, None, 16, 40, 128),
    (FAKE + 4, FAKE, FAKE, 16, 40, 128), (FAKE, FAKE, FAKE, 0, 40, 128),
    (FAKE, FAKE, FAKE, 16, 0, 128), (FAKE, FAKE, FAKE, 16, 40, 100),
])
def test_append_rejects(args):
    k_new, v_new, seq, batch, hkv, dim = args
    d = desc()
    assert B.lib().instattn_kv_append(ctypes.byref(d), k_new, v_new, seq, batch, hkv, dim,
                                      None) == B.ERR_INVALID_ARG


def test_probe_rejects():
    L = B.lib()
    assert L.instattn_probe_read(None, 1024, FAKE, None) == B.ERR_INVALID_ARG
    assert L.instattn_probe_read(FAKE, 1000, FAKE, None) == B.ERR_INVALID_ARG
    assert L.instattn_probe_copy(FAKE, None, 1024, None) == B.ERR_INVALID_ARG
    assert L.instattn_probe_copy(FAKE, FAKE, 0, None) == B.ERR_INVALID_ARG
    cols = lambda *a: L.instattn_probe_read_columns(*a)
    assert cols(None, 128 * 4112 * 2, 4112 * 2, 640, 128, 16, 4096, FAKE, None) == B.ERR_INVALID_ARG
    assert cols(FAKE, 128 * 4112 * 2, 4112 * 2, 640, 128, 129, 4096, FAKE, None) == B.ERR_INVALID_ARG   # r > dims
    assert cols(FAKE, 128 * 4112 * 2, 4112 * 2, 640, 128, 16, 4100, FAKE, None) == B.ERR_INVALID_ARG    # not a multiple of 8
    assert cols(FAKE, 128 * 4112 * 2, 4112 * 2, 640, 128, 16, 4120, FAKE, None) == B.ERR_INVALID_ARG    # behind the column
    assert cols(FAKE, 100 * 4112 * 2, 4112 * 2, 640, 128, 16, 4096, FAKE, None) == B.ERR_INVALID_ARG    # columns overlap rows


# ------------------------------------------------------------------ split plan (host arithmetic)
@pytest.mark.parametrize("shape", [
    (2, 4, 4, 64, 257), (16, 40, 40, 128, 4097), (8, 40, 40, 128, 32769),
    (64, 40, 40, 128, 16385), (32, 64, 8, 128, 16385), (1, 40, 40, 128, 131072), (1, 1, 1, 64, 1),
])
def test_plan_covers_the_sequence_and_fills_the_chip(shape):
    batch, hq, hkv, dim, max_len = shape
    chunk, splits = B.decode_plan(*shape)
    assert chunk % 128 == 0 and chunk >= 128
    assert (splits - 1) * chunk < max_len <= splits * chunk
    streams = batch * (hq if hq == hkv else hkv)
    if max_len * streams >= 1024 * 1024:           # enough work to want every CU busy twice over
        assert streams * splits >= 512
    if hq == hkv and streams >= 512 and max_len <= 8192:
        # enough short streams: whole sequences, or the fewest equal splits that fill every
        # block slot of the chip (no merge pass from 1280 streams on)
        assert splits == max(1, -(-1280 // streams)) or chunk == 384
    if chunk < max_len:                            # split: chunk is an odd multiple of 128
        assert (chunk // 128) % 2 == 1
    ws = B.decode_workspace_size(*shape)
    assert ws >= batch * hq * splits * (dim + 1) * 4 and ws % 256 == 0


def test_plan_units_of_the_ring_form(options):
    """Large launches of the vector-ALU kernel: units of 2944 or 5504 rows (or whole sequences up to
    that length), whichever gives the fewest rounds over 256 compute units times the unit length
    (the longer must win by 3 %), and only when those rounds come out at least 88 % full; else the
    register form's short units."""
    plan = lambda b, h, L: B.decode_plan(b, h, h, 128, L)
    assert plan(8, 40, 32769) == (2944, 12)          # 15 rounds of 2944 against 8 of 5504: level, the shorter
    assert plan(6, 40, 32769) == (5504, 6)           # 12 rounds of 2944 against 6 of 5504
    assert plan(1, 40, 131073) == (5504, 24)
    assert plan(64, 40, 16385) == (5504, 3)
    assert plan(32, 8, 16385) == (5504, 3)           # 768 units: three full rounds
    assert plan(2, 40, 16385) == (5504, 3)           # 240 units: one round
    assert plan(12, 40, 3073) == (3200, 1)           # 480 whole sequences: two rounds, no merge
    assert plan(1, 40, 1 << 20) == (2944, 357)
    # rounds that would stay partly empty: the register form (1280 block slots) in short units
    assert plan(24, 8, 16385) == (896, 19)           # 1152 units of 2944 rows fill 83 % of five rounds
    assert plan(3, 8, 65537) == (384, 171)           # 552 units: 72 % of three rounds
    assert plan(5, 40, 8193) == (384, 22)
    assert plan(10, 40, 6145) == (640, 10)           # a third unit of 257 rows per sequence
    # below 2^20 rows in all, or sequences shorter than 2048 rows: the register form
    assert plan(1, 40, 16385) == (384, 43) and plan(64, 8, 1537)[0] < 2048
    # forced either way
    options.setenv("INSTATTN_MHA_RING", 1)
    assert plan(3, 8, 65537) == (2944, 23) and plan(1, 4, 4000) == (2944, 2)
    options.setenv("INSTATTN_MHA_RING", 0)
    assert plan(6, 40, 32769)[0] <= 1408


def test_plan_units_of_the_grouped_query_kernel():
    """About three units per four compute units, at most 5504 rows; sequences of more than three
    units of 8832 rows take that length when it saves rounds over the kernel's 512 block slots."""
    plan = lambda b, L: B.decode_plan(b, 64, 8, 128, L)
    assert plan(32, 16385) == (5504, 3)              # the 80-layer configuration: 768 units
    assert plan(8, 65537) == (8832, 8)               # 512 units in one round instead of 768 in one and a half
    assert plan(4, 131073) == (8832, 15) and plan(16, 32769) == (8832, 4)
    assert plan(64, 32769) == (5504, 6)              # 3072 units: six full rounds either way
    assert plan(16, 26496) == (5504, 5)              # three units of 8832 rows: too few
    assert plan(2, 32769) == (2688, 13)              # few streams: short units for every compute unit


def test_plan_rejects_bad_shapes():
    assert B.decode_workspace_size(0, 4, 4, 64, 100) == 0
    assert B.decode_workspace_size(1, 4, 4, 80, 100) == 0
    with pytest.raises(B.InstattnError):
        B.decode_plan(1, 4, 3, 64, 100)


def test_forced_chunk_env(options):
    options.setenv("INSTATTN_CHUNK", "512")
    assert B.decode_plan(16, 40, 40, 128, 4097) == (512, 9)
    options.setenv("INSTATTN_CHUNK", "500")      # rounded up to the tile quantum
    assert B.decode_plan(16, 40, 40, 128, 4097) == (512, 9)
    options.delenv("INSTATTN_CHUNK")
    assert B.decode_plan(16, 40, 40, 128, 4097) == (2176, 2)      # 640 streams in two halves
    assert B.decode_plan(32, 40, 40, 128, 4097) == (4224, 1)      # 1280 streams fill the chip: one unit each


def test_switches_are_set_and_read_back(options):
    for name in B.OPTIONS:
        assert B.get_option(name) == -1
        B.set_option(name, 1)
        assert B.get_option(name) == 1
        B.set_option(name, -7)                      # any negative value hands the choice back
        assert B.get_option(name) == -1
    L = B.lib()
    assert L.instattn_set_option(b"INSTATTN_NO_SUCH_SWITCH", 1) == B.ERR_INVALID_ARG
    assert L.instattn_set_option(None, 1) == B.ERR_INVALID_ARG
    assert L.instattn_get_option(b"INSTATTN_CHUNK", None) == B.ERR_INVALID_ARG


def test_switches_start_from_the_environment():
    """Read once per process: a child that finds INSTATTN_CHUNK in its environment plans with it,
    and a later change of the variable inside that process changes nothing."""
    import subprocess
    import sys
    code = ("import os, sys; sys.path.insert(0, %r); from paper_2409_04992_amd import binding as B; "
            "a = B.decode_plan(16, 40, 40, 128, 4097); os.environ['INSTATTN_CHUNK'] = '1024'; "
            "print(a, B.decode_plan(16, 40, 40, 128, 4097), B.get_option('INSTATTN_CHUNK'))" % ROOT)
    env = dict(os.environ, INSTATTN_CHUNK="512")
    out = subprocess.run([sys.executable, "-c", code], check=True, capture_output=True, text=True, env=env).stdout
    assert out.strip() == "(512, 9) (512, 9) 512"


def test_decode_launches(options):
    # the four timed shapes: only the paged one lists its units first
    assert B.decode_launches(16, 40, 40, 128, 4097, True) == \
        {"append": False, "unit_list": False, "split_pass": True, "merge": True}
    assert not B.decode_launches(8, 40, 40, 128, 32769, True)["unit_list"]
    assert B.decode_launches(64, 40, 40, 128, 16385, True, paged=True)["unit_list"]
    assert not B.decode_launches(64, 40, 40, 128, 16385, True)["unit_list"]      # the same batch, contiguous
    assert not B.decode_launches(32, 64, 8, 128, 16385, True)["unit_list"]
    assert B.decode_launches(32, 40, 40, 128, 4097) == \
        {"append": False, "unit_list": False, "split_pass": True, "merge": False}  # whole sequences as units
    assert B.decode_launches(32, 40, 40, 128, 4097, paged=True)["unit_list"]     # ... listed all the same when paged
    assert not B.decode_launches(2, 4, 4, 128, 4097, paged=True)["unit_list"]    # too little to pay for the launch
    assert not B.decode_launches(1, 40, 40, 128, 131072, paged=True)["unit_list"]  # one sequence: nothing to order
    # a group of more than 16 query heads: the append is a launch of its own, and no list
    assert B.decode_launches(64, 48, 1, 128, 16385, True, paged=True) == \
        {"append": True, "unit_list": False, "split_pass": True, "merge": True}
    assert not B.decode_launches(64, 48, 1, 128, 16385, False)["append"]
    options.setenv("INSTATTN_COMPACT", 1)
    assert B.decode_launches(8, 40, 40, 128, 32769)["unit_list"]
    assert B.decode_launches(32, 40, 40, 128, 4097)["unit_list"]
    assert not B.decode_launches(1, 40, 40, 128, 131072)["unit_list"]
    assert not B.decode_launches(64, 48, 1, 128, 16385)["unit_list"]
    assert not B.decode_launches(5000, 8, 8, 128, 4097)["unit_list"]             # more sequences than the list's block holds
    options.setenv("INSTATTN_COMPACT", 0)
    assert not B.decode_launches(64, 40, 40, 128, 16385, paged=True)["unit_list"]
    # the workspace has room for the list whatever the switch and the layout say
    sizes = set()
    for v in (None, 0, 1):
        options.setenv("INSTATTN_COMPACT", -1 if v is None else v)
        sizes.add(B.decode_workspace_size(64, 40, 40, 128, 16385))
    assert len(sizes) == 1 and sizes.pop() >= 64 * 40 * 3 * 129 * 4 + 64 * 3 * 4
    L = B.lib()
    assert L.instattn_decode_launches(8, 40, 40, 128, 32769, 7, 0, (ctypes.c_int32 * 4)()) == B.ERR_INVALID_ARG
    assert L.instattn_decode_launches(8, 40, 40, 128, 32769, 0, 0, None) == B.ERR_INVALID_ARG


def test_limits_of_the_launch_grids_are_checked_before_anything_is_launched(options):
    """More splits than a grid dimension holds, or more blocks than a one-dimensional grid:
    unsupported, from the plan call and from the decode calls alike, and in front of the
    separate append launch of a large group (on a box without a GPU a launch would come
    back as a runtime error instead)."""
    options.setenv("INSTATTN_CHUNK", 128)
    long_len = 128 * 65536
    assert B.lib().instattn_decode_plan(1, 8, 8, 128, long_len, None, None) == B.ERR_UNSUPPORTED
    assert B.decode_workspace_size(1, 8, 8, 128, long_len) == 0
    big = desc(capacity=long_len, stride_h=long_len * 128, stride_b=8 * long_len * 128)
    assert decode_status(d=big, batch=1, hq=8, hkv=8, max_len=long_len) == B.ERR_UNSUPPORTED
    assert B.decode_plan(1, 8, 8, 128, 128 * 65535) == (128, 65535)
    options.delenv("INSTATTN_CHUNK")
    # 65535 sequences x 1927 KV heads x 6 splits x 3 blocks per unit do not fit an int32
    shape = dict(batch=65535, hq=1927 * 34, hkv=1927, max_len=27521)
    assert B.lib().instattn_decode_plan(65535, 1927 * 34, 1927, 128, 27521, None, None) == B.ERR_UNSUPPORTED
    assert decode_status(desc(capacity=27600), ws_bytes=1 << 50, **shape) == B.ERR_UNSUPPORTED
    L = B.lib()
    d = desc(capacity=27600)
    st = L.instattn_append_decode(FAKE, FAKE, FAKE, ctypes.byref(d), FAKE, 65535, 1927 * 34, 1927, 128, 0.088,
                                  FAKE, B.F16, None, FAKE & ~255, 1 << 50, 27521, None)
    assert st == B.ERR_UNSUPPORTED


# ------------------------------------------------------------------ SparF entry points
def aux_desc(**kw):
    a = B.SparfAux()
    a.kt, a.vsum = FAKE, FAKE
    a.stride_b, a.stride_h, a.stride_d = 40 * 128 * 4112, 128 * 4112, 4112
    a.capacity, a.page_size, a.page_table = 4112, 0, None
    for k, v in kw.items():
        setattr(a, k, v)
    return a


def paged_aux_desc(**kw):
    a = B.SparfAux()
    a.kt, a.vsum, a.page_table = FAKE, FAKE, FAKE
    a.stride_b, a.stride_h, a.stride_d = 40 * 128 * 256, 128 * 256, 256
    a.page_size, a.max_pages_per_seq, a.num_pages = 256, 17, 16 * 17
    a.capacity = 256 * 17
    for k, v in kw.items():
        setattr(a, k, v)
    return a


def sparf_status(d=None, a=None, q=FAKE, seq=FAKE, batch=16, hq=40, hkv=40, dim=128, scale=0.088,
                 r=16, k=256, l=16, out=FAKE, out_dtype=B.F16, ws=FAKE & ~255, ws_bytes=1 << 30,
                 max_len=4097):
    d = desc() if d is None else d
    a = aux_desc() if a is None else a
    return B.lib().instattn_sparf_decode(q, ctypes.byref(d), ctypes.byref(a), seq, batch, hq, hkv, dim,
                                         scale, r, k, l, out, out_dtype, None, None, ws, ws_bytes,
                                         max_len, None)


@pytest.mark.parametrize("kw,want", [
    (dict(q=None), B.ERR_INVALID_ARG), (dict(seq=None), B.ERR_INVALID_ARG),
    (dict(out=None), B.ERR_INVALID_ARG), (dict(r=0), B.ERR_INVALID_ARG),
    (dict(r=129), B.ERR_INVALID_ARG), (dict(k=0), B.ERR_INVALID_ARG), (dict(l=-1), B.ERR_INVALID_ARG),
    (dict(dim=96), B.ERR_UNSUPPORTED), (dict(hq=40, hkv=16), B.ERR_INVALID_ARG),
    (dict(max_len=5000), B.ERR_INVALID_ARG), (dict(out_dtype=3), B.ERR_INVALID_ARG),
    (dict(ws=None), B.ERR_WORKSPACE), (dict(ws_bytes=4096), B.ERR_WORKSPACE),
    (dict(d=paged_desc(page_table=None)), B.ERR_INVALID_ARG),
    (dict(a=aux_desc(kt=None)), B.ERR_INVALID_ARG), (dict(a=aux_desc(vsum=None)), B.ERR_INVALID_ARG),
    (dict(a=aux_desc(capacity=4100)), B.ERR_INVALID_ARG), (dict(a=aux_desc(stride_d=4000)), B.ERR_INVALID_ARG),
    (dict(a=aux_desc(capacity=4000, stride_d=4000)), B.ERR_INVALID_ARG),
    (dict(a=aux_desc(page_table=FAKE)), B.ERR_INVALID_ARG),              # table without a page size
    (dict(a=paged_aux_desc(page_table=None)), B.ERR_INVALID_ARG),
    (dict(a=paged_aux_desc(page_size=100)), B.ERR_INVALID_ARG),
    (dict(a=paged_aux_desc(page_size=4)), B.ERR_INVALID_ARG),
    (dict(a=paged_aux_desc(capacity=4096)), B.ERR_INVALID_ARG),          # != page_size * max_pages
    (dict(a=paged_aux_desc(stride_d=128)), B.ERR_INVALID_ARG),
    (dict(a=paged_aux_desc(num_pages=0)), B.ERR_INVALID_ARG),
    (dict(d=desc(stride_t=(1 << 24) + 8)), B.ERR_UNSUPPORTED),
])
def test_sparf_decode_rejects(kw, want):
    assert sparf_status(**kw) == want


def test_sparf_accepts_either_layout_of_either_copy():
    """Validation only reaches the launch when everything is in order; stop it there
    with a workspace that is too small."""
    for d in (desc(), paged_desc()):
        for a in (aux_desc(), paged_aux_desc()):
            assert sparf_status(d=d, a=a, ws_bytes=4096) == B.ERR_WORKSPACE


def test_sparf_append_decode_rejects():
    L = B.lib()
    d, a = desc(), aux_desc()
    args = [FAKE, FAKE, FAKE, ctypes.byref(d), ctypes.byref(a), FAKE, 16, 40, 40, 128, 0.088, 16, 256, 16,
            FAKE, B.F16, None, None, FAKE & ~255, 1 << 30, 4097, None]
    for i in (0, 1, 2, 5, 14):
        bad = list(args)
        bad[i] = None
        assert L.instattn_sparf_append_decode(*bad) == B.ERR_INVALID_ARG, i
    bad = list(args)
    bad[19] = 4096
    assert L.instattn_sparf_append_decode(*bad) == B.ERR_WORKSPACE
    for i in (1, 2):                             # new rows are read with 128-bit loads
        bad = list(args)
        bad[i] = FAKE + 2
        assert L.instattn_sparf_append_decode(*bad) == B.ERR_INVALID_ARG, i


def test_sparf_build_and_append_reject():
    L = B.lib()
    d, a = desc(), aux_desc()
    assert L.instattn_sparf_build(ctypes.byref(d), ctypes.byref(a), None, 16, 40, 128, None, 0, None) == B.ERR_INVALID_ARG
    assert L.instattn_sparf_build(None, ctypes.byref(a), FAKE, 16, 40, 128, None, 0, None) == B.ERR_INVALID_ARG
    assert L.instattn_sparf_build(ctypes.byref(d), None, FAKE, 16, 40, 128, None, 0, None) == B.ERR_INVALID_ARG
    # scratch for the V sum: none wanted with 640 pairs; with 8 pairs 64 blocks each, and a
    # scratch that is given must be large enough and aligned
    assert B.sparf_build_workspace_size(16, 40, 128) == 0
    assert B.sparf_build_workspace_size(1, 8, 128) == 8 * 64 * 128 * 4
    assert B.sparf_build_workspace_size(1, 40, 64) == 40 * 26 * 64 * 4
    assert B.sparf_build_workspace_size(0, 8, 128) == 0 and B.sparf_build_workspace_size(1, 8, 96) == 0
    small = ctypes.c_void_p(0x100000)
    assert L.instattn_sparf_build(ctypes.byref(d), ctypes.byref(a), FAKE, 1, 8, 128, small, 1000, None) == B.ERR_WORKSPACE
    assert L.instattn_sparf_build(ctypes.byref(d), ctypes.byref(a), FAKE, 1, 8, 128, ctypes.c_void_p(0x100010),
                                  1 << 20, None) == B.ERR_WORKSPACE
    assert L.instattn_sparf_append(ctypes.byref(d), ctypes.byref(a), None, FAKE, FAKE, 16, 40, 128,
                                   None) == B.ERR_INVALID_ARG
    assert L.instattn_sparf_append(ctypes.byref(d), ctypes.byref(a), FAKE, FAKE, FAKE, 0, 40, 128,
                                   None) == B.ERR_INVALID_ARG
    assert B.sparf_workspace_size(16, 40, 128, 4097, 256) >= 16 * 40 * (6144 + 256 + 1) * 4
    assert B.sparf_workspace_size(16, 40, 100, 4097, 256) == 0
    # a k beyond the row length (every row kept = the dense result) asks for no more room than k = row length
    assert B.sparf_workspace_size(16, 40, 128, 4097, 1 << 30) == B.sparf_workspace_size(16, 40, 128, 4097, 4097)


def test_kv_write_rejects():
    L = B.lib()
    d = desc()
    ok = [ctypes.byref(d), FAKE, FAKE, FAKE, FAKE, 16, 40, 128, 512, None]
    for idx, bad, want in [(1, None, B.ERR_INVALID_ARG), (2, None, B.ERR_INVALID_ARG),
                           (3, None, B.ERR_INVALID_ARG), (4, None, B.ERR_INVALID_ARG),
                           (1, FAKE + 2, B.ERR_INVALID_ARG), (5, 0, B.ERR_INVALID_ARG),
                           (6, 0, B.ERR_INVALID_ARG), (7, 96, B.ERR_UNSUPPORTED),
                           (8, 0, B.ERR_INVALID_ARG), (0, None, B.ERR_INVALID_ARG)]:
        args = list(ok)
        args[idx] = bad
        assert L.instattn_kv_write(*args) == want, idx


# ------------------------------------------------------------------ what a SparF decode launches
SPARF_ENV = ("INSTATTN_SPARF_THREE_LAUNCHES", "INSTATTN_SPARF_WIDE", "INSTATTN_SPARF_SPLIT_TAIL",
             "INSTATTN_SPARF_DISTRIBUTED")


@pytest.fixture
def no_sparf_env(options):
    return options


def test_sparf_plan_of_the_measured_shapes(no_sparf_env):
    # 16 x 40 heads x 4K: everything in one launch of 256 threads per head, append included
    p = B.sparf_plan(16, 40, 40, 128, 4097, 256, with_append=True)
    assert p == {"launches": 1, "one_launch_threads": 256, "append_fused": True, "selection": 0,
                 "select_and_gather": False, "slices": 1}
    # grouped queries: another head reads what the block would store, so the append stays a launch
    p = B.sparf_plan(4, 32, 8, 128, 4097, 256, with_append=True)
    assert p["launches"] == 2 and not p["append_fused"] and p["one_launch_threads"] == 256
    # 64 ragged sequences up to 16K: the 512-thread form
    p = B.sparf_plan(64, 40, 40, 128, 16385, 1024, with_append=True)
    assert p["launches"] == 1 and p["one_launch_threads"] == 512 and p["append_fused"]
    # 8 x 40 heads x 32K: score pass (which stores the new token), one block per head selects,
    # sliced gather, merge
    p = B.sparf_plan(8, 40, 40, 128, 32769, 2048, with_append=True)
    assert p == {"launches": 4, "one_launch_threads": 0, "append_fused": True, "selection": 1,
                 "select_and_gather": False, "slices": 4}
    # the same with grouped queries: the append is a launch of its own
    p = B.sparf_plan(8, 40, 8, 128, 32769, 2048, with_append=True)
    assert p["launches"] == 5 and not p["append_fused"]
    # 1 x 40 heads x 128K: selection spread over the stretches
    p = B.sparf_plan(1, 40, 40, 128, 131073, 8192)
    assert p["selection"] == 2 and p["slices"] == 8 and p["launches"] == 6


def test_sparf_plan_one_block_per_head_or_one_per_stretch(no_sparf_env):
    sel = lambda batch, L: B.sparf_plan(batch, 40, 40, 128, L, L // 16)["selection"]
    # up to 40K positions one block per head, whatever the number of heads
    for batch in (1, 2, 8, 16, 32):
        assert sel(batch, 32769) == 1 and sel(batch, 40960) == 1
    # from 96K on one block per stretch
    for batch in (1, 4, 16):
        assert sel(batch, 98304) == 2 and sel(batch, 262145) == 2
    assert sel(4, 98303) == 1
    # in between: few heads (at most 128) and many (more than 512) spread, about one round of blocks does not
    assert sel(1, 40961) == 2 and sel(2, 65537) == 2 and sel(3, 65537) == 2
    assert sel(4, 65537) == 1 and sel(8, 65537) == 1 and sel(12, 65537) == 1
    assert sel(13, 65537) == 2 and sel(16, 65537) == 2 and sel(32, 65537) == 2


def test_sparf_plan_limits_of_the_one_launch_kernel(no_sparf_env):
    assert B.sparf_plan(1, 1, 1, 64, 8192, 10)["one_launch_threads"] == 256        # any number of heads
    assert B.sparf_plan(1, 1, 1, 64, 8193, 10)["one_launch_threads"] == 0          # few heads: pipeline
    assert B.sparf_plan(4, 24, 24, 64, 8193, 10)["one_launch_threads"] == 512      # 96 heads
    assert B.sparf_plan(95, 1, 1, 64, 8193, 10)["one_launch_threads"] == 0
    assert B.sparf_plan(4, 32, 32, 64, 18432, 10)["one_launch_threads"] == 512
    assert B.sparf_plan(4, 32, 32, 64, 18433, 10)["one_launch_threads"] == 1024    # 128 heads: one round
    assert B.sparf_plan(8, 32, 32, 64, 36864, 10)["one_launch_threads"] == 1024    # 256 heads
    assert B.sparf_plan(8, 32, 32, 64, 36865, 10)["one_launch_threads"] == 0
    assert B.sparf_plan(3, 32, 32, 64, 18433, 10)["one_launch_threads"] == 1024    # 96 heads
    assert B.sparf_plan(1, 95, 95, 64, 18433, 10)["one_launch_threads"] == 0
    assert B.sparf_plan(1, 257, 257, 64, 18433, 10)["one_launch_threads"] == 0


def test_sparf_plan_pipeline_tail(no_sparf_env):
    # many heads, rows too long for one launch, few kept rows: one block per head selects and gathers
    p = B.sparf_plan(32, 40, 40, 128, 20000, 1000)
    assert p == {"launches": 2, "one_launch_threads": 0, "append_fused": False, "selection": 1,
                 "select_and_gather": True, "slices": 1}
    # ... not behind 65535 positions, where the one-block selection passes over memory (and the
    # host prefers the spread form: 5 launches)
    p = B.sparf_plan(32, 40, 40, 128, 70000, 1000)
    assert not p["select_and_gather"] and p["selection"] == 2 and p["launches"] == 5
    no_sparf_env.setenv("INSTATTN_SPARF_DISTRIBUTED", "0")
    p = B.sparf_plan(32, 40, 40, 128, 70000, 1000)
    assert not p["select_and_gather"] and p["selection"] == 1 and p["launches"] == 3
    no_sparf_env.delenv("INSTATTN_SPARF_DISTRIBUTED")
    # few heads with many kept rows: the gather is sliced, never more than 8 ways, never below 256 rows
    assert B.sparf_plan(1, 8, 8, 128, 20000, 20000)["slices"] == 8
    assert B.sparf_plan(1, 8, 8, 128, 20000, 600)["slices"] == 2
    assert B.sparf_plan(1, 8, 8, 128, 20000, 255)["slices"] == 1


def test_sparf_plan_environment_switches(no_sparf_env):
    m = no_sparf_env
    m.setenv("INSTATTN_SPARF_THREE_LAUNCHES", "1")
    p = B.sparf_plan(16, 40, 40, 128, 4097, 256, with_append=True)
    assert p["one_launch_threads"] == 0 and p["append_fused"] and p["launches"] == 2
    p = B.sparf_plan(16, 40, 8, 128, 4097, 256, with_append=True)
    assert p["one_launch_threads"] == 0 and not p["append_fused"] and p["launches"] == 3
    m.setenv("INSTATTN_SPARF_SPLIT_TAIL", "1")
    assert B.sparf_plan(16, 40, 40, 128, 4097, 256)["launches"] == 3
    m.delenv("INSTATTN_SPARF_THREE_LAUNCHES")
    m.setenv("INSTATTN_SPARF_WIDE", "1")
    assert B.sparf_plan(1, 2, 2, 128, 9000, 100)["one_launch_threads"] == 512
    m.setenv("INSTATTN_SPARF_WIDE", "0")
    assert B.sparf_plan(64, 40, 40, 128, 16385, 1024)["one_launch_threads"] == 0
    m.setenv("INSTATTN_SPARF_DISTRIBUTED", "1")
    assert B.sparf_plan(64, 40, 40, 128, 16385, 1024)["selection"] == 2
    m.setenv("INSTATTN_SPARF_DISTRIBUTED", "0")
    assert B.sparf_plan(1, 40, 40, 128, 131073, 8192)["selection"] == 1


def test_sparf_plan_rejects():
    for args in [(0, 4, 4, 128, 100, 10), (1, 4, 3, 128, 100, 10), (1, 4, 4, 128, 0, 10), (1, 4, 4, 128, 100, 0)]:
        with pytest.raises(B.InstattnError) as e:
            B.sparf_plan(*args)
        assert e.value.status == B.ERR_INVALID_ARG
    longest = 65535 * 8192              # the stretches of a row are a grid dimension of the distributed selection
    for args in [(1, 4, 4, 96, 100, 10), (1, 4, 4, 128, longest + 1, 10)]:
        with pytest.raises(B.InstattnError) as e:
            B.sparf_plan(*args)
        assert e.value.status == B.ERR_UNSUPPORTED
    assert B.sparf_workspace_size(1, 4, 128, longest + 1, 10) == 0
    assert B.sparf_workspace_size(1, 4, 128, longest, 10) > longest * 4 * 4


# ------------------------------------------------------------------ the header as plain C
def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """include/instattn.h compiles as C99 with every warning on, and a C program that
    uses it links against the library and runs its host-only entry points."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_header.c"
    src.write_text(r'''
#include <stdio.h>
#include "instattn.h"
int main(void) {
    int chunk = 0, splits = 0;
    int32_t plan[6];
    instattn_kv_desc kv = {0};
    instattn_sparf_aux aux = {0};
    (void)kv; (void)aux;
    if (instattn_version() < 100) return 1;
    if (instattn_decode_plan(16, 40, 40, 128, 4097, &chunk, &splits) != INSTATTN_OK) return 2;
    if (instattn_sparf_plan(16, 40, 40, 128, 4097, 256, 1, plan) != INSTATTN_OK) return 3;
    if (instattn_decode(NULL, NULL, NULL, 1, 1, 1, 128, 1.0f, NULL, INSTATTN_F16, NULL, NULL, 0, 1, NULL)
        != INSTATTN_ERR_INVALID_ARG) return 4;
    printf("%d %d %d %s\n", chunk, splits, plan[0], instattn_status_string(INSTATTN_ERR_WORKSPACE));
    return 0;
}
''')
    exe = tmp_path / "use_header"
    lib_dir = os.path.dirname(B.LIB_PATH)
    B.lib()                                    # raises if the library is not built
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", lib_dir, "-l:libinstattn.so", "-Wl,-rpath," + lib_dir],
                   check=True)
    env = dict(os.environ)
    for name in list(env):
        if name.startswith("INSTATTN_"):
            del env[name]
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True, env=env).stdout.split(None, 3)
    assert (int(out[0]), int(out[1]), int(out[2])) == (2176, 2, 1)
    assert out[3].strip() == "workspace missing, misaligned or too small"


# ------------------------------------------------------------------ bench.py's command line
def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU only" in r.stderr and r.stdout.strip() == ""


def test_smoke_and_bench_fail_loudly_without_a_gpu():
    """No CPU fallback anywhere on the product path: without a GPU the smoke run and the
    bench raise instead of computing something else."""
    import subprocess
    import sys
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "1", "--warmup", "0",
                        "--no-cpu-baseline"], capture_output=True, text=True)
    assert r.returncode != 0 and r.stdout.strip() == ""
    r = subprocess.run([sys.executable, "-c", "import __graft_entry__ as g; g.smoke()"], cwd=ROOT,
                       capture_output=True, text=True)
    assert r.returncode != 0


def test_descriptors_keep_their_tensors_alive():
    """The C structs hold bare addresses; the binding's objects must own what they point
    at, or a caller that drops its tensors hands the kernels freed memory."""
    import gc
    import weakref

    import torch
    k = torch.zeros(2, 1, 16, 64, dtype=torch.float16)
    v = torch.zeros_like(k)
    table = torch.zeros(1, 2, dtype=torch.int32)
    kt = torch.zeros(1, 1, 64, 32, dtype=torch.float16)
    vsum = torch.zeros(1, 1, 64, dtype=torch.float32)
    desc, aux = B.kv_desc(k, v, table), B.sparf_aux(kt, vsum)
    refs = [weakref.ref(t) for t in (k, v, table, kt, vsum)]
    addr = (k.data_ptr(), v.data_ptr(), table.data_ptr(), kt.data_ptr(), vsum.data_ptr())
    del k, v, table, kt, vsum
    gc.collect()
    assert all(r() is not None for r in refs)
    assert (desc.k, desc.v, desc.page_table, aux.kt) == addr[:4]
    assert ctypes.cast(aux.vsum, ctypes.c_void_p).value == addr[4]
    del desc, aux
    gc.collect()
    assert all(r() is None for r in refs)
