"""CPU sanitizer leg: the host side of the library (argument checks, plans, workspace
carving) and the C form of the oracle, built with AddressSanitizer and
UndefinedBehaviorSanitizer and run on the CPU.  No GPU is touched: the library's kernel
launchers are replaced by stubs that write, on the host, into the parts of the workspace
their kernels address (tests/host/stub_launch.hip)."""
import os
import struct
import subprocess

import numpy as np
import pytest

from oracle import decode_attention as np_oracle
from paper_2409_04992_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HOST = os.path.join(ROOT, "tests", "host")
CSRC = os.path.join(ROOT, "paper_2409_04992_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def test_host_side_of_the_library_under_sanitizers(tmp_path):
    """Every entry point over a sweep of shapes and of the switches that force a form, with
    a workspace of exactly the size the library asked for: a region carved too small or
    behind the end (as the distributed SparF selection's state once was for short rows) is a
    heap overflow here, overlapping regions and grids beyond the launch limits abort."""
    if not os.path.exists(HIPCC):
        pytest.skip("no hipcc")
    exe = tmp_path / "san_host"
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17",
           # host pass only: the device pass has no sanitizers on this target
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           os.path.join(CSRC, "api.hip"), os.path.join(CSRC, "api_sparf.hip"),
           os.path.join(HOST, "stub_launch.hip"), "-x", "hip", os.path.join(HOST, "san_main.cpp"), "-o", str(exe)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=ENV, timeout=600)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    assert "no report" in r.stdout and "ERROR" not in r.stderr
    calls, launches = (int(x) for x in r.stdout.split() if x.isdigit())
    assert calls > 20000 and launches > calls


def run_c_oracle(exe, tmp_path, case):
    wl = case.wl
    k, v = case.k_cache.numpy(), case.v_cache.numpy()
    paged = case.page_table is not None
    head = [wl.batch, wl.num_q_heads, wl.num_kv_heads, wl.head_dim, 0 if paged else k.shape[2],
            k.shape[2] if paged else 0, case.page_table.shape[1] if paged else 0, k.shape[0]]
    src, dst = tmp_path / "case.bin", tmp_path / "result.bin"
    with open(src, "wb") as f:
        f.write(struct.pack("8i", *head))
        f.write(struct.pack("f", case.scale))
        for t in (case.q, case.k_cache, case.v_cache, case.k_new, case.v_new, case.seq_lens):
            f.write(np.ascontiguousarray(t.numpy()).tobytes())
        if paged:
            f.write(np.ascontiguousarray(case.page_table.numpy()).tobytes())
    r = subprocess.run([str(exe), str(src), str(dst)], capture_output=True, text=True, env=ENV, timeout=300)
    assert r.returncode == 0, (r.stdout + r.stderr)[-4000:]
    raw = open(dst, "rb").read()
    n = k.size
    got_k = np.frombuffer(raw, np.uint16, n).reshape(k.shape)
    got_v = np.frombuffer(raw, np.uint16, n, offset=2 * n).reshape(k.shape)
    out = np.frombuffer(raw, np.float64, wl.batch * wl.num_q_heads * wl.head_dim, offset=4 * n)
    lse = np.frombuffer(raw, np.float64, wl.batch * wl.num_q_heads, offset=4 * n + 8 * out.size)
    return got_k, got_v, out.reshape(wl.batch, wl.num_q_heads, wl.head_dim), lse.reshape(wl.batch, wl.num_q_heads)


def test_c_oracle_under_sanitizers(tmp_path):
    """oracle/decode_attention.c built with -fsanitize=address,undefined: ragged and empty
    sequences, a sequence that fills its cache, both layouts, grouped heads, poisoned slack -
    against the numpy form (bit-exact caches, rows to 1e-12) and against closed forms."""
    exe = tmp_path / "san_oracle"
    r = subprocess.run(["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                        "-Wall", os.path.join(HOST, "san_oracle.c"), os.path.join(ROOT, "oracle", "decode_attention.c"),
                        "-o", str(exe), "-lm"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    shapes = [W.Workload("san_contig", 5, 6, 3, 64, 300, seq_len_min=1, seed=51),
              W.Workload("san_paged", 6, 4, 4, 128, 200, seq_len_min=1, paged=True, seed=52),
              W.Workload("san_paged_gqa", 4, 8, 1, 64, 97, seq_len_min=1, paged=True, page_size=32, seed=53)]
    for wl in shapes:
        lens = [int(x) for x in W.draw_seq_lens(wl)]
        lens[0], lens[1], lens[2] = 0, wl.seq_len + 1, 1          # empty, filling the cache, a single row
        case = W.make_case(wl, "cpu", poison=True, lens=lens)
        got_k, got_v, out, lse = run_c_oracle(exe, tmp_path, case)
        k, v = case.k_cache.numpy().copy(), case.v_cache.numpy().copy()
        pt = None if case.page_table is None else case.page_table.numpy()
        np_oracle.kv_append(k, v, case.k_new.numpy(), case.v_new.numpy(), case.seq_lens.numpy(), pt)
        want, want_lse = np_oracle.decode(case.q.numpy(), k, v, case.seq_lens.numpy(), case.scale, pt)
        assert np.array_equal(got_k, k.view(np.uint16)) and np.array_equal(got_v, v.view(np.uint16))
        assert np.abs(out - want).max() < 1e-12
        assert np.array_equal(np.isinf(lse), np.isinf(want_lse))
        fin = np.isfinite(want_lse)
        assert np.abs(lse[fin] - want_lse[fin]).max() < 1e-12
        # closed forms on the sanitized build itself: an empty sequence gives a zero row, a
        # single row returns that row of V exactly
        assert not out[0].any() and np.isneginf(lse[0]).all()
        g = wl.group
        assert np.array_equal(out[2], np.repeat(case.v_new.numpy()[2].astype(np.float64), g, axis=0))
    # identical keys => the mean of V (closed form), through the sanitized build
    wl = W.Workload("san_mean", 2, 2, 2, 64, 40, seed=54)
    case = W.make_case(wl, "cpu")
    case.k_cache[:] = case.k_cache[:, :, :1]
    case.k_new[:] = case.k_cache[:, :, 0]
    _, got_v, out, _ = run_c_oracle(exe, tmp_path, case)
    mean_v = got_v.view(np.float16)[:, :, :41].astype(np.float64).mean(axis=2)
    assert np.abs(out - mean_v).max() < 1e-12
