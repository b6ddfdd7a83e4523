#!/usr/bin/env python3
"""Decode-attention benchmark on one MI355X.

A step is one pass of the whole hot path over one batch: for every layer of the
workload the new token's k, v are appended to the cache and the query attends over
it (split pass + LSE merge where the plan splits), through the C ABI
(instattn_append_decode, or the two separate calls with --two-calls), with every
input already resident in HBM.  Steps rotate over several distinct layer caches so
that no step starts with its KV in the last-level cache.

With no --workload the ONE JSON line it prints has the largest single-GPU
configuration as its headline (gqa70b_16k: 80 layers, 172 GB of KV resident, a step
walks all 80) and carries the other timed configurations under "per_config"
(mha13b_4k, mha13b_32k, ragged_paged; same fields) and the SparF path (Algorithm 1)
at 1/8 of the dense bytes on those three shapes under "sparf".  --workload NAME times
that configuration alone (the form the rocprofv3 summaries under profiles/ are made
with).  --steps / --warmup apply to the headline; the per_config and sparf entries
use fixed counts of their own, stated in each entry.

Fields: whole-job KV GB/s (algorithmic K+V bytes / wall time of the timed steps),
the roofline of the split-pass kernel timed live with HIP events on the launch
stream (the split pass of the fused call the step makes), HBM traffic per launch
as read from the matching rocprofv3 summary under profiles/, and the CPU oracle
timed on the host cores as a baseline.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
HEADLINE = "gqa70b_16k"
# name -> (steps, warmup, resident layer caches) of the per_config entries
PER_CONFIG = {"mha13b_4k": (400, 40, 8), "mha13b_32k": (200, 20, 3), "ragged_paged": (100, 10, 2)}
# name -> ("r,k,l", steps, warmup) of the sparf entries: r = d_h/8 columns, k = L/16 rows, i.e. 1/8 of the dense bytes
SPARF = {"mha13b_4k": ("16,256,16", 300, 30), "mha13b_32k": ("16,2048,16", 200, 20),
         "ragged_paged": ("16,1024,16", 100, 10)}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default=None,
                    help="time this configuration alone: one of the named ones, or custom:{json fields of "
                         "Workload} for sweeps (default: headline %s plus per_config and sparf entries)" % HEADLINE)
    ap.add_argument("--layers-resident", type=int, default=None,
                    help="distinct layer caches the steps rotate over (single-layer workloads)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="default run without the per_config and sparf entries")
    ap.add_argument("--kt-page", type=int, default=None,
                    help="with --sparf: positions per page of the component-major K copy "
                         "(0: contiguous; default 256 for a paged workload, else 0)")
    ap.add_argument("--kt-capacity", type=int, default=None,
                    help="with --sparf and a contiguous component-major copy: positions it is allocated "
                         "for (multiple of 8; default: the cache's capacity)")
    ap.add_argument("--sparf", default=None, metavar="r,k,l",
                    help="time the SparF path (Algorithm 1) with these parameters instead of the "
                         "dense path, next to the dense step on the same caches")
    ap.add_argument("--kv-write", action="store_true",
                    help="time instattn_kv_write of a whole prompt (the prefill-side bulk store)")
    ap.add_argument("--graph", action="store_true",
                    help="replay the step's launches from a captured HIP graph instead of launching them "
                         "one by one (dense path)")
    ap.add_argument("--two-calls", action="store_true",
                    help="step = instattn_kv_append + instattn_decode instead of instattn_append_decode")
    return ap.parse_args()


# ----------------------------------------------------------------------------- profiles/
def profile_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` on `workload` from the rocprofv3 summary under
    profiles/ named for that kernel and workload (FETCH_SIZE and WRITE_SIZE runs scaled by
    what the same counters read for the 256 MiB copy kernel; the summary states the
    factors), or None when there is no such summary."""
    path = os.path.join(ROOT, "profiles", "%s__%s.txt" % (kernel, workload))
    if not os.path.exists(path):
        return None
    m = re.search(r"total HBM traffic (\d+) B", open(path).read())
    return int(m.group(1)) if m else None


def sparf_profile_traffic(workload, rkl):
    """The same for all launches of a SparF step (fetched + written), from the summary
    profiles/sparf_step__<workload>.txt made with the same r,k,l."""
    path = os.path.join(ROOT, "profiles", "sparf_step__%s.txt" % workload)
    if not os.path.exists(path):
        return None
    text = open(path).read()
    if "--sparf %s " % rkl not in text:
        return None
    m = re.search(r"all launches of a step: fetched (\d+) B.*?written (\d+) B", text)
    return int(m.group(1)) + int(m.group(2)) if m else None


# ----------------------------------------------------------------------------- CPU baseline
def cpu_baseline(cases, kv_bytes_layer, positions_layer):
    """The C oracle as it stands, on the host cores, on a bounded sample: whole
    layers of the same workload (every (sequence, head) pair, or every n-th pair if
    one layer alone would take much longer than the budget), about 10-30 s of CPU
    work in total."""
    from oracle import c_oracle
    cores = min(len(os.sched_getaffinity(0)), 16)
    wl = cases[0].wl
    pairs = wl.batch * wl.num_q_heads
    budget_cpu_s = 20.0

    def host(case):
        pt = None if case.page_table is None else case.page_table.cpu().numpy()
        return (case.q.cpu().numpy(), case.k_cache.cpu().numpy(), case.v_cache.cpu().numpy(),
                case.seq_lens.cpu().numpy(), case.scale, pt)

    # calibrate on a thin sample of the first layer
    args0 = host(cases[0])
    stride = max(1, pairs // (2 * cores))
    t = time.perf_counter()
    c_oracle.decode(*args0, pair_stride=stride, nthreads=cores)
    per_pair_cpu_s = (time.perf_counter() - t) * cores / len(range(0, pairs, stride))
    # every n-th pair only if one whole layer would take much longer than the budget;
    # then whole layers until about 12 s of CPU work are done (the thin calibration
    # sample overestimates, so the clock decides, not the estimate)
    want_pairs = 1.5 * budget_cpu_s / per_pair_cpu_s
    stride = max(1, int(pairs // want_pairs)) if want_pairs < pairs else 1
    done, dt, layers = 0, 0.0, 0
    while layers < len(cases) and dt * cores < 12.0:
        args = args0 if layers == 0 else host(cases[layers])
        t = time.perf_counter()
        c_oracle.decode(*args, pair_stride=stride, nthreads=cores)
        dt += time.perf_counter() - t
        done += len(range(0, pairs, stride))
        layers += 1
    frac = done / pairs          # in units of one layer
    # the same oracle on one core, on a sixteenth of the pairs of the first layer
    stride1 = max(16, stride * 16)
    t = time.perf_counter()
    c_oracle.decode(*args0, pair_stride=stride1, nthreads=1)
    dt1 = time.perf_counter() - t
    single = kv_bytes_layer * len(range(0, pairs, stride1)) / pairs / dt1 / 1e9
    return {
        "value": kv_bytes_layer * frac / dt / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
        "sample": "%d (sequence, head) pairs = every %d-th pair of %d layer(s) of workload %s, "
                  "fp64 C oracle, %d OpenMP threads, %.1f s wall" % (done, stride, layers, wl.name, cores, dt),
        "single_core_value": single,
        "attended_tokens_per_s": positions_layer * frac / dt,
    }


# ----------------------------------------------------------------------------- SparF
def sparf_setup(cases, descs, kt_page, kt_capacity=None):
    """Component-major K copy and V sum for every resident layer (instattn_sparf_build)."""
    import torch
    from paper_2409_04992_amd import binding as B
    wl = cases[0].wl
    dev = cases[0].q.device
    auxs = []
    for c, d in zip(cases, descs):
        Bn, Hkv, cap, D = wl.batch, wl.num_kv_heads, c.capacity, wl.head_dim
        vsum = torch.zeros(Bn, Hkv, D, dtype=torch.float32, device=dev)
        if kt_page == 0:
            kt, kt_table = torch.zeros(Bn, Hkv, D, max(cap, kt_capacity or 0), dtype=torch.float16, device=dev), None
        else:
            # the component-major copy in pages of its own size behind a shuffled table
            need = [(int(L) + kt_page - 1) // kt_page for L in c.seq_lens.cpu().tolist()]
            pool = sum(need)
            kt = torch.zeros(pool, Hkv, D, kt_page, dtype=torch.float16, device=dev)
            perm = torch.randperm(pool, generator=torch.Generator().manual_seed(wl.seed)).to(torch.int32)
            kt_table = torch.full((Bn, (cap + kt_page - 1) // kt_page), -1, dtype=torch.int32)
            at = 0
            for b in range(Bn):
                kt_table[b, :need[b]] = perm[at:at + need[b]]
                at += need[b]
            kt_table = kt_table.to(dev)
        a = B.sparf_aux(kt, vsum, kt_table)
        B.sparf_build(d, a, (c.seq_lens - 1).contiguous(), Hkv, D)
        auxs.append(a)
    return auxs


def time_sparf(cases, descs, rkl, steps, warmup, kt_page, two_calls=False, kt_capacity=None):
    """SparF step (sparf_append_decode) and the dense step on the same caches."""
    import torch
    from paper_2409_04992_amd import binding as B
    wl = cases[0].wl
    dev = cases[0].q.device
    r, k, l = (int(x) for x in rkl.split(","))
    R = len(cases)
    auxs = sparf_setup(cases, descs, kt_page, kt_capacity)
    max_len = int(cases[0].seq_lens.max().item())
    lens = cases[0].seq_lens.cpu().tolist()
    D, Hq = wl.head_dim, wl.num_q_heads
    ws = torch.empty(B.sparf_workspace_size(wl.batch, Hq, D, max_len, k), dtype=torch.uint8, device=dev)
    wsd = B.alloc_workspace(wl.batch, Hq, wl.num_kv_heads, D, max_len, dev)
    out = torch.empty(wl.batch, Hq, D, dtype=torch.float16, device=dev)
    dense_bytes = cases[0].kv_read_bytes()
    sparf_bytes = sum(Hq * 2 * (r * L + 2 * min(k, L) * D) for L in lens)
    score_bytes = sum(Hq * 4 * L * 2 for L in lens)          # fp32 scores written, then read by the selection

    def sparf_step(i):
        c, d, a = cases[i % R], descs[i % R], auxs[i % R]
        if two_calls:
            B.sparf_append(d, a, c.k_new, c.v_new, c.seq_lens)
            B.sparf_decode(c.q, d, a, c.seq_lens, wl.num_kv_heads, c.scale, r, k, l, out, ws, max_len)
        else:
            B.sparf_append_decode(c.q, c.k_new, c.v_new, d, a, c.seq_lens, wl.num_kv_heads, c.scale,
                                  r, k, l, out, ws, max_len)

    def dense_step(i):
        c, d = cases[i % R], descs[i % R]
        B.append_decode(c.q, c.k_new, c.v_new, d, c.seq_lens, wl.num_kv_heads, c.scale, out, wsd, max_len)

    def timed(fn):
        for i in range(warmup):
            fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            fn(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    t_sparf, t_dense = timed(sparf_step), timed(dense_step)
    # What the memory system gives on the addresses of the score pass: a bare read of r of
    # the D columns of every head over the same copies (contiguous copies of equal lengths only).
    column_read = None
    if kt_page == 0 and len(set(lens)) == 1 and lens[0] >= 16:
        sink = torch.zeros(4096, dtype=torch.int32, device=dev)
        positions = lens[0] // 8 * 8
        ev = []
        for i in range(12):
            a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a0.record()
            B.probe_read_columns(auxs[i % R].tensors[0], r, positions, sink)
            a1.record()
            ev.append((a0, a1))
        torch.cuda.synchronize()
        ms = sorted(x.elapsed_time(y) for x, y in ev[2:])
        col_bytes = wl.batch * wl.num_kv_heads * r * positions * 2
        column_read = {"GBps": col_bytes / (ms[len(ms) // 2] * 1e-3) / 1e9, "bytes": col_bytes,
                       "us": ms[len(ms) // 2] * 1e3,
                       "what": "bare read of r of the D columns of every KV head's component-major copy (no arithmetic)"}
    plan = B.sparf_plan(wl.batch, Hq, wl.num_kv_heads, D, max_len, k, with_append=not two_calls)
    default_page = kt_page == (256 if wl.paged else 0)
    return {
        "metric": "sparf_decode_attention_dense_equivalent_kv_bandwidth",
        "value": dense_bytes / t_sparf / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": t_sparf * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": wl.name, "r": r, "k": k, "l": l, "layers_resident": R,
                   "kt_page": kt_page, "launches": plan["launches"],
                   "step": ("sparf_append + sparf_decode" if two_calls else "sparf_append_decode") +
                           " (column scores, selection, gather attention)"},
        "dense_ms_per_step": t_dense * 1e3, "speedup_over_dense_step": t_dense / t_sparf,
        "bytes_read_algorithm1": sparf_bytes, "bytes_read_dense": dense_bytes,
        "compression": sparf_bytes / dense_bytes, "score_bytes_written_and_read": score_bytes,
        "column_read_probe": column_read,
        # the whole step (one or several launches) against the bytes Algorithm 1 must read
        "roofline": {"bound": "hbm", "achieved": sparf_bytes / t_sparf / 1e9, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": sparf_bytes / t_sparf / 1e9 / HBM_PEAK_GBPS,
                     "traffic": sparf_profile_traffic(wl.name, rkl) if default_page and not two_calls else None,
                     "kernel": "whole SparF step", "algorithmic_bytes_per_launch": sparf_bytes},
    }


def sparf_cpu_baseline(cases, r, k, l, budget_s=10.0):
    """The fp64 numpy oracle of Algorithm 1 as it stands, one (sequence, head) pair after
    the other on one core, over the resident layers in order until about 10 s of CPU
    work are done (a pair's rows are gathered on the device and copied over, outside
    the clock)."""
    from oracle import sparf_attention as sparf_oracle
    wl = cases[0].wl
    done, bytes_done, dt = 0, 0, 0.0
    for case in cases:
        lens = case.seq_lens.cpu().numpy()
        ps = case.k_cache.shape[2]
        for b in range(wl.batch):
            for h in range(wl.num_q_heads):
                if dt >= budget_s:
                    break
                hk, L = h // wl.group, int(lens[b])
                if case.page_table is None:
                    K, V = case.k_cache[b, hk, :L], case.v_cache[b, hk, :L]
                else:
                    pages = case.page_table[b, :(L + ps - 1) // ps].long()
                    K = case.k_cache[pages, hk].reshape(-1, wl.head_dim)[:L]
                    V = case.v_cache[pages, hk].reshape(-1, wl.head_dim)[:L]
                q, K, V = case.q[b, h].cpu().numpy(), K.cpu().numpy(), V.cpu().numpy()
                t = time.perf_counter()
                sparf_oracle.sparf_one(q, K, V, case.scale, r, k, l)
                dt += time.perf_counter() - t
                done += 1
                bytes_done += 2 * L * wl.head_dim * 2 // wl.group     # this head's share of the dense K + V bytes
    return {"value": bytes_done / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "%d (sequence, head) pairs of the same workload's layers in order, fp64 numpy "
                      "oracle of Algorithm 1, 1 thread, %.1f s; value in dense-equivalent KV bytes like the "
                      "metric" % (done, dt)}


def bench_sparf(args):
    from paper_2409_04992_amd import binding as B
    from paper_2409_04992_amd import workloads as W
    wl = W.get_workload(args.workload or "mha13b_4k")
    kt_page = args.kt_page if args.kt_page is not None else (256 if wl.paged else 0)
    R = max(1, args.layers_resident or 8)
    cases = [W.make_case(wl, "cuda:0", layer=i) for i in range(R)]
    descs = [B.kv_desc(c.k_cache, c.v_cache, c.page_table) for c in cases]
    res = time_sparf(cases, descs, args.sparf, args.steps or 200, args.warmup or 20, kt_page,
                     two_calls=args.two_calls, kt_capacity=args.kt_capacity)
    if not args.no_cpu_baseline:
        r, k, l = (int(x) for x in args.sparf.split(","))
        res["cpu_baseline"] = sparf_cpu_baseline(cases, r, k, l)
    print(json.dumps(res), flush=True)


# ----------------------------------------------------------------------------- bulk write
def bench_kv_write(args):
    """Bulk store of seq_len prompt rows per sequence into the cache (one layer)."""
    import torch
    from paper_2409_04992_amd import binding as B
    from paper_2409_04992_amd import workloads as W
    dev = "cuda:0"
    wl = W.get_workload(args.workload or "mha13b_4k")
    steps, warmup = args.steps or 50, args.warmup or 5
    R = 3
    cases = [W.make_case(wl, dev, layer=i) for i in range(R)]
    descs = [B.kv_desc(c.k_cache, c.v_cache, c.page_table) for c in cases]
    S = wl.seq_len
    srcs = [(torch.randn(wl.batch, wl.num_kv_heads, S, wl.head_dim, device=dev).half(),
             torch.randn(wl.batch, wl.num_kv_heads, S, wl.head_dim, device=dev).half()) for _ in range(R)]
    start = torch.zeros(wl.batch, dtype=torch.int32, device=dev)
    count = (cases[0].seq_lens - 1).contiguous()
    nbytes = int(count.sum().item()) * wl.num_kv_heads * wl.head_dim * 2 * 2

    def step(i):
        B.kv_write(descs[i % R], srcs[i % R][0], srcs[i % R][1], start, count)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    print(json.dumps({
        "metric": "kv_write_bandwidth_read_plus_write", "value": 2 * nbytes / dt / 1e9, "unit": "GB/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": dt * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic", "config": {"workload": wl.name, "rows_per_sequence": "seq_len",
                                        "kv_layout": "paged16" if wl.paged else "contiguous"},
        "bytes_stored": nbytes, "pct_of_hbm_peak": 100.0 * 2 * nbytes / dt / 1e9 / HBM_PEAK_GBPS}), flush=True)


# ----------------------------------------------------------------------------- dense path
def time_dense(cases, descs, steps, warmup, two_calls=False, graph=False, probes=True):
    """Times `steps` steps of the dense path over the given resident layer caches and the
    split pass on its own; returns the fields of one bench entry."""
    import torch
    from paper_2409_04992_amd import binding as B
    wl = cases[0].wl
    dev = cases[0].q.device
    R, lps = len(cases), wl.layers
    max_len = int(cases[0].seq_lens.max().item())
    ws = B.alloc_workspace(wl.batch, wl.num_q_heads, wl.num_kv_heads, wl.head_dim, max_len, dev)
    out_dtype = torch.float32 if wl.out_dtype == "f32" else torch.float16
    out = torch.empty(wl.batch, wl.num_q_heads, wl.head_dim, dtype=out_dtype, device=dev)
    kv_bytes_layer = cases[0].kv_read_bytes()
    kv_bytes = kv_bytes_layer * lps                      # per step
    positions = int(cases[0].seq_lens.sum().item()) * lps
    chunk, splits = B.decode_plan(wl.batch, wl.num_q_heads, wl.num_kv_heads, wl.head_dim, max_len)
    launches = B.decode_launches(wl.batch, wl.num_q_heads, wl.num_kv_heads, wl.head_dim, max_len, not two_calls,
                                 paged=wl.paged)

    def step(i):
        for j in range(lps):
            c, d = cases[(i * lps + j) % R], descs[(i * lps + j) % R]
            if two_calls:
                B.kv_append(d, c.k_new, c.v_new, c.seq_lens)
                B.decode(c.q, d, c.seq_lens, wl.num_kv_heads, c.scale, out, ws, max_len)
            else:
                B.append_decode(c.q, c.k_new, c.v_new, d, c.seq_lens, wl.num_kv_heads, c.scale,
                                out, ws, max_len)

    if graph:
        # One graph holds as many consecutive steps as it takes to come back to the first
        # resident layer cache; the timed loop replays it.
        per_graph = max(1, R // lps)
        steps = max(per_graph, steps // per_graph * per_graph)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(0)                                    # warm everything the capture touches
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(per_graph):
                step(i)

        def run(n_steps):
            for _ in range(n_steps // per_graph):
                g.replay()
    else:
        def run(n_steps):
            for i in range(n_steps):
                step(i)
    run(warmup if not graph else max(1, warmup // max(1, R // lps)) * max(1, R // lps))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(steps)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / steps * 1e3
    value = kv_bytes * steps / wall / 1e9

    # Dominant kernel on its own: the split pass of the call the step makes (the fused
    # append included; where the plan lists the units first, that small launch too), HIP
    # events on the launch stream.
    n_k = min(steps * lps, 200)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(n_k)]
    for i in range(n_k):
        c, d = cases[i % R], descs[i % R]
        ev[i][0].record()
        if two_calls:
            B.decode_partial(c.q, d, c.seq_lens, wl.num_kv_heads, c.scale, out, ws, max_len)
        else:
            B.append_decode_partial(c.q, c.k_new, c.v_new, d, c.seq_lens, wl.num_kv_heads, c.scale, out, ws,
                                    max_len)
        ev[i][1].record()
    torch.cuda.synchronize()
    k_ms = sorted(a.elapsed_time(b) for a, b in ev)
    k_avg_ms = sum(k_ms) / len(k_ms)
    achieved = kv_bytes_layer / (k_avg_ms * 1e-3) / 1e9
    kernel = "decode_mha_kernel" if wl.group == 1 else "decode_gqa_kernel"

    res = {
        "metric": "decode_attention_kv_bandwidth", "value": value, "unit": "GB/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": wl.name, "batch": wl.batch, "num_q_heads": wl.num_q_heads,
                   "num_kv_heads": wl.num_kv_heads, "head_dim": wl.head_dim,
                   "seq_len": wl.seq_len, "kv_layout": "paged16" if wl.paged else "contiguous",
                   "out_dtype": wl.out_dtype, "layers_resident": R, "layers_per_step": lps,
                   "step": ("kv_append; decode" if two_calls else "append_decode (append fused into "
                            "the split pass)") + (", LSE merge" if splits > 1 else ", single split: no merge")
                           + (", unit list built on the device in front" if launches["unit_list"] else "")
                           + ", for each layer of the step"
                           + ("; launches replayed from a HIP graph" if graph else ""),
                   "chunk_tokens": chunk, "num_splits": splits,
                   "kv_bytes_per_step": kv_bytes},
        "pct_of_hbm_peak": 100.0 * value / HBM_PEAK_GBPS,
        "attended_tokens_per_s": positions * steps / wall,
        "attended_head_tokens_per_s": positions * wl.num_q_heads * steps / wall,
        # a step that walks every layer produces one token per sequence (attention only)
        "decode_tokens_per_s_attention_only": wl.batch * steps / wall if lps > 1 else None,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": profile_traffic(kernel, wl.name),
                     "kernel": kernel + (" (split pass of the step's call" +
                                         ("; the unit-list launch in front of it is inside the events" if launches["unit_list"] else "") + ")"),
                     "kernel_ms_avg": k_avg_ms, "kernel_ms_median": k_ms[len(k_ms) // 2],
                     "kernel_ms_min": k_ms[0], "launches_timed": n_k,
                     "algorithmic_bytes_per_launch": kv_bytes_layer},
    }
    if probes:
        res.update(time_probes(kv_bytes_layer, dev))
    return res


def time_probes(kv_bytes_layer, dev):
    """Read ceiling: a plain streaming-read kernel over a buffer of the size one launch of
    the split pass reads (K and V of a layer), two buffers in turn so that none is warm.
    And a plain copy of known size (256 MiB read + 256 MiB written per launch): the
    reference kernel for scaling the hardware traffic counters."""
    import torch
    from paper_2409_04992_amd import binding as B
    sink = torch.zeros(4096, dtype=torch.int32, device=dev)
    n_probe = (kv_bytes_layer + 4095) // 4096 * 4096
    flat = [torch.empty(n_probe, dtype=torch.uint8, device=dev).random_(0, 255) for _ in range(2)]
    rd = []
    for i in range(12):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        B.probe_read(flat[i % 2], sink)
        b.record()
        rd.append((a, b))
    torch.cuda.synchronize()
    rd_ms = sorted(a.elapsed_time(b) for a, b in rd[2:])
    ceiling = n_probe / (sum(rd_ms) / len(rd_ms) * 1e-3) / 1e9
    del flat
    csrc = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
    cdst = torch.empty_like(csrc)
    cp = []
    for i in range(6):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        B.probe_copy(csrc, cdst)
        b.record()
        cp.append((a, b))
    torch.cuda.synchronize()
    cp_ms = sorted(a.elapsed_time(b) for a, b in cp[1:])
    copy_gbps = 2 * csrc.numel() / (sum(cp_ms) / len(cp_ms) * 1e-3) / 1e9
    return {"read_ceiling_GBps": ceiling, "copy_GBps_read_plus_write": copy_gbps}


def release():
    """Hands the freed device memory back to the driver and waits for it.  Behind a large
    free the device reads slower for a while, whatever process runs there (measured with
    the 4K configuration next to the 172 GB of the headline: 85.4 % of peak while those
    stay resident, 83.2 ... 81.9 % during the first 4 s after they are freed, 84.8 % from
    8 s on): the wait scales with the bytes freed."""
    import torch
    before = torch.cuda.memory_reserved()
    torch.cuda.empty_cache()
    freed = before - torch.cuda.memory_reserved()
    time.sleep(1.0 + 0.06 * freed / 1e9)


def make_cases(wl, R):
    from paper_2409_04992_amd import binding as B
    from paper_2409_04992_amd import workloads as W
    cases = [W.make_case(wl, "cuda:0", layer=i) for i in range(R)]
    return cases, [B.kv_desc(c.k_cache, c.v_cache, c.page_table) for c in cases]


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2409_04992_amd import binding as B
    from paper_2409_04992_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.lib()                                   # fail loudly if the HIP library is missing
    if args.sparf:
        return bench_sparf(args)
    if args.kv_write:
        return bench_kv_write(args)

    extras = args.workload is None and not args.no_extras and not args.graph and not args.two_calls
    wl = W.get_workload(args.workload or HEADLINE)
    # a multi-layer workload keeps all its layers resident and a step walks them all
    R = wl.layers if wl.layers > 1 else max(1, args.layers_resident or 8)
    # The headline first, before this process has freed anything (see release()).
    cases, descs = make_cases(wl, R)
    steps = args.steps if args.steps is not None else (400 if wl.layers == 1 else 20)
    warmup = args.warmup if args.warmup is not None else (40 if wl.layers == 1 else 2)
    res = time_dense(cases, descs, steps, warmup, two_calls=args.two_calls, graph=args.graph)
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cases, cases[0].kv_read_bytes(),
                                           int(cases[0].seq_lens.sum().item()))
    if extras:
        del cases, descs
        release()
        per_config, sparf = {}, {}
        # the smaller configurations, each freed before the next
        for name, (c_steps, c_warmup, c_R) in PER_CONFIG.items():
            R_sparf = 8 if name == "mha13b_4k" else c_R        # the 4K SparF step touches 168 MB: 8 caches keep it out of the last-level cache
            cases, descs = make_cases(W.get_workload(name), max(c_R, R_sparf))
            e = time_dense(cases[:c_R], descs[:c_R], c_steps, c_warmup, probes=False)
            per_config[name] = {k: e[k] for k in ("value", "unit", "steps", "warmup", "ms_per_step", "pct_of_hbm_peak",
                                                  "attended_tokens_per_s", "config", "roofline")}
            rkl, s_steps, s_warmup = SPARF[name]
            e = time_sparf(cases, descs, rkl, s_steps, s_warmup, 256 if cases[0].wl.paged else 0)
            sparf[name] = {k: e[k] for k in ("value", "unit", "steps", "warmup", "ms_per_step", "dense_ms_per_step",
                                             "speedup_over_dense_step", "bytes_read_algorithm1", "compression",
                                             "column_read_probe", "config", "roofline")}
            del cases, descs, e
            release()
        res["per_config"] = per_config
        res["sparf"] = sparf
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
