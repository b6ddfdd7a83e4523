// Host-only stand-ins for the kernel launchers, for the sanitizer build of the host side of
// the library (tests/test_sanitizers.py): the real argument checks, plans and workspace
// carving of csrc/api.hip and csrc/api_sparf.hip run on the CPU under AddressSanitizer and
// UndefinedBehaviorSanitizer, and every "launch" touches, on the host, exactly the parts of
// the workspace its kernel addresses (extents as documented with the argument structs).
// The workspace is a host allocation of exactly the size the library asked for, so a
// region carved too small, or carved behind the end, is an out-of-bounds write here; regions
// that overlap are reported by the interval check.  Caches, queries and outputs are never
// touched (the driver passes small dummy allocations for them).
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "../../paper_2409_04992_amd/csrc/common.h"
#include "../../paper_2409_04992_amd/csrc/sparf.h"

namespace instattn {

namespace {

struct Region {
    const char* name;
    char* begin;
    size_t bytes;
};

int g_launches = 0;

[[noreturn]] void fail(const char* what, const char* name)
{
    fprintf(stderr, "stub_launch: %s (%s)\n", what, name);
    abort();
}

// Writes into every region - its first and last byte and one byte per 64 KB, which is enough
// for AddressSanitizer to see a region that reaches outside the workspace - and checks that
// no two overlap.
void touch(std::vector<Region> regions)
{
    ++g_launches;
    for (const Region& r : regions) {
        if (r.bytes == 0) continue;
        if (r.begin == nullptr) fail("null region", r.name);
        for (size_t i = 0; i < r.bytes; i += 65536) r.begin[i] = 0x5A;
        r.begin[r.bytes - 1] = 0x5A;
    }
    std::sort(regions.begin(), regions.end(), [](const Region& x, const Region& y) { return x.begin < y.begin; });
    for (size_t i = 1; i < regions.size(); ++i)
        if (regions[i - 1].bytes && regions[i].bytes && regions[i - 1].begin + regions[i - 1].bytes > regions[i].begin)
            fail("regions overlap", regions[i].name);
}

std::vector<Region> decode_regions(const DecodeArgs& a, int batch, int head_dim)
{
    const size_t units = (size_t)batch * a.num_q_heads * a.num_splits;
    std::vector<Region> r;
    if (a.num_splits > 1) {
        r.push_back({"o_part", (char*)a.o_part, units * head_dim * sizeof(float)});
        r.push_back({"lse_part", (char*)a.lse_part, units * sizeof(float)});
    }
    if (a.unit_list) r.push_back({"unit_list", (char*)a.unit_list, (size_t)a.list_len * sizeof(int32_t)});
    return r;
}

void check_grid(const DecodeArgs& a, int batch, int heads)
{
    if (a.chunk <= 0 || a.chunk % 128 || (int64_t)a.chunk * a.num_splits < a.max_len) fail("units do not cover the rows", "plan");
    if (a.unit_list) {
        if (a.list_len != batch * a.num_splits) fail("list length", "unit_list");
        if (((int64_t)a.list_len + 7) / 8 * 8 * heads > (int64_t)INT32_MAX) fail("one-dimensional grid too large", "unit_list");
    } else if (a.group_blocks > 1) {
        if (((int64_t)batch * a.num_kv_heads * a.num_splits + 8) * a.group_blocks > (int64_t)INT32_MAX)
            fail("one-dimensional grid too large", "group_blocks");
    } else if (a.num_splits > 65535 || batch > 65535) {
        fail("grid dimension beyond 65535", "grid");
    }
}

size_t sparf_rows(const SparfArgs& a) { return (size_t)a.batch * a.num_q_heads; }

Region sel_region(const SparfArgs& a) { return {"sel", (char*)a.sel, sparf_rows(a) * (size_t)a.k * sizeof(int32_t)}; }
Region alpha_region(const SparfArgs& a) { return {"alpha", (char*)a.alpha, sparf_rows(a) * sizeof(float)}; }

}  // namespace

int stub_launch_count() { return g_launches; }

hipError_t launch_decode_mha(const DecodeArgs& a, int batch, int head_dim, hipStream_t)
{
    check_grid(a, batch, a.num_q_heads);
    touch(decode_regions(a, batch, head_dim));
    return hipSuccess;
}

hipError_t launch_decode_gqa(const DecodeArgs& a, int batch, int head_dim, hipStream_t)
{
    check_grid(a, batch, a.num_kv_heads);
    touch(decode_regions(a, batch, head_dim));
    return hipSuccess;
}

hipError_t launch_list_units(const DecodeArgs& a, int batch, hipStream_t)
{
    if (batch > 4096 || a.list_len != batch * a.num_splits) fail("list launch outside its limits", "unit_list");
    touch({{"unit_list", (char*)a.unit_list, (size_t)a.list_len * sizeof(int32_t)}});
    return hipSuccess;
}

hipError_t launch_merge(const MergeArgs& a, int batch, int head_dim, hipStream_t)
{
    const size_t units = (size_t)batch * a.num_q_heads * a.num_splits;
    touch({{"o_part", (char*)a.o_part, units * head_dim * sizeof(float)}, {"lse_part", (char*)a.lse_part, units * sizeof(float)}});
    return hipSuccess;
}

hipError_t launch_kv_append(const AppendArgs&, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_kv_write(const WriteArgs&, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_probe_read(const void*, size_t, void*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_probe_copy(const void*, void*, size_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_probe_columns(const void*, size_t, size_t, int, int, int, int, void*, hipStream_t) { ++g_launches; return hipSuccess; }

hipError_t launch_sparf_build(const SparfArgs& a, hipStream_t)
{
    std::vector<Region> r;
    if (a.vsum_part)
        r.push_back({"vsum_part", (char*)a.vsum_part,
                     (size_t)a.batch * a.num_kv_heads * a.vsum_parts * a.head_dim * sizeof(float)});
    touch(r);
    return hipSuccess;
}

hipError_t launch_sparf_append(const SparfArgs&, hipStream_t) { ++g_launches; return hipSuccess; }

hipError_t launch_sparf_logits(const SparfArgs& a, hipStream_t)
{
    if (a.lpad < a.max_len || a.lpad % kSparfChunk || a.nstat * kSparfStatRun != a.lpad) fail("padded row", "logits");
    touch({{"logits", (char*)a.logits, sparf_rows(a) * a.lpad * sizeof(float)},
           {"stats", (char*)a.stats, sparf_rows(a) * a.nstat * 3 * sizeof(float)}});
    return hipSuccess;
}

hipError_t launch_sparf_select(const SparfArgs& a, hipStream_t)
{
    const size_t rows = sparf_rows(a);
    std::vector<Region> r = {sel_region(a), {"logits", (char*)a.logits, rows * a.lpad * sizeof(float)},
                             {"stats", (char*)a.stats, rows * a.nstat * 3 * sizeof(float)}};
    if (a.distributed) {
        if (a.nparts < 1 || a.nparts > kSparfHistParts || a.nparts > a.nchunk) fail("histogram parts", "hist");
        r.push_back({"hist", (char*)a.hist, rows * a.nparts * 256 * sizeof(uint32_t)});
        r.push_back({"gt1", (char*)a.gt1, rows * a.nchunk * sizeof(uint32_t)});
        r.push_back({"counters", (char*)a.counters, rows * 2 * sizeof(uint32_t)});
        r.push_back({"state", (char*)a.state, rows * 2 * sizeof(uint32_t)});
        r.push_back({"members", (char*)a.members, rows * a.member_cap * 2 * sizeof(uint32_t)});
        r.push_back({"mass_part", (char*)a.mass_part, rows * a.nchunk * sizeof(float)});
        r.push_back({"rowstat", (char*)a.rowstat, rows * 4 * sizeof(float)});
    } else {
        r.push_back(alpha_region(a));
    }
    touch(r);
    return hipSuccess;
}

hipError_t launch_sparf_attend(const SparfArgs& a, hipStream_t)
{
    const size_t rows = sparf_rows(a);
    if (a.nslices < 1 || a.nslices > kSparfMaxSlices || (int64_t)a.nslices * a.slice_rows < std::min(a.k, a.max_len))
        fail("slices do not cover the kept rows", "part");
    std::vector<Region> r = {sel_region(a), alpha_region(a)};
    if (a.nslices > 1) r.push_back({"part", (char*)a.part, rows * a.nslices * (a.head_dim + 2) * sizeof(float)});
    if (a.distributed) {
        r.push_back({"mass_part", (char*)a.mass_part, rows * a.nchunk * sizeof(float)});
        r.push_back({"rowstat", (char*)a.rowstat, rows * 4 * sizeof(float)});
    }
    touch(r);
    return hipSuccess;
}

hipError_t launch_sparf_select_attend(const SparfArgs& a, hipStream_t)
{
    const size_t rows = sparf_rows(a);
    touch({sel_region(a), alpha_region(a), {"logits", (char*)a.logits, rows * a.lpad * sizeof(float)},
           {"stats", (char*)a.stats, rows * a.nstat * 3 * sizeof(float)}});
    return hipSuccess;
}

hipError_t launch_sparf_fused(const SparfArgs& a, hipStream_t)
{
    if (a.fused_threads != 256 && a.fused_threads != 512 && a.fused_threads != 1024) fail("threads per head", "fused");
    const int cap = a.fused_threads == 256 ? kSparfFusedMaxLen
                                           : (a.fused_threads == 512 ? kSparfFusedWideMaxLen : kSparfFusedWidestMaxLen);
    if (a.max_len > cap) fail("row longer than the one-launch kernel's scores in LDS", "fused");
    touch({sel_region(a), alpha_region(a)});
    return hipSuccess;
}

}  // namespace instattn
