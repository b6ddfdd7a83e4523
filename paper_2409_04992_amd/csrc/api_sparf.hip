// Host side of the SparF entry points: argument checks, workspace carving, launches.
#include "../../include/instattn.h"

#include <math.h>
#include <stdlib.h>

#include "host_checks.h"
#include "options.h"
#include "sparf.h"

using namespace instattn;

namespace {

size_t up256(size_t x) { return (x + 255) / 256 * 256; }

// Room in the distributed selection's list of threshold-bin members: with 256 level-1
// bins a row of L evenly spread scores puts about L / 200 of them into the bin (5000 at
// a million positions), so the list grows with the row.
int member_cap_for(int max_seq_len)
{
    int cap = kSparfMemberCap;
    while (cap < max_seq_len / 64 && cap < 65536) cap *= 2;
    return cap;
}

struct Carve {
    size_t logits, stats, sel, alpha, part, hist, gt1, counters, state, members, mass_part, rowstat, total;
    int lpad, nchunk, nstat, member_cap;
};

Carve carve(int batch, int num_q_heads, int head_dim, int max_seq_len, int k)
{
    Carve c;
    if (k > max_seq_len) k = max_seq_len;       // no head keeps more rows than it has
    c.nchunk = (max_seq_len + kSparfChunk - 1) / kSparfChunk;
    c.lpad = c.nchunk * kSparfChunk;
    c.nstat = c.lpad / kSparfStatRun;
    c.member_cap = member_cap_for(max_seq_len);
    const size_t rows = (size_t)batch * num_q_heads;
    c.logits = 0;
    c.stats = c.logits + up256(rows * c.lpad * sizeof(float));
    c.sel = c.stats + up256(rows * c.nstat * 3 * sizeof(float));
    c.alpha = c.sel + up256(rows * (size_t)k * sizeof(int32_t));
    c.part = c.alpha + up256(rows * sizeof(float));
    c.hist = c.part + up256(rows * kSparfMaxSlices * (size_t)(head_dim + 2) * sizeof(float));
    // the distributed selection's state (small next to the scores; any row length may be
    // sent that way through the environment switches)
    const size_t lr = rows;
    c.gt1 = c.hist + up256(lr * c.nchunk * 256 * sizeof(uint32_t));
    c.counters = c.gt1 + up256(lr * c.nchunk * sizeof(uint32_t));
    c.state = c.counters + up256(lr * 2 * sizeof(uint32_t));
    c.members = c.state + up256(lr * 2 * sizeof(uint32_t));
    c.mass_part = c.members + up256(lr * c.member_cap * 2 * sizeof(uint32_t));
    c.rowstat = c.mass_part + up256(lr * c.nchunk * sizeof(float));
    c.total = c.rowstat + up256(lr * 4 * sizeof(float));
    return c;
}

// Blocks over which the set-up spreads the V sum of one (sequence, KV head): about a
// thousand blocks in all, at most 64 per pair (one block per pair reads at 60-250 GB/s:
// 8 pairs of a million rows took 4.6 ms).
int vsum_parts_for(int batch, int num_kv_heads)
{
    const int64_t pairs = (int64_t)batch * num_kv_heads;
    if (pairs >= 512) return 1;
    const int64_t parts = (1024 + pairs - 1) / pairs;
    return (int)(parts > 64 ? 64 : parts);
}

// Which kernels a decode of these sizes launches: host arithmetic only.
struct SparfPlan {
    bool one_launch;      // sparf_fused_kernel does everything
    int fused_threads;    // ... with this many threads per head (0: the pipeline runs)
    bool append_fused;    // the decode's launch stores the new token itself
    bool distributed;     // selection spread over one block per stretch (three launches)
    bool fused_tail;      // one block per head selects and gathers
    int nslices, slice_rows;
    int launches;
};

SparfPlan plan_sparf(const Options& opt, int batch, int num_q_heads, int num_kv_heads, int max_seq_len, int k,
                     bool append)
{
    SparfPlan p = {};
    const int64_t heads = (int64_t)batch * num_q_heads;
    // One block per head, or the selection of a head spread over its stretches (three
    // launches)?  From step times measured with either form forced (40 to 1280 heads, rows
    // of 20K to 256K positions): up to 40K positions one block per head is ahead for any
    // number of heads (by 2 to 15 %); from 96K on the spread form is (40 heads x 128K: 111
    // against 205 us, 640 heads x 128K: 1.31 against 1.48 ms); in between the spread form
    // wins with few heads, which leave most of the chip idle otherwise (80 heads x 64K:
    // 104 against 111 us), and with many, whose blocks come in several rounds (640 heads x
    // 64K: 616 against 623 us), but not with about one round of them (160 heads x 64K: 190
    // against 182 us).
    {
        const bool few = heads <= kSparfSpreadFewHeads, many = heads > kSparfSpreadManyHeads;
        const int forced = opt[kOptSparfDistributed];
        p.distributed = forced >= 0 ? forced == 1
                                    : max_seq_len >= kSparfSpreadAlwaysLen ||
                                          (max_seq_len > kSparfSpreadMinLen && (few || many));
    }
    // Slices of a head's kept rows for the attend kernel: enough blocks to fill the
    // chip when there are few heads, none smaller than 256 rows.
    {
        const int kept = k < max_seq_len ? k : max_seq_len;      // no head keeps more rows than it has
        int ns = (int)((1024 + heads - 1) / heads);
        ns = ns < kept / 256 ? ns : kept / 256;
        ns = ns < 1 ? 1 : (ns > kSparfMaxSlices ? kSparfMaxSlices : ns);
        p.nslices = ns;
        p.slice_rows = ((kept + ns - 1) / ns + 15) / 16 * 16;
    }
    // Rows behind the 256-thread form's limit take the one-launch kernel's 512-thread form
    // (up to 18432 positions; up to 36864 one of 1024 threads) when there are heads enough
    // for one block each.  Step times at 16K rows: 160 heads 48 us against the pipeline's 58,
    // 80 heads 42 against 41, 40 heads 40 against 33; at 12K rows: 120 heads 37 against 42,
    // 80 heads 35 against 34.  INSTATTN_SPARF_WIDE forces either way.
    const bool force_wide = opt[kOptSparfWide] == 1, forbid_wide = opt[kOptSparfWide] == 0;
    p.fused_threads = 0;
    if (max_seq_len <= kSparfFusedMaxLen) p.fused_threads = 256;
    else if (max_seq_len <= kSparfFusedWideMaxLen && !forbid_wide && (force_wide || heads >= kSparfWideMinHeads)) p.fused_threads = 512;
    else if (max_seq_len > kSparfFusedWideMaxLen && max_seq_len <= kSparfFusedWidestMaxLen && !forbid_wide &&
             (force_wide || (heads >= kSparfWideMinHeads && heads <= kSparfWidestMaxHeads)))
        p.fused_threads = 1024;   // one block per compute unit: pays when the heads fit in one round of those
                                  // (step times at 32K rows: 120 heads 78 us against the pipeline's 81, 240
                                  // heads 112 against 132; 80 heads 73 against 62, 280 heads 179 against 164)
    if (opt[kOptSparfThreeLaunches] == 1) p.fused_threads = 0;
    p.one_launch = p.fused_threads != 0;
    // The decode's first launch (the one-launch kernel, or the pipeline's score pass) stores
    // the new token itself when one block is the only reader of what it stores during that
    // launch, which takes one query head per KV head; otherwise the append is a launch of
    // its own.
    p.append_fused = append && num_q_heads == num_kv_heads;
    // One block per head and no slices: that block also gathers the rows it kept.
    p.fused_tail = !p.one_launch && !p.distributed && p.nslices == 1 && max_seq_len < kSparfTailMaxLen &&
                   opt[kOptSparfSplitTail] != 1;
    p.launches = (append && !p.append_fused) ? 1 : 0;
    if (p.one_launch) p.launches += 1;
    else if (p.fused_tail) p.launches += 2;
    else p.launches += 1 + (p.distributed ? 3 : 1) + 1 + (p.nslices > 1 ? 1 : 0);
    return p;
}

int check_common(const instattn_kv_desc* kv, const instattn_sparf_aux* aux, int batch, int num_kv_heads,
                 int head_dim)
{
    if (batch <= 0 || num_kv_heads <= 0) return INSTATTN_ERR_INVALID_ARG;
    if (head_dim != 64 && head_dim != 128) return head_dim > 0 ? INSTATTN_ERR_UNSUPPORTED : INSTATTN_ERR_INVALID_ARG;
    const int st = check_kv(kv, head_dim);
    if (st != INSTATTN_OK) return st;
    // the gather packs pool page and row inside the page into one 32-bit row id
    if (kv->layout == INSTATTN_KV_PAGED && (int64_t)kv->num_pages * kv->page_size > INT32_MAX)
        return INSTATTN_ERR_UNSUPPORTED;
    if (!aux || !aux->kt || !aux->vsum || !aligned16(aux->kt)) return INSTATTN_ERR_INVALID_ARG;
    if (aux->capacity <= 0 || aux->capacity % 8) return INSTATTN_ERR_INVALID_ARG;
    if (aux->stride_b <= 0 || aux->stride_h <= 0) return INSTATTN_ERR_INVALID_ARG;
    if (aux->stride_b % 8 || aux->stride_h % 8 || aux->stride_d % 8) return INSTATTN_ERR_INVALID_ARG;
    if (aux->page_size == 0) {
        if (aux->page_table != nullptr || aux->stride_d < aux->capacity) return INSTATTN_ERR_INVALID_ARG;
    } else {
        if (!pow2(aux->page_size) || aux->page_size < 8 || !aux->page_table) return INSTATTN_ERR_INVALID_ARG;
        if (aux->max_pages_per_seq <= 0 || aux->num_pages <= 0) return INSTATTN_ERR_INVALID_ARG;
        if (aux->stride_d < aux->page_size) return INSTATTN_ERR_INVALID_ARG;
        if ((int64_t)aux->capacity != (int64_t)aux->page_size * aux->max_pages_per_seq)
            return INSTATTN_ERR_INVALID_ARG;
    }
    return INSTATTN_OK;
}

void fill_views(SparfArgs& a, const instattn_kv_desc* kv, const instattn_sparf_aux* aux)
{
    a.kv = make_view(kv);
    a.aux.kt = (half_t*)aux->kt;
    a.aux.stride_b = aux->stride_b;
    a.aux.stride_h = aux->stride_h;
    a.aux.stride_d = aux->stride_d;
    a.aux.capacity = aux->capacity;
    a.aux.vsum = aux->vsum;
    const bool paged = aux->page_size != 0;
    a.aux.page_table = paged ? aux->page_table : nullptr;
    a.aux.page_shift = paged ? ilog2(aux->page_size) : 0;
    a.aux.page_mask = paged ? aux->page_size - 1 : 0;
    a.aux.max_pages = paged ? aux->max_pages_per_seq : 0;
    a.aux.last_page = paged ? aux->num_pages - 1 : 0;
}

int status_of(hipError_t e) { return e == hipSuccess ? INSTATTN_OK : INSTATTN_ERR_RUNTIME; }

}  // namespace

extern "C" {

size_t instattn_sparf_build_workspace_size(int batch, int num_kv_heads, int head_dim)
{
    if (batch <= 0 || num_kv_heads <= 0 || (head_dim != 64 && head_dim != 128)) return 0;
    const int parts = vsum_parts_for(batch, num_kv_heads);
    if (parts == 1) return 0;
    return up256((size_t)batch * num_kv_heads * parts * head_dim * sizeof(float));
}

int instattn_sparf_build(const instattn_kv_desc* kv, const instattn_sparf_aux* aux,
                         const int32_t* seq_lens, int batch, int num_kv_heads, int head_dim,
                         void* workspace, size_t workspace_bytes, void* stream)
{
    int st = check_common(kv, aux, batch, num_kv_heads, head_dim);
    if (st != INSTATTN_OK) return st;
    if (!seq_lens || batch > 65535) return INSTATTN_ERR_INVALID_ARG;
    SparfArgs a = {};
    fill_views(a, kv, aux);
    a.seq_lens = seq_lens;
    a.batch = batch;
    a.num_kv_heads = num_kv_heads;
    a.head_dim = head_dim;
    const size_t need = instattn_sparf_build_workspace_size(batch, num_kv_heads, head_dim);
    if (workspace != nullptr && need > 0) {
        if (((uintptr_t)workspace & 255) || workspace_bytes < need) return INSTATTN_ERR_WORKSPACE;
        const int rows = kv->capacity < aux->capacity ? kv->capacity : aux->capacity;
        a.vsum_part = (float*)workspace;
        a.vsum_parts = vsum_parts_for(batch, num_kv_heads);
        a.vsum_rows = ((rows + a.vsum_parts - 1) / a.vsum_parts + 63) / 64 * 64;
    }
    return status_of(launch_sparf_build(a, (hipStream_t)stream));
}

int instattn_sparf_append(const instattn_kv_desc* kv, const instattn_sparf_aux* aux,
                          const void* k_new, const void* v_new, const int32_t* seq_lens,
                          int batch, int num_kv_heads, int head_dim, void* stream)
{
    int st = check_common(kv, aux, batch, num_kv_heads, head_dim);
    if (st != INSTATTN_OK) return st;
    if (!seq_lens || !k_new || !v_new) return INSTATTN_ERR_INVALID_ARG;
    SparfArgs a = {};
    fill_views(a, kv, aux);
    a.seq_lens = seq_lens;
    a.batch = batch;
    a.num_kv_heads = num_kv_heads;
    a.head_dim = head_dim;
    a.k_new = (const half_t*)k_new;
    a.v_new = (const half_t*)v_new;
    return status_of(launch_sparf_append(a, (hipStream_t)stream));
}

int instattn_sparf_plan(int batch, int num_q_heads, int num_kv_heads, int head_dim, int max_seq_len, int k,
                        int with_append, int32_t* plan)
{
    if (!plan || batch <= 0 || num_q_heads <= 0 || num_kv_heads <= 0 || num_q_heads % num_kv_heads ||
        max_seq_len <= 0 || k <= 0)
        return INSTATTN_ERR_INVALID_ARG;
    if (max_seq_len > kSparfMaxSeqLen) return INSTATTN_ERR_UNSUPPORTED;
    if (head_dim != 64 && head_dim != 128) return head_dim > 0 ? INSTATTN_ERR_UNSUPPORTED : INSTATTN_ERR_INVALID_ARG;
    const SparfPlan p = plan_sparf(options_snapshot(), batch, num_q_heads, num_kv_heads, max_seq_len, k, with_append != 0);
    plan[0] = p.launches;
    plan[1] = p.fused_threads;
    plan[2] = p.append_fused;
    plan[3] = p.one_launch ? 0 : (p.distributed ? 2 : 1);
    plan[4] = p.fused_tail;
    plan[5] = p.one_launch || p.fused_tail ? 1 : p.nslices;
    return INSTATTN_OK;
}

size_t instattn_sparf_workspace_size(int batch, int num_q_heads, int head_dim, int max_seq_len, int k)
{
    if (batch <= 0 || num_q_heads <= 0 || max_seq_len <= 0 || max_seq_len > kSparfMaxSeqLen || k <= 0) return 0;
    if (head_dim != 64 && head_dim != 128) return 0;
    return carve(batch, num_q_heads, head_dim, max_seq_len, k).total;
}

}  // extern "C"

namespace {

int run_sparf_decode(const void* q, const void* k_new, const void* v_new, bool append,
                     const instattn_kv_desc* kv, const instattn_sparf_aux* aux, const int32_t* seq_lens,
                     int batch, int num_q_heads, int num_kv_heads, int head_dim, float scale, int r, int k,
                     int l, void* out, int out_dtype, int32_t* sel_rows, float* alpha, void* workspace,
                     size_t workspace_bytes, int max_seq_len, void* stream)
{
    int st = check_common(kv, aux, batch, num_kv_heads, head_dim);
    if (st != INSTATTN_OK) return st;
    if (num_q_heads <= 0 || num_q_heads % num_kv_heads || max_seq_len <= 0) return INSTATTN_ERR_INVALID_ARG;
    if (batch > 65535 || num_q_heads > 65535) return INSTATTN_ERR_UNSUPPORTED;
    if (!q || !aligned16(q) || !seq_lens || !isfinite(scale)) return INSTATTN_ERR_INVALID_ARG;
    if (append && (!k_new || !v_new || !aligned16(k_new) || !aligned16(v_new))) return INSTATTN_ERR_INVALID_ARG;
    if (!out || !aligned16(out)) return INSTATTN_ERR_INVALID_ARG;
    if (out_dtype != INSTATTN_F16 && out_dtype != INSTATTN_F32) return INSTATTN_ERR_INVALID_ARG;
    if (r < 1 || r > head_dim || k < 1 || l < 0) return INSTATTN_ERR_INVALID_ARG;
    if (max_seq_len > kv->capacity || max_seq_len > aux->capacity) return INSTATTN_ERR_INVALID_ARG;
    if (max_seq_len > kSparfMaxSeqLen) return INSTATTN_ERR_UNSUPPORTED;
    const Carve c = carve(batch, num_q_heads, head_dim, max_seq_len, k);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < c.total)
        return INSTATTN_ERR_WORKSPACE;

    SparfArgs a = {};
    fill_views(a, kv, aux);
    a.q = (const half_t*)q;
    a.seq_lens = seq_lens;
    a.batch = batch;
    a.num_q_heads = num_q_heads;
    a.num_kv_heads = num_kv_heads;
    a.head_dim = head_dim;
    a.max_len = max_seq_len;
    a.scale_log2 = scale * kLog2e;
    a.r = r;
    // kept rows are stored k apart in the caller's sel_rows; the library's own list needs
    // no more room per head than a row has positions
    a.k = sel_rows || k < max_seq_len ? k : max_seq_len;
    a.l = l;
    char* ws = (char*)workspace;
    a.logits = (float*)(ws + c.logits);
    a.lpad = c.lpad;
    a.nchunk = c.nchunk;
    a.nstat = c.nstat;
    a.stats = (float*)(ws + c.stats);
    a.sel = sel_rows ? sel_rows : (int32_t*)(ws + c.sel);
    a.alpha = alpha ? alpha : (float*)(ws + c.alpha);
    a.part = (float*)(ws + c.part);
    a.hist = (uint32_t*)(ws + c.hist);
    a.gt1 = (uint32_t*)(ws + c.gt1);
    a.counters = (uint32_t*)(ws + c.counters);
    a.state = (uint32_t*)(ws + c.state);
    a.members = (uint32_t*)(ws + c.members);
    a.member_cap = c.member_cap;
    a.nparts = c.nchunk < kSparfHistParts ? c.nchunk : kSparfHistParts;
    a.mass_part = (float*)(ws + c.mass_part);
    a.rowstat = (float*)(ws + c.rowstat);
    const SparfPlan plan = plan_sparf(options_snapshot(), batch, num_q_heads, num_kv_heads, max_seq_len, k, append);
    a.distributed = plan.distributed;
    a.nslices = plan.nslices;
    a.slice_rows = plan.slice_rows;
    a.fused_threads = plan.fused_threads;
    a.out = out;
    a.out_f32 = out_dtype == INSTATTN_F32;
    a.k_new = append ? (const half_t*)k_new : nullptr;
    a.v_new = append ? (const half_t*)v_new : nullptr;
    hipStream_t s = (hipStream_t)stream;
    if (append && !plan.append_fused) {
        if (launch_sparf_append(a, s) != hipSuccess) return INSTATTN_ERR_RUNTIME;
        a.k_new = a.v_new = nullptr;
    }
    if (plan.one_launch) return status_of(launch_sparf_fused(a, s));
    if (launch_sparf_logits(a, s) != hipSuccess) return INSTATTN_ERR_RUNTIME;
    a.k_new = a.v_new = nullptr;                  // stored by now, one way or the other
    if (plan.fused_tail) return status_of(launch_sparf_select_attend(a, s));
    if (launch_sparf_select(a, s) != hipSuccess) return INSTATTN_ERR_RUNTIME;
    return status_of(launch_sparf_attend(a, s));
}

}  // namespace

extern "C" {

int instattn_sparf_decode(const void* q, const instattn_kv_desc* kv, const instattn_sparf_aux* aux,
                          const int32_t* seq_lens, int batch, int num_q_heads, int num_kv_heads,
                          int head_dim, float scale, int r, int k, int l, void* out, int out_dtype,
                          int32_t* sel_rows, float* alpha, void* workspace, size_t workspace_bytes,
                          int max_seq_len, void* stream)
{
    return run_sparf_decode(q, nullptr, nullptr, false, kv, aux, seq_lens, batch, num_q_heads, num_kv_heads,
                            head_dim, scale, r, k, l, out, out_dtype, sel_rows, alpha, workspace,
                            workspace_bytes, max_seq_len, stream);
}

int instattn_sparf_append_decode(const void* q, const void* k_new, const void* v_new,
                                 const instattn_kv_desc* kv, const instattn_sparf_aux* aux,
                                 const int32_t* seq_lens, int batch, int num_q_heads, int num_kv_heads,
                                 int head_dim, float scale, int r, int k, int l, void* out, int out_dtype,
                                 int32_t* sel_rows, float* alpha, void* workspace, size_t workspace_bytes,
                                 int max_seq_len, void* stream)
{
    return run_sparf_decode(q, k_new, v_new, true, kv, aux, seq_lens, batch, num_q_heads, num_kv_heads,
                            head_dim, scale, r, k, l, out, out_dtype, sel_rows, alpha, workspace,
                            workspace_bytes, max_seq_len, stream);
}

}  // extern "C"
