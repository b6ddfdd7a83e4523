// Host side of the C ABI: argument checks, the split plan, kernel launches.
// Nothing here touches device memory or synchronises.
#include "../../include/instattn.h"

#include <math.h>
#include <limits.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <mutex>

#include "common.h"
#include "host_checks.h"
#include "options.h"

using namespace instattn;

// ---------------------------------------------------------------------------
// Implementation switches: process-wide atomics, first filled from the environment.
namespace instattn {
namespace {

const char* const kOptionNames[kNumOptions] = {
    "INSTATTN_CHUNK", "INSTATTN_ROTATE", "INSTATTN_SPARF_DISTRIBUTED", "INSTATTN_SPARF_THREE_LAUNCHES",
    "INSTATTN_SPARF_WIDE", "INSTATTN_SPARF_SPLIT_TAIL", "INSTATTN_COMPACT", "INSTATTN_MHA_RING",
};
std::atomic<int> g_options[kNumOptions];
std::once_flag g_options_once;

void options_from_environment()
{
    for (int o = 0; o < kNumOptions; ++o) {
        const char* e = getenv(kOptionNames[o]);
        g_options[o].store(e && e[0] ? atoi(e) : -1, std::memory_order_relaxed);
    }
}

}  // namespace

Options options_snapshot()
{
    std::call_once(g_options_once, options_from_environment);
    Options s;
    for (int o = 0; o < kNumOptions; ++o) s.v[o] = g_options[o].load(std::memory_order_relaxed);
    return s;
}

const char* option_name(int o) { return o >= 0 && o < kNumOptions ? kOptionNames[o] : nullptr; }

}  // namespace instattn

namespace {

int option_index(const char* name)
{
    if (!name) return -1;
    for (int o = 0; o < kNumOptions; ++o)
        if (strcmp(name, kOptionNames[o]) == 0) return o;
    return -1;
}

constexpr int kVersion = 200;          // 0.2.0
constexpr int kChunkQuantum = 128;     // every kernel's block tile divides this
constexpr int kMinChunk = 384;
// Work units wanted per launch and largest unit, per kernel.  The vector-ALU kernel has
// two forms.  Large launches stage their tiles through an LDS ring, one block per CU, in
// long units that amortise its prologue and epilogue (below).  Small launches (below
// kRingMinRows rows in all, an upper bound: 0.5 GB at head_dim 128) hold two tiles in
// registers, five blocks per CU, and take shorter units, so that 1280 block slots hide
// each other's start and end (4 x 40 heads x 1.5K: 24.5 us against 27.3 us through the
// ring); so do launches of sequences shorter than kRingMinChunk rows (32 x 40 heads x 1.5K
// as whole sequences: 83.0 % of peak against 81.3 %).  The MFMA kernel runs 2 blocks per CU
// and pays more per unit (prologue, cross-wave epilogue), so it gets fewer, larger units:
// about three per four compute units measured best from 16 x 16K down to 128 x 1K rows in all.
constexpr int kTargetUnitsMhaSmall = 4096, kMaxChunkMhaSmall = 1408;
// The ring form of the vector-ALU kernel (one block per compute unit) takes launches of 2^20
// rows or more in units of 2048 rows or more.  Its units are 2944 or 5504 rows long: lengths
// whose byte size, taken modulo 512 KB, lies near the middle of that period - units of a
// stream that start nearly a multiple of 512 KB apart (2176, 4224, 8320 rows of 256 bytes)
// walk the HBM channels in step and lose 3 to 6 % (measured on every shape tried).  Between
// the two the launch's rounds decide (units over 256 compute units, rounded up, times the
// unit length); the longer unit must win by 3 % (8 x 40 heads x 32K: 88.5 % of peak with
// 2944, 87.7 % with 5504, equal rounds; 6 x 40 x 32K: 86.9 against 87.3 %, 1 x 40 x 128K:
// 86.6 against 87.8 %, 24 x 8 x 16K: 84.0 against 77.8 %, where 5504 leaves a quarter of the
// last round empty).
constexpr long kRingMinRows = 1L << 20;
constexpr int kRingMinChunk = 2048;
constexpr int kRingChunk = 2944, kRingLongChunk = 5504;
constexpr long kRingMinFill = 88;      // per cent of the rounds' rows that the launch must hold
constexpr int kComputeUnits = 256;
constexpr int kTargetUnitsGqa = 192, kMaxChunkGqa = 5504;
constexpr int kLongChunkGqa = 8832, kSlotsGqa = 512;   // both sizes, modulo 512 KB, sit near the middle (see the ring form's units)
constexpr int kSingleSplitStreams = 512, kSingleSplitMaxLen = 8192 + kChunkQuantum;
constexpr int kResidentUnits = 1280;   // five blocks of the vector-ALU kernel on each of 256 compute units
// The unit list of a paged cache: rows (an upper bound: max_seq_len x KV streams) from
// which on its small launch in front pays, and the most (sequence, split) pairs the one
// block of that launch sorts.
constexpr long kCompactMinRows = 2L << 20;
constexpr int kCompactMaxEntries = 8192, kCompactMaxBatch = 4096;

struct Plan {
    int chunk;
    int num_splits;
    int group_blocks;     // MFMA kernel: blocks per KV head and unit (16 query heads each)
    bool compact;         // the split pass walks a device-built list of the units that hold rows
    bool staged;          // vector-ALU kernel: tiles through the LDS ring (large launches)
    bool rotate;
};

// Sequence split: units of `chunk` positions, enough of them to fill the chip
// from host-known sizes alone.  The chunk is an ODD multiple of 128 rows: units
// that start a large power of two apart walk the same HBM channels in lockstep
// and lose up to a fifth of the bandwidth (measured), an odd multiple staggers them.
Plan make_plan(const Options& opt, int batch, int num_q_heads, int num_kv_heads, int max_seq_len, bool paged)
{
    const int group = num_q_heads / num_kv_heads;
    // the MFMA path walks a KV head once for its whole query group
    const long streams = (long)batch * (group == 1 ? num_q_heads : num_kv_heads);
    auto odd_multiple = [](long rows) { return ((rows + kChunkQuantum - 1) / kChunkQuantum | 1) * kChunkQuantum; };
    // unit length from the units wanted and the longest unit allowed
    auto unit_length = [&](long target, long cap) {
        long chunk = ((long)max_seq_len * streams + target - 1) / target;
        if (chunk < kMinChunk) chunk = kMinChunk;
        if (chunk > cap) chunk = cap;
        chunk = (chunk / kChunkQuantum | 1) * kChunkQuantum;
        // Enough short independent streams already fill the chip with whole sequences as
        // units: one unit per stream (the split pass writes the result itself, no merge) when
        // the streams fill every block slot of the chip, else the fewest equal splits that do
        // (640 streams in two halves: +1 % on the step; 520 in three thirds: +10 %).
        if (group == 1 && streams >= kSingleSplitStreams && max_seq_len <= kSingleSplitMaxLen) {
            const long n = (kResidentUnits + streams - 1) / streams;       // 1 from 1280 streams on
            chunk = odd_multiple(((long)max_seq_len + n - 1) / n);
        }
        // The MFMA kernel holds two blocks per compute unit.  With a stream or more per
        // compute unit and short sequences, whole sequences are the best units when they
        // come out even over the 256 compute units (256 or 512 streams: 84.5 % of peak
        // against 79 % in two splits, and no merge); otherwise equal splits, three units or
        // more per compute unit, dilute the uneven last round (384 streams of 8K rows in
        // halves: 82 % against 78 % at the longest allowed unit).
        if (group > 1 && streams >= 256 && max_seq_len <= kSingleSplitMaxLen) {
            const long n = streams % 256 == 0 ? 1 : (3 * 256 + streams - 1) / streams;
            chunk = odd_multiple(((long)max_seq_len + n - 1) / n);
            if (chunk < kMinChunk) chunk = kMinChunk;
        }
        return chunk;
    };
    long chunk;
    bool staged = false;
    if (group > 1) {
        chunk = unit_length(kTargetUnitsGqa, kMaxChunkGqa);
        // Long sequences in a large launch: units of 8832 rows when they save rounds over the
        // kernel's 512 block slots (8 x 8 KV heads x 64K: 512 units in one round, 85.2 % of peak,
        // against 768 units of 5504 rows in a round and a half, 83.9 %; 16 x 8 x 32K 85.0 against
        // 83.7 %).  Not for sequences of fewer than four such units: 32 x 8 x 16K is level
        // either way, and more, shorter units spread a ragged batch better.
        if (chunk == kMaxChunkGqa && max_seq_len > 3 * kLongChunkGqa) {
            auto rounds_times_length = [&](long c) {
                const long units = streams * (((long)max_seq_len + c - 1) / c);
                return (units + kSlotsGqa - 1) / kSlotsGqa * c;
            };
            if (100 * rounds_times_length(kLongChunkGqa) <= 97 * rounds_times_length(kMaxChunkGqa)) chunk = kLongChunkGqa;
        }
    } else {
        // the ring form wants a large launch of long units; everything else takes the register form
        chunk = unit_length(kTargetUnitsMhaSmall, kMaxChunkMhaSmall);
        const bool whole_sequences = streams >= kSingleSplitStreams && max_seq_len <= kSingleSplitMaxLen;
        const bool large = (long)max_seq_len * streams >= kRingMinRows;
        if (whole_sequences) {
            staged = large && chunk >= kRingMinChunk;
        } else {
            auto rounds_times_length = [&](long c) {
                const long units = streams * (((long)max_seq_len + c - 1) / c);
                return (units + kComputeUnits - 1) / kComputeUnits * c;
            };
            long ring_chunk = kRingChunk;
            if (100 * rounds_times_length(kRingLongChunk) <= 97 * rounds_times_length(ring_chunk)) ring_chunk = kRingLongChunk;
            // sequences of at most the longer unit (+ a tile): one unit each, and no merge (12 x 40
            // heads x 3K: whole step 82.1 % of peak against 78.9 % in the register form's short units)
            const long whole_rows = ((long)max_seq_len + kChunkQuantum - 1) / kChunkQuantum * kChunkQuantum;
            if (whole_rows <= kRingLongChunk + kChunkQuantum &&
                100 * rounds_times_length(whole_rows) <= 97 * rounds_times_length(ring_chunk))
                ring_chunk = whole_rows;
            // ... and the rounds must come out nearly full: with one block per compute unit a last
            // round of few units, or of short ends of sequences, idles most of the chip (3 x 8 heads x
            // 64K: 552 units of 2944 rows fill 72 % of three rounds and run at 72.5 % of peak, the
            // register form's 4104 short units at 82.8 %)
            const bool full_rounds =
                100 * (long)max_seq_len * streams >= kRingMinFill * rounds_times_length(ring_chunk) * kComputeUnits;
            staged = large && max_seq_len >= kRingMinChunk && full_rounds;
            if (opt[kOptMhaRing] == 1 || (staged && opt[kOptMhaRing] != 0)) chunk = ring_chunk;
        }
        if (opt[kOptMhaRing] >= 0) staged = opt[kOptMhaRing] == 1;
    }
    if (opt[kOptChunk] > 0)
        chunk = ((long)opt[kOptChunk] + kChunkQuantum - 1) / kChunkQuantum * kChunkQuantum;
    const long whole = ((long)max_seq_len + kChunkQuantum - 1) / kChunkQuantum * kChunkQuantum;
    if (chunk > whole) chunk = whole;
    Plan p;
    p.staged = staged;
    p.chunk = (int)chunk;
    p.num_splits = (int)((max_seq_len + chunk - 1) / chunk);
    p.group_blocks = (group + 15) / 16;
    // A paged cache is read in scattered pieces (4 KB per page and head), every one behind an
    // address translation of its own.  There one block first lists the units that hold
    // rows - the full ones in front, the partly filled ones behind them from long to short -
    // and the split pass walks that list with the blocks of a unit (its heads) on ONE XCD:
    // they read the same pages of the pool together, so a translation serves all of them,
    // and the list's order deals the units out evenly over the XCDs and ends the launch on
    // its shortest units.  Measured on the same caches: 64 ragged sequences of 1K..16K rows,
    // 40 heads, 16-token pages 82.1 -> 84.8 % of peak (the same list without the XCD grouping:
    // 81.8 %); 64 x 8.7K rows 81.9 -> 85.8 %.  A contiguous cache gains nothing from it (ragged
    // 87.8 % without, 86.6 % with) and keeps the plain grid.
    const long entries = (long)batch * p.num_splits;
    const bool can = batch > 1 && batch <= kCompactMaxBatch && entries <= kCompactMaxEntries && p.group_blocks == 1;
    p.compact = can && (opt[kOptCompact] >= 0 ? opt[kOptCompact] == 1
                                               : paged && (long)max_seq_len * streams >= kCompactMinRows);
    // Streams whose strides walk the HBM channels in step (a contiguous cache of 2064
    // rows per head does) lose a tenth to a half of the bandwidth; starting every unit
    // at its own tile undoes most of that and costs about 1 % elsewhere: off by default.
    p.rotate = opt[kOptRotate] == 1;
    return p;
}

int check_shape(int batch, int num_q_heads, int num_kv_heads, int head_dim, int max_seq_len)
{
    if (batch <= 0 || num_q_heads <= 0 || num_kv_heads <= 0 || head_dim <= 0 || max_seq_len <= 0)
        return INSTATTN_ERR_INVALID_ARG;
    if (num_q_heads % num_kv_heads != 0) return INSTATTN_ERR_INVALID_ARG;
    if (head_dim != 64 && head_dim != 128) return INSTATTN_ERR_UNSUPPORTED;
    if (batch > 65535 || num_q_heads > 65535) return INSTATTN_ERR_UNSUPPORTED;  // grid y, z
    return INSTATTN_OK;
}

// What the launch grids can hold, known once the plan is: the split index is a grid
// dimension of its own, and a group of more than 16 query heads runs on a one-dimensional
// grid of units x blocks per unit.
int check_plan(const Plan& p, int batch, int num_kv_heads)
{
    if (p.num_splits > 65535) return INSTATTN_ERR_UNSUPPORTED;
    if (p.group_blocks > 1 &&
        ((int64_t)batch * num_kv_heads * p.num_splits + 8) * p.group_blocks > (int64_t)INT32_MAX)
        return INSTATTN_ERR_UNSUPPORTED;
    return INSTATTN_OK;
}

// The caller's workspace: partial rows, their log-sum-exp, the list of units.
struct Carve {
    size_t o_part, lse_part, unit_list, total;
};

Carve carve(int batch, int num_q_heads, int head_dim, const Plan& p)
{
    const size_t units = (size_t)batch * num_q_heads * p.num_splits;
    const size_t entries = (size_t)batch * p.num_splits;
    Carve c;
    c.o_part = 0;
    c.lse_part = c.o_part + units * (size_t)head_dim * sizeof(float);
    c.unit_list = (c.lse_part + units * sizeof(float) + 255) / 256 * 256;
    // room for the list whenever the plan could use it, so that the size does not depend on the switches
    c.total = c.unit_list + (entries <= (size_t)kCompactMaxEntries ? (entries * sizeof(int32_t) + 255) / 256 * 256 : 0);
    // (the layout changes neither the units nor this size, only whether the list is used)
    return c;
}

int check_out(void* out, int out_dtype, const void* workspace, size_t workspace_bytes, size_t need)
{
    if (!out || !aligned16(out)) return INSTATTN_ERR_INVALID_ARG;
    if (out_dtype != INSTATTN_F16 && out_dtype != INSTATTN_F32) return INSTATTN_ERR_INVALID_ARG;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need)
        return INSTATTN_ERR_WORKSPACE;
    return INSTATTN_OK;
}

// Every host check of a decode, in one place and in front of the first launch; leaves the plan.
int check_decode(const void* q, const void* k_new, const void* v_new, bool fused,
                 const instattn_kv_desc* kv, const int32_t* seq_lens, int batch, int num_q_heads,
                 int num_kv_heads, int head_dim, float scale, void* out, int out_dtype,
                 const void* workspace, size_t workspace_bytes, int max_seq_len, Plan* plan)
{
    int st = check_shape(batch, num_q_heads, num_kv_heads, head_dim, max_seq_len);
    if (st != INSTATTN_OK) return st;
    st = check_kv(kv, head_dim);
    if (st != INSTATTN_OK) return st;
    if (!q || !aligned16(q) || !seq_lens || !isfinite(scale)) return INSTATTN_ERR_INVALID_ARG;
    if (max_seq_len > kv->capacity) return INSTATTN_ERR_INVALID_ARG;
    if (fused && (!k_new || !v_new || !aligned16(k_new) || !aligned16(v_new)))
        return INSTATTN_ERR_INVALID_ARG;
    *plan = make_plan(options_snapshot(), batch, num_q_heads, num_kv_heads, max_seq_len,
                      kv->layout == INSTATTN_KV_PAGED);
    st = check_plan(*plan, batch, num_kv_heads);
    if (st != INSTATTN_OK) return st;
    return check_out(out, out_dtype, workspace, workspace_bytes, carve(batch, num_q_heads, head_dim, *plan).total);
}

int status_of(hipError_t e) { return e == hipSuccess ? INSTATTN_OK : INSTATTN_ERR_RUNTIME; }

AppendArgs append_args(const instattn_kv_desc* kv, const void* k_new, const void* v_new,
                       const int32_t* seq_lens, int batch, int num_kv_heads, int head_dim)
{
    const KvView w = make_view(kv);
    AppendArgs a;
    a.k = (half_t*)kv->k;
    a.v = (half_t*)kv->v;
    a.page_table = w.page_table;
    a.stride_b = w.stride_b;
    a.stride_h = w.stride_h;
    a.stride_t = w.stride_t;
    a.capacity = w.capacity;
    a.page_shift = w.page_shift;
    a.page_mask = w.page_mask;
    a.max_pages = w.max_pages;
    a.last_page = w.last_page;
    a.k_new = (const half_t*)k_new;
    a.v_new = (const half_t*)v_new;
    a.seq_lens = seq_lens;
    a.batch = batch;
    a.num_kv_heads = num_kv_heads;
    a.head_dim = head_dim;
    return a;
}

// The split pass of a checked decode (with the store of the new token when k_new is given).
int enqueue_partial(const Plan& p, const void* q, const void* k_new, const void* v_new,
                    const instattn_kv_desc* kv, const int32_t* seq_lens, int batch, int num_q_heads,
                    int num_kv_heads, int head_dim, float scale, void* out, int out_dtype, float* lse,
                    void* workspace, int max_seq_len, hipStream_t stream)
{
    // The split pass stores the new token itself where one block per KV head and unit reads
    // it; a group of more than 16 query heads is shared out over several blocks, so there the
    // store is a launch of its own in front.
    if (k_new && p.group_blocks > 1) {
        if (launch_kv_append(append_args(kv, k_new, v_new, seq_lens, batch, num_kv_heads, head_dim), stream) !=
            hipSuccess)
            return INSTATTN_ERR_RUNTIME;
        k_new = v_new = nullptr;
    }
    const Carve c = carve(batch, num_q_heads, head_dim, p);
    DecodeArgs a;
    a.group_blocks = p.group_blocks;
    a.units = 0;
    a.k_new = (const half_t*)k_new;
    a.v_new = (const half_t*)v_new;
    a.rotate = p.rotate;
    a.q = (const half_t*)q;
    a.kv = make_view(kv);
    a.seq_lens = seq_lens;
    a.num_q_heads = num_q_heads;
    a.num_kv_heads = num_kv_heads;
    a.chunk = p.chunk;
    a.num_splits = p.num_splits;
    a.max_len = max_seq_len;
    a.scale_log2 = scale * kLog2e;
    a.o_part = (float*)((char*)workspace + c.o_part);
    a.lse_part = (float*)((char*)workspace + c.lse_part);
    a.unit_list = nullptr;
    a.list_len = 0;
    a.staged = p.staged;
    a.out = out;
    a.lse = lse;
    a.out_f32 = out_dtype == INSTATTN_F32;
    if (p.compact) {
        a.unit_list = (int32_t*)((char*)workspace + c.unit_list);
        a.list_len = batch * p.num_splits;
        if (launch_list_units(a, batch, stream) != hipSuccess) return INSTATTN_ERR_RUNTIME;
    }
    return status_of(num_q_heads == num_kv_heads ? launch_decode_mha(a, batch, head_dim, stream)
                                                 : launch_decode_gqa(a, batch, head_dim, stream));
}

// The merge of a checked decode; nothing to do when the split pass wrote out/lse itself.
int enqueue_merge(const Plan& p, const int32_t* seq_lens, int batch, int num_q_heads, int head_dim,
                  void* out, int out_dtype, float* lse, const void* workspace, int max_seq_len,
                  hipStream_t stream)
{
    if (p.num_splits == 1) return INSTATTN_OK;
    const Carve c = carve(batch, num_q_heads, head_dim, p);
    MergeArgs m;
    m.seq_lens = seq_lens;
    m.o_part = (const float*)((const char*)workspace + c.o_part);
    m.lse_part = (const float*)((const char*)workspace + c.lse_part);
    m.out = out;
    m.lse = lse;
    m.num_q_heads = num_q_heads;
    m.chunk = p.chunk;
    m.num_splits = p.num_splits;
    m.max_len = max_seq_len;
    m.out_f32 = out_dtype == INSTATTN_F32;
    return status_of(launch_merge(m, batch, head_dim, stream));
}

// One call = one set of checks, one plan, then the launches.
int run_decode(const void* q, const void* k_new, const void* v_new, bool fused, bool partial, bool merge,
               const instattn_kv_desc* kv, const int32_t* seq_lens, int batch, int num_q_heads,
               int num_kv_heads, int head_dim, float scale, void* out, int out_dtype, float* lse,
               void* workspace, size_t workspace_bytes, int max_seq_len, void* stream)
{
    Plan p;
    int st = check_decode(q, k_new, v_new, fused, kv, seq_lens, batch, num_q_heads, num_kv_heads, head_dim,
                          scale, out, out_dtype, workspace, workspace_bytes, max_seq_len, &p);
    if (st != INSTATTN_OK) return st;
    if (partial) {
        st = enqueue_partial(p, q, fused ? k_new : nullptr, fused ? v_new : nullptr, kv, seq_lens, batch,
                             num_q_heads, num_kv_heads, head_dim, scale, out, out_dtype, lse, workspace,
                             max_seq_len, (hipStream_t)stream);
        if (st != INSTATTN_OK) return st;
    }
    if (merge)
        st = enqueue_merge(p, seq_lens, batch, num_q_heads, head_dim, out, out_dtype, lse, workspace,
                           max_seq_len, (hipStream_t)stream);
    return st;
}

}  // namespace

extern "C" {

int instattn_version(void) { return kVersion; }

const char* instattn_status_string(int status)
{
    switch (status) {
        case INSTATTN_OK: return "ok";
        case INSTATTN_ERR_INVALID_ARG: return "invalid argument";
        case INSTATTN_ERR_UNSUPPORTED: return "unsupported configuration";
        case INSTATTN_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case INSTATTN_ERR_RUNTIME: return "HIP launch failed";
        default: return "unknown status";
    }
}

int instattn_set_option(const char* name, int value)
{
    const int o = option_index(name);
    if (o < 0) return INSTATTN_ERR_INVALID_ARG;
    options_snapshot();                       // the environment first, so that it never overwrites this value
    g_options[o].store(value < 0 ? -1 : value, std::memory_order_relaxed);
    return INSTATTN_OK;
}

int instattn_get_option(const char* name, int* value)
{
    const int o = option_index(name);
    if (o < 0 || !value) return INSTATTN_ERR_INVALID_ARG;
    *value = options_snapshot()[(Option)o];
    return INSTATTN_OK;
}

int instattn_kv_append(const instattn_kv_desc* kv, const void* k_new, const void* v_new,
                       const int32_t* seq_lens, int batch, int num_kv_heads, int head_dim,
                       void* stream)
{
    if (batch <= 0 || num_kv_heads <= 0 || head_dim <= 0 || head_dim % 8) return INSTATTN_ERR_INVALID_ARG;
    int st = check_kv(kv, head_dim);
    if (st != INSTATTN_OK) return st;
    if (!k_new || !v_new || !seq_lens || !aligned16(k_new) || !aligned16(v_new))
        return INSTATTN_ERR_INVALID_ARG;
    return status_of(launch_kv_append(append_args(kv, k_new, v_new, seq_lens, batch, num_kv_heads, head_dim),
                                      (hipStream_t)stream));
}

int instattn_kv_write(const instattn_kv_desc* kv, const void* k_src, const void* v_src,
                      const int32_t* start, const int32_t* count, int batch, int num_kv_heads,
                      int head_dim, int max_new, void* stream)
{
    if (batch <= 0 || num_kv_heads <= 0 || max_new <= 0) return INSTATTN_ERR_INVALID_ARG;
    if (head_dim != 64 && head_dim != 128) return head_dim > 0 ? INSTATTN_ERR_UNSUPPORTED : INSTATTN_ERR_INVALID_ARG;
    if (batch > 65535 || num_kv_heads > 65535) return INSTATTN_ERR_UNSUPPORTED;
    int st = check_kv(kv, head_dim);
    if (st != INSTATTN_OK) return st;
    if (!k_src || !v_src || !start || !count || !aligned16(k_src) || !aligned16(v_src))
        return INSTATTN_ERR_INVALID_ARG;
    WriteArgs a;
    a.kv = make_view(kv);
    a.k_src = (const half_t*)k_src;
    a.v_src = (const half_t*)v_src;
    a.start = start;
    a.count = count;
    a.batch = batch;
    a.num_kv_heads = num_kv_heads;
    a.head_dim = head_dim;
    a.max_new = max_new;
    return status_of(launch_kv_write(a, (hipStream_t)stream));
}

int instattn_decode_plan(int batch, int num_q_heads, int num_kv_heads, int head_dim,
                         int max_seq_len, int* chunk_tokens, int* num_splits)
{
    int st = check_shape(batch, num_q_heads, num_kv_heads, head_dim, max_seq_len);
    if (st != INSTATTN_OK) return st;
    const Plan p = make_plan(options_snapshot(), batch, num_q_heads, num_kv_heads, max_seq_len, false);
    st = check_plan(p, batch, num_kv_heads);
    if (st != INSTATTN_OK) return st;
    if (chunk_tokens) *chunk_tokens = p.chunk;
    if (num_splits) *num_splits = p.num_splits;
    return INSTATTN_OK;
}

int instattn_decode_launches(int batch, int num_q_heads, int num_kv_heads, int head_dim, int max_seq_len,
                             int kv_layout, int with_append, int32_t* launches)
{
    int st = check_shape(batch, num_q_heads, num_kv_heads, head_dim, max_seq_len);
    if (st != INSTATTN_OK) return st;
    if (!launches || (kv_layout != INSTATTN_KV_CONTIGUOUS && kv_layout != INSTATTN_KV_PAGED))
        return INSTATTN_ERR_INVALID_ARG;
    const Plan p = make_plan(options_snapshot(), batch, num_q_heads, num_kv_heads, max_seq_len,
                             kv_layout == INSTATTN_KV_PAGED);
    st = check_plan(p, batch, num_kv_heads);
    if (st != INSTATTN_OK) return st;
    launches[0] = with_append && p.group_blocks > 1;   // the store of the new token as a launch of its own
    launches[1] = p.compact;                           // the list of units
    launches[2] = 1;                                   // the split pass
    launches[3] = p.num_splits > 1;                    // the merge
    return INSTATTN_OK;
}

size_t instattn_decode_workspace_size(int batch, int num_q_heads, int num_kv_heads, int head_dim,
                                      int max_seq_len)
{
    if (check_shape(batch, num_q_heads, num_kv_heads, head_dim, max_seq_len) != INSTATTN_OK) return 0;
    const Plan p = make_plan(options_snapshot(), batch, num_q_heads, num_kv_heads, max_seq_len, false);
    if (check_plan(p, batch, num_kv_heads) != INSTATTN_OK) return 0;
    return carve(batch, num_q_heads, head_dim, p).total;
}

int instattn_decode_partial(const void* q, const instattn_kv_desc* kv, const int32_t* seq_lens,
                            int batch, int num_q_heads, int num_kv_heads, int head_dim,
                            float scale, void* out, int out_dtype, float* lse, void* workspace,
                            size_t workspace_bytes, int max_seq_len, void* stream)
{
    return run_decode(q, nullptr, nullptr, false, true, false, kv, seq_lens, batch, num_q_heads, num_kv_heads,
                      head_dim, scale, out, out_dtype, lse, workspace, workspace_bytes, max_seq_len, stream);
}

int instattn_append_decode_partial(const void* q, const void* k_new, const void* v_new,
                                   const instattn_kv_desc* kv, const int32_t* seq_lens, int batch,
                                   int num_q_heads, int num_kv_heads, int head_dim, float scale, void* out,
                                   int out_dtype, float* lse, void* workspace, size_t workspace_bytes,
                                   int max_seq_len, void* stream)
{
    return run_decode(q, k_new, v_new, true, true, false, kv, seq_lens, batch, num_q_heads, num_kv_heads,
                      head_dim, scale, out, out_dtype, lse, workspace, workspace_bytes, max_seq_len, stream);
}

int instattn_append_decode(const void* q, const void* k_new, const void* v_new,
                           const instattn_kv_desc* kv, const int32_t* seq_lens, int batch,
                           int num_q_heads, int num_kv_heads, int head_dim, float scale, void* out,
                           int out_dtype, float* lse, void* workspace, size_t workspace_bytes,
                           int max_seq_len, void* stream)
{
    return run_decode(q, k_new, v_new, true, true, true, kv, seq_lens, batch, num_q_heads, num_kv_heads,
                      head_dim, scale, out, out_dtype, lse, workspace, workspace_bytes, max_seq_len, stream);
}

int instattn_decode_merge(const int32_t* seq_lens, int batch, int num_q_heads, int num_kv_heads,
                          int head_dim, int capacity, void* out, int out_dtype, float* lse,
                          const void* workspace, size_t workspace_bytes, int max_seq_len,
                          void* stream)
{
    int st = check_shape(batch, num_q_heads, num_kv_heads, head_dim, max_seq_len);
    if (st != INSTATTN_OK) return st;
    if (!seq_lens || capacity <= 0 || max_seq_len > capacity) return INSTATTN_ERR_INVALID_ARG;
    const Plan p = make_plan(options_snapshot(), batch, num_q_heads, num_kv_heads, max_seq_len, false);
    st = check_plan(p, batch, num_kv_heads);
    if (st != INSTATTN_OK) return st;
    st = check_out(out, out_dtype, workspace, workspace_bytes, carve(batch, num_q_heads, head_dim, p).total);
    if (st != INSTATTN_OK) return st;
    return enqueue_merge(p, seq_lens, batch, num_q_heads, head_dim, out, out_dtype, lse, workspace, max_seq_len,
                         (hipStream_t)stream);
}

int instattn_decode(const void* q, const instattn_kv_desc* kv, const int32_t* seq_lens, int batch,
                    int num_q_heads, int num_kv_heads, int head_dim, float scale, void* out,
                    int out_dtype, float* lse, void* workspace, size_t workspace_bytes,
                    int max_seq_len, void* stream)
{
    return run_decode(q, nullptr, nullptr, false, true, true, kv, seq_lens, batch, num_q_heads, num_kv_heads,
                      head_dim, scale, out, out_dtype, lse, workspace, workspace_bytes, max_seq_len, stream);
}

// ---------------------------------------------------------------------------
// The entry point that allocates nothing: instattn_decode with the library's own scratch
// as its workspace.  `scratch` is a host-side stand-in for the device array, not an address
// a kernel can take; the device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[INSTATTN_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];       // per device: its own copy of the array, at its own address
std::mutex g_scratch_mutex;

// Address of the current device's copy of `scratch`; nullptr (and *status set) on failure.
void* scratch_of_current_device(int* status)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        *status = INSTATTN_ERR_RUNTIME;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
            *status = INSTATTN_ERR_RUNTIME;
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

}  // namespace

int instattn_decode_static(const void* q, const instattn_kv_desc* kv, const int32_t* seq_lens, int batch,
                           int num_q_heads, int num_kv_heads, int head_dim, float scale, void* out,
                           int out_dtype, float* lse, int max_seq_len, void* stream)
{
    // sizes first: a call that does not fit is rejected whatever the device says
    if (check_shape(batch, num_q_heads, num_kv_heads, head_dim, max_seq_len) == INSTATTN_OK) {
        const size_t need = instattn_decode_workspace_size(batch, num_q_heads, num_kv_heads, head_dim, max_seq_len);
        if (need > (size_t)INSTATTN_STATIC_SCRATCH_BYTES) return INSTATTN_ERR_WORKSPACE;
    }
    int st = INSTATTN_OK;
    void* ws = scratch_of_current_device(&st);
    if (ws == nullptr) return st;
    return run_decode(q, nullptr, nullptr, false, true, true, kv, seq_lens, batch, num_q_heads, num_kv_heads,
                      head_dim, scale, out, out_dtype, lse, ws, (size_t)INSTATTN_STATIC_SCRATCH_BYTES, max_seq_len,
                      stream);
}

int instattn_probe_read(const void* src, size_t bytes, void* sink, void* stream)
{
    if (!src || !sink || bytes == 0 || bytes % 16 || !aligned16(src)) return INSTATTN_ERR_INVALID_ARG;
    return status_of(launch_probe_read(src, bytes, sink, (hipStream_t)stream));
}

int instattn_probe_read_columns(const void* base, size_t row_stride, size_t col_stride, int rows, int dims, int r,
                                int positions, void* sink, void* stream)
{
    if (!base || !sink || !aligned16(base) || row_stride % 16 || col_stride % 16) return INSTATTN_ERR_INVALID_ARG;
    if (rows < 1 || dims < 1 || r < 1 || r > dims) return INSTATTN_ERR_INVALID_ARG;
    if (positions < 8 || positions % 8 || (size_t)positions * 2 > col_stride || (size_t)dims * col_stride > row_stride)
        return INSTATTN_ERR_INVALID_ARG;
    if ((positions + 2047) / 2048 > 65535) return INSTATTN_ERR_UNSUPPORTED;
    return status_of(launch_probe_columns(base, row_stride, col_stride, rows, dims, r, positions, sink,
                                          (hipStream_t)stream));
}

int instattn_probe_copy(const void* src, void* dst, size_t bytes, void* stream)
{
    if (!src || !dst || bytes == 0 || bytes % 16 || !aligned16(src) || !aligned16(dst))
        return INSTATTN_ERR_INVALID_ARG;
    return status_of(launch_probe_copy(src, dst, bytes, (hipStream_t)stream));
}

}  // extern "C"
