// Host side of the C ABI: argument checks, the split plan, kernel launches.
// Nothing here touches device memory or synchronises.
#include "../../include/instattn.h"

#include <math.h>
#include <limits.h>
#include <stdlib.h>

#include "common.h"
#include "host_checks.h"

using namespace instattn;

namespace {

constexpr int kVersion = 100;          // 0.1.0
constexpr int kChunkQuantum = 128;     // every kernel's block tile divides this
constexpr int kMinChunk = 384;
// Work units wanted per launch and largest unit, per kernel family.  The
// vector-ALU kernel runs 5 blocks per CU and is insensitive to the unit size, so
// units stay small enough to balance ragged batches; the MFMA kernel runs 2
// blocks per CU and pays more per unit (prologue, cross-wave epilogue), so it gets
// fewer, larger units: about three per four compute units measured best from
// 16 x 16K down to 128 x 1K rows in all.
constexpr int kTargetUnitsMha = 4096, kMaxChunkMha = 1408;
constexpr int kTargetUnitsGqa = 192, kMaxChunkGqa = 5504;
constexpr int kSingleSplitStreams = 512, kSingleSplitMaxLen = 8192 + kChunkQuantum;
constexpr int kResidentUnits = 1280;   // five blocks of the vector-ALU kernel on each of 256 compute units

struct Plan {
    int chunk;
    int num_splits;
};

// Sequence split: units of `chunk` positions, enough of them to fill the chip
// from host-known sizes alone.  The chunk is an ODD multiple of 128 rows: units
// that start a large power of two apart walk the same HBM channels in lockstep
// and lose up to a fifth of the bandwidth (measured), an odd multiple staggers them.
Plan make_plan(int batch, int num_q_heads, int num_kv_heads, int max_seq_len)
{
    const int group = num_q_heads / num_kv_heads;
    // the MFMA path walks a KV head once for its whole query group
    const long streams = (long)batch * (group == 1 ? num_q_heads : num_kv_heads);
    const long target = group == 1 ? kTargetUnitsMha : kTargetUnitsGqa;
    const long cap = group == 1 ? kMaxChunkMha : kMaxChunkGqa;
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
        chunk = ((((long)max_seq_len + n - 1) / n + kChunkQuantum - 1) / kChunkQuantum | 1) * kChunkQuantum;
    }
    // The MFMA kernel holds two blocks per compute unit.  With a stream or more per
    // compute unit and short sequences, whole sequences are the best units when they
    // come out even over the 256 compute units (256 or 512 streams: 84.5 % of peak
    // against 79 % in two splits, and no merge); otherwise equal splits, three units or
    // more per compute unit, dilute the uneven last round (384 streams of 8K rows in
    // halves: 82 % against 78 % at the longest allowed unit).
    if (group > 1 && streams >= 256 && max_seq_len <= kSingleSplitMaxLen) {
        const long n = streams % 256 == 0 ? 1 : (3 * 256 + streams - 1) / streams;
        chunk = ((((long)max_seq_len + n - 1) / n + kChunkQuantum - 1) / kChunkQuantum | 1) * kChunkQuantum;
        if (chunk < kMinChunk) chunk = kMinChunk;
    }
    const char* forced = getenv("INSTATTN_CHUNK");
    if (forced && atoi(forced) > 0)
        chunk = ((long)atoi(forced) + kChunkQuantum - 1) / kChunkQuantum * kChunkQuantum;
    const long whole = ((long)max_seq_len + kChunkQuantum - 1) / kChunkQuantum * kChunkQuantum;
    if (chunk > whole) chunk = whole;
    Plan p;
    p.chunk = (int)chunk;
    p.num_splits = (int)((max_seq_len + chunk - 1) / chunk);
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

size_t workspace_bytes_for(int batch, int num_q_heads, int head_dim, const Plan& p)
{
    size_t units = (size_t)batch * num_q_heads * p.num_splits;
    size_t bytes = units * (size_t)(head_dim + 1) * sizeof(float);
    return (bytes + 255) / 256 * 256;
}

int check_out(void* out, int out_dtype, const void* workspace, size_t workspace_bytes, size_t need)
{
    if (!out || !aligned16(out)) return INSTATTN_ERR_INVALID_ARG;
    if (out_dtype != INSTATTN_F16 && out_dtype != INSTATTN_F32) return INSTATTN_ERR_INVALID_ARG;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need)
        return INSTATTN_ERR_WORKSPACE;
    return INSTATTN_OK;
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

int instattn_kv_append(const instattn_kv_desc* kv, const void* k_new, const void* v_new,
                       const int32_t* seq_lens, int batch, int num_kv_heads, int head_dim,
                       void* stream)
{
    if (batch <= 0 || num_kv_heads <= 0 || head_dim <= 0 || head_dim % 8) return INSTATTN_ERR_INVALID_ARG;
    int st = check_kv(kv, head_dim);
    if (st != INSTATTN_OK) return st;
    if (!k_new || !v_new || !seq_lens || !aligned16(k_new) || !aligned16(v_new))
        return INSTATTN_ERR_INVALID_ARG;
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
    return launch_kv_append(a, (hipStream_t)stream) == hipSuccess ? INSTATTN_OK : INSTATTN_ERR_RUNTIME;
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
    return launch_kv_write(a, (hipStream_t)stream) == hipSuccess ? INSTATTN_OK : INSTATTN_ERR_RUNTIME;
}

int instattn_decode_plan(int batch, int num_q_heads, int num_kv_heads, int head_dim,
                         int max_seq_len, int* chunk_tokens, int* num_splits)
{
    int st = check_shape(batch, num_q_heads, num_kv_heads, head_dim, max_seq_len);
    if (st != INSTATTN_OK) return st;
    const Plan p = make_plan(batch, num_q_heads, num_kv_heads, max_seq_len);
    if (chunk_tokens) *chunk_tokens = p.chunk;
    if (num_splits) *num_splits = p.num_splits;
    return INSTATTN_OK;
}

size_t instattn_decode_workspace_size(int batch, int num_q_heads, int num_kv_heads, int head_dim,
                                      int max_seq_len)
{
    if (check_shape(batch, num_q_heads, num_kv_heads, head_dim, max_seq_len) != INSTATTN_OK) return 0;
    return workspace_bytes_for(batch, num_q_heads, head_dim,
                               make_plan(batch, num_q_heads, num_kv_heads, max_seq_len));
}

static int run_partial(const void* q, const void* k_new, const void* v_new, bool fused,
                       const instattn_kv_desc* kv, const int32_t* seq_lens,
                       int batch, int num_q_heads, int num_kv_heads, int head_dim,
                       float scale, void* out, int out_dtype, float* lse, void* workspace,
                       size_t workspace_bytes, int max_seq_len, void* stream)
{
    int st = check_shape(batch, num_q_heads, num_kv_heads, head_dim, max_seq_len);
    if (st != INSTATTN_OK) return st;
    st = check_kv(kv, head_dim);
    if (st != INSTATTN_OK) return st;
    if (!q || !aligned16(q) || !seq_lens || !isfinite(scale)) return INSTATTN_ERR_INVALID_ARG;
    if (max_seq_len > kv->capacity) return INSTATTN_ERR_INVALID_ARG;
    if (fused && (!k_new || !v_new || !aligned16(k_new) || !aligned16(v_new)))
        return INSTATTN_ERR_INVALID_ARG;
    const Plan p = make_plan(batch, num_q_heads, num_kv_heads, max_seq_len);
    st = check_out(out, out_dtype, workspace, workspace_bytes,
                   workspace_bytes_for(batch, num_q_heads, head_dim, p));
    if (st != INSTATTN_OK) return st;

    // The split pass stores the new token itself where one block per KV head and unit reads
    // it; a group of more than 16 query heads is shared out over several blocks, so there the
    // store is a launch of its own in front.
    const int group = num_q_heads / num_kv_heads;
    if (fused && group > 16) {
        st = instattn_kv_append(kv, k_new, v_new, seq_lens, batch, num_kv_heads, head_dim, stream);
        if (st != INSTATTN_OK) return st;
        fused = false;
    }
    DecodeArgs a;
    a.group_blocks = (group + 15) / 16;
    a.units = 0;
    // such a group runs on a one-dimensional grid of units x blocks per unit
    if (a.group_blocks > 1 &&
        ((int64_t)batch * num_kv_heads * p.num_splits + 8) * a.group_blocks > (int64_t)INT32_MAX)
        return INSTATTN_ERR_UNSUPPORTED;
    a.k_new = fused ? (const half_t*)k_new : nullptr;
    a.v_new = fused ? (const half_t*)v_new : nullptr;
    // Streams whose strides walk the HBM channels in step (a contiguous cache of 2064
    // rows per head does) lose a tenth to a half of the bandwidth; starting every unit
    // at its own tile undoes most of that and costs about 1 % elsewhere: off by default.
    {
        const char* e = getenv("INSTATTN_ROTATE");
        a.rotate = e && e[0] == '1';
    }
    a.q = (const half_t*)q;
    a.kv = make_view(kv);
    a.seq_lens = seq_lens;
    a.num_q_heads = num_q_heads;
    a.num_kv_heads = num_kv_heads;
    a.chunk = p.chunk;
    a.num_splits = p.num_splits;
    a.max_len = max_seq_len;
    a.scale_log2 = scale * kLog2e;
    a.o_part = (float*)workspace;
    a.lse_part = a.o_part + (size_t)batch * num_q_heads * p.num_splits * head_dim;
    a.out = out;
    a.lse = lse;
    a.out_f32 = out_dtype == INSTATTN_F32;
    hipError_t e = num_q_heads == num_kv_heads
                       ? launch_decode_mha(a, batch, head_dim, (hipStream_t)stream)
                       : launch_decode_gqa(a, batch, head_dim, (hipStream_t)stream);
    return e == hipSuccess ? INSTATTN_OK : INSTATTN_ERR_RUNTIME;
}

int instattn_decode_partial(const void* q, const instattn_kv_desc* kv, const int32_t* seq_lens,
                            int batch, int num_q_heads, int num_kv_heads, int head_dim,
                            float scale, void* out, int out_dtype, float* lse, void* workspace,
                            size_t workspace_bytes, int max_seq_len, void* stream)
{
    return run_partial(q, nullptr, nullptr, false, kv, seq_lens, batch, num_q_heads, num_kv_heads,
                       head_dim, scale, out, out_dtype, lse, workspace, workspace_bytes, max_seq_len,
                       stream);
}

int instattn_append_decode(const void* q, const void* k_new, const void* v_new,
                           const instattn_kv_desc* kv, const int32_t* seq_lens, int batch,
                           int num_q_heads, int num_kv_heads, int head_dim, float scale, void* out,
                           int out_dtype, float* lse, void* workspace, size_t workspace_bytes,
                           int max_seq_len, void* stream)
{
    int st = run_partial(q, k_new, v_new, true, kv, seq_lens, batch, num_q_heads, num_kv_heads,
                         head_dim, scale, out, out_dtype, lse, workspace, workspace_bytes,
                         max_seq_len, stream);
    if (st != INSTATTN_OK) return st;
    return instattn_decode_merge(seq_lens, batch, num_q_heads, num_kv_heads, head_dim,
                                 kv->capacity, out, out_dtype, lse, workspace, workspace_bytes,
                                 max_seq_len, stream);
}

int instattn_decode_merge(const int32_t* seq_lens, int batch, int num_q_heads, int num_kv_heads,
                          int head_dim, int capacity, void* out, int out_dtype, float* lse,
                          const void* workspace, size_t workspace_bytes, int max_seq_len,
                          void* stream)
{
    int st = check_shape(batch, num_q_heads, num_kv_heads, head_dim, max_seq_len);
    if (st != INSTATTN_OK) return st;
    if (!seq_lens || capacity <= 0 || max_seq_len > capacity) return INSTATTN_ERR_INVALID_ARG;
    const Plan p = make_plan(batch, num_q_heads, num_kv_heads, max_seq_len);
    st = check_out(out, out_dtype, workspace, workspace_bytes,
                   workspace_bytes_for(batch, num_q_heads, head_dim, p));
    if (st != INSTATTN_OK) return st;
    if (p.num_splits == 1) return INSTATTN_OK;   // the split pass already wrote out/lse

    MergeArgs m;
    m.seq_lens = seq_lens;
    m.o_part = (const float*)workspace;
    m.lse_part = m.o_part + (size_t)batch * num_q_heads * p.num_splits * head_dim;
    m.out = out;
    m.lse = lse;
    m.num_q_heads = num_q_heads;
    m.chunk = p.chunk;
    m.num_splits = p.num_splits;
    m.max_len = max_seq_len;
    m.out_f32 = out_dtype == INSTATTN_F32;
    return launch_merge(m, batch, head_dim, (hipStream_t)stream) == hipSuccess ? INSTATTN_OK
                                                                                : INSTATTN_ERR_RUNTIME;
}

int instattn_decode(const void* q, const instattn_kv_desc* kv, const int32_t* seq_lens, int batch,
                    int num_q_heads, int num_kv_heads, int head_dim, float scale, void* out,
                    int out_dtype, float* lse, void* workspace, size_t workspace_bytes,
                    int max_seq_len, void* stream)
{
    int st = instattn_decode_partial(q, kv, seq_lens, batch, num_q_heads, num_kv_heads, head_dim,
                                     scale, out, out_dtype, lse, workspace, workspace_bytes,
                                     max_seq_len, stream);
    if (st != INSTATTN_OK) return st;
    return instattn_decode_merge(seq_lens, batch, num_q_heads, num_kv_heads, head_dim,
                                 kv->capacity, out, out_dtype, lse, workspace, workspace_bytes,
                                 max_seq_len, stream);
}

int instattn_probe_read(const void* src, size_t bytes, void* sink, void* stream)
{
    if (!src || !sink || bytes == 0 || bytes % 16 || !aligned16(src)) return INSTATTN_ERR_INVALID_ARG;
    return launch_probe_read(src, bytes, sink, (hipStream_t)stream) == hipSuccess ? INSTATTN_OK
                                                                                    : INSTATTN_ERR_RUNTIME;
}

int instattn_probe_copy(const void* src, void* dst, size_t bytes, void* stream)
{
    if (!src || !dst || bytes == 0 || bytes % 16 || !aligned16(src) || !aligned16(dst))
        return INSTATTN_ERR_INVALID_ARG;
    return launch_probe_copy(src, dst, bytes, (hipStream_t)stream) == hipSuccess ? INSTATTN_OK
                                                                                  : INSTATTN_ERR_RUNTIME;
}

}  // extern "C"
