// Device-side declarations of the SparF (sparse decode attention) kernels.
#pragma once

#include "common.h"

namespace instattn {

constexpr int kSparfChunk = 8192;      // positions per block of the approximate-score pass
constexpr int kSparfMaxSeqLen = 65535 * kSparfChunk;   // longest row accepted: its stretches are a grid dimension (and the padded row length stays an int32)
constexpr int kSparfStatRun = 512;     // scores per entry of the score statistics (a wave's share of a unit)
constexpr int kSparfAttendWaves = 8;
constexpr int kSparfMemberCap = 1024;  // members of the threshold bin the distributed selection ranks through LDS
constexpr int kSparfHistParts = 32;    // most level-1 histograms kept per row by the distributed selection
constexpr int kSparfMaxSlices = 8;      // most slices the attend kernel cuts a head's kept rows into
constexpr int kSparfAttendIds = 4096;   // kept rows staged in LDS at a time by the attend kernel

// K stored a second time, component-major (the paper's hidden-embedding-indexed
// copy, Sec. IV-C): element (b, hk, d, t) at b*stride_b + hk*stride_h + d*stride_d + t,
// or, paged, at page*stride_b + hk*stride_h + d*stride_d + (t & page_mask) with
// page = page_table[b*max_pages + (t >> page_shift)].
struct KtView {
    half_t* kt;
    int64_t stride_b, stride_h, stride_d;
    int32_t capacity;                  // max positions per sequence, multiple of 8
    float* vsum;                       // [B][Hkv][D] running sum of the first L_b rows of V
    const int32_t* page_table;         // nullptr: contiguous
    int32_t page_shift, page_mask, max_pages, last_page;
};

// Where column 0 of KV head hk holds position t; the 8 positions of an aligned
// run of 8 are contiguous there, and column d is d*stride_d further on.
__device__ __forceinline__ half_t* kt_col0(const KtView& v, int b, int hk, int t) {
    if (v.page_table == nullptr) return v.kt + (int64_t)b * v.stride_b + (int64_t)hk * v.stride_h + t;
    const int page = pool_page(v.page_table[(int64_t)b * v.max_pages + (t >> v.page_shift)], v.last_page);
    return v.kt + (int64_t)page * v.stride_b + (int64_t)hk * v.stride_h + (t & v.page_mask);
}

struct SparfArgs {
    const half_t* q;                   // [B][Hq][D]
    KvView kv;
    KtView aux;
    const int32_t* seq_lens;
    int32_t batch, num_q_heads, num_kv_heads, head_dim, max_len;
    float scale_log2;
    int32_t r, k, l;
    float* logits;                     // [B][Hq][lpad] approximate scores, log2 domain
    int32_t lpad, nchunk, nstat;       // padded row, its stretches of kSparfChunk, its runs of kSparfStatRun
    float* stats;                      // [B][Hq][nstat][3]: a run's max, sum of 2^(x - max), min
    int32_t* sel;                      // [B][Hq][k] selected rows, ascending
    float* alpha;                      // [B][Hq] selected share of the approximate softmax
    float* part;                       // [B][Hq][nslices][D + 2] shares of the attend kernel's slices
    int32_t nslices, slice_rows;       // slices per head and kept rows per slice (multiple of 16)
    int32_t fused_threads;             // one-launch kernel: threads per head (256, 512 or 1024)
    // selection of a head spread over one block per stretch (few heads, long rows)
    int32_t distributed;
    uint32_t* hist;                    // [B][Hq][nparts][256] level-1 histograms: part p covers stretches p, p + nparts, ...
    int32_t nparts;                    // min(nchunk, kSparfHistParts)
    uint32_t* gt1;                     // [B][Hq][nchunk] scores of the stretch in bins above the threshold bin
    uint32_t* counters;                // [B][Hq][2]: members gathered, spare
    uint32_t* state;                   // [B][Hq][2]: threshold bin, rows still wanted inside it
    uint32_t* members;                 // [B][Hq][member_cap][2]: key and stretch of the bin's members
    int32_t member_cap;                // room in that list: kSparfMemberCap, more for very long rows
    float* mass_part;                  // [B][Hq][nchunk] softmax mass kept per stretch
    float* rowstat;                    // [B][Hq][4]: a row's max, min and sum of 2^(x - max), folded by sparf_hist_kernel
    // set-up: the V sum of a (sequence, KV head) spread over vsum_parts blocks of vsum_rows rows each
    float* vsum_part;                  // [B][Hkv][vsum_parts][D] or nullptr (one block per pair)
    int32_t vsum_parts, vsum_rows;
    void* out;
    int32_t out_f32;
    const half_t* k_new;               // append, or decode with the append fused in
    const half_t* v_new;
};

hipError_t launch_sparf_build(const SparfArgs& a, hipStream_t stream);
hipError_t launch_sparf_append(const SparfArgs& a, hipStream_t stream);
hipError_t launch_sparf_logits(const SparfArgs& a, hipStream_t stream);
hipError_t launch_sparf_select(const SparfArgs& a, hipStream_t stream);
hipError_t launch_sparf_attend(const SparfArgs& a, hipStream_t stream);
hipError_t launch_sparf_select_attend(const SparfArgs& a, hipStream_t stream);
hipError_t launch_sparf_fused(const SparfArgs& a, hipStream_t stream);

constexpr int kSparfFusedMaxLen = 8192;   // rows up to this length take the one-launch kernel with 256 threads
// ... and up to this length its form with 512 threads, when there are heads enough to
// fill the chip with one block each (two blocks of 72 KB of LDS + 8 KB fit a compute unit)
constexpr int kSparfFusedWideMaxLen = 18432;
// ... and up to this length its form with 1024 threads (one block of 144 KB + 8 KB per compute unit)
constexpr int kSparfFusedWidestMaxLen = 36864;
// The wide forms are taken from this many (sequence, query head) pairs on, the 1024-thread form
// up to one block per compute unit.
constexpr int kSparfWideMinHeads = 96;
constexpr int kSparfWidestMaxHeads = 256;

// Floats at the end of the one-launch kernel's dynamic LDS that take the partial
// sums of the gather (NG row groups of D sums, a maximum and a weight each) ...
__host__ __device__ constexpr int sparf_fused_acc_floats(int ng, int d) { return ng * d + 2 * ng; }
// ... and the size of that LDS: one score per position, and never less than those
// sums plus room for 1024 row ids.
__host__ __device__ constexpr int sparf_fused_lds_floats(int max_len, int ng, int d)
{
    const int scores = (max_len + 7) / 8 * 8;
    const int least = sparf_fused_acc_floats(ng, d) + 1024;
    return scores > least ? scores : least;
}
constexpr int kSparfTailMaxLen = 65536;   // rows below this length can be selected and gathered by one block
// Rows up to this length are selected by one block per head, rows from kSparfSpreadAlwaysLen on by one
// block per stretch; in between by one block per stretch when there are at most kSparfSpreadFewHeads
// heads or more than kSparfSpreadManyHeads.
constexpr int kSparfSpreadMinLen = 5 * kSparfChunk;
constexpr int kSparfSpreadAlwaysLen = 12 * kSparfChunk;
constexpr int kSparfSpreadFewHeads = 128;
constexpr int kSparfSpreadManyHeads = 512;

}  // namespace instattn
