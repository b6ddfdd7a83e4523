// SparF attention (Algorithm 1 of the paper) on the HBM-resident cache.
//
// The algorithm reads r of the d_h columns of K to approximate every score, keeps
// the k best positions plus the l most recent ones and runs exact attention over
// those rows only, blended with the mean of V.  On flash its loads are page-wise
// with a filter behind them; in HBM a 256-byte row or a run of 8 positions of one column
// is already an efficient access, so the loads are exact: only selected columns
// and selected rows are read.
//
// Kernels (the device functions they are made of are in sparf_score.h, approximate
// scores; sparf_select.h, selection; sparf_gather.h, attention over the kept rows):
//   sparf_fused_kernel    the whole algorithm in one launch, one block per query
//                         head, scores kept in LDS: 256 threads for rows of at most
//                         8192 positions, 512 up to 18432, 1024 up to 36864.
// Longer rows (or too few heads for the wider forms):
//   sparf_logits_kernel   approximate scores up to the softmax normaliser: blocks walk units
//                         of 2048 positions of one query head; reads the component-
//                         major K copy, writes fp32 scores (log2 domain) and every
//                         wave's max / sum / min.
//   sparf_select_attend_kernel  everything behind the scores: one block per query head
//                         selects (scores in registers) and gathers the rows it
//                         kept; taken when the kept rows of a head are not sliced.
//   sparf_select_kernel   normaliser and selection: one block per query head; an
//                         exact two-level selection over the scores (held in
//                         registers for rows below 65536), ordered compaction
//                         (ties towards the lower position), alpha.
//   sparf_hist_kernel,    the same selection for few heads with long rows, one block
//   sparf_members_kernel, per stretch of 8192 scores in three launches (described
//   sparf_compact_kernel  with the kernels).
//   sparf_attend_kernel   attention and blend: one block per query head (or per slice of its
//                         kept rows, then sparf_merge_kernel combines the slices)
//                         gathers the selected rows of K and V (online softmax as in
//                         the dense vector-ALU kernel) and blends with the mean of V.
// Set-up and append:
//   sparf_build_kernel,   build the component-major K copy and the running sum of V
//   sparf_vsum_kernel     from an existing cache (prefill side).
//   sparf_append_kernel   kv_append plus the new column entry and sum update (the
//                         one-launch kernel and sparf_logits_kernel do this
//                         themselves when asked to and every KV head has a single
//                         query head).
#include <stdlib.h>

#include <atomic>

#include "sparf.h"
#include "sparf_gather.h"
#include "sparf_score.h"
#include "sparf_select.h"

#ifndef INSTATTN_SPARF_WAVES_PER_SIMD
#define INSTATTN_SPARF_WAVES_PER_SIMD 4   // register budget: blocks of 4 waves resident per compute unit
#endif

namespace instattn {

// ---------------------------------------------------------------------------
// Approximate scores (without the normaliser), long rows.  A block of 256 threads ranks the
// query once and walks units of 2048 positions of its head, every gridDim.y-th one;
// a thread owns 8 consecutive positions of a unit and adds up the kept columns in
// rank order, 8 columns per step (the same sums, in the same order, as the column
// pass of the one-launch kernel).  The steps of all its units form one sequence:
// the loads of step i+1 are in flight while step i is consumed, across units, and
// every step issues its 8 loads unconditionally (a last group of fewer than 8
// columns repeats the last column, steps behind the row's end re-read its last 8
// positions) so that the count of loads in flight is known at every wait.  The
// columns of a step and their q components come out of two registers by lane index
// (lane j holds the component ranked j): no LDS, no barrier after the query ranking.
// Scores go to the workspace; every wave leaves the max / sum of 2^(x - max) / min
// of its 512 positions.
#ifndef INSTATTN_SPARF_LOGITS_CG
// Columns per step; with 4 or 2 a thread takes 2 or 4 runs of 8 positions, 2048 apart,
// of each (fewer address streams per block, same bytes in flight: measured the same).
#define INSTATTN_SPARF_LOGITS_CG 8
#endif
template <bool PAGED>
__global__ __launch_bounds__(256, INSTATTN_SPARF_WAVES_PER_SIMD) void sparf_logits_kernel(SparfArgs a)
{
    constexpr int NT = 256, CG = INSTATTN_SPARF_LOGITS_CG, NV = 8 / CG, SPAN = NT * 8, UNIT = SPAN * NV;
    static_assert(SPAN == 4 * kSparfStatRun, "one statistics entry per wave and span");
    const int h = blockIdx.x, b = blockIdx.z;
    const int G = a.num_q_heads / a.num_kv_heads;
    const int hk = h / G;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t row = (int64_t)b * a.num_q_heads + h;
    const int L_raw = a.seq_lens[b];
    const int L = clamp_len(L_raw, a.max_len);
    const int nunits = (L + UNIT - 1) / UNIT;
    const int stride = gridDim.y;
    if (a.k_new != nullptr) {
        // Fused append (one query head per KV head only).  The new token's column entries
        // are read by one block of the head alone, the one that walks the unit of position
        // L_raw - 1: that block stores the token (row, column entries, sum) before its first
        // load and synchronises, so that its own loads see the new bits; the launches behind
        // this one see them anyway.  A position behind the attended range is read by nobody:
        // the head's first block stores it.
        const int t_new = L_raw - 1;
        const int owner = t_new >= 0 && t_new < L ? (t_new / UNIT) % stride : 0;
        if ((int)blockIdx.y == owner) {                       // block-uniform
            if (tid < a.head_dim) append_component(a, b, hk, tid, L_raw);
            __syncthreads();
        }
    }
    if ((int)blockIdx.y >= nunits) return;                    // block-uniform
    __shared__ float s_q[128];
    __shared__ __align__(16) float s_abs[128];
    __shared__ int s_dim[128];
    __shared__ float s_red[48];
    const float factor = prepare_query(a, row, s_q, s_abs, s_dim, s_red);

    // lane j: component ranked j (and 64 + j) and its q times the factor
    const int D = a.head_dim;
    const int dim_lo = s_dim[lane];
    const int dim_hi = 64 + lane < D ? s_dim[64 + lane] : 0;
    const int qw_lo = __builtin_bit_cast(int, s_q[dim_lo] * factor);
    const int qw_hi = __builtin_bit_cast(int, s_q[dim_hi] * factor);

    const int ng = (a.r + CG - 1) / CG;                       // steps per unit
    const int t_last = (L - 1) & ~7;                          // last run of 8 that holds a position
    struct Step {
        int u, g;                                             // unit, column group
    };
    auto advance = [&](Step& s) {
        if (++s.g == ng) {
            s.g = 0;
            s.u += stride;
        }
    };
    // This thread's v-th run of 8 positions in a unit, pulled back into the row.
    auto run_of = [&](const Step& s, int v) { return min(s.u * UNIT + v * SPAN + tid * 8, t_last); };
    // Where column 0 holds such a run: the page of the component-major copy (paged
    // form) is looked up one step before it is needed.
    struct Pages {
        int p[NV];
    };
    auto pages_of = [&](const Step& s) {
        Pages pg;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            if constexpr (!PAGED) pg.p[v] = b;
            else pg.p[v] = a.aux.page_table[(int64_t)b * a.aux.max_pages + (run_of(s, v) >> a.aux.page_shift)];
        }
        return pg;
    };
    auto ptr = [&](const Step& s, int v, int page) {
        const int t = run_of(s, v);
        if constexpr (PAGED) page = pool_page(page, a.aux.last_page);   // at the use: the id was fetched a step ahead
        return a.aux.kt + (int64_t)page * a.aux.stride_b + (int64_t)hk * a.aux.stride_h + (PAGED ? (t & a.aux.page_mask) : t);
    };
    // columns (as offsets) and q components of a step, wave-uniform
    auto setup = [&](const Step& s, int64_t (&coff)[CG], float (&qv)[CG]) {
        const int c0 = s.g * CG;
        const int dsel = c0 < 64 ? dim_lo : dim_hi;           // a group never straddles 64
        const int qsel = c0 < 64 ? qw_lo : qw_hi;
#pragma unroll
        for (int j = 0; j < CG; ++j) {
            const int rk = min(c0 + j, a.r - 1) & 63;
            coff[j] = (int64_t)__builtin_amdgcn_readlane(dsel, rk) * a.aux.stride_d;
            qv[j] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(qsel, rk));
        }
    };
    auto load = [&](half8_t (&T)[NV][CG], const Step& s, const Pages& pg, const int64_t (&coff)[CG]) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const half_t* p = ptr(s, v, pg.p[v]);
#pragma unroll
            for (int j = 0; j < CG; ++j) T[v][j] = __builtin_nontemporal_load((const half8_t*)(p + coff[j]));
        }
    };

    float x[NV][8];
    auto finish = [&](int u) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int t = u * UNIT + v * SPAN + tid * 8;
            if (t < L) {
                float* dst = a.logits + row * a.lpad + t;
                *(float4_t*)dst = float4_t{x[v][0], x[v][1], x[v][2], x[v][3]};
                *(float4_t*)(dst + 4) = float4_t{x[v][4], x[v][5], x[v][6], x[v][7]};
            }
            const int t_w = u * UNIT + v * SPAN + wave * kSparfStatRun;
            if (t_w < L) {                                    // wave-uniform
                float mx = kNegBig, mn = -kNegBig;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (t + e < L) {
                        mx = fmaxf(mx, x[v][e]);
                        mn = fminf(mn, x[v][e]);
                    }
                float zs = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (t + e < L) zs += fast_exp2(x[v][e] - mx);
                const float mw = wave_max(mx);
                const float zw = wave_sum(zs * fast_exp2(mx - mw));
                const float nw_min = -wave_max(-mn);
                if (lane == 0) {
                    float* st = a.stats + (row * a.nstat + t_w / kSparfStatRun) * 3;
                    st[0] = mw;
                    st[1] = zw;
                    st[2] = nw_min;
                }
            }
        }
    };
    auto consume = [&](const half8_t (&T)[NV][CG], const float (&qv)[CG], const Step& s) {
        if (s.g == 0) {
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int e = 0; e < 8; ++e) x[v][e] = 0.f;
        }
        const int cnt = a.r - s.g * CG;                       // columns of this group (CG or more: all)
#pragma unroll
        for (int j = 0; j < CG; ++j)
            if (cnt >= CG || j < cnt) {
#pragma unroll
                for (int v = 0; v < NV; ++v)
#pragma unroll
                    for (int e = 0; e < 8; ++e) x[v][e] = __builtin_fmaf(qv[j], (float)T[v][j][e], x[v][e]);
            }
        if (s.g == ng - 1) finish(s.u);
    };

    const int n = (nunits - (int)blockIdx.y + stride - 1) / stride * ng;   // this block's steps
    Step sa{(int)blockIdx.y, 0};                              // step whose columns go to A next
    Step sb = sa;                                             // ... to B next
    advance(sb);
    Pages page_a = pages_of(sa), page_b = pages_of(sb);
    half8_t A[NV][CG], B[NV][CG];
    int64_t coff[CG];
    float qa[CG], qb[CG];
    setup(sa, coff, qa);
    load(A, sa, page_a, coff);
    for (int i = 0; i < n; i += 2) {
        const Step ca = sa, cb = sb;                          // the steps consumed in this round
        setup(sb, coff, qb);
        const Step la = sb;
        advance(sa);
        advance(sa);
        const Pages next_a = pages_of(sa);                    // in flight behind B's loads
        load(B, la, page_b, coff);
        pin_order();
        consume(A, qa, ca);
        setup(sa, coff, qa);
        advance(sb);
        advance(sb);
        page_b = pages_of(sb);
        page_a = next_a;
        load(A, sa, page_a, coff);
        pin_order();
        if (i + 1 < n) consume(B, qb, cb);
    }
}

// Maximum, minimum and sum of 2^(x - maximum) of a row from those of its runs of
// 512 scores: lane c folds runs c, 64 + c, ... in that order (independent loads, no
// cross-lane traffic inside the loop), then the 64 lanes are combined once.  The
// order is fixed; every wave (and every block) gets the same values.
__device__ __forceinline__ void row_stats(const SparfArgs& a, int64_t row, int L, float& M, float& xmin, float& Z)
{
    const int nc = (L + kSparfStatRun - 1) / kSparfStatRun;
    const float* st = a.stats + row * a.nstat * 3;
    const int lane = threadIdx.x & 63;
    float m = kNegBig, mn = -kNegBig, z = 0.f;
    for (int c = lane; c < nc; c += 64) {
        const float mc = st[3 * c], zc = st[3 * c + 1], nc_min = st[3 * c + 2];
        const float m2 = fmaxf(m, mc);
        z = z * fast_exp2(m - m2) + zc * fast_exp2(mc - m2);
        m = m2;
        mn = fminf(mn, nc_min);
    }
    M = wave_max(m);
    Z = wave_sum(z * fast_exp2(m - M));
    xmin = -wave_max(-mn);
}

// Normaliser and selection, long rows: one block per head over the stored scores.
// STEPS > 0: the row has at most NT * 8 * STEPS positions, every thread reads its
// scores once and keeps them in registers; STEPS == 0: the selection passes over
// the workspace.
template <int NT, int STEPS>
__global__ __launch_bounds__(NT) void sparf_select_kernel(SparfArgs a)
{
    const int h = blockIdx.x, b = blockIdx.y;
    const int64_t row = (int64_t)b * a.num_q_heads + h;
    const int L = clamp_len(a.seq_lens[b], a.max_len);
    if (L == 0) {
        if (threadIdx.x == 0) a.alpha[row] = 0.f;
        return;
    }
    __shared__ SelectScratch S;
    const float* x = a.logits + row * a.lpad;
    float xr[STEPS > 0 ? STEPS : 1][8];
    if constexpr (STEPS > 0) own_scores<NT, STEPS>(x, L, xr);   // in flight while the statistics are combined
    float M, xmin, Z;
    row_stats(a, row, L, M, xmin, Z);
    float alpha;
    if constexpr (STEPS > 0) alpha = select_rows_reg<NT, STEPS>(xr, x, L, a.k, a.l, M, xmin, Z, a.sel + row * a.k, S);
    else alpha = select_rows<NT>(x, L, a.k, a.l, M, xmin, Z, a.sel + row * a.k, S);
    if (threadIdx.x == 0) a.alpha[row] = alpha;
}

// ---------------------------------------------------------------------------
// Normaliser and selection for few heads with long rows: the selection of a head
// is spread over one block of 256 threads per stretch of 8192 scores (held in
// registers), in three launches that pass small integers through the workspace:
//   sparf_hist_kernel     level-1 histogram of every stretch;
//   sparf_members_kernel  every block adds the histograms up and finds the threshold
//                         bin (same result in all of them), then gathers its members
//                         of that bin into the head's list and counts its scores in
//                         higher bins;
//   sparf_compact_kernel  every block ranks the members (same threshold key in all
//                         of them), derives how many kept rows lie in front of its
//                         stretch, compacts it and leaves its share of the kept
//                         softmax mass; the attend kernel adds the shares up in
//                         stretch order (alpha).  Nothing crosses blocks inside a
//                         launch except one integer atomic per block: fences between
//                         the chip's L2 caches cost more than a launch.
// The kept rows are those of the one-block selection.  If the threshold bin holds
// more than kSparfMemberCap scores (many equal scores), the block of stretch 0 runs
// the one-block selection over the whole row instead.
struct StretchView {
    int L, want, leff, ncand, t0, ncc;     // ncc: stretches that hold candidates
};

__device__ __forceinline__ StretchView stretch_view(const SparfArgs& a, int b, int chunk)
{
    StretchView v;
    v.L = clamp_len(a.seq_lens[b], a.max_len);
    const int keff = min(a.k, v.L);
    v.leff = min(a.l, keff);
    v.want = keff - v.leff;
    v.ncand = v.L - v.leff;
    v.t0 = chunk * kSparfChunk;
    v.ncc = (v.ncand + kSparfChunk - 1) / kSparfChunk;
    return v;
}

__global__ __launch_bounds__(256) void sparf_hist_kernel(SparfArgs a)
{
    constexpr int NT = 256, STEPS = kSparfChunk / (NT * 8);
    const int h = blockIdx.x, part = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int64_t row = (int64_t)b * a.num_q_heads + h;
    const StretchView v = stretch_view(a, b, part);
    if (part == 0 && tid < 2) a.counters[row * 2 + tid] = 0;
    const bool idle = v.want <= 0 || v.t0 >= v.ncand;      // no stretch with candidates for this block
    if (v.L == 0 || (idle && part != 0)) return;
    float M, xmin, Z;
    row_stats(a, row, v.L, M, xmin, Z);
    // the row's statistics, folded once, for the launches behind this one
    if (part == 0 && tid == 0) {
        float* rs = a.rowstat + row * 4;
        rs[0] = M;
        rs[1] = xmin;
        rs[2] = Z;
    }
    if (idle) return;
    const ScoreRange range(M, xmin);
    const Level1 level1(range);
    __shared__ uint32_t s_hist[257];                       // slot 0: places behind the last candidate
    s_hist[1 + tid] = 0;
    __syncthreads();
    // this block's stretches: every nparts-th one (a very long row has more stretches than
    // histograms are kept for it)
    for (int t0 = v.t0; t0 < v.ncand; t0 += a.nparts * kSparfChunk) {
        float xr[STEPS][8];
        own_scores<NT, STEPS>(a.logits + row * a.lpad + t0, v.ncand - t0, xr);
        mark_candidates<NT, STEPS>(xr, t0, v.ncand, range);
#pragma unroll
        for (int i = 0; i < STEPS; ++i)
#pragma unroll
            for (int e = 0; e < 8; ++e) atomicAdd(&s_hist[1 + level1(xr[i][e])], 1u);
    }
    __syncthreads();
    a.hist[(row * a.nparts + part) * 256 + tid] = s_hist[1 + tid];
}

__global__ __launch_bounds__(256) void sparf_members_kernel(SparfArgs a)
{
    constexpr int NT = 256, STEPS = kSparfChunk / (NT * 8);
    const int h = blockIdx.x, chunk = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int64_t row = (int64_t)b * a.num_q_heads + h;
    const StretchView v = stretch_view(a, b, chunk);
    if (v.want <= 0 || v.t0 >= v.ncand) return;
    float xr[STEPS][8];
    own_scores<NT, STEPS>(a.logits + row * a.lpad + v.t0, v.ncand - v.t0, xr);
    const float M = a.rowstat[row * 4], xmin = a.rowstat[row * 4 + 1];
    const ScoreRange range(M, xmin);
    const Level1 level1(range);
    mark_candidates<NT, STEPS>(xr, v.t0, v.ncand, range);

    __shared__ SelectScratch S;
    __shared__ uint32_t s_keys[kSparfMemberCap];
    __shared__ uint32_t s_n, s_above, s_base;
    uint32_t total = 0;
    const uint32_t* hp = a.hist + row * a.nparts * 256 + tid;
    const int np = min(a.nparts, v.ncc);                   // histograms that were written
    int c = 0;
    for (; c + 4 <= np; c += 4) {
        const uint32_t h0 = hp[c * 256], h1 = hp[(c + 1) * 256], h2 = hp[(c + 2) * 256], h3 = hp[(c + 3) * 256];
        total += (h0 + h1) + (h2 + h3);
    }
    for (; c < np; ++c) total += hp[c * 256];
    S.hist(tid) = total;
    if (tid == 0) s_n = s_above = 0;
    __syncthreads();
    if (tid < 64) locate_bin(S, (uint32_t)v.want, tid);
    __syncthreads();
    const int bin1 = (int)S.prefix;
    if (chunk == 0 && tid == 0) {
        a.state[row * 2] = (uint32_t)bin1;
        a.state[row * 2 + 1] = S.remaining;
    }
    uint32_t above = 0;
#pragma unroll
    for (int i = 0; i < STEPS; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) {                      // places without a candidate: bin -1
            const int bin = level1(xr[i][e]);
            above += bin > bin1;
            if (bin == bin1) {
                const uint32_t j = atomicAdd(&s_n, 1u);
                if (j < (uint32_t)kSparfMemberCap) s_keys[j] = order_key(xr[i][e]);
            }
        }
    above = (uint32_t)wave_sum((float)above);              // at most 32 per lane: exact in fp32
    if ((tid & 63) == 0) atomicAdd(&s_above, above);
    __syncthreads();
    const uint32_t n = s_n;
    if (tid == 0) {
        a.gt1[row * a.nchunk + chunk] = s_above;
        s_base = atomicAdd(&a.counters[row * 2], n);       // more than the cap in all: the list is not used
        // more members in this stretch alone than are staged here: the list is not used either
        if (n > (uint32_t)kSparfMemberCap) atomicOr(&a.counters[row * 2 + 1], 1u);
    }
    __syncthreads();
    const uint32_t base = s_base, cap = (uint32_t)a.member_cap;
    for (uint32_t j = tid; j < n && j < (uint32_t)kSparfMemberCap; j += NT) {
        if (base + j < cap) {
            uint32_t* m = a.members + ((uint64_t)row * cap + base + j) * 2;
            m[0] = s_keys[j];
            m[1] = (uint32_t)chunk;
        }
    }
}

__global__ __launch_bounds__(256) void sparf_compact_kernel(SparfArgs a)
{
    constexpr int NT = 256, STEPS = kSparfChunk / (NT * 8);
    const int h = blockIdx.x, chunk = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int64_t row = (int64_t)b * a.num_q_heads + h;
    const StretchView v = stretch_view(a, b, chunk);
    float* share = a.mass_part + row * a.nchunk;           // kept softmax mass per stretch; alpha = sum / Z
    if (v.L == 0) {
        if (tid == 0) share[chunk] = 0.f;
        return;
    }
    __shared__ SelectScratch S;
    const float* x = a.logits + row * a.lpad;
    int32_t* sel = a.sel + row * a.k;
    const float M = a.rowstat[row * 4], xmin = a.rowstat[row * 4 + 1], Z = a.rowstat[row * 4 + 2];
    const uint32_t nmem = v.want > 0 ? a.counters[row * 2] : 0u;
    const uint32_t cap = (uint32_t)a.member_cap;
    const uint32_t* mem = a.members + (uint64_t)row * cap * 2;     // key, stretch
    // The members of the threshold bin are ranked against each other: the threshold key
    // has fewer than rem1 keys above it and at least rem1 at or above.  Up to
    // kSparfMemberCap of them go through LDS; longer lists (rows of hundreds of thousands
    // of positions) are ranked from the workspace: 256 finer buckets over the whole list,
    // then the members of the one bucket that holds the threshold directly.
    __shared__ __align__(16) uint32_t s_mkey[kSparfMemberCap];
    __shared__ __align__(16) uint32_t s_mkey2[kSparfMemberCap];
    __shared__ uint16_t s_mchunk[kSparfMemberCap];
    __shared__ uint32_t s_gtb, s_eqb;
    const ScoreRange range(M, xmin);
    const Level1 level1(range);
    const uint32_t rem1 = v.want > 0 ? a.state[row * 2 + 1] : 0u;
    bool one_block = v.want <= 0 || nmem > cap || a.counters[row * 2 + 1] != 0;
    const bool long_list = !one_block && nmem > (uint32_t)kSparfMemberCap;
    uint32_t rem2 = 0, nsub = 0;
    if (long_list) {
        // every block of the head takes the same decisions from the same list
        S.hist(tid) = 0;
        if (tid == 0) S.nsub = 0;
        __syncthreads();
        for (uint32_t i = tid; i < nmem; i += NT) atomicAdd(&S.hist((int)level1.sub(key_score(mem[2 * i]))), 1u);
        __syncthreads();
        if (tid < 64) locate_bin(S, rem1, tid);
        __syncthreads();
        const uint32_t bucket = S.prefix;
        rem2 = S.remaining;
        for (uint32_t i = tid; i < nmem; i += NT) {
            const uint32_t key = mem[2 * i];
            if (level1.sub(key_score(key)) == bucket) {
                const uint32_t j = atomicAdd(&S.nsub, 1u);
                if (j < (uint32_t)kSparfMemberCap) s_mkey2[j] = key;
            }
        }
        __syncthreads();
        nsub = S.nsub;
        if (nsub > (uint32_t)kSparfMemberCap) one_block = true;     // that many near-equal scores
    }
    if (one_block) {
        // nothing to pick among the candidates, or too many scores in the threshold bin:
        // the block of stretch 0 does the whole row the one-block way
        if (chunk == 0) {
            const float alpha = select_rows<NT>(x, v.L, a.k, a.l, M, xmin, Z, sel, S);
            if (tid == 0) share[0] = alpha * Z;
        } else if (tid == 0) {
            share[chunk] = 0.f;
        }
        return;
    }
    if (v.t0 >= v.ncand) {
        if (tid == 0) share[chunk] = 0.f;
        return;
    }
    float xr[STEPS][8];
    own_scores<NT, STEPS>(x + v.t0, v.ncand - v.t0, xr);
    mark_candidates<NT, STEPS>(xr, v.t0, v.ncand, range);

    if (tid == 0) s_gtb = s_eqb = 0;
    uint32_t thr, rem_eq;
    // kept rows in front of this stretch: scores in higher bins and members above the
    // threshold key of earlier stretches; rows at the threshold key likewise
    // (every thread counts its share, one LDS atomic per wave; all loads in flight at once)
    uint32_t gtb = 0, eqb = 0;
    if (long_list) {
        if (tid < 3 && nsub + tid < (uint32_t)kSparfMemberCap) s_mkey2[nsub + tid] = 0;
        __syncthreads();
        rank_directly<NT>(s_mkey2, nsub, rem2, S);
        __syncthreads();
        thr = S.prefix;
        rem_eq = S.remaining;
        for (uint32_t i = tid; i < nmem; i += NT) {
            const uint32_t key = mem[2 * i];
            if ((int)mem[2 * i + 1] < chunk) {
                gtb += key > thr;
                eqb += key == thr;
            }
        }
    } else {
        for (uint32_t i = tid; i < nmem; i += NT) {
            s_mkey[i] = mem[2 * i];
            s_mchunk[i] = (uint16_t)mem[2 * i + 1];
        }
        __syncthreads();
        rank_members<NT>(s_mkey, s_mkey2, nmem, (uint32_t)kSparfMemberCap, rem1, level1, S);
        __syncthreads();
        thr = S.prefix;
        rem_eq = S.remaining;
        for (uint32_t i = tid; i < nmem; i += NT) {
            if ((int)s_mchunk[i] < chunk) {
                gtb += s_mkey[i] > thr;
                eqb += s_mkey[i] == thr;
            }
        }
    }
    for (int c = tid; c < chunk; c += NT) gtb += a.gt1[row * a.nchunk + c];
#pragma unroll
    for (int sft = 32; sft > 0; sft >>= 1) {
        gtb += __shfl_xor(gtb, sft, 64);
        eqb += __shfl_xor(eqb, sft, 64);
    }
    if ((tid & 63) == 0) {
        atomicAdd(&s_gtb, gtb);
        atomicAdd(&s_eqb, eqb);
    }
    __syncthreads();
    uint32_t gt_base = s_gtb, eq_base = s_eqb;

    float mass = 0.f;
    compact_tile<NT, STEPS>(xr, v.t0, v.ncand, thr, rem_eq, gt_base, eq_base, &S.wave_cnt[0][0], M, sel,
                            (uint32_t)v.want, mass);
    if (chunk == 0) {
        // the l most recent positions are always kept
        for (int i = tid; i < v.leff; i += NT) {
            const int t = v.ncand + i;
            sel[v.want + i] = t;
            mass += fast_exp2(x[t] - M);
        }
    }
    mass = block_sum(mass, S.red);
    if (tid == 0) share[chunk] = mass;                      // alpha is finished by the attend kernel
}

// Alpha after the distributed selection: the stretches' shares in stretch order.
__device__ __forceinline__ float distributed_alpha(const SparfArgs& a, int64_t row, int L)
{
    const float Z = a.rowstat[row * 4 + 2];
    float kept = 0.f;
    for (int c = 0; c < a.nchunk; ++c) kept += a.mass_part[row * a.nchunk + c];
    return kept / Z;
}

// Attention and blend, long rows: one block per query head and slice of its kept rows.
// With one slice the block writes the output row; with more, each writes its
// share and sparf_merge_kernel finishes (few heads with many kept rows would
// otherwise leave most of the chip idle).
template <int D>
__global__ __launch_bounds__(kSparfAttendWaves * 64) void sparf_attend_kernel(SparfArgs a)
{
    constexpr int NG = kSparfAttendWaves * (kWave / (D / 8));
    const int h = blockIdx.x, slice = blockIdx.y, b = blockIdx.z;
    const int64_t row = (int64_t)b * a.num_q_heads + h;
    const int L = clamp_len(a.seq_lens[b], a.max_len);
    if (L == 0) {
        if (a.nslices == 1) write_zero_row<D>(a, row);     // else the merge writes it
        if (a.distributed && slice == 0 && threadIdx.x == 0) a.alpha[row] = 0.f;
        return;
    }
    __shared__ float s_acc[NG][D];
    __shared__ float s_m[NG];
    __shared__ float s_l[NG];
    __shared__ int32_t s_ids[kSparfAttendIds];
    const int n = min(a.k, L);
    const int p_begin = min(slice * a.slice_rows, n), p_end = min(p_begin + a.slice_rows, n);
    float* part = a.nslices == 1 ? nullptr : a.part + (row * a.nslices + slice) * (D + 2);
    float alpha;
    if (a.distributed) {
        alpha = distributed_alpha(a, row, L);
        if (slice == 0 && threadIdx.x == 0) a.alpha[row] = alpha;
    } else {
        alpha = a.alpha[row];
    }
    attend_rows<D, kSparfAttendWaves>(a, b, h, L, p_begin, p_end, a.sel + row * a.k, alpha, part, s_ids,
                                      kSparfAttendIds, s_acc, s_m, s_l);
}

// Combines the slices of a head (attention and blend finished): one thread per output dim.
template <int D>
__global__ __launch_bounds__(D) void sparf_merge_kernel(SparfArgs a)
{
    const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int64_t row = (int64_t)b * a.num_q_heads + h;
    const int L = clamp_len(a.seq_lens[b], a.max_len);
    if (L == 0) {
        write_zero_row<D>(a, row);
        return;
    }
    const float* part = a.part + row * a.nslices * (D + 2);
    float M = kNegBig;
    for (int s = 0; s < a.nslices; ++s) M = fmaxf(M, part[s * (D + 2) + D]);
    float lsum = 0.f, o = 0.f;
    for (int s = 0; s < a.nslices; ++s) {
        const float w = fast_exp2(part[s * (D + 2) + D] - M);
        lsum += w * part[s * (D + 2) + D + 1];
        o += w * part[s * (D + 2) + tid];
    }
    o /= lsum;
    const int hk = h / (a.num_q_heads / a.num_kv_heads);
    const float alpha = a.alpha[row];
    const float vbar = a.aux.vsum[((int64_t)b * a.num_kv_heads + hk) * D + tid] / (float)L;
    o = alpha * o + (1.f - alpha) * vbar;
    if (a.out_f32) ((float*)a.out)[row * D + tid] = o;
    else ((half_t*)a.out)[row * D + tid] = (half_t)o;
}

// The whole of Algorithm 1 for one query head in one block of NT threads; the
// scores live in dynamic LDS (one float per position, rows of at most
// STEPS * NT * 8 positions).  Three forms: 256 threads for rows up to 8192 (four blocks
// per compute unit), 512 threads for rows up to kSparfFusedWideMaxLen (two blocks per
// compute unit: 72 KB of LDS each) and 1024 threads up to kSparfFusedWidestMaxLen (one
// block: 144 KB).  Once the scores are dead the same LDS holds
// the row ids of the gather and, at its end, the partial sums of its waves.
template <int D, int NT, int STEPS>
__global__ __launch_bounds__(NT, INSTATTN_SPARF_WAVES_PER_SIMD) void sparf_fused_kernel(SparfArgs a)
{
    constexpr int NG = (NT / 64) * (kWave / (D / 8));
    const int h = blockIdx.x, b = blockIdx.y;
    const int G = a.num_q_heads / a.num_kv_heads;
    const int hk = h / G;
    const int tid = threadIdx.x;
    const int64_t row = (int64_t)b * a.num_q_heads + h;
    extern __shared__ __align__(16) float xs[];   // scores, log2 domain
    __shared__ float s_q[128];
    __shared__ __align__(16) float s_abs[128];
    __shared__ int s_dim[128];
    __shared__ SelectScratch S;
    // the gather's partial sums sit at the end of the dynamic LDS, its row ids in front
    const int lds_floats = sparf_fused_lds_floats(a.max_len, NG, D);
    const int ids_cap = lds_floats - sparf_fused_acc_floats(NG, D);
    float(*s_acc)[D] = (float(*)[D])(xs + ids_cap);
    float* s_m = xs + ids_cap + NG * D;
    float* s_l = s_m + NG;

    // approximate scores; the length is not needed before the column pass, so its load and
    // the load of q are in flight together
    const int L_raw = a.seq_lens[b];
    // Fused append (one query head per KV head only: this block is the only reader
    // of the row, the column entries and the sum of this KV head).  The new token is
    // stored when everything else is done, so that nothing waits for those scattered
    // stores; until then its score and its row are taken from k_new / v_new.
    const bool fresh = a.k_new != nullptr && L_raw >= 1 && L_raw <= a.kv.capacity && L_raw <= a.aux.capacity;
    const int t_new = L_raw - 1;
    const float factor = prepare_query(a, row, s_q, s_abs, s_dim, S.red);
    const int L = clamp_len(L_raw, a.max_len);
    if (L == 0) {
        write_zero_row<D>(a, row);
        if (tid == 0) a.alpha[row] = 0.f;
        return;
    }
    // the new token's score comes from k_new below: when it is the row's last position the
    // column pass stops in front of it (a row of 2^n + 1 positions then takes no step for
    // that one position)
    const int L_cols = fresh && t_new == L - 1 ? L - 1 : L;
    if (L_cols > 0) column_passes<NT, STEPS>(a, b, hk, 0, L_cols, factor, s_q, s_dim, xs);
    if (fresh && t_new < L && tid == ((t_new >> 3) % NT)) {
        // the score of the new position, from k_new, by the thread that owns it and with
        // the arithmetic of the column pass
        const half_t* kn = a.k_new + ((int64_t)b * a.num_kv_heads + hk) * D;
        float x = 0.f;
        for (int j = 0; j < a.r; ++j) {
            const int d = s_dim[j];
            x = __builtin_fmaf(s_q[d] * factor, (float)kn[d], x);
        }
        xs[t_new] = x;
    }
    // the thread's own scores stay in registers for the statistics and the selection
    float xr[STEPS][8];
    own_scores<NT, STEPS>(xs, L, xr);
    float M, xmin, Z;
    block_stats<NT, STEPS>(xr, L, S.red, M, xmin, Z);

    // selection
    int32_t* sel = a.sel + row * a.k;
    const float alpha = select_rows_reg<NT, STEPS>(xr, xs, L, a.k, a.l, M, xmin, Z, sel, S);
    if (tid == 0) a.alpha[row] = alpha;

    // attention and blend; the scores are dead, their LDS takes the row ids (the barrier
    // in front of that also makes the kept positions visible to the whole block)
    attend_rows<D, NT / 64>(a, b, h, L, 0, min(a.k, L), sel, alpha, nullptr, (int32_t*)xs, ids_cap, s_acc, s_m, s_l,
                            fresh, t_new);
    if (fresh && tid < D) append_component(a, b, hk, tid, L_raw);
}

// ---------------------------------------------------------------------------
// Everything behind the scores, long rows, one block per head: the selection of
// sparf_select_kernel on register-resident scores, then the same block gathers the
// rows it kept.  With many heads the blocks drift apart, and the latency-bound
// selection of some overlaps the memory-bound gather of others.
template <int D, int NT, int STEPS>
__global__ __launch_bounds__(NT) void sparf_select_attend_kernel(SparfArgs a)
{
    static_assert(STEPS > 0, "scores in registers");
    constexpr int NG = (NT / 64) * (kWave / (D / 8));
    const int h = blockIdx.x, b = blockIdx.y;
    const int64_t row = (int64_t)b * a.num_q_heads + h;
    const int L = clamp_len(a.seq_lens[b], a.max_len);
    if (L == 0) {
        write_zero_row<D>(a, row);
        if (threadIdx.x == 0) a.alpha[row] = 0.f;
        return;
    }
    __shared__ SelectScratch S;
    __shared__ float s_acc[NG][D];
    __shared__ float s_m[NG];
    __shared__ float s_l[NG];
    __shared__ int32_t s_ids[kSparfAttendIds];
    const float* x = a.logits + row * a.lpad;
    float xr[STEPS][8];
    own_scores<NT, STEPS>(x, L, xr);                          // in flight while the statistics are combined
    float M, xmin, Z;
    row_stats(a, row, L, M, xmin, Z);
    int32_t* sel = a.sel + row * a.k;
    const float alpha = select_rows_reg<NT, STEPS>(xr, x, L, a.k, a.l, M, xmin, Z, sel, S);
    if (threadIdx.x == 0) a.alpha[row] = alpha;
    // the barrier in front of the row ids also makes the kept positions visible to the block
    attend_rows<D, NT / 64>(a, b, h, L, 0, min(a.k, L), sel, alpha, nullptr, s_ids, kSparfAttendIds, s_acc, s_m,
                            s_l);
}

// ---------------------------------------------------------------------------
// Component-major copy of K for rows [0, L_b): one block per stretch of 512 rows and
// group of 32 components of one (sequence, KV head).  A thread loads an 8 x 8 block (8 rows, 16 bytes each),
// transposes it in registers, and the 16-byte pieces (8 positions of one component)
// change hands through LDS so that adjacent lanes store adjacent pieces of a column:
// every LDS access is 128 bits wide.  Slots are swizzled by the column group, so the
// lanes of a store hit different banks.
constexpr int kBuildRows = 512;

#ifndef INSTATTN_SPARF_BUILD_COLS
#define INSTATTN_SPARF_BUILD_COLS 32             // components per block of the copy (128: -11 %, 64: -3 %)
#endif
// A block copies DP of the D components of a stretch: fewer components per block mean
// more rows per tile, so longer contiguous runs of every column it writes (DP = 32: 1 KB).
// A copy in short pages cannot take runs that long; there whole rows (DP = D) read better.
template <int D, int DP>
__global__ __launch_bounds__(256) void sparf_build_kernel(SparfArgs a)
{
    constexpr int CS = D / DP;                   // blocks that share a row
    constexpr int COLS8 = DP / 8;                // 16-byte pieces of a row this block reads
    constexpr int RUNS = 256 / COLS8;            // runs of 8 rows per tile: one 8 x 8 block per thread
    constexpr int TILE = 8 * RUNS;               // rows per tile
    static_assert(kBuildRows % TILE == 0, "a stretch is a whole number of tiles");
    const int hk = blockIdx.x / CS, d0 = (blockIdx.x % CS) * DP, b = blockIdx.z;
    const int tid = threadIdx.x;
    const int L = clamp_len(a.seq_lens[b], min(a.kv.capacity, a.aux.capacity));
    const int t_begin = blockIdx.y * kBuildRows, t_end = min(t_begin + kBuildRows, L);
    if (t_begin >= L) return;

    __shared__ u32x4 s_piece[DP][RUNS];          // [component][run of 8 positions, swizzled]
    const int c8 = tid % COLS8, run = tid / COLS8;
    for (int t0 = t_begin; t0 < t_end; t0 += TILE) {
        // rows t0 + 8 run .. + 7 (rows at or behind L are not read; their slots become 0)
        half8_t rows[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int t = t0 + run * 8 + j;
            const half8_t z = {0, 0, 0, 0, 0, 0, 0, 0};
            rows[j] = t < L ? *(const half8_t*)(a.kv.k + row_offset(a.kv, b, hk, t) + d0 + c8 * 8) : z;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const half8_t col = {rows[0][e], rows[1][e], rows[2][e], rows[3][e],
                                 rows[4][e], rows[5][e], rows[6][e], rows[7][e]};
            s_piece[c8 * 8 + e][run ^ (c8 % RUNS)] = __builtin_bit_cast(u32x4, col);
        }
        __syncthreads();
        for (int i = tid; i < DP * RUNS; i += 256) {
            const int d = i / RUNS, r8 = i % RUNS;
            const int t = t0 + r8 * 8;
            if (t < L)
                *(u32x4*)(kt_col0(a.aux, b, hk, t) + (int64_t)(d0 + d) * a.aux.stride_d) =
                    s_piece[d][r8 ^ ((d / 8) % RUNS)];
        }
        __syncthreads();
    }
}

// Column sums of V over rows [0, L_b): one block of 512 threads per (sequence, KV
// head), or, with scratch from the caller, several blocks per pair that take
// vsum_rows rows each and leave their shares for sparf_vsum_fold_kernel; D / 8
// adjacent threads read a row, each of the 512 / (D / 8) row groups takes runs of 8
// consecutive rows (one page lookup per run, eight loads in flight); the groups'
// sums are added in a fixed order.
constexpr int kVsumThreads = 512;

__global__ __launch_bounds__(kVsumThreads) void sparf_vsum_kernel(SparfArgs a)
{
    constexpr int NT = kVsumThreads, U = 8;
    const int hk = blockIdx.x, b = blockIdx.y, part_of_pair = blockIdx.z;
    const int D = a.head_dim;
    const int tid = threadIdx.x;
    // this block's rows: all of the pair's, or its share when the sum is spread over blocks
    const int L_all = clamp_len(a.seq_lens[b], min(a.kv.capacity, a.aux.capacity));
    const int t_first = part_of_pair * a.vsum_rows;          // a multiple of 8
    const int L = a.vsum_part ? min(L_all, t_first + a.vsum_rows) : L_all;
    const int cols8 = D / 8;                 // 8 or 16
    const int c8 = tid % cols8, part = tid / cols8, parts = NT / cols8;
    __shared__ float s_sum[NT * 8];          // [row group][column]: 32 x 128 or 64 x 64
    float vs[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) vs[e] = 0.f;
    for (int t = t_first + part * U; t < L; t += parts * U) {
        // rows t .. t + 7 lie in one page (pages hold a multiple of 8 rows, t is a multiple of 8)
        const half_t* p = a.kv.v + row_offset(a.kv, b, hk, t) + c8 * 8;
        if (t + U <= L) {
            half8_t vr[U];
#pragma unroll
            for (int j = 0; j < U; ++j) vr[j] = __builtin_nontemporal_load((const half8_t*)(p + (int64_t)j * a.kv.stride_t));
#pragma unroll
            for (int j = 0; j < U; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) vs[e] += (float)vr[j][e];
        } else {
            for (int j = 0; t + j < L; ++j) {
                const half8_t vr = *(const half8_t*)(p + (int64_t)j * a.kv.stride_t);
#pragma unroll
                for (int e = 0; e < 8; ++e) vs[e] += (float)vr[e];
            }
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) s_sum[part * D + c8 * 8 + e] = vs[e];
    __syncthreads();
    if (tid < D) {
        float s = 0.f;
        for (int p = 0; p < parts; ++p) s += s_sum[p * D + tid];
        const int64_t pair = (int64_t)b * a.num_kv_heads + hk;
        if (a.vsum_part) a.vsum_part[(pair * a.vsum_parts + part_of_pair) * D + tid] = s;
        else a.aux.vsum[pair * D + tid] = s;
    }
}

// The blocks' shares of a pair's V sum, added in block order.
__global__ __launch_bounds__(128) void sparf_vsum_fold_kernel(SparfArgs a)
{
    const int hk = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    if (tid >= a.head_dim) return;
    const int64_t pair = (int64_t)b * a.num_kv_heads + hk;
    const float* p = a.vsum_part + pair * a.vsum_parts * a.head_dim + tid;
    float s = 0.f;
    for (int i = 0; i < a.vsum_parts; ++i) s += p[(int64_t)i * a.head_dim];
    a.aux.vsum[pair * a.head_dim + tid] = s;
}

// kv_append plus the new entry of every K column and the update of the V sum.
__global__ __launch_bounds__(256) void sparf_append_kernel(SparfArgs a)
{
    const int D = a.head_dim;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)a.batch * a.num_kv_heads * D;
    if (i >= total) return;
    const int d = (int)(i % D);
    const int hk = (int)((i / D) % a.num_kv_heads);
    const int b = (int)(i / ((int64_t)D * a.num_kv_heads));
    append_component(a, b, hk, d, a.seq_lens[b]);
}

// ---------------------------------------------------------------------------
hipError_t launch_sparf_build(const SparfArgs& a, hipStream_t stream)
{
    const int rows = a.kv.capacity < a.aux.capacity ? a.kv.capacity : a.aux.capacity;
    // components per block: few where the copy can be written in long runs
    const bool long_runs = a.aux.page_table == nullptr || (a.aux.page_mask + 1) >= kBuildRows;
    const int cols = long_runs && a.head_dim > INSTATTN_SPARF_BUILD_COLS ? INSTATTN_SPARF_BUILD_COLS : a.head_dim;
    dim3 grid(a.num_kv_heads * (a.head_dim / cols), (rows + kBuildRows - 1) / kBuildRows, a.batch);
    constexpr int kFew = INSTATTN_SPARF_BUILD_COLS;
    if (a.head_dim == 128) {
        if (cols == kFew) hipLaunchKernelGGL((sparf_build_kernel<128, kFew>), grid, dim3(256), 0, stream, a);
        else hipLaunchKernelGGL((sparf_build_kernel<128, 128>), grid, dim3(256), 0, stream, a);
    } else {
        if (cols == kFew) hipLaunchKernelGGL((sparf_build_kernel<64, kFew>), grid, dim3(256), 0, stream, a);
        else hipLaunchKernelGGL((sparf_build_kernel<64, 64>), grid, dim3(256), 0, stream, a);
    }
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    const int parts = a.vsum_part ? a.vsum_parts : 1;
    hipLaunchKernelGGL(sparf_vsum_kernel, dim3(a.num_kv_heads, a.batch, parts), dim3(kVsumThreads), 0, stream, a);
    if (a.vsum_part) hipLaunchKernelGGL(sparf_vsum_fold_kernel, dim3(a.num_kv_heads, a.batch), dim3(128), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_sparf_append(const SparfArgs& a, hipStream_t stream)
{
    const int64_t total = (int64_t)a.batch * a.num_kv_heads * a.head_dim;
    hipLaunchKernelGGL(sparf_append_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_sparf_logits(const SparfArgs& a, hipStream_t stream)
{
    // about 1024 blocks (four per compute unit) at most: a block walks several stretches of
    // its head when there are more, and ranks the query once for all of them
    // about as many blocks as are resident at once (5 per compute unit), so that each
    // ranks its query once and then streams
    const int64_t heads = (int64_t)a.num_q_heads * a.batch;
    const int unit = 2048 * (8 / INSTATTN_SPARF_LOGITS_CG);
    const int nunits = (a.max_len + unit - 1) / unit;
    int per_head = (int)(1280 / heads);
    per_head = per_head < 1 ? 1 : (per_head > nunits ? nunits : per_head);
    const dim3 grid(a.num_q_heads, per_head, a.batch);
    if (a.aux.page_table) hipLaunchKernelGGL(sparf_logits_kernel<true>, grid, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(sparf_logits_kernel<false>, grid, dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_sparf_select(const SparfArgs& a, hipStream_t stream)
{
    if (a.distributed) {
        dim3 dgrid(a.num_q_heads, a.nchunk, a.batch);
        hipLaunchKernelGGL(sparf_hist_kernel, dim3(a.num_q_heads, a.nparts, a.batch), dim3(256), 0, stream, a);
        hipLaunchKernelGGL(sparf_members_kernel, dgrid, dim3(256), 0, stream, a);
        hipLaunchKernelGGL(sparf_compact_kernel, dgrid, dim3(256), 0, stream, a);
        return hipGetLastError();
    }
    dim3 grid(a.num_q_heads, a.batch);
    // Smallest block whose threads hold the row in registers, 32 or 40 scores each
    // (sequence lengths like to sit just behind a power of two), 64 as the last
    // resort: small blocks share a compute unit and overlap each other's barriers.
#define INSTATTN_SELECT(NT, STEPS) \
    hipLaunchKernelGGL((sparf_select_kernel<NT, STEPS>), grid, dim3(NT), 0, stream, a)
    if (a.max_len <= 256 * 32) INSTATTN_SELECT(256, 4);
    else if (a.max_len <= 256 * 40) INSTATTN_SELECT(256, 5);
    else if (a.max_len <= 512 * 32) INSTATTN_SELECT(512, 4);
    else if (a.max_len <= 512 * 40) INSTATTN_SELECT(512, 5);
    else if (a.max_len <= 1024 * 32) INSTATTN_SELECT(1024, 4);
    else if (a.max_len <= 1024 * 40) INSTATTN_SELECT(1024, 5);
    else if (a.max_len < 1024 * 64) INSTATTN_SELECT(1024, 8);   // the packed 16-bit counts hold at most 65535
    else INSTATTN_SELECT(1024, 0);
#undef INSTATTN_SELECT
    return hipGetLastError();
}

template <int D>
static void launch_select_attend(const SparfArgs& a, hipStream_t stream)
{
    dim3 grid(a.num_q_heads, a.batch);
    // block sizes as in launch_sparf_select
#define INSTATTN_TAIL(NT, STEPS) \
    hipLaunchKernelGGL((sparf_select_attend_kernel<D, NT, STEPS>), grid, dim3(NT), 0, stream, a)
    if (a.max_len <= 256 * 32) INSTATTN_TAIL(256, 4);
    else if (a.max_len <= 256 * 40) INSTATTN_TAIL(256, 5);
    else if (a.max_len <= 512 * 32) INSTATTN_TAIL(512, 4);
    else if (a.max_len <= 512 * 40) INSTATTN_TAIL(512, 5);
    else if (a.max_len <= 1024 * 32) INSTATTN_TAIL(1024, 4);
    else if (a.max_len <= 1024 * 40) INSTATTN_TAIL(1024, 5);
    else INSTATTN_TAIL(1024, 8);
#undef INSTATTN_TAIL
}

// Selection and gather of a head in one block; rows shorter than kSparfTailMaxLen,
// kept rows not sliced.
hipError_t launch_sparf_select_attend(const SparfArgs& a, hipStream_t stream)
{
    if (a.head_dim == 128) launch_select_attend<128>(a, stream);
    else launch_select_attend<64>(a, stream);
    return hipGetLastError();
}

template <int D, int NT, int STEPS>
static hipError_t launch_fused(const SparfArgs& a, hipStream_t stream)
{
    constexpr int NG = (NT / 64) * (kWave / (D / 8));
    const size_t lds = (size_t)sparf_fused_lds_floats(a.max_len, NG, D) * sizeof(float);
    auto kernel = sparf_fused_kernel<D, NT, STEPS>;
    if (lds > 48 * 1024) {
        // more dynamic LDS than a launch gets by default: raise this kernel's limit to the
        // largest it can ask for, once per device (the attribute belongs to the device's copy
        // of the kernel)
        constexpr int kDevices = 64;
        static std::atomic<bool> raised[kDevices];    // zero-initialised; two host threads may both raise it: harmless
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        const bool tracked = dev >= 0 && dev < kDevices;
        if (!tracked || !raised[dev].load(std::memory_order_acquire)) {
            constexpr int most = kSparfFusedWidestMaxLen * (int)sizeof(float);
            e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, most);
            if (e != hipSuccess) return e;
            if (tracked) raised[dev].store(true, std::memory_order_release);
        }
    }
    hipLaunchKernelGGL(kernel, dim3(a.num_q_heads, a.batch), dim3(NT), lds, stream, a);
    return hipGetLastError();
}

hipError_t launch_sparf_fused(const SparfArgs& a, hipStream_t stream)
{
    if (a.fused_threads == 256)
        return a.head_dim == 128 ? launch_fused<128, 256, 4>(a, stream) : launch_fused<64, 256, 4>(a, stream);
    if (a.fused_threads == 512)
        return a.head_dim == 128 ? launch_fused<128, 512, 5>(a, stream) : launch_fused<64, 512, 5>(a, stream);
    return a.head_dim == 128 ? launch_fused<128, 1024, 5>(a, stream) : launch_fused<64, 1024, 5>(a, stream);
}

hipError_t launch_sparf_attend(const SparfArgs& a, hipStream_t stream)
{
    dim3 grid(a.num_q_heads, a.nslices, a.batch), block(kSparfAttendWaves * 64);
    if (a.head_dim == 128) hipLaunchKernelGGL(sparf_attend_kernel<128>, grid, block, 0, stream, a);
    else hipLaunchKernelGGL(sparf_attend_kernel<64>, grid, block, 0, stream, a);
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    if (a.nslices > 1) {
        dim3 mgrid(a.num_q_heads, a.batch);
        if (a.head_dim == 128) hipLaunchKernelGGL(sparf_merge_kernel<128>, mgrid, dim3(128), 0, stream, a);
        else hipLaunchKernelGGL(sparf_merge_kernel<64>, mgrid, dim3(64), 0, stream, a);
    }
    return hipGetLastError();
}

}  // namespace instattn
