// SparF attention (Algorithm 1 of the paper) on the HBM-resident cache.
//
// The algorithm reads r of the d_h columns of K to approximate every score
// (steps 1-4), keeps the k best positions plus the l most recent ones (steps 5-7)
// and runs exact attention over those rows only, blended with the mean of V
// (steps 10-11).  On flash the loads are page-wise with a filter behind them
// (steps 2-3, 8-9); in HBM a 256-byte row or a run of 8 positions of one column
// is already an efficient access, so the loads are exact: only selected columns
// and selected rows are read.
//
// Kernels, in launch order:
//   sparf_logits_kernel   steps 1-4 up to the softmax normaliser: one block per
//                         8192 positions of one query head; reads the component-
//                         major K copy, writes fp32 scores (log2 domain) and the
//                         block's max / sum / min.
//   sparf_select_kernel   steps 4 (normaliser), 5-7: one block per query head; an
//                         exact two-level selection over the scores (held in
//                         registers for rows up to 32768), ordered compaction
//                         (ties towards the lower position), alpha.
//   sparf_hist_kernel,    the same selection for few heads with long rows, one block
//   sparf_members_kernel, per stretch of 8192 scores in three launches (described
//   sparf_compact_kernel  with the kernels).
//   sparf_attend_kernel   steps 10-11: one block per query head (or per slice of its
//                         kept rows, then sparf_merge_kernel combines the slices)
//                         gathers the selected rows of K and V (online softmax as in
//                         the dense vector-ALU kernel) and blends with the mean of V.
//   sparf_fused_kernel    all of the above in one launch, one block per query head,
//                         scores kept in LDS: used when a row has at most 8192
//                         positions.
//   sparf_build_kernel,   build the component-major K copy and the running sum of V
//   sparf_vsum_kernel     from an existing cache (prefill side).
//   sparf_append_kernel   kv_append plus the new column entry and sum update (the
//                         one-launch kernel does this itself when asked to and
//                         every KV head has a single query head).
#include "sparf.h"

#include <stdlib.h>

#include <type_traits>

// Compile-time knobs of the one-launch kernel (defaults are the measured best).
#ifndef INSTATTN_SPARF_CGMAX
#define INSTATTN_SPARF_CGMAX 8       // most kept columns loaded per step of the column pass (16: -5..-14 %)
#endif
#ifndef INSTATTN_SPARF_WAVES_PER_SIMD
#define INSTATTN_SPARF_WAVES_PER_SIMD 4   // register budget: blocks of 4 waves resident per compute unit
#endif

namespace instattn {

namespace {

// Wave-wide reductions: four DPP steps inside each row of 16 lanes, then the four
// row results through scalar registers (no LDS crossbar traffic).  Every lane gets
// the result; the order of the operations is fixed.
__device__ __forceinline__ float lane_value(float x, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), lane));
}
__device__ __forceinline__ float wave_max(float x) {
    x = fmaxf(x, dpp_f32<kDppXor1>(x));
    x = fmaxf(x, dpp_f32<kDppXor2>(x));
    x = fmaxf(x, dpp_f32<kDppHalfMirror>(x));
    x = fmaxf(x, dpp_f32<kDppMirror>(x));
    return fmaxf(fmaxf(lane_value(x, 0), lane_value(x, 16)), fmaxf(lane_value(x, 32), lane_value(x, 48)));
}
__device__ __forceinline__ float wave_sum(float x) {
    x = group_sum<16>(x);
    return (lane_value(x, 0) + lane_value(x, 16)) + (lane_value(x, 32) + lane_value(x, 48));
}

// Block-wide reductions through a small LDS array (one slot per wave); every
// thread gets the result.  `red` must hold blockDim.x / 64 floats.
__device__ __forceinline__ float block_max(float x, float* red) {
    x = wave_max(x);
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = x;
    __syncthreads();
    float m = red[0];
    for (int i = 1; i < nw; ++i) m = fmaxf(m, red[i]);
    return m;
}
__device__ __forceinline__ float block_min(float x, float* red) { return -block_max(-x, red); }
__device__ __forceinline__ float block_sum(float x, float* red) {
    x = wave_sum(x);
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[w] = x;
    __syncthreads();
    float s = 0.f;
    for (int i = 0; i < nw; ++i) s += red[i];   // fixed order: deterministic
    return s;
}

// Monotone map from float to unsigned: a < b  <=>  key(a) < key(b).
__device__ __forceinline__ uint32_t order_key(float x) {
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Step 1 and the temperature of step 4.  Leaves q (fp32) in s_q and the components
// ordered by decreasing |q| (ties towards the lower index) in s_dim; returns the
// factor that turns a column dot product into a log2-domain score.  Needs at least
// head_dim threads and is called by the whole block; `red` holds 32 floats and is
// free again once every thread has passed the next barrier.
__device__ __forceinline__ float prepare_query(const SparfArgs& a, int64_t row, float* s_q, float* s_abs,
                                               int* s_dim, float* red)
{
    const int D = a.head_dim, tid = threadIdx.x;
    uint32_t* s_key = (uint32_t*)s_abs;     // 16-byte aligned by its callers
    float mine = 0.f;
    uint32_t key = 0;
    if (tid < D) {
        const half_t qh = a.q[row * D + tid];
        const float qd = (float)qh;
        s_q[tid] = qd;
        mine = fabsf(qd);
        // one integer per component that orders them as step 1 wants: by magnitude (the
        // fp16 bit pattern without its sign is monotone in it), ties to the lower index
        key = ((uint32_t)(__builtin_bit_cast(uint16_t, qh) & 0x7FFFu) << 8) | (uint32_t)(255 - tid);
        s_key[tid] = key;
    }
    __syncthreads();
    float kept = 0.f;
    if (tid < D) {
        // rank = number of keys above this one (keys are distinct); 128-bit LDS reads
        const u32x4* k4 = (const u32x4*)s_key;
        int rank = 0;
#pragma unroll 8
        for (int i = 0; i < D / 4; ++i) {
            const u32x4 o = k4[i];
            rank += (int)(o.x > key) + (int)(o.y > key) + (int)(o.z > key) + (int)(o.w > key);
        }
        s_dim[rank] = tid;
        if (rank < a.r) kept = mine;
    }
    // sqrt(d_h * |q_kept|_1 / |q|_1); 1/sqrt(d_h) is in `scale`.  Both sums in one
    // block reduction (fixed order: deterministic).
    const float tot_w = wave_sum(mine), kept_w = wave_sum(kept);
    const int w = tid >> 6, nw = blockDim.x >> 6;
    if ((tid & 63) == 0) {
        red[w] = tot_w;
        red[16 + w] = kept_w;
    }
    __syncthreads();
    float tot = 0.f, kp = 0.f;
    for (int i = 0; i < nw; ++i) {
        tot += red[i];
        kp += red[16 + i];
    }
    const float rho = tot > 0.f ? kp / tot : 1.f;
    return rho > 0.f ? a.scale_log2 / sqrtf(rho) : 0.f;
}

// Column pass of a whole row by one block (steps 2-4 without the softmax): adds
// to xs[t], t < L, the contribution of CG kept columns, the ones ranked
// j0 .. j0+CG-1, for the L positions that start at t_base (a multiple of 8).  The columns' offsets and the q components are the same for
// every lane and are kept in scalar registers; a thread takes 8 consecutive
// positions per step with one 128-bit load per column, and the loads of step i+1
// are in flight while step i is consumed.  The steps are unrolled and every load
// is issued unconditionally (steps behind the row's end re-read its last 8
// positions, a cache hit) so that the count of loads in flight is known at every
// wait.  first: xs is written, not added to.
template <int CG, int NT, int STEPS>
__device__ __forceinline__ void column_pass(const SparfArgs& a, int b, int hk, int t_base, int L, int j0,
                                            bool first, float factor, const float* s_q, const int* s_dim,
                                            float* xs)
{

    int64_t coff[CG];
    float qv[CG];
#pragma unroll
    for (int j = 0; j < CG; ++j) {
        const int d = __builtin_amdgcn_readfirstlane(s_dim[j0 + j]);
        coff[j] = (int64_t)d * a.aux.stride_d;
        qv[j] = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, s_q[d] * factor)));
    }
    const int tid = threadIdx.x;
    const int t_last = (L - 1) & ~7;                 // last run of 8 that holds a position
    const half_t* p0[STEPS];
#pragma unroll
    for (int i = 0; i < STEPS; ++i) p0[i] = kt_col0(a.aux, b, hk, t_base + min((i * NT + tid) * 8, t_last));

    half8_t A[CG], B[CG];
    auto load = [&](half8_t (&T)[CG], const half_t* p) {
#pragma unroll
        for (int j = 0; j < CG; ++j) T[j] = __builtin_nontemporal_load((const half8_t*)(p + coff[j]));
    };
    auto consume = [&](const half8_t (&T)[CG], int i) {
        const int t = (i * NT + tid) * 8;
        float4_t* dst = (float4_t*)(xs + min(t, t_last));
        const float4_t lo = dst[0], hi = dst[1];
        float x[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[e] = first ? 0.f : lo[e];
            x[4 + e] = first ? 0.f : hi[e];
        }
#pragma unroll
        for (int j = 0; j < CG; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = __builtin_fmaf(qv[j], (float)T[j][e], x[e]);
        if (t <= t_last) {
            dst[0] = float4_t{x[0], x[1], x[2], x[3]};
            dst[1] = float4_t{x[4], x[5], x[6], x[7]};
        }
    };
    load(A, p0[0]);
#pragma unroll
    for (int i = 0; i < STEPS; i += 2) {
        if (i * NT * 8 >= L) break;                  // block-uniform: the row ended before this pair of steps
        if (i + 1 < STEPS) load(B, p0[i + 1]);
        pin_order();
        consume(A, i);
        if (i + 2 < STEPS) load(A, p0[i + 2]);
        pin_order();
        if (i + 1 < STEPS) consume(B, i + 1);
    }
}

constexpr int kSelMembers = 512;     // members of the threshold bin ranked directly

struct SelectScratch {
    uint32_t hist[256];
    uint32_t prefix, remaining, nmem, nsub;
    alignas(16) uint32_t mem_key[kSelMembers];
    alignas(16) uint32_t mem_key2[kSelMembers];
    uint32_t wave_cnt[8][16];        // per round parity (or step) and wave: rows above the threshold | rows at it << 16
    float red[48];
};

// Executed by wave 0 after a histogram is complete: finds the bin that holds the
// remaining-th largest entry (higher bins rank first) and leaves
//   S.prefix = that bin,  S.remaining = entries still to take inside it.
// Lane i owns bins 4i .. 4i+3; suffix sums over the lanes locate the bin.
__device__ __forceinline__ void locate_bin(SelectScratch& S, uint32_t remaining, int lane)
{
    const uint32_t c0 = S.hist[4 * lane], c1 = S.hist[4 * lane + 1];
    const uint32_t c2 = S.hist[4 * lane + 2], c3 = S.hist[4 * lane + 3];
    const uint32_t mine = c0 + c1 + c2 + c3;
    uint32_t suffix = mine;                       // inclusive, over lanes >= this one
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_down(suffix, d, 64);
        if (lane + d < 64) suffix += o;
    }
    uint32_t above = suffix - mine;               // entries in bins above this lane's
    if (above < remaining && remaining <= suffix) {
        int bin = 4 * lane + 3;
        const uint32_t cs[4] = {c0, c1, c2, c3};
#pragma unroll
        for (int j = 3; j > 0; --j) {
            if (above + cs[j] >= remaining) break;
            above += cs[j];
            --bin;
        }
        S.prefix = (uint32_t)bin;
        S.remaining = remaining - above;
    }
}

// All kept columns of one stretch of at most STEPS * NT * 8 positions, in groups
// of INSTATTN_SPARF_CGMAX columns, then halves of that down to one.
template <int CG, int NT, int STEPS>
__device__ __forceinline__ void column_groups(const SparfArgs& a, int b, int hk, int t_base, int L, float factor,
                                              const float* s_q, const int* s_dim, float* xs, int& j0)
{
    if constexpr (CG <= INSTATTN_SPARF_CGMAX)
        for (; a.r - j0 >= CG; j0 += CG)
            column_pass<CG, NT, STEPS>(a, b, hk, t_base, L, j0, j0 == 0, factor, s_q, s_dim, xs);
}

template <int NT, int STEPS>
__device__ __forceinline__ void column_passes(const SparfArgs& a, int b, int hk, int t_base, int L, float factor,
                                              const float* s_q, const int* s_dim, float* xs)
{
    int j0 = 0;
    column_groups<16, NT, STEPS>(a, b, hk, t_base, L, factor, s_q, s_dim, xs, j0);
    column_groups<8, NT, STEPS>(a, b, hk, t_base, L, factor, s_q, s_dim, xs, j0);
    column_groups<4, NT, STEPS>(a, b, hk, t_base, L, factor, s_q, s_dim, xs, j0);
    column_groups<2, NT, STEPS>(a, b, hk, t_base, L, factor, s_q, s_dim, xs, j0);
    column_groups<1, NT, STEPS>(a, b, hk, t_base, L, factor, s_q, s_dim, xs, j0);
}

// The scores of positions (i * NT + tid) * 8 + e, e < 8, of a row of L scores at x
// (what the column pass gave this thread, so no barrier is needed to read them back
// from LDS); 0 where the run of 8 starts at or behind L.
template <int NT, int STEPS>
__device__ __forceinline__ void own_scores(const float* x, int L, float (&xr)[STEPS][8])
{
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < STEPS; ++i) {
        const int t = (i * NT + tid) * 8;
        float4_t lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
        if (t < L) {
            lo = *(const float4_t*)(x + t);
            hi = *(const float4_t*)(x + t + 4);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            xr[i][e] = lo[e];
            xr[i][4 + e] = hi[e];
        }
    }
}

// Softmax statistics of step 4 over the first L positions of such a register
// tile: maximum, minimum and sum of 2^(x - maximum), to every thread.  Own max,
// min and sum first, then one block reduction for all three (fixed order).  red
// holds 48 floats.
template <int NT, int STEPS>
__device__ __forceinline__ void block_stats(const float (&xr)[STEPS][8], int L, float* red, float& M, float& xmin,
                                            float& Z)
{
    const int tid = threadIdx.x;
    float mx = kNegBig, mn = -kNegBig;
#pragma unroll
    for (int i = 0; i < STEPS; ++i) {
        if (i * NT * 8 < L) {                                  // block-uniform
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if ((i * NT + tid) * 8 + e < L) {
                    mx = fmaxf(mx, xr[i][e]);
                    mn = fminf(mn, xr[i][e]);
                }
        }
    }
    float zs = 0.f;
#pragma unroll
    for (int i = 0; i < STEPS; ++i) {
        if (i * NT * 8 < L) {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if ((i * NT + tid) * 8 + e < L) zs += fast_exp2(xr[i][e] - mx);
        }
    }
    const float mw = wave_max(mx);
    const float zw = wave_sum(zs * fast_exp2(mx - mw));
    const float nw_min = -wave_max(-mn);
    const int w = tid >> 6;
    __syncthreads();                       // red is free (earlier readers are done)
    if ((tid & 63) == 0) {
        red[w] = mw;
        red[16 + w] = zw;
        red[32 + w] = nw_min;
    }
    __syncthreads();
    M = kNegBig;
    xmin = -kNegBig;
#pragma unroll
    for (int i = 0; i < NT / 64; ++i) {
        M = fmaxf(M, red[i]);
        xmin = fminf(xmin, red[32 + i]);
    }
    Z = 0.f;
#pragma unroll
    for (int i = 0; i < NT / 64; ++i) Z += red[16 + i] * fast_exp2(red[i] - M);
}

// Level-1 bucket of a score: linear between the row's minimum and maximum,
// monotone in the score, so every score in a higher bucket is >= every score in a
// lower one.
struct Level1 {
    float M, binscale;
    __device__ __forceinline__ Level1(float M_, float xmin) : M(M_), binscale(M_ > xmin ? 255.99f / (M_ - xmin) : 0.f) {}
    __device__ __forceinline__ uint32_t operator()(float v) const {
        return 255u - (uint32_t)min(255, max(0, (int)((M - v) * binscale)));
    }
    // 256 finer buckets inside a level-1 bucket, monotone in the score like the bucket
    __device__ __forceinline__ uint32_t sub(float v) const {
        const float t = (M - v) * binscale;
        const float f = t - (float)min(255, max(0, (int)t));
        return 255u - (uint32_t)min(255, max(0, (int)(f * 256.f)));
    }
};

// Inverse of order_key.
__device__ __forceinline__ float key_score(uint32_t key) {
    return __builtin_bit_cast(float, (key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key);
}

// Ranks the n keys at `keys` (LDS, 16-byte aligned, room for n rounded up to 4)
// against each other: the threshold key is the one with fewer than `remaining` keys
// above it and at least `remaining` at or above.  The tail of the last vector must
// hold 0, a key no finite score has.  Leaves the key in S.prefix and the number of
// rows with exactly that key still wanted in S.remaining.
template <int NT>
__device__ __forceinline__ void rank_directly(const uint32_t* keys, uint32_t n, uint32_t remaining,
                                              SelectScratch& S)
{
    const int tid = threadIdx.x;
    const u32x4* k4 = (const u32x4*)keys;
    const uint32_t n4 = (n + 3) / 4;
    for (uint32_t i = tid; i < n; i += NT) {
        const uint32_t mine = keys[i];
        uint32_t gt = 0, ge = 0;
#pragma unroll 4
        for (uint32_t j = 0; j < n4; ++j) {
            const u32x4 o = k4[j];
            gt += (uint32_t)(o.x > mine) + (uint32_t)(o.y > mine) + (uint32_t)(o.z > mine) + (uint32_t)(o.w > mine);
            ge += (uint32_t)(o.x >= mine) + (uint32_t)(o.y >= mine) + (uint32_t)(o.z >= mine) + (uint32_t)(o.w >= mine);
        }
        if (gt < remaining && remaining <= ge) {         // same values from every such member
            S.prefix = mine;
            S.remaining = remaining - gt;
        }
    }
}

// The threshold key among the n members of the threshold bin (keys, n <= cap; keys2:
// scratch of the same size; both 16-byte aligned LDS).  A handful is ranked
// directly; more go through 256 finer buckets first (linear in n instead of
// quadratic: the members of a long row's bin run into the hundreds) and only the
// members of the one finer bucket that holds the threshold are ranked.  Called by
// the whole block, synchronised on entry; the results are in S.prefix and
// S.remaining after the caller's next barrier.
template <int NT>
__device__ __forceinline__ void rank_members(uint32_t* keys, uint32_t* keys2, uint32_t n, uint32_t cap,
                                             uint32_t remaining, const Level1& level1, SelectScratch& S)
{
    const int tid = threadIdx.x;
    if (n <= 64u) {
        if (tid < 3 && n + tid < cap) keys[n + tid] = 0;
        __syncthreads();
        rank_directly<NT>(keys, n, remaining, S);
        return;
    }
    if (tid < 256) S.hist[tid] = 0;
    if (tid == 0) S.nsub = 0;
    __syncthreads();
    for (uint32_t i = tid; i < n; i += NT) atomicAdd(&S.hist[level1.sub(key_score(keys[i]))], 1u);
    __syncthreads();
    if (tid < 64) locate_bin(S, remaining, tid);
    __syncthreads();
    const uint32_t bucket = S.prefix, rem2 = S.remaining;
    for (uint32_t i = tid; i < n; i += NT) {
        const uint32_t key = keys[i];
        if (level1.sub(key_score(key)) == bucket) keys2[atomicAdd(&S.nsub, 1u)] = key;
    }
    __syncthreads();                                   // also: everyone has read bucket and rem2
    const uint32_t m = S.nsub;
    if (tid < 3 && m + tid < cap) keys2[m + tid] = 0;
    __syncthreads();
    rank_directly<NT>(keys2, m, rem2, S);
}

// The threshold of the top-`want` candidates, exactly, in two levels.  Level 1
// buckets the scores into 256 bins (scores spread evenly over these, unlike over
// the exponent byte of a float).  Level 2 works on the members of the one bin that
// holds the threshold: normally a few dozen, which are gathered and ranked against
// each other directly; if there are more than kSelMembers (e.g. all scores equal)
// a 4-pass radix select on order-preserving keys takes over.  The outcome: the
// kept candidates are those in a bin above bin1, those in bin1 with a key above
// `prefix`, and the first `remaining` (in position order) with exactly that key.
// for_each(f) calls f(score, its level-1 bin) for every candidate of the calling
// thread; it is called several times and must visit the same candidates each time.
template <int NT, class ForEach>
__device__ __forceinline__ void find_threshold(ForEach&& for_each, int want, const Level1& level1,
                                               SelectScratch& S, uint32_t& bin1, uint32_t& prefix,
                                               uint32_t& remaining)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    bin1 = 0;
    prefix = 0;
    remaining = (uint32_t)want;
    if (want <= 0) return;
    // level 1
    if (tid < 256) S.hist[tid] = 0;
    if (tid == 0) S.nmem = 0;
    __syncthreads();
    for_each([&](float, uint32_t bin) { atomicAdd(&S.hist[bin], 1u); });
    __syncthreads();
    if (wave == 0) locate_bin(S, remaining, lane);
    __syncthreads();
    bin1 = S.prefix;
    remaining = S.remaining;
    // level 2: gather the members of bin1
    const uint32_t b1 = bin1;
    for_each([&](float v, uint32_t bin) {
        if (bin == b1) {
            const uint32_t i = atomicAdd(&S.nmem, 1u);
            if (i < (uint32_t)kSelMembers) S.mem_key[i] = order_key(v);
        }
    });
    __syncthreads();
    const uint32_t nmem = S.nmem;
    if (nmem <= (uint32_t)kSelMembers) {
        rank_members<NT>(S.mem_key, S.mem_key2, nmem, (uint32_t)kSelMembers, remaining, level1, S);
        __syncthreads();
        prefix = S.prefix;
        remaining = S.remaining;
    } else {
        for (int shift = 24; shift >= 0; shift -= 8) {
            __syncthreads();
            if (tid < 256) S.hist[tid] = 0;
            __syncthreads();
            const uint32_t hi_mask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
            const uint32_t pfx = prefix;
            for_each([&](float v, uint32_t bin) {
                const uint32_t key = order_key(v);
                if (bin == b1 && (key & hi_mask) == (pfx & hi_mask))
                    atomicAdd(&S.hist[(key >> shift) & 255u], 1u);
            });
            __syncthreads();
            if (wave == 0) locate_bin(S, remaining, lane);
            __syncthreads();
            prefix |= S.prefix << shift;
            remaining = S.remaining;
        }
    }
}

// Ordered compaction of one register tile: xr[i][e] is the score of position
// t_off + (i * NT + tid) * 8 + e, candidates are the positions below ncand.  Writes
// the kept positions of the tile to their slots of sel and adds their softmax mass.
// Position order is (i, wave, lane, e): a shuffle scan over the lanes of a wave per
// step i, the wave totals per step through LDS (step_cnt, STEPS * NT / 64 words),
// one barrier.  The output slot of a row is (rows above the threshold before it) +
// min(rows at the threshold before it, number of those still wanted), so ties go
// to the lower position and the result is deterministic.  gt_base / eq_base count
// the rows above / at the threshold in earlier tiles and are advanced.
template <int NT, int STEPS, class BinOf>
__device__ __forceinline__ void compact_tile(const float (&xr)[STEPS][8], BinOf&& bin_of, int t_off, int ncand,
                                             uint32_t bin1, uint32_t prefix, uint32_t remaining,
                                             uint32_t& gt_base, uint32_t& eq_base, uint32_t* step_cnt,
                                             float M, int32_t* sel, float& mass)
{
    constexpr int NW = NT / 64;
    typedef typename std::conditional<(STEPS > 4), uint64_t, uint32_t>::type bits_t;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // the score whose key is the threshold key (inverse of order_key)
    const float mass_at_key = fast_exp2(key_score(prefix) - M);
    bits_t gtbits = 0, eqbits = 0;                         // bit 8i + e
    uint32_t excl[STEPS];                                  // kept before this lane in its wave, per step
#pragma unroll
    for (int i = 0; i < STEPS; ++i) {
        uint32_t c = 0;
        if (t_off + i * NT * 8 < ncand) {                  // block-uniform
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const bool valid = t_off + (i * NT + tid) * 8 + e < ncand;
                const uint32_t b1 = bin_of(i, e);
                const uint32_t key = order_key(xr[i][e]);
                const bool gt = valid && (b1 > bin1 || (b1 == bin1 && key > prefix));
                const bool eq = valid && b1 == bin1 && key == prefix;
                gtbits |= (bits_t)gt << (8 * i + e);
                eqbits |= (bits_t)eq << (8 * i + e);
                c += (uint32_t)gt + ((uint32_t)eq << 16);
                if (gt) mass += fast_exp2(xr[i][e] - M);   // here, where the score is at hand in a register
            }
        }
        uint32_t incl = c;                                 // 16-bit halves: at most 512 each
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const uint32_t o = __shfl_up(incl, d, 64);
            if (lane >= d) incl += o;
        }
        excl[i] = incl - c;
        if (lane == 63) step_cnt[i * NW + wave] = incl;
    }
    __syncthreads();
    uint32_t run = 0;                                      // halves: at most 65535 each in a tile
#pragma unroll
    for (int i = 0; i < STEPS; ++i) {
        uint32_t mine = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            mine = w == wave ? run : mine;
            run += step_cnt[i * NW + w];
        }
        const uint32_t gb = gt_base + ((mine + excl[i]) & 0xFFFFu), eb = eq_base + ((mine + excl[i]) >> 16);
        // the few flagged slots of this lane, in position order
        const uint32_t g8 = (uint32_t)(gtbits >> (8 * i)) & 0xFFu, e8 = (uint32_t)(eqbits >> (8 * i)) & 0xFFu;
        uint32_t todo = g8 | e8;
        while (todo) {
            const int e = __builtin_ctz(todo);
            todo &= todo - 1;
            const uint32_t below = (1u << e) - 1u;
            const uint32_t eq_before = eb + (uint32_t)__popc(e8 & below);
            const bool above = (g8 >> e) & 1u;
            if (above || eq_before < remaining) {
                sel[gb + (uint32_t)__popc(g8 & below) + min(eq_before, remaining)] = t_off + (i * NT + tid) * 8 + e;
                if (!above) mass += mass_at_key;           // rows at the threshold key share one score
            }
        }
    }
    gt_base += run & 0xFFFFu;
    eq_base += run >> 16;
}

// Steps 5-7 for one head of any length: x[0..L) are the log2-domain scores in
// global memory, M their maximum, xmin their minimum and Z the sum of 2^(x - M).
// Writes the kept positions in ascending order to sel and returns alpha to every
// thread.  The row goes through register tiles of NT * 32 positions (two 128-bit
// loads per thread and step, all of a tile in flight at once): twice for the
// threshold, once for the compaction.
template <int NT>
__device__ __forceinline__ float select_rows(const float* x, int L, int k, int l, float M, float xmin, float Z,
                                             int32_t* sel, SelectScratch& S)
{
    constexpr int STEPS = 4, TILE = NT * 8 * STEPS;
    const int tid = threadIdx.x;
    const int keff = min(k, L);
    const int leff = min(l, keff);
    const int want = keff - leff;          // rows to pick among the candidates
    const int ncand = L - leff;            // candidates: positions [0, ncand)
    const Level1 level1(M, xmin);

    uint32_t bin1, prefix, remaining;
    find_threshold<NT>(
        [&](auto&& f) {
            for (int t_off = 0; t_off < ncand; t_off += TILE) {
                float xr[STEPS][8];
                own_scores<NT, STEPS>(x + t_off, ncand - t_off, xr);
#pragma unroll
                for (int i = 0; i < STEPS; ++i)
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (t_off + (i * NT + tid) * 8 + e < ncand) f(xr[i][e], level1(xr[i][e]));
            }
        },
        want, level1, S, bin1, prefix, remaining);

    float mass = 0.f;
    uint32_t gt_base = 0, eq_base = 0;
    int parity = 0;
    for (int t_off = 0; want > 0 && t_off < ncand; t_off += TILE, parity ^= 1) {
        float xr[STEPS][8];
        own_scores<NT, STEPS>(x + t_off, ncand - t_off, xr);
        compact_tile<NT, STEPS>(
            xr, [&](int i, int e) { return level1(xr[i][e]); }, t_off, ncand, bin1, prefix, remaining, gt_base,
            eq_base, &S.wave_cnt[parity * 4][0], M, sel, mass);
    }
    // step 5: the l most recent positions are always kept
    for (int i = tid; i < leff; i += NT) {
        const int t = ncand + i;
        sel[want + i] = t;
        mass += fast_exp2(x[t] - M);
    }
    return block_sum(mass, S.red) / Z;     // step 7
}

// The same for a row of at most STEPS * NT * 8 positions whose scores the threads
// hold in registers already: xr[i][e] is the score of position (i * NT + tid) * 8 + e
// (what the column pass gave this thread); xs holds the same scores in memory.
template <int NT, int STEPS>
__device__ __forceinline__ float select_rows_reg(const float (&xr)[STEPS][8], const float* xs, int L, int k,
                                                 int l, float M, float xmin, float Z, int32_t* sel,
                                                 SelectScratch& S)
{
    static_assert(STEPS * (NT / 64) <= 128 && STEPS * 8 <= 64, "counts and flag words");
    const int tid = threadIdx.x;
    const int keff = min(k, L);
    const int leff = min(l, keff);
    const int want = keff - leff;
    const int ncand = L - leff;
    const Level1 level1(M, xmin);

    // level-1 bins of the own scores, one byte each, computed once (where the register
    // budget allows: with 40 or 64 scores per thread they are recomputed instead)
    constexpr bool kCacheBins = STEPS <= 4;
    uint32_t bins[kCacheBins ? STEPS : 1][2];
    if constexpr (kCacheBins) {
#pragma unroll
        for (int i = 0; i < STEPS; ++i) {
            bins[i][0] = bins[i][1] = 0;
            if (want > 0 && i * NT * 8 < ncand) {              // block-uniform
#pragma unroll
                for (int e = 0; e < 8; ++e) bins[i][e >> 2] |= level1(xr[i][e]) << (8 * (e & 3));
            }
        }
    }
    auto bin_of = [&](int i, int e) -> uint32_t {
        if constexpr (kCacheBins) return (bins[i][e >> 2] >> (8 * (e & 3))) & 255u;
        else return level1(xr[i][e]);
    };

    uint32_t bin1, prefix, remaining;
    find_threshold<NT>(
        [&](auto&& f) {
#pragma unroll
            for (int i = 0; i < STEPS; ++i) {
                if (i * NT * 8 < ncand) {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if ((i * NT + tid) * 8 + e < ncand) f(xr[i][e], bin_of(i, e));
                }
            }
        },
        want, level1, S, bin1, prefix, remaining);

    float mass = 0.f;
    if (want > 0) {
        uint32_t gt_base = 0, eq_base = 0;
        compact_tile<NT, STEPS>(xr, bin_of, 0, ncand, bin1, prefix, remaining, gt_base, eq_base, &S.wave_cnt[0][0],
                                M, sel, mass);
    }
    // step 5: the l most recent positions are always kept
    for (int i = tid; i < leff; i += NT) {
        const int t = ncand + i;
        sel[want + i] = t;
        mass += fast_exp2(xs[t] - M);
    }
    return block_sum(mass, S.red) / Z;     // step 7
}

// Steps 10-11 for one head over the n kept rows listed in sel, by WAVES waves:
// 16 (or 8) lanes read a row, every row group runs its own online softmax, the
// groups are combined in LDS, the result is blended with the mean of V.
// The kept positions are first turned into row ids in LDS (`ids`, room for
// ids_cap of them; longer lists go through in pieces): the position itself, or,
// for a paged cache, pool page and row inside it packed into one word, so that
// the gather loop has no global load between the id and the row.  Two register
// tiles: the rows of step i+1 are in flight while step i is consumed.
//
// The block handles entries [p_begin, p_end) of the list.  part == nullptr: that is
// the whole list and the block writes the output row.  Otherwise it writes its
// share as D unnormalised sums, their reference maximum and the sum of weights
// (D + 2 floats at part) for sparf_merge_kernel.
//
// fresh: the new token of this step is not in the cache yet (the one-launch kernel
// stores it when everything else is done): its row, position t_new, comes from
// k_new / v_new, and v_new is added to the V sum here.
template <int D, int WAVES>
__device__ __forceinline__ void attend_rows(const SparfArgs& a, int b, int h, int L, int p_begin, int p_end,
                                            const int32_t* sel, float alpha, float* part, int32_t* ids,
                                            int ids_cap, float (*s_acc)[D], float* s_m, float* s_l,
                                            bool fresh = false, int t_new = -1)
{
    constexpr int LPR = D / 8;
    constexpr int RPW = kWave / LPR;
    constexpr int U = 16 / RPW;            // 16 rows per wave and step
    constexpr int TILE = WAVES * 16;
    constexpr int NG = WAVES * RPW;
    const int G = a.num_q_heads / a.num_kv_heads;
    const int hk = h / G;
    const int tid = threadIdx.x;
    const int64_t row = (int64_t)b * a.num_q_heads + h;
    const int wave = tid >> 6, lane = tid & 63;
    const int r = lane / LPR, c = lane % LPR;
    const half8_t q8 = *(const half8_t*)(a.q + row * D + c * 8);
    const bool paged = a.kv.page_table != nullptr;
    const int shift = a.kv.page_shift, mask = a.kv.page_mask;
    const int64_t base = (paged ? 0 : (int64_t)b * a.kv.stride_b) + (int64_t)hk * a.kv.stride_h + c * 8;
    const int64_t stride_page = paged ? a.kv.stride_b : 0;
    const int64_t new_off = ((int64_t)b * a.num_kv_heads + hk) * D + c * 8;
    if (!fresh) t_new = -1;

    float m = kNegBig, l = 0.f;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;

    struct Tile {
        u32x4 k[U], v[U];
    };
    for (int c0 = p_begin; c0 < p_end; c0 += ids_cap) {
        const int nc = min(ids_cap, p_end - c0);
        __syncthreads();                   // whatever used this LDS before is done with it
        for (int i = tid; i < nc; i += WAVES * 64) {
            const int t = sel[c0 + i];
            if (t == t_new) ids[i] = -1;
            else
                ids[i] =
                    paged ? (a.kv.page_table[(int64_t)b * a.kv.max_pages + (t >> shift)] << shift) | (t & mask) : t;
        }
        __syncthreads();
        auto load = [&](Tile& T, int it) {
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const int raw = ids[min(it * TILE + wave * 16 + j * RPW + r, nc - 1)];
                const int id = max(raw, 0);
                const int64_t off = base + (int64_t)(paged ? id >> shift : 0) * stride_page +
                                    (int64_t)(paged ? id & mask : id) * a.kv.stride_t;
                T.k[j] = __builtin_nontemporal_load((const u32x4*)(raw < 0 ? a.k_new + new_off : a.kv.k + off));
                T.v[j] = __builtin_nontemporal_load((const u32x4*)(raw < 0 ? a.v_new + new_off : a.kv.v + off));
            }
        };
        auto consume = [&](const Tile& T, int it) {
            float s[U];
            float mx = m;
#pragma unroll
            for (int j = 0; j < U; ++j) {
                float d = dot8(__builtin_bit_cast(half8_t, T.k[j]), q8, 0.f);
                d = group_sum<LPR>(d);
                s[j] = it * TILE + wave * 16 + j * RPW + r < nc ? d * a.scale_log2 : -__builtin_inff();
                mx = fmaxf(mx, s[j]);
            }
            const float al = fast_exp2(m - mx);
            m = mx;
            l *= al;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] *= al;
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const float p = fast_exp2(s[j] - mx);
                l += p;
                const half8_t vh = __builtin_bit_cast(half8_t, T.v[j]);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] = __builtin_fmaf((float)vh[e], p, acc[e]);
            }
        };
        const int n_it = (nc + TILE - 1) / TILE;
        Tile A, B;
        load(A, 0);
        for (int it = 0; it < n_it; it += 2) {
            load(B, it + 1);
            pin_order();
            consume(A, it);
            load(A, it + 2);
            pin_order();
            if (it + 1 < n_it) consume(B, it + 1);
        }
    }

    const int g = wave * RPW + r;
#pragma unroll
    for (int e = 0; e < 8; ++e) s_acc[g][c * 8 + e] = acc[e];
    if (c == 0) {
        s_m[g] = m;
        s_l[g] = l;
    }
    __syncthreads();
    if (tid < D) {
        float M = kNegBig;
#pragma unroll 8
        for (int i = 0; i < NG; ++i) M = fmaxf(M, s_m[i]);
        float lsum = 0.f, o = 0.f;
#pragma unroll 8
        for (int i = 0; i < NG; ++i) {
            const float w = fast_exp2(s_m[i] - M);
            lsum += w * s_l[i];
            o += w * s_acc[i][tid];
        }
        if (part != nullptr) {
            part[tid] = o;
            if (tid == 0) {
                part[D] = M;
                part[D + 1] = lsum;
            }
            return;
        }
        o /= lsum;
        // step 11: alpha * (attention over the kept rows) + (1 - alpha) * mean of V
        const int64_t vi = ((int64_t)b * a.num_kv_heads + hk) * D + tid;
        float vs = a.aux.vsum[vi];
        if (fresh) vs += (float)a.v_new[vi];
        const float vbar = vs / (float)L;
        o = alpha * o + (1.f - alpha) * vbar;
        if (a.out_f32) ((float*)a.out)[row * D + tid] = o;
        else ((half_t*)a.out)[row * D + tid] = (half_t)o;
    }
}

// Component d of the new token of (sequence b, KV head hk) goes into the cache row,
// the column copy and the V sum; L is the length including that token.
__device__ __forceinline__ void append_component(const SparfArgs& a, int b, int hk, int d, int L)
{
    if (L < 1 || L > a.kv.capacity || L > a.aux.capacity) return;
    const int t = L - 1;
    const int64_t i = ((int64_t)b * a.num_kv_heads + hk) * a.head_dim + d;
    const half_t kn = a.k_new[i], vn = a.v_new[i];
    const int64_t off = row_offset(a.kv, b, hk, t) + d;
    const_cast<half_t*>(a.kv.k)[off] = kn;
    const_cast<half_t*>(a.kv.v)[off] = vn;
    kt_col0(a.aux, b, hk, t)[(int64_t)d * a.aux.stride_d] = kn;
    a.aux.vsum[i] += (float)vn;
}

template <int D>
__device__ __forceinline__ void write_zero_row(const SparfArgs& a, int64_t row)
{
    if ((int)threadIdx.x < D) {
        if (a.out_f32) ((float*)a.out)[row * D + threadIdx.x] = 0.f;
        else ((half_t*)a.out)[row * D + threadIdx.x] = (half_t)0.f;
    }
}

}  // namespace

// ---------------------------------------------------------------------------
// Steps 1-4 (without the normaliser), long rows.  A block of 256 threads ranks the
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
    const int L = clamp_len(a.seq_lens[b], a.max_len);
    const int nunits = (L + UNIT - 1) / UNIT;
    if ((int)blockIdx.y >= nunits) return;                    // block-uniform, before any barrier
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
    const int stride = gridDim.y;
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
// 512 scores: lane c takes run c (then 64 + c ...), every wave (and every block)
// gets the same values.
__device__ __forceinline__ void row_stats(const SparfArgs& a, int64_t row, int L, float& M, float& xmin, float& Z)
{
    const int nc = (L + kSparfStatRun - 1) / kSparfStatRun;
    const float* st = a.stats + row * a.nstat * 3;
    const int lane = threadIdx.x & 63;
    M = kNegBig;
    xmin = -kNegBig;
    Z = 0.f;
    for (int c0 = 0; c0 < nc; c0 += 64) {
        const bool in = c0 + lane < nc;
        const float mc = in ? st[3 * (c0 + lane)] : kNegBig;
        const float zc = in ? st[3 * (c0 + lane) + 1] : 0.f;
        const float nc_min = in ? st[3 * (c0 + lane) + 2] : -kNegBig;
        const float Mn = fmaxf(M, wave_max(mc));
        Z = Z * fast_exp2(M - Mn) + wave_sum(zc * fast_exp2(mc - Mn));
        M = Mn;
        xmin = fminf(xmin, -wave_max(-nc_min));
    }
}

// Steps 4 (normaliser) to 7, long rows: one block per head over the stored scores.
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
// Steps 4 (normaliser) to 7 for few heads with long rows: the selection of a head
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
    const int h = blockIdx.x, chunk = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int64_t row = (int64_t)b * a.num_q_heads + h;
    const StretchView v = stretch_view(a, b, chunk);
    if (chunk == 0 && tid < 2) a.counters[row * 2 + tid] = 0;
    if (v.want <= 0 || v.t0 >= v.ncand) return;
    float xr[STEPS][8];
    own_scores<NT, STEPS>(a.logits + row * a.lpad + v.t0, v.ncand - v.t0, xr);
    float M, xmin, Z;
    row_stats(a, row, v.L, M, xmin, Z);
    const Level1 level1(M, xmin);
    __shared__ uint32_t s_hist[256];
    s_hist[tid] = 0;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < STEPS; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (v.t0 + (i * NT + tid) * 8 + e < v.ncand) atomicAdd(&s_hist[level1(xr[i][e])], 1u);
    __syncthreads();
    a.hist[(row * a.nchunk + chunk) * 256 + tid] = s_hist[tid];
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
    float M, xmin, Z;
    row_stats(a, row, v.L, M, xmin, Z);
    const Level1 level1(M, xmin);

    __shared__ SelectScratch S;
    __shared__ uint32_t s_keys[kSparfMemberCap];
    __shared__ uint32_t s_n, s_above, s_base;
    uint32_t total = 0;
    const uint32_t* hp = a.hist + row * a.nchunk * 256 + tid;
    int c = 0;
    for (; c + 4 <= v.ncc; c += 4) {
        const uint32_t h0 = hp[c * 256], h1 = hp[(c + 1) * 256], h2 = hp[(c + 2) * 256], h3 = hp[(c + 3) * 256];
        total += (h0 + h1) + (h2 + h3);
    }
    for (; c < v.ncc; ++c) total += hp[c * 256];
    S.hist[tid] = total;
    if (tid == 0) s_n = s_above = 0;
    __syncthreads();
    if (tid < 64) locate_bin(S, (uint32_t)v.want, tid);
    __syncthreads();
    const uint32_t bin1 = S.prefix;
    if (chunk == 0 && tid == 0) {
        a.state[row * 2] = bin1;
        a.state[row * 2 + 1] = S.remaining;
    }
    uint32_t above = 0;
#pragma unroll
    for (int i = 0; i < STEPS; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (v.t0 + (i * NT + tid) * 8 + e < v.ncand) {
                const uint32_t bin = level1(xr[i][e]);
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
    }
    __syncthreads();
    const uint32_t base = s_base;
    for (uint32_t j = tid; j < n && j < (uint32_t)kSparfMemberCap; j += NT) {
        if (base + j < (uint32_t)kSparfMemberCap) {
            uint32_t* m = a.members + (row * kSparfMemberCap + base + j) * 2;
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
    float M, xmin, Z;
    row_stats(a, row, v.L, M, xmin, Z);
    const uint32_t nmem = v.want > 0 ? a.counters[row * 2] : 0u;
    if (v.want <= 0 || nmem > (uint32_t)kSparfMemberCap) {
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
    const Level1 level1(M, xmin);
    const uint32_t bin1 = a.state[row * 2], rem1 = a.state[row * 2 + 1];

    // the members of the threshold bin: rank them against each other (the threshold key
    // has fewer than rem1 keys above it and at least rem1 at or above)
    __shared__ __align__(16) uint32_t s_mkey[kSparfMemberCap];
    __shared__ __align__(16) uint32_t s_mkey2[kSparfMemberCap];
    __shared__ uint16_t s_mchunk[kSparfMemberCap];
    __shared__ uint32_t s_gtb, s_eqb;
    for (uint32_t i = tid; i < nmem; i += NT) {
        const uint32_t* m = a.members + (row * kSparfMemberCap + i) * 2;
        s_mkey[i] = m[0];
        s_mchunk[i] = (uint16_t)m[1];
    }
    if (tid == 0) s_gtb = s_eqb = 0;
    __syncthreads();
    rank_members<NT>(s_mkey, s_mkey2, nmem, (uint32_t)kSparfMemberCap, rem1, level1, S);
    __syncthreads();
    const uint32_t thr = S.prefix, rem_eq = S.remaining;
    // kept rows in front of this stretch: scores in higher bins and members above the
    // threshold key of earlier stretches; rows at the threshold key likewise
    // (every thread counts its share, one LDS atomic per wave; all loads in flight at once)
    uint32_t gtb = 0, eqb = 0;
    for (uint32_t i = tid; i < nmem; i += NT) {
        if ((int)s_mchunk[i] < chunk) {
            gtb += s_mkey[i] > thr;
            eqb += s_mkey[i] == thr;
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
    compact_tile<NT, STEPS>(
        xr, [&](int i, int e) { return level1(xr[i][e]); }, v.t0, v.ncand, bin1, thr, rem_eq, gt_base, eq_base,
        &S.wave_cnt[0][0], M, sel, mass);
    if (chunk == 0) {
        // step 5: the l most recent positions are always kept
        for (int i = tid; i < v.leff; i += NT) {
            const int t = v.ncand + i;
            sel[v.want + i] = t;
            mass += fast_exp2(x[t] - M);
        }
    }
    mass = block_sum(mass, S.red);
    if (tid == 0) share[chunk] = mass;                      // step 7 is finished by the attend kernel
}

// Step 7 after the distributed selection: the stretches' shares in stretch order.
__device__ __forceinline__ float distributed_alpha(const SparfArgs& a, int64_t row, int L)
{
    float M, xmin, Z;
    row_stats(a, row, L, M, xmin, Z);
    float kept = 0.f;
    for (int c = 0; c < a.nchunk; ++c) kept += a.mass_part[row * a.nchunk + c];
    return kept / Z;
}

// Steps 10-11, long rows: one block per query head and slice of its kept rows.
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

// Combines the slices of a head (steps 10-11 finished): one thread per output dim.
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

    // steps 1-4; the length is not needed before the column pass, so its load and
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
    column_passes<NT, STEPS>(a, b, hk, 0, L, factor, s_q, s_dim, xs);
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
    // the thread's own scores stay in registers for the rest of steps 4-7
    float xr[STEPS][8];
    own_scores<NT, STEPS>(xs, L, xr);
    float M, xmin, Z;
    block_stats<NT, STEPS>(xr, L, S.red, M, xmin, Z);

    // steps 5-7
    int32_t* sel = a.sel + row * a.k;
    const float alpha = select_rows_reg<NT, STEPS>(xr, xs, L, a.k, a.l, M, xmin, Z, sel, S);
    if (tid == 0) a.alpha[row] = alpha;

    // steps 10-11; the scores are dead, their LDS takes the row ids (the barrier
    // in front of that also makes the kept positions visible to the whole block)
    attend_rows<D, NT / 64>(a, b, h, L, 0, min(a.k, L), sel, alpha, nullptr, (int32_t*)xs, ids_cap, s_acc, s_m, s_l,
                            fresh, t_new);
    if (fresh && tid < D) append_component(a, b, hk, tid, L_raw);
}

// ---------------------------------------------------------------------------
// Steps 4 (normaliser) to 11, long rows, one block per head: the selection of
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
// Component-major copy of K for rows [0, L_b): one block per stretch of 512 rows of
// one (sequence, KV head).  A thread loads an 8 x 8 block (8 rows, 16 bytes each),
// transposes it in registers, and the 16-byte pieces (8 positions of one component)
// change hands through LDS so that adjacent lanes store adjacent pieces of a column:
// every LDS access is 128 bits wide.  Slots are swizzled by the column group, so the
// lanes of a store hit different banks.
constexpr int kBuildRows = 512;

template <int D>
__global__ __launch_bounds__(256) void sparf_build_kernel(SparfArgs a)
{
    constexpr int COLS8 = D / 8;                 // 16-byte pieces per row
    constexpr int RUNS = 256 / COLS8;            // runs of 8 rows per tile: one 8 x 8 block per thread
    constexpr int TILE = 8 * RUNS;               // 128 rows (D = 128) or 256 (D = 64)
    const int hk = blockIdx.x, b = blockIdx.z;
    const int tid = threadIdx.x;
    const int L = clamp_len(a.seq_lens[b], min(a.kv.capacity, a.aux.capacity));
    const int t_begin = blockIdx.y * kBuildRows, t_end = min(t_begin + kBuildRows, L);
    if (t_begin >= L) return;

    __shared__ u32x4 s_piece[D][RUNS];           // [component][run of 8 positions, swizzled]
    const int c8 = tid % COLS8, run = tid / COLS8;
    for (int t0 = t_begin; t0 < t_end; t0 += TILE) {
        // rows t0 + 8 run .. + 7 (rows at or behind L are not read; their slots become 0)
        half8_t rows[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int t = t0 + run * 8 + j;
            const half8_t z = {0, 0, 0, 0, 0, 0, 0, 0};
            rows[j] = t < L ? *(const half8_t*)(a.kv.k + row_offset(a.kv, b, hk, t) + c8 * 8) : z;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const half8_t col = {rows[0][e], rows[1][e], rows[2][e], rows[3][e],
                                 rows[4][e], rows[5][e], rows[6][e], rows[7][e]};
            s_piece[c8 * 8 + e][run ^ (c8 % RUNS)] = __builtin_bit_cast(u32x4, col);
        }
        __syncthreads();
        for (int i = tid; i < D * RUNS; i += 256) {
            const int d = i / RUNS, r8 = i % RUNS;
            const int t = t0 + r8 * 8;
            if (t < L)
                *(u32x4*)(kt_col0(a.aux, b, hk, t) + (int64_t)d * a.aux.stride_d) = s_piece[d][r8 ^ ((d / 8) % RUNS)];
        }
        __syncthreads();
    }
}

// Column sums of V over rows [0, L_b): one block of 1024 threads per (sequence, KV
// head); D / 8 adjacent threads read a row, the 1024 / (D / 8) row groups take every
// such-th row with four loads in flight and are added in a fixed order.
__global__ __launch_bounds__(1024) void sparf_vsum_kernel(SparfArgs a)
{
    const int hk = blockIdx.x, b = blockIdx.y;
    const int D = a.head_dim;
    const int tid = threadIdx.x;
    const int L = clamp_len(a.seq_lens[b], min(a.kv.capacity, a.aux.capacity));
    const int cols8 = D / 8;                 // 8 or 16
    const int c8 = tid % cols8, part = tid / cols8, parts = 1024 / cols8;
    __shared__ float s_sum[8192];            // [row group][column]: 64 x 128 or 128 x 64
    float vs[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) vs[e] = 0.f;
    int t = part;
    for (; t + 3 * parts < L; t += 4 * parts) {
        half8_t vr[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            vr[j] = *(const half8_t*)(a.kv.v + row_offset(a.kv, b, hk, t + j * parts) + c8 * 8);
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) vs[e] += (float)vr[j][e];
    }
    for (; t < L; t += parts) {
        const half8_t vr = *(const half8_t*)(a.kv.v + row_offset(a.kv, b, hk, t) + c8 * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) vs[e] += (float)vr[e];
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) s_sum[part * D + c8 * 8 + e] = vs[e];
    __syncthreads();
    if (tid < D) {
        float s = 0.f;
        for (int p = 0; p < parts; ++p) s += s_sum[p * D + tid];
        a.aux.vsum[((int64_t)b * a.num_kv_heads + hk) * D + tid] = s;
    }
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
    dim3 grid(a.num_kv_heads, (rows + kBuildRows - 1) / kBuildRows, a.batch);
    if (a.head_dim == 128) hipLaunchKernelGGL(sparf_build_kernel<128>, grid, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(sparf_build_kernel<64>, grid, dim3(256), 0, stream, a);
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    hipLaunchKernelGGL(sparf_vsum_kernel, dim3(a.num_kv_heads, a.batch), dim3(1024), 0, stream, a);
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
        hipLaunchKernelGGL(sparf_hist_kernel, dgrid, dim3(256), 0, stream, a);
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
        // more dynamic LDS than a launch gets by default
        const hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
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
