// SparF device code, the approximate scores of Algorithm 1: reductions, ranking of the query's
// components, the column pass over the component-major K copy, softmax statistics.
#pragma once

#include "sparf.h"

// Compile-time knobs of the one-launch kernel (defaults are the measured best).
#ifndef INSTATTN_SPARF_CGMAX
#define INSTATTN_SPARF_CGMAX 8       // most kept columns loaded per step of the column pass (16: -5..-14 %)
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

// The kept components and the temperature of the approximate softmax.  Leaves q (fp32) in s_q and the components
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
        // one integer per component that orders them as the algorithm wants: by magnitude (the
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

// Column pass of a whole row by one block (the approximate scores, without the softmax): adds
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

// What the selection works on instead of a raw score: the score pulled into the range
// of the row's numbers, [lo, hi] = [minimum, maximum] cut off at the largest finite
// float.  A score that is not a number becomes lo, an infinite one the end of the
// range: the selection then orders every candidate, whatever the inputs held, and a
// place of a register tile that holds no candidate can be marked by a NaN.
struct ScoreRange {
    float lo, hi;
    __device__ __forceinline__ ScoreRange(float M, float xmin) {
        hi = fminf(M, 3.4028235e38f);
        lo = fminf(fmaxf(xmin, -3.4028235e38f), hi);       // a row without a number: lo = hi
    }
    __device__ __forceinline__ float operator()(float x) const { return fminf(fmaxf(x, lo), hi); }
};

// Candidates of a register tile: xr[i][e], the score of position t_off + (i * NT + tid) * 8 + e,
// is pulled into the range; a NaN marks the places at or behind ncand.
template <int NT, int STEPS>
__device__ __forceinline__ void mark_candidates(float (&xr)[STEPS][8], int t_off, int ncand, const ScoreRange& range)
{
    const int tid = threadIdx.x;
#pragma unroll
    for (int i = 0; i < STEPS; ++i) {
        const int t = t_off + (i * NT + tid) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) xr[i][e] = range(xr[i][e]);
        if (t + 8 > ncand) {                                   // few lanes: the row's end
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (t + e >= ncand) xr[i][e] = __builtin_nanf("");
        }
    }
}

// Statistics of the approximate softmax over the first L positions of such a register
// tile: maximum, minimum and sum of 2^(x - maximum), to every thread.  Own max,
// min and sum first, then one block reduction for all three (fixed order).  red
// holds 48 floats.  A step that lies wholly inside the row (block-uniform) takes no
// per-position tests.
template <int NT, int STEPS>
__device__ __forceinline__ void block_stats(const float (&xr)[STEPS][8], int L, float* red, float& M, float& xmin,
                                            float& Z)
{
    const int tid = threadIdx.x;
    float mx = kNegBig, mn = -kNegBig;
#pragma unroll
    for (int i = 0; i < STEPS; ++i) {
        if ((i + 1) * NT * 8 <= L) {                           // block-uniform
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                mx = fmaxf(mx, xr[i][e]);
                mn = fminf(mn, xr[i][e]);
            }
        } else if (i * NT * 8 < L) {
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
        if ((i + 1) * NT * 8 <= L) {
#pragma unroll
            for (int e = 0; e < 8; ++e) zs += fast_exp2(xr[i][e] - mx);
        } else if (i * NT * 8 < L) {
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

}  // namespace

}  // namespace instattn
