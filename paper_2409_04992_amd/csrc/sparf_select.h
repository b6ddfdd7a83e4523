// SparF device code, the selection of Algorithm 1: exact two-level selection of the k best
// positions, ordered compaction, the kept share of the approximate softmax.
#pragma once

#include <type_traits>

#include "sparf_score.h"

namespace instattn {

namespace {

constexpr int kSelMembers = 512;     // members of the threshold bin ranked directly

struct SelectScratch {
    // level-1 histogram: slot 0 takes the scores that are no candidates (see Level1),
    // slot 1 + b counts bin b
    uint32_t slots[260];
    uint32_t prefix, remaining, nmem, nsub;
    alignas(16) uint32_t mem_key[kSelMembers];
    alignas(16) uint32_t mem_key2[kSelMembers];
    uint32_t wave_cnt[8][16];        // per round parity (or step) and wave: rows above the threshold | rows at it << 16
    float red[48];
    __device__ __forceinline__ uint32_t& hist(int bin) { return slots[bin + 1]; }
};

// Executed by wave 0 after a histogram is complete: finds the bin that holds the
// remaining-th largest entry (higher bins rank first) and leaves
//   S.prefix = that bin,  S.remaining = entries still to take inside it.
// Lane i owns bins 4i .. 4i+3; suffix sums over the lanes locate the bin.
__device__ __forceinline__ void locate_bin(SelectScratch& S, uint32_t remaining, int lane)
{
    const uint32_t c0 = S.hist(4 * lane), c1 = S.hist(4 * lane + 1);
    const uint32_t c2 = S.hist(4 * lane + 2), c3 = S.hist(4 * lane + 3);
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

// Level-1 bucket of a candidate (a score inside the row's range, see ScoreRange):
// linear between the ends of the range, 0 .. 255, monotone in the score (a
// subtraction, a product with a positive factor, a clamp and a truncation are each
// monotone), so every score in a higher bucket is >= every score in a lower one.
// The NaN that marks a place without a candidate gets bucket -1: it is counted
// nowhere and is a member of no bucket.
struct Level1 {
    float lo, scale;
    __device__ __forceinline__ Level1(const ScoreRange& r) : lo(r.lo) {
        const float d = r.hi - r.lo;                       // >= 0, may overflow to infinity
        scale = d > 0.f ? (d < __builtin_inff() ? 255.99f / d : 1e-36f) : 1.f;
    }
    __device__ __forceinline__ float place(float v) const {
        // the maximum first: it turns the NaN into -1
        return fminf(fmaxf((v - lo) * scale, -1.f), 255.99f);
    }
    __device__ __forceinline__ int operator()(float v) const { return (int)place(v); }
    // 256 finer buckets inside a level-1 bucket, monotone in the score like the bucket
    __device__ __forceinline__ uint32_t sub(float v) const {
        const float t = place(v);
        const float f = t - (float)(int)t;
        return (uint32_t)min(255, max(0, (int)(f * 256.f)));
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
    if (tid < 256) S.hist(tid) = 0;
    if (tid == 0) S.nsub = 0;
    __syncthreads();
    for (uint32_t i = tid; i < n; i += NT) atomicAdd(&S.hist((int)level1.sub(key_score(keys[i]))), 1u);
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
// kept candidates are those with a key above `prefix` and the first `remaining`
// (in position order) with exactly that key.
// for_each(f) calls f(score) for every place of the calling thread's register tiles
// (candidates as mark_candidates leaves them: inside the row's range, NaN where a
// place holds none); it is called several times and must visit the same scores each
// time.
template <int NT, class ForEach>
__device__ __forceinline__ void find_threshold(ForEach&& for_each, int want, const Level1& level1,
                                               SelectScratch& S, uint32_t& prefix, uint32_t& remaining)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    prefix = 0;
    remaining = (uint32_t)want;
    if (want <= 0) return;
    // level 1
    if (tid < 256) S.hist(tid) = 0;
    if (tid == 0) S.nmem = 0;
    __syncthreads();
    for_each([&](float v) { atomicAdd(&S.hist(level1(v)), 1u); });
    __syncthreads();
    if (wave == 0) locate_bin(S, remaining, lane);
    __syncthreads();
    const int b1 = (int)S.prefix;
    remaining = S.remaining;
    // level 2: gather the members of that bin
    for_each([&](float v) {
        if (level1(v) == b1) {
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
            if (tid < 256) S.hist(tid) = 0;
            __syncthreads();
            const uint32_t hi_mask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
            const uint32_t pfx = prefix;
            for_each([&](float v) {
                const uint32_t key = order_key(v);
                if (level1(v) == b1 && (key & hi_mask) == (pfx & hi_mask))
                    atomicAdd(&S.hist((int)((key >> shift) & 255u)), 1u);
            });
            __syncthreads();
            if (wave == 0) locate_bin(S, remaining, lane);
            __syncthreads();
            prefix |= S.prefix << shift;
            remaining = S.remaining;
        }
    }
}

// Number of set bits of a wave-wide mask in the lanes below the calling one, added to n.
__device__ __forceinline__ uint32_t lanes_below(uint64_t mask, uint32_t n) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, n));
}

// Ordered compaction of one register tile: xr[i][e] is the candidate at position
// t_off + (i * NT + tid) * 8 + e (inside the row's range), or NaN where that position
// is no candidate.  Writes the kept positions of the tile to their slots of sel and adds
// their softmax mass.  A score is kept when it lies above the threshold score (the one
// whose key is `prefix`; comparing the scores orders them as comparing their keys
// does: the sums the scores come from never give a negative zero), or equals it
// and fewer than `remaining` such rows lie before it.  Position order is (i, wave,
// lane, e): per step i and place e one wave-wide compare, whose mask gives every lane
// the number of kept rows in the lanes below it; the wave totals per step go through
// LDS (step_cnt, STEPS * NT / 64 words), one barrier.  The output slot of a row is
// (rows above the threshold before it) + min(rows at the threshold before it, number
// of those still wanted), so ties go to the lower position and the result is
// deterministic.  gt_base / eq_base count the rows above / at the threshold in earlier
// tiles and are advanced.
template <int NT, int STEPS>
__device__ __forceinline__ void compact_tile(const float (&xr)[STEPS][8], int t_off, int ncand, uint32_t prefix,
                                             uint32_t remaining, uint32_t& gt_base, uint32_t& eq_base,
                                             uint32_t* step_cnt, float M, int32_t* sel, uint32_t room, float& mass)
{
    constexpr int NW = NT / 64;
    typedef typename std::conditional<(STEPS > 4), uint64_t, uint32_t>::type bits_t;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float thr = key_score(prefix);                   // the score whose key is the threshold key
    const float mass_at_key = fast_exp2(thr - M);
    bits_t gtbits = 0, eqbits = 0;                         // bit 8i + e
    uint32_t excl[STEPS];                                  // kept in the lanes below this one, per step (halves)
#pragma unroll
    for (int i = 0; i < STEPS; ++i) {
        uint32_t below = 0, total = 0;                     // halves: at most 512 each
        if (t_off + i * NT * 8 < ncand) {                  // block-uniform
            uint32_t g8 = 0;
            uint64_t any_eq = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const bool gt = xr[i][e] > thr;
                const uint64_t m = __ballot(gt);
                below = lanes_below(m, below);
                total += (uint32_t)__popcll(m);
                g8 |= gt ? 1u << e : 0u;
                mass += gt ? fast_exp2(xr[i][e] - M) : 0.f;
                any_eq |= __ballot(xr[i][e] == thr);
            }
            gtbits |= (bits_t)g8 << (8 * i);
            if (any_eq != 0) {                             // wave-uniform; few waves hold a row at the threshold
                uint32_t e8 = 0, eq_below = 0, eq_total = 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bool eq = xr[i][e] == thr;
                    const uint64_t m = __ballot(eq);
                    eq_below = lanes_below(m, eq_below);
                    eq_total += (uint32_t)__popcll(m);
                    e8 |= eq ? 1u << e : 0u;
                }
                eqbits |= (bits_t)e8 << (8 * i);
                below |= eq_below << 16;
                total |= eq_total << 16;
            }
        }
        excl[i] = below;
        if (lane == 0) step_cnt[i * NW + wave] = total;
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
        // the few flagged places of this lane, in position order
        const uint32_t g8 = (uint32_t)(gtbits >> (8 * i)) & 0xFFu, e8 = (uint32_t)(eqbits >> (8 * i)) & 0xFFu;
        uint32_t todo = g8 | e8;
        while (todo) {
            const int e = __builtin_ctz(todo);
            todo &= todo - 1;
            const uint32_t below = (1u << e) - 1u;
            const uint32_t eq_before = eb + (uint32_t)__popc(e8 & below);
            const bool above = (g8 >> e) & 1u;
            if (above || eq_before < remaining) {
                // slot < room whenever the counts behind the threshold agree with these predicates,
                // which they do by construction; the test keeps a disagreement (scores that are
                // not numbers) from ever becoming a store behind the list
                const uint32_t slot = gb + (uint32_t)__popc(g8 & below) + min(eq_before, remaining);
                if (slot < room) sel[slot] = t_off + (i * NT + tid) * 8 + e;
                if (!above) mass += mass_at_key;           // rows at the threshold key share one score
            }
        }
    }
    gt_base += run & 0xFFFFu;
    eq_base += run >> 16;
}

// The selection for one head of any length: x[0..L) are the log2-domain scores in
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
    const ScoreRange range(M, xmin);
    const Level1 level1(range);

    uint32_t prefix, remaining;
    find_threshold<NT>(
        [&](auto&& f) {
            for (int t_off = 0; t_off < ncand; t_off += TILE) {
                float xr[STEPS][8];
                own_scores<NT, STEPS>(x + t_off, ncand - t_off, xr);
                mark_candidates<NT, STEPS>(xr, t_off, ncand, range);
#pragma unroll
                for (int i = 0; i < STEPS; ++i) {
                    if (t_off + i * NT * 8 < ncand) {          // block-uniform
#pragma unroll
                        for (int e = 0; e < 8; ++e) f(xr[i][e]);
                    }
                }
            }
        },
        want, level1, S, prefix, remaining);

    float mass = 0.f;
    uint32_t gt_base = 0, eq_base = 0;
    int parity = 0;
    for (int t_off = 0; want > 0 && t_off < ncand; t_off += TILE, parity ^= 1) {
        float xr[STEPS][8];
        own_scores<NT, STEPS>(x + t_off, ncand - t_off, xr);
        mark_candidates<NT, STEPS>(xr, t_off, ncand, range);
        compact_tile<NT, STEPS>(xr, t_off, ncand, prefix, remaining, gt_base, eq_base, &S.wave_cnt[parity * 4][0], M,
                                sel, (uint32_t)want, mass);
    }
    // the l most recent positions are always kept
    for (int i = tid; i < leff; i += NT) {
        const int t = ncand + i;
        sel[want + i] = t;
        mass += fast_exp2(x[t] - M);
    }
    return block_sum(mass, S.red) / Z;     // alpha: the kept share of the approximate softmax
}

// The same for a row of at most STEPS * NT * 8 positions whose scores the threads
// hold in registers already: xr[i][e] is the score of position (i * NT + tid) * 8 + e
// (what the column pass gave this thread); xs holds the same scores in memory.  xr is
// turned into candidates in place.
template <int NT, int STEPS>
__device__ __forceinline__ float select_rows_reg(float (&xr)[STEPS][8], const float* xs, int L, int k, int l,
                                                 float M, float xmin, float Z, int32_t* sel, SelectScratch& S)
{
    static_assert(STEPS * (NT / 64) <= 128 && STEPS * 8 <= 64, "counts and flag words");
    const int tid = threadIdx.x;
    const int keff = min(k, L);
    const int leff = min(l, keff);
    const int want = keff - leff;
    const int ncand = L - leff;
    const ScoreRange range(M, xmin);
    const Level1 level1(range);
    mark_candidates<NT, STEPS>(xr, 0, ncand, range);

    uint32_t prefix, remaining;
    find_threshold<NT>(
        [&](auto&& f) {
#pragma unroll
            for (int i = 0; i < STEPS; ++i) {
                if (i * NT * 8 < ncand) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) f(xr[i][e]);
                }
            }
        },
        want, level1, S, prefix, remaining);

    float mass = 0.f;
    if (want > 0) {
        uint32_t gt_base = 0, eq_base = 0;
        compact_tile<NT, STEPS>(xr, 0, ncand, prefix, remaining, gt_base, eq_base, &S.wave_cnt[0][0], M, sel,
                                (uint32_t)want, mass);
    }
    // the l most recent positions are always kept
    for (int i = tid; i < leff; i += NT) {
        const int t = ncand + i;
        sel[want + i] = t;
        mass += fast_exp2(xs[t] - M);
    }
    return block_sum(mass, S.red) / Z;     // alpha: the kept share of the approximate softmax
}

}  // namespace

}  // namespace instattn
