// SparF device code, the end of Algorithm 1: attention over the kept rows, blend
// with the mean of V; and the store of a new token's components.
#pragma once

#include "sparf.h"

namespace instattn {

namespace {


// Attention and blend for one head over the n kept rows listed in sel, by WAVES waves:
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
            const int t = min(max(sel[c0 + i], 0), L - 1);   // a kept position, whatever the list holds
            if (t == t_new) ids[i] = -1;
            else
                ids[i] =
                    paged ? (pool_page(a.kv.page_table[(int64_t)b * a.kv.max_pages + (t >> shift)], a.kv.last_page) << shift) | (t & mask) : t;
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
        // the blend: alpha * (attention over the kept rows) + (1 - alpha) * mean of V
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

}  // namespace instattn
