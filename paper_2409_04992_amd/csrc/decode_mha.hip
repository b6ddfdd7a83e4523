// Split pass of decode attention on the vector ALUs (one query head per KV stream).
//
// Paper: Sec. II-B (decode attention is two matrix-vector products over the
// cached K and V) and Sec. III-B (these "Logit" and "Attend" operators are bound
// by KV bandwidth).  With one query row per KV head there is one multiply-add per
// fp16 loaded, so the work stays on the VALU and the kernel is built around
// keeping 128-bit KV loads in flight:
//
//   * A row of D fp16 is read by D/8 adjacent lanes, 16 B each, so one wave load
//     covers 64/(D/8) consecutive rows = 1 KB of contiguous memory.
//   * q.K: four v_dot2_f32_f16 per lane, then a DPP butterfly inside the 8- or
//     16-lane row group (no LDS).
//   * Every row group runs its own online softmax (running max m, sum l, fp32
//     accumulator of its 8 output dims) over the rows it reads, so the loop has
//     no communication between groups; groups are combined once per unit in LDS.
//   * Two register tiles: the loads of tile i+1 are issued before tile i is
//     consumed.  Positions at or behind the unit's end are redirected to its
//     last valid row (a cache hit) and their score is set to -inf, so rows behind
//     the sequence length are never read.
#include "common.h"

// Compile-time knobs (defaults are the measured best).
#ifndef INSTATTN_MHA_NT
#define INSTATTN_MHA_NT 1        // 1: KV loads carry the non-temporal hint
#endif
#ifndef INSTATTN_MHA_WAVES
#define INSTATTN_MHA_WAVES 4     // waves per block
#endif
#ifndef INSTATTN_MHA_WTILE
#define INSTATTN_MHA_WTILE 16    // rows per wave per iteration, contiguous layout (paged: always 16)
#endif

#ifndef INSTATTN_MHA_LDS_PAD
#define INSTATTN_MHA_LDS_PAD 0   // extra LDS bytes per block (experiments: caps blocks per CU)
#endif

namespace instattn {

template <int U>
struct MhaTile {
    u32x4 k[U];
    u32x4 v[U];
};

// 128-bit load at (uniform 64-bit base) + (32-bit per-lane byte offset): the form
// the hardware addresses with a scalar base register pair and one VGPR.
__device__ __forceinline__ u32x4 load16(const char* base, uint32_t lane_off) {
#if INSTATTN_MHA_NT
    return __builtin_nontemporal_load((const u32x4*)(base + (uint64_t)lane_off));
#else
    return *(const u32x4*)(base + (uint64_t)lane_off);
#endif
}

template <int D, bool PAGED>
__global__ __launch_bounds__(INSTATTN_MHA_WAVES * 64) void decode_mha_kernel(DecodeArgs a)
{
    constexpr int LPR = D / 8;             // lanes per row
    constexpr int RPW = kWave / LPR;       // rows per wave load
    constexpr int WAVES = INSTATTN_MHA_WAVES;
    // rows per wave per iteration; 16 never straddles a page
    constexpr int WTILE = PAGED ? 16 : INSTATTN_MHA_WTILE;
    constexpr int U = WTILE / RPW;         // loads of K (and of V) per lane per iteration
    constexpr int TILE = WAVES * WTILE;    // rows per block per iteration
    constexpr int NG = WAVES * RPW;        // independent softmax streams per block

    const int h = blockIdx.x;
    int split, b;
    if (!unit_of_block(a, b, split)) return;       // block-uniform
    const int G = a.num_q_heads / a.num_kv_heads;
    const int hk = h / G;
    const int L = clamp_len(a.seq_lens[b], a.max_len);
    const int t0 = split * a.chunk;
    const int tid = threadIdx.x;
    const int64_t row = (int64_t)b * a.num_q_heads + h;
#if INSTATTN_MHA_LDS_PAD > 0
    __shared__ char s_pad[INSTATTN_MHA_LDS_PAD];
    if (a.chunk < 0) s_pad[tid] = 1;   // never true; keeps the allocation
#endif

    if (G == 1) fused_append<D>(a, b, hk, split, tid);

    if (t0 >= L) {
        // Nothing to attend in this unit.  The merge ignores units behind L; with a
        // single split this block owns the output row of an empty sequence.
        if (a.num_splits == 1 && tid < D) {
            if (a.out_f32) ((float*)a.out)[row * D + tid] = 0.f;
            else ((half_t*)a.out)[row * D + tid] = (half_t)0.f;
            if (a.lse && tid == 0) a.lse[row] = -__builtin_inff();
        }
        return;
    }
    const int t1 = min(t0 + a.chunk, L);
    const int last = t1 - 1;

    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int r = lane / LPR;              // row inside a wave load
    const int c = lane % LPR;              // 16-byte column of the row

    // q stays in registers as fp16 pairs; the softmax scale is applied in fp32.
    const half8_t q8 = *(const half8_t*)(a.q + row * D + c * 8);

    const char* kp = (const char*)a.kv.k;
    const char* vp = (const char*)a.kv.v;
    const uint32_t row_bytes = (uint32_t)a.kv.stride_t * 2u;
    const int64_t head_off = (int64_t)hk * a.kv.stride_h;
    const int32_t* table = PAGED ? a.kv.page_table + (int64_t)b * a.kv.max_pages : nullptr;

    const int n_it = (t1 - t0 + TILE - 1) / TILE;
    // Tile visited in iteration `it`: in order, or (a.rotate) from a start of the unit's
    // own and round; iterations behind the end stay behind it.
    const int rot = a.rotate ? (int)((((uint32_t)row * 0x9E3779B1u) >> 16) % (uint32_t)n_it) : 0;
    auto tile_of = [&](int it) { return it < n_it ? (it + rot < n_it ? it + rot : it + rot - n_it) : it; };
    // First row this wave touches in iteration `it`, pulled back into the unit.
    auto wave_row = [&](int it) { return min(t0 + tile_of(it) * TILE + wave * WTILE, last); };
    // Pool page (paged) of that row; fetched one iteration ahead of its use.
    auto page_of = [&](int tw) { return PAGED ? table[tw >> a.kv.page_shift] : b; };

    auto load_tile = [&](MhaTile<U>& T, int it, int page) {
        const int tw = wave_row(it);                         // wave-uniform
        const int in_page = PAGED ? (tw & a.kv.page_mask) : tw;
        if constexpr (PAGED) page = pool_page_valu(page, a.kv.last_page);   // here, not at the fetch: the id stays in flight until now
        const int64_t tile_off =
            2 * ((int64_t)page * a.kv.stride_b + head_off + (int64_t)in_page * a.kv.stride_t);
        const int first = t0 + tile_of(it) * TILE + wave * WTILE + r;  // this lane's row for j = 0
#pragma unroll
        for (int j = 0; j < U; ++j) {
            // rows behind the unit's end are redirected to its last row
            const uint32_t lane_off = (uint32_t)(min(first + j * RPW, last) - tw) * row_bytes + c * 16;
            T.k[j] = load16(kp + tile_off, lane_off);
            T.v[j] = load16(vp + tile_off, lane_off);
        }
    };

    float m = kNegBig, l = 0.f;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;

    auto consume = [&](const MhaTile<U>& T, int it) {
        const int first = t0 + tile_of(it) * TILE + wave * WTILE + r;
        float s[U];
        float mx = m;
#pragma unroll
        for (int j = 0; j < U; ++j) {
            float d = dot8(__builtin_bit_cast(half8_t, T.k[j]), q8, 0.f);
            d = group_sum<LPR>(d);
            s[j] = (first + j * RPW < t1) ? d * a.scale_log2 : -__builtin_inff();
            mx = fmaxf(mx, s[j]);
        }
        const float alpha = fast_exp2(m - mx);
        m = mx;
        l *= alpha;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= alpha;
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const float p = fast_exp2(s[j] - mx);
            l += p;
            const half8_t vh = __builtin_bit_cast(half8_t, T.v[j]);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = __builtin_fmaf((float)vh[e], p, acc[e]);
        }
    };

    // Two register tiles: tile i+1 is in flight while tile i is consumed; the page
    // id of tile i+2 is in flight behind it.
    MhaTile<U> A, B;
    int page_a = page_of(wave_row(0));
    int page_b = page_of(wave_row(1));
    load_tile(A, 0, page_a);
    for (int it = 0; it < n_it; it += 2) {
        page_a = page_of(wave_row(it + 2));
        load_tile(B, it + 1, page_b);
        pin_order();
        consume(A, it);
        page_b = page_of(wave_row(it + 3));
        load_tile(A, it + 2, page_a);
        pin_order();
        if (it + 1 < n_it) consume(B, it + 1);
    }

    // Combine the NG streams of this block.
    __shared__ float s_acc[NG][D];
    __shared__ float s_m[NG];
    __shared__ float s_l[NG];
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
#pragma unroll
        for (int i = 0; i < NG; ++i) M = fmaxf(M, s_m[i]);
        float lsum = 0.f, o = 0.f;
#pragma unroll
        for (int i = 0; i < NG; ++i) {
            const float w = fast_exp2(s_m[i] - M);
            lsum += w * s_l[i];
            o += w * s_acc[i][tid];
        }
        o /= lsum;
        const float lse2 = M + fast_log2(lsum);
        if (a.num_splits == 1) {
            if (a.out_f32) ((float*)a.out)[row * D + tid] = o;
            else ((half_t*)a.out)[row * D + tid] = (half_t)o;
            if (a.lse && tid == 0) a.lse[row] = lse2 * kLn2;
        } else {
            const int64_t u = row * a.num_splits + split;
            a.o_part[u * D + tid] = o;
            if (tid == 0) a.lse_part[u] = lse2;
        }
    }
}

template <int D>
static hipError_t launch_mha(const DecodeArgs& a, int batch, hipStream_t stream)
{
    // blockIdx.x walks the heads: consecutive blocks go round-robin over the XCDs, so every
    // XCD gets the same mix of units whatever the sequence lengths are
    const dim3 grid = a.unit_list ? dim3(a.num_q_heads, a.list_len, 1) : dim3(a.num_q_heads, a.num_splits, batch);
    if (a.kv.page_table)
        hipLaunchKernelGGL((decode_mha_kernel<D, true>), grid, dim3(INSTATTN_MHA_WAVES * 64), 0, stream, a);
    else
        hipLaunchKernelGGL((decode_mha_kernel<D, false>), grid, dim3(INSTATTN_MHA_WAVES * 64), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_decode_mha(const DecodeArgs& a, int batch, int head_dim, hipStream_t stream)
{
    if (head_dim == 128) return launch_mha<128>(a, batch, stream);
    return launch_mha<64>(a, batch, stream);
}

}  // namespace instattn
