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
//   * Tiles are staged through LDS: every wave owns a ring of STAGES tiles (16 rows
//     of K and of V each) that direct-to-LDS loads (global_load_lds_dwordx4) fill
//     without holding a register while they are in flight; the wave reads a stage
//     back with ds_read_b128 when its turn comes and requests the next tile into
//     the stage it has just emptied, so STAGES tiles are always in flight behind
//     the one being consumed.  A wave touches only its own ring: no barrier in the
//     loop, only the wave's own load counter.  One block of four waves per compute
//     unit.  The other form of the kernel (STAGES = 0) holds two tiles in registers
//     instead and runs five blocks per compute unit; measured on the same caches in
//     one process the ring is ahead on large launches (+0.7 % on 16 x 40 heads x 4K,
//     +1.3 % on 8 x 40 x 32K at equal unit length and +2.5 % with the longer units it
//     allows, +1 % at head_dim 64) and behind on small ones, where 256 block slots
//     are too few for short units (4 x 40 heads x 1.5K: -10 %), so the host picks
//     the form by the size of the launch.
//   * q.K: four v_dot2_f32_f16 per lane, then a DPP butterfly inside the 8- or
//     16-lane row group (no LDS).
//   * Every row group runs its own online softmax (running max m, sum l, fp32
//     accumulator of its 8 output dims) over the rows it reads, so the loop has
//     no communication between groups; groups are combined once per unit in LDS
//     (in the ring's memory, dead by then).
//   * Positions at or behind the unit's end are redirected to its last valid row
//     (a cache hit) and their score is set to -inf, so rows behind the sequence
//     length are never read and every iteration issues the same number of loads
//     (the count of loads in flight is known at every wait).
//   * Paged caches: the page id of a tile is fetched two iterations ahead with a
//     SCALAR load.  Vector loads return in order, so a page id fetched with one
//     would arrive behind every tile requested before it and the ring could never
//     be more than one tile deep.
#include "common.h"

// Compile-time knobs (defaults are the measured best).
#ifndef INSTATTN_MHA_LDS_STAGES
#define INSTATTN_MHA_LDS_STAGES 3   // tiles per wave in the LDS ring (2: -1 %, 4 and 5: level)
#endif
#ifndef INSTATTN_MHA_NT
#define INSTATTN_MHA_NT 1           // 1: KV loads carry the non-temporal hint (without it: -10 %)
#endif
#ifndef INSTATTN_MHA_WAVES
#define INSTATTN_MHA_WAVES 4        // waves per block (2: -1 to -7 %, 6: -0.5 %, 8 with two stages: -1.5 %)
#endif
#ifndef INSTATTN_MHA_WTILE
#define INSTATTN_MHA_WTILE 16       // rows per wave per iteration, contiguous layout (paged: always 16; 8: -1 %)
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

template <int D, bool PAGED, int STAGES>
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

    // One LDS buffer: the staged form's ring of tiles while the unit is walked, then (both
    // forms) the partial sums of the block's streams.
    constexpr int kSumBytes = (NG * D + 2 * NG) * (int)sizeof(float);
    constexpr int kRingBytes = WAVES * STAGES * 2 * U * 1024;
    __shared__ __align__(16) char s_lds[kRingBytes > kSumBytes ? kRingBytes : kSumBytes];

    int split, b, h;
    if (!unit_of_block(a, a.num_q_heads, b, split, h)) return;       // block-uniform
    const int G = a.num_q_heads / a.num_kv_heads;
    const int hk = h / G;
    const int L = clamp_len(a.seq_lens[b], a.max_len);
    const int t0 = split * a.chunk;
    const int tid = threadIdx.x;
    const int64_t row = (int64_t)b * a.num_q_heads + h;

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
    half8_t q8 = *(const half8_t*)(a.q + row * D + c * 8);
    // q arrives before the first tile is requested: the wait for it then does not wait for the tiles
    if constexpr (STAGES > 0) asm volatile("" : "+v"(q8));

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

    if constexpr (STAGES > 0) {
        // Stage s of a wave holds one tile: U wave loads of K (1 KB each, the 16 bytes of lane i
        // at byte 16 i) and U of V.  Every iteration issues one full stage (tiles behind the end
        // are pulled back to the last row), which keeps the count of loads in flight known.
        constexpr int STAGE_BYTES = 2 * U * 1024;
        static_assert(U == 4 || U == 2 || U == 1, "the ds_read sequences below are written for 1, 2 or 4 loads per tensor");
        char (*s_ring)[STAGES][STAGE_BYTES] = (char (*)[STAGES][STAGE_BYTES])s_lds;
        typedef __attribute__((address_space(3))) char lds_char;
        typedef const __attribute__((address_space(1))) char glb_char;
        // Pool page of iteration `it` (paged): a scalar load through the constant address
        // space, so that it is counted apart from the vector loads of the stages (vector loads
        // return in order: a page id fetched with one would arrive behind every stage
        // requested before it, and the ring would never be more than one stage deep).
        typedef const __attribute__((address_space(4))) int32_t const_i32;
        auto page_of_s = [&](int it) { return PAGED ? *(const_i32*)(table + (wave_row(it) >> a.kv.page_shift)) : b; };
        auto issue = [&](int st, int it, int page) {
            const int tw = wave_row(it);
            const int in_page = PAGED ? (tw & a.kv.page_mask) : tw;
            if constexpr (PAGED) page = pool_page(page, a.kv.last_page);
            const int64_t tile_off = 2 * ((int64_t)page * a.kv.stride_b + head_off + (int64_t)in_page * a.kv.stride_t);
            const int first = t0 + tile_of(it) * TILE + wave * WTILE + r;
            lds_char* dst = (lds_char*)&s_ring[wave][st][0];
#pragma unroll
            for (int j = 0; j < U; ++j) {
                const uint32_t lane_off = (uint32_t)(min(first + j * RPW, last) - tw) * row_bytes + c * 16;
                // last argument: cache policy bits of the instruction, 2 = non-temporal
                __builtin_amdgcn_global_load_lds((glb_char*)(kp + tile_off + lane_off), dst + j * 1024, 16, 0,
                                                 INSTATTN_MHA_NT ? 2 : 0);
                __builtin_amdgcn_global_load_lds((glb_char*)(vp + tile_off + lane_off), dst + (U + j) * 1024, 16, 0,
                                                 INSTATTN_MHA_NT ? 2 : 0);
            }
        };
        // Reads a stage back once its loads have landed: the wait allows exactly the loads of
        // the STAGES - 1 younger tiles to be outstanding.  The compiler does not see these LDS
        // reads as depending on the direct-to-LDS loads, so wait, reads and the wait for the
        // reads are one block of instructions.
        auto fetch = [&](MhaTile<U>& T, int st) {
            const uint32_t addr = (uint32_t)(uintptr_t)(lds_char*)&s_ring[wave][st][0] + lane * 16;
            if constexpr (U == 4) {
                asm volatile(
                    "s_waitcnt vmcnt(%9)\n\t"
                    "ds_read_b128 %0, %8\n\t"
                    "ds_read_b128 %1, %8 offset:1024\n\t"
                    "ds_read_b128 %2, %8 offset:2048\n\t"
                    "ds_read_b128 %3, %8 offset:3072\n\t"
                    "ds_read_b128 %4, %8 offset:4096\n\t"
                    "ds_read_b128 %5, %8 offset:5120\n\t"
                    "ds_read_b128 %6, %8 offset:6144\n\t"
                    "ds_read_b128 %7, %8 offset:7168\n\t"
                    "s_waitcnt lgkmcnt(0)"
                    : "=&v"(T.k[0]), "=&v"(T.k[1]), "=&v"(T.k[2]), "=&v"(T.k[3]), "=&v"(T.v[0]), "=&v"(T.v[1]),
                      "=&v"(T.v[2]), "=&v"(T.v[3])
                    : "v"(addr), "n"((STAGES - 1) * 2 * U)
                    : "memory");
            } else if constexpr (U == 2) {
                asm volatile(
                    "s_waitcnt vmcnt(%5)\n\t"
                    "ds_read_b128 %0, %4\n\t"
                    "ds_read_b128 %1, %4 offset:1024\n\t"
                    "ds_read_b128 %2, %4 offset:2048\n\t"
                    "ds_read_b128 %3, %4 offset:3072\n\t"
                    "s_waitcnt lgkmcnt(0)"
                    : "=&v"(T.k[0]), "=&v"(T.k[1]), "=&v"(T.v[0]), "=&v"(T.v[1])
                    : "v"(addr), "n"((STAGES - 1) * 2 * U)
                    : "memory");
            } else {
                asm volatile(
                    "s_waitcnt vmcnt(%3)\n\t"
                    "ds_read_b128 %0, %2\n\t"
                    "ds_read_b128 %1, %2 offset:1024\n\t"
                    "s_waitcnt lgkmcnt(0)"
                    : "=&v"(T.k[0]), "=&v"(T.v[0])
                    : "v"(addr), "n"((STAGES - 1) * 2 * U)
                    : "memory");
            }
        };
        int page_first[STAGES];
#pragma unroll
        for (int p = 0; p < STAGES; ++p) page_first[p] = page_of_s(p);   // all in flight together
#pragma unroll
        for (int p = 0; p < STAGES; ++p) issue(p, p, page_first[p]);
        int st = 0;
        int page_next = page_of_s(STAGES);                    // of the tile the next iteration requests
        for (int it = 0; it < n_it; ++it) {
            MhaTile<U> T;
            fetch(T, st);                                     // leaves the STAGES - 1 younger tiles in flight
            issue(st, it + STAGES, page_next);                // into the stage just read: STAGES tiles in flight again
            page_next = page_of_s(it + STAGES + 1);           // lands while this tile is consumed
            pin_order();
            consume(T, it);
            st = st + 1 == STAGES ? 0 : st + 1;
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // the stages still in flight land before the wave moves on
        __syncthreads();                                      // the ring is dead in every wave: its LDS takes the partial sums
    } else {
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
    }

    // Combine the NG streams of this block.
    float (*s_acc)[D] = (float (*)[D])s_lds;
    float* s_m = (float*)s_lds + NG * D;
    float* s_l = s_m + NG;
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
    dim3 grid(a.num_q_heads, a.num_splits, batch);
    if (a.unit_list) grid = dim3((unsigned)((a.list_len + 7) / 8 * 8 * a.num_q_heads), 1, 1);   // see unit_of_block
    const dim3 block(INSTATTN_MHA_WAVES * 64);
    constexpr int S = INSTATTN_MHA_LDS_STAGES;
    if (a.staged) {
        if (a.kv.page_table) hipLaunchKernelGGL((decode_mha_kernel<D, true, S>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((decode_mha_kernel<D, false, S>), grid, block, 0, stream, a);
    } else {
        if (a.kv.page_table) hipLaunchKernelGGL((decode_mha_kernel<D, true, 0>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((decode_mha_kernel<D, false, 0>), grid, block, 0, stream, a);
    }
    return hipGetLastError();
}

hipError_t launch_decode_mha(const DecodeArgs& a, int batch, int head_dim, hipStream_t stream)
{
    if (head_dim == 128) return launch_mha<128>(a, batch, stream);
    return launch_mha<64>(a, batch, stream);
}

}  // namespace instattn
