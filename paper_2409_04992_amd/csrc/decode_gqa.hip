// Split pass of decode attention for grouped queries on the matrix cores
// (head_dim 64 or 128; up to 16 query heads of a KV head per block, a larger group
// takes one block per 16 of its heads).
//
// Paper: Sec. II-A/II-B give the operation; the paper's engine runs one query
// head per K/V stream.  With G query heads sharing a KV head every fp16 loaded
// feeds G multiply-adds, which is more than the vector ALUs sustain at HBM speed,
// while the two products become small dense contractions:
//     S^T [16 rows x 16 heads] = K_tile [16 x D] . Q^T [D x 16]
//     O^T [D dims x 16 heads] += V_tile^T [D x 32] . P^T [32 x 16]
// done with v_mfma_f32_16x16x32_f16 (heads padded to 16 with zero queries).
// The comments below give the numbers for D = 128; for D = 64 a lane moves 8 bytes
// of a row instead of 16 (a row is still read by 16 adjacent lanes), the first
// product takes 2 instructions per 16 rows instead of 4 and the second 4 per 32
// rows instead of 8.
//
// Operand layouts of that instruction (lane l, g = l / 16, c = l % 16):
//     A[i][k]: i = c, k = 8g .. 8g+7      B[k][j]: j = c, k = 8g .. 8g+7
//     C[i][j]: j = c, i = 4g + r  (r = 0..3)
//
// Data movement per wave and iteration (32 rows of K and of V, 16 KB):
//   * Global loads are 128-bit and row-contiguous: lane (g, c) reads bytes
//     [16c, 16c+16) of row  base + 16m + 4x + g  (m = 0,1; x = 0..3), so one wave
//     load covers four consecutive rows (1 KB).  K and V use the same offsets.
//   * K goes through a wave-private LDS tile (row stride 272 B, conflict-free
//     128-bit reads): the row loaded as (m, x) by lane group g is stored as LDS
//     row 16m + 4g + x, and read back as the A operand, so that the score a lane
//     gets in C register r of sub-tile m belongs to row 16m + 4r + g -- exactly
//     the rows whose V it loaded.
//   * V never touches LDS.  A lane holds 8 rows x 8 dims of V; contraction slot
//     8g + 4m + r of the second product is defined to be "the row this lane group
//     loaded as (m, r)", so the A operand V^T for output dims {8c + e} is an
//     in-lane 8x8 transpose of fp16 values, and the softmax weights the lane
//     already holds are the B operand as they are.
//   * Softmax statistics are per head = per lane column c: the running maximum
//     is agreed across the four lane groups with two cross-lane exchanges per
//     tile; the running sum stays a per-lane partial until the unit ends.
//   * Weights enter the matrix core as fp16.  When fp32 output is requested a
//     second product with the fp16 remainder of each weight restores fp32
//     accuracy.
#include "common.h"

namespace instattn {

namespace {

constexpr int kGqWaves = 4;
constexpr int kGqWaveRows = 32;                   // rows per wave per iteration
constexpr int kGqTile = kGqWaves * kGqWaveRows;   // rows per block per iteration

// Per head_dim: a lane holds EL = D/16 fp16 of a row (one 16- or 8-byte load).
template <int D>
struct GqTraits {
    static constexpr int EL = D / 16;                 // fp16 per lane and row; also MFMAs of the second product
    static constexpr int KK = D / 32;                 // MFMAs of the first product per 16 rows
    static constexpr int kLaneBytes = 2 * EL;
    static constexpr int kRowBytes = 2 * D + 16;      // padded LDS row: conflict-free A-operand reads
    static constexpr int kWaveLds = kGqWaveRows * kRowBytes;
    static constexpr int kLds = kGqWaves * kWaveLds;  // 34816 B (D = 128), 18432 B (D = 64)
    typedef _Float16 vec_t __attribute__((ext_vector_type(EL)));
};

template <int D>
struct GqaTile {
    typename GqTraits<D>::vec_t k[8];   // index 4m + x
    typename GqTraits<D>::vec_t v[8];
};

// One lane's share of a row.  A row that one block alone reads carries the non-temporal
// hint (measured +10 %); KEEP: several blocks of the XCD read it (a group of more than
// 16 query heads), so it should stay in the L2 for the ones behind the first.
template <int D, bool KEEP>
__device__ __forceinline__ typename GqTraits<D>::vec_t gq_load(const char* base, uint32_t lane_off) {
    typedef typename GqTraits<D>::vec_t vec_t;
    if constexpr (KEEP) return *(const vec_t*)(base + (uint64_t)lane_off);
    else return __builtin_nontemporal_load((const vec_t*)(base + (uint64_t)lane_off));
}

__device__ __forceinline__ float xor_lanes(float x, int mask) {
    return __shfl_xor(x, mask, 64);
}

// Orders this wave's LDS stores before its following LDS loads (and the reverse)
// for the compiler; the hardware executes one wave's LDS operations in order.
__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace

template <int D, bool PAGED, bool SPLIT_P, bool KEEP>
__global__ __launch_bounds__(256, 2) void decode_gqa_kernel(DecodeArgs a)
{
    typedef GqTraits<D> TR;
    typedef typename TR::vec_t vec_t;
    constexpr int EL = TR::EL, KK = TR::KK;
    // blockIdx.x walks KV heads: consecutive blocks go round-robin over the XCDs,
    // so every XCD gets the same mix of units whatever the lengths are.
    // A group of more than 16 query heads is shared out over group_blocks blocks, 16 heads
    // each (the last one the rest): every one of them streams the KV head again.
    // Those blocks of a unit are 8 apart in a one-dimensional grid: same XCD, dispatched
    // together, so that the passes behind the first find the rows in that XCD's L2.
    int split, b, hk, sub = 0;
    if (!unit_of_block(a, a.num_kv_heads, b, split, hk)) return;   // block-uniform
    if (a.group_blocks > 1) {
        const int span = 8 * a.group_blocks;
        const int chunk = (int)blockIdx.x / span, within = (int)blockIdx.x - chunk * span;
        sub = within >> 3;
        const int u = chunk * 8 + (within & 7);              // unit: KV head fastest, then split, then sequence
        if (u >= a.units) return;                            // block-uniform: the grid is rounded up
        hk = u % a.num_kv_heads;
        const int rest = u / a.num_kv_heads;
        split = rest % a.num_splits;
        b = rest / a.num_splits;
    }
    const int group = a.num_q_heads / a.num_kv_heads;
    const int G = min(16, group - 16 * sub);                 // query heads of this block
    const int L = clamp_len(a.seq_lens[b], a.max_len);
    const int t0 = split * a.chunk;
    const int tid = threadIdx.x;
    const int64_t row0 = (int64_t)b * a.num_q_heads + (int64_t)hk * group + 16 * sub;   // first query head of the block

    fused_append<D>(a, b, hk, split, tid);

    if (t0 >= L) {
        if (a.num_splits == 1) {
            for (int i = tid; i < G * D; i += 256) {
                if (a.out_f32) ((float*)a.out)[row0 * D + i] = 0.f;
                else ((half_t*)a.out)[row0 * D + i] = (half_t)0.f;
            }
            if (a.lse && tid < G) a.lse[row0 + tid] = -__builtin_inff();
        }
        return;
    }
    const int t1 = min(t0 + a.chunk, L);
    const int last = t1 - 1;

    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int g = lane >> 4;
    const int c = lane & 15;

    __shared__ __align__(16) char lds[TR::kLds];
    char* my_lds = lds + wave * TR::kWaveLds;

    // Q^T as B operand of the first product: head c, dims 32kk + 8g .. +7.
    half8_t qb[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        half8_t z = {0, 0, 0, 0, 0, 0, 0, 0};
        qb[kk] = c < G ? *(const half8_t*)(a.q + (row0 + c) * D + kk * 32 + g * 8) : z;
    }

    const char* kp = (const char*)a.kv.k;
    const char* vp = (const char*)a.kv.v;
    const uint32_t row_bytes = (uint32_t)a.kv.stride_t * 2u;
    const int64_t head_off = (int64_t)hk * a.kv.stride_h;
    const int32_t* table = PAGED ? a.kv.page_table + (int64_t)b * a.kv.max_pages : nullptr;

    const int n_it = (t1 - t0 + kGqTile - 1) / kGqTile;
    // Tile visited in iteration `it`: in order, or (a.rotate) from a start of the unit's
    // own and round; iterations behind the end stay behind it.
    const int rot =
        a.rotate ? (int)((((uint32_t)(b * a.num_kv_heads + hk) * 0x9E3779B1u) >> 16) % (uint32_t)n_it) : 0;
    auto tile_of = [&](int it) { return it < n_it ? (it + rot < n_it ? it + rot : it + rot - n_it) : it; };
    // First row of sub-tile m of this wave in iteration `it`, pulled back into the unit.
    auto sub_row = [&](int it, int m) {
        return min(t0 + tile_of(it) * kGqTile + wave * kGqWaveRows + 16 * m, last);
    };
    auto page_of = [&](int t) { return PAGED ? table[t >> a.kv.page_shift] : b; };

    auto load_tile = [&](GqaTile<D>& T, int it, int page0, int page1) {
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const int tm = sub_row(it, m);                      // wave-uniform
            const int in_page = PAGED ? (tm & a.kv.page_mask) : tm;
            const int page = PAGED ? pool_page_valu(m == 0 ? page0 : page1, a.kv.last_page) : b;
            const int64_t base =
                2 * ((int64_t)page * a.kv.stride_b + head_off + (int64_t)in_page * a.kv.stride_t);
            const int first = t0 + tile_of(it) * kGqTile + wave * kGqWaveRows + 16 * m + g;
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                // rows behind the unit's end are redirected to its last row
                const uint32_t off = (uint32_t)(min(first + 4 * x, last) - tm) * row_bytes + c * TR::kLaneBytes;
                T.k[4 * m + x] = gq_load<D, KEEP>(kp + base, off);
                T.v[4 * m + x] = gq_load<D, KEEP>(vp + base, off);
            }
        }
    };

    float m_run = kNegBig, l_run = 0.f;
    float4_t acc[EL];
#pragma unroll
    for (int e = 0; e < EL; ++e) acc[e] = float4_t{0.f, 0.f, 0.f, 0.f};

    auto consume = [&](const GqaTile<D>& T, int it) {
        // K tile -> LDS: the row loaded as (m, x) by group g becomes LDS row 16m + 4g + x.
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int lrow = 16 * (i >> 2) + 4 * g + (i & 3);
            *(vec_t*)(my_lds + lrow * TR::kRowBytes + c * TR::kLaneBytes) = T.k[i];
        }
        wave_lds_fence();
        float4_t s[2];
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            s[m] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const half8_t ka =
                    *(const half8_t*)(my_lds + (16 * m + c) * TR::kRowBytes + kk * 64 + g * 16);
                s[m] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka, qb[kk], s[m], 0, 0, 0);
            }
        }
        wave_lds_fence();

        // Scores of head c for rows first + 16m + 4r (slot 4m + r).
        const int first = t0 + tile_of(it) * kGqTile + wave * kGqWaveRows + g;
        float sc[8];
        float mx = -__builtin_inff();
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int t = first + 16 * (i >> 2) + 4 * (i & 3);
            sc[i] = t < t1 ? s[i >> 2][i & 3] * a.scale_log2 : -__builtin_inff();
            mx = fmaxf(mx, sc[i]);
        }
        mx = fmaxf(mx, xor_lanes(mx, 16));
        mx = fmaxf(mx, xor_lanes(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = fast_exp2(m_run - m_new);
        m_run = m_new;

        half8_t p_hi, p_lo = {0, 0, 0, 0, 0, 0, 0, 0};
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float p = fast_exp2(sc[i] - m_new);
            p_hi[i] = (half_t)p;
            if (SPLIT_P) {
                p_lo[i] = (half_t)(p - (float)p_hi[i]);
                psum += p;
            } else {
                psum += (float)p_hi[i];     // normalise by the weights actually used
            }
        }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int e = 0; e < EL; ++e) acc[e] *= alpha;

        // V^T operand for output dims EL*c + e: element e of each of the 8 rows held.
#pragma unroll
        for (int e = 0; e < EL; ++e) {
            const half8_t va = {T.v[0][e], T.v[1][e], T.v[2][e], T.v[3][e],
                                T.v[4][e], T.v[5][e], T.v[6][e], T.v[7][e]};
            acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va, p_hi, acc[e], 0, 0, 0);
            if (SPLIT_P) acc[e] = __builtin_amdgcn_mfma_f32_16x16x32_f16(va, p_lo, acc[e], 0, 0, 0);
        }
    };

    GqaTile<D> A, B;
    int pa0 = page_of(sub_row(0, 0)), pa1 = page_of(sub_row(0, 1));
    int pb0 = page_of(sub_row(1, 0)), pb1 = page_of(sub_row(1, 1));
    load_tile(A, 0, pa0, pa1);
    for (int it = 0; it < n_it; it += 2) {
        pa0 = page_of(sub_row(it + 2, 0));
        pa1 = page_of(sub_row(it + 2, 1));
        load_tile(B, it + 1, pb0, pb1);
        pin_order();
        consume(A, it);
        pb0 = page_of(sub_row(it + 3, 0));
        pb1 = page_of(sub_row(it + 3, 1));
        load_tile(A, it + 2, pa0, pa1);
        pin_order();
        if (it + 1 < n_it) consume(B, it + 1);
    }

    // Unit result: combine the four waves through LDS (the K tiles are dead now).
    l_run += xor_lanes(l_run, 16);
    l_run += xor_lanes(l_run, 32);
    __syncthreads();
    float* s_o = (float*)lds;                       // [wave][G][D]
    float* s_m = s_o + kGqWaves * G * D;            // [wave][16]
    float* s_l = s_m + kGqWaves * 16;               // [wave][16]
    if (c < G) {
        // register r of product e holds output dim EL * (4g + r) + e of head c
        float* dst = s_o + ((int64_t)wave * G + c) * D + 4 * EL * g;
#pragma unroll
        for (int e = 0; e < EL; ++e)
#pragma unroll
            for (int r = 0; r < 4; ++r) dst[EL * r + e] = acc[e][r];
        if (g == 0) {
            s_m[wave * 16 + c] = m_run;
            s_l[wave * 16 + c] = l_run;
        }
    }
    __syncthreads();
    for (int i = tid; i < G * D; i += 256) {
        const int head = i / D, d = i % D;
        float M = kNegBig;
#pragma unroll
        for (int w = 0; w < kGqWaves; ++w) M = fmaxf(M, s_m[w * 16 + head]);
        float lsum = 0.f, o = 0.f;
#pragma unroll
        for (int w = 0; w < kGqWaves; ++w) {
            const float wgt = fast_exp2(s_m[w * 16 + head] - M);
            lsum += wgt * s_l[w * 16 + head];
            o += wgt * s_o[((int64_t)w * G + head) * D + d];
        }
        o /= lsum;
        const float lse2 = M + fast_log2(lsum);
        const int64_t row = row0 + head;
        if (a.num_splits == 1) {
            if (a.out_f32) ((float*)a.out)[row * D + d] = o;
            else ((half_t*)a.out)[row * D + d] = (half_t)o;
            if (a.lse && d == 0) a.lse[row] = lse2 * kLn2;
        } else {
            const int64_t u = row * a.num_splits + split;
            a.o_part[u * D + d] = o;
            if (d == 0) a.lse_part[u] = lse2;
        }
    }
}

template <int D>
static hipError_t launch_gqa(const DecodeArgs& args, int batch, hipStream_t stream)
{
    DecodeArgs a = args;
    dim3 grid(a.num_kv_heads, a.num_splits, batch);
    if (a.unit_list) grid = dim3((unsigned)((a.list_len + 7) / 8 * 8 * a.num_kv_heads), 1, 1);   // see unit_of_block
    if (a.group_blocks > 1) {
        a.units = a.num_kv_heads * a.num_splits * batch;
        grid = dim3((unsigned)((a.units + 7) / 8 * 8 * a.group_blocks), 1, 1);
    }
    const bool paged = a.kv.page_table != nullptr, keep = a.group_blocks > 1;
#define INSTATTN_GQA(P, S, K) hipLaunchKernelGGL((decode_gqa_kernel<D, P, S, K>), grid, dim3(256), 0, stream, a)
    if (keep) {
        if (a.out_f32) { if (paged) INSTATTN_GQA(true, true, true); else INSTATTN_GQA(false, true, true); }
        else { if (paged) INSTATTN_GQA(true, false, true); else INSTATTN_GQA(false, false, true); }
    } else {
        if (a.out_f32) { if (paged) INSTATTN_GQA(true, true, false); else INSTATTN_GQA(false, true, false); }
        else { if (paged) INSTATTN_GQA(true, false, false); else INSTATTN_GQA(false, false, false); }
    }
#undef INSTATTN_GQA
    return hipGetLastError();
}

hipError_t launch_decode_gqa(const DecodeArgs& a, int batch, int head_dim, hipStream_t stream)
{
    return head_dim == 128 ? launch_gqa<128>(a, batch, stream) : launch_gqa<64>(a, batch, stream);
}

}  // namespace instattn
