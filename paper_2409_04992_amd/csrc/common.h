// Shared device-side declarations of the instattn kernels (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace instattn {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
// Running maxima start at a large finite negative value so that a unit whose
// positions are all masked never forms (-inf) - (-inf).
constexpr float kNegBig = -1.0e30f;

// Geometry of the cached keys/values as the kernels see it (copied from the
// caller's descriptor after validation).
struct KvView {
    const half_t* k;
    const half_t* v;
    const int32_t* page_table;  // nullptr: contiguous
    int64_t stride_b, stride_h, stride_t;
    int32_t capacity;
    int32_t page_shift;         // log2(page_size), paged only
    int32_t page_mask;          // page_size - 1
    int32_t max_pages;
    int32_t last_page;          // num_pages - 1, paged only
};

// Arguments of the split pass (both the vector-ALU and the MFMA kernel).
struct DecodeArgs {
    const half_t* q;            // [B][Hq][D]
    KvView kv;
    const int32_t* seq_lens;    // [B]
    int32_t num_q_heads, num_kv_heads;
    int32_t chunk;              // positions per unit
    int32_t num_splits;
    int32_t max_len;            // min(capacity, max_seq_len)
    float scale_log2;           // scale * log2(e)
    float* o_part;              // [B][Hq][num_splits][D] fp32, normalised rows
    float* lse_part;            // [B][Hq][num_splits]   fp32, log2 domain
    void* out;                  // final rows when num_splits == 1
    float* lse;                 // may be nullptr
    int32_t out_f32;
    // Fused append (both nullptr otherwise): [B][Hkv][D] rows stored at position
    // seq_lens[b] - 1 by the unit that owns that position, before it reads it.
    const half_t* k_new;
    const half_t* v_new;
    // 1: every unit starts its walk over its rows at a tile of its own (and wraps
    // round) instead of at its first row.
    int32_t rotate;
    // MFMA kernel: blocks per KV head and unit; each takes up to 16 of the group's
    // query heads (1 for groups of at most 16).
    int32_t group_blocks;
    int32_t units;              // with group_blocks > 1: KV heads x splits x sequences (the grid is one-dimensional then)
    // Unit list (nullptr: the grid itself spans sequences x splits): entry j is
    // (sequence << 16 | split) of the j-th unit that holds rows, -1 behind the last one;
    // list_len = sequences x splits entries, filled by list_units_kernel in front of the pass;
    // the pass then runs on a one-dimensional grid (unit_of_block).
    int32_t* unit_list;
    int32_t list_len;
    int32_t staged;             // vector-ALU kernel: 1 = tiles through the LDS ring, 0 = two register tiles
};

// Arguments of the log-sum-exp merge.
struct MergeArgs {
    const int32_t* seq_lens;
    const float* o_part;   // [B][Hq][num_splits][D]
    const float* lse_part; // [B][Hq][num_splits], log2 domain
    void* out;
    float* lse;
    int32_t num_q_heads, chunk, num_splits, max_len, out_f32;
};

// Arguments of the KV append.
struct AppendArgs {
    half_t* k;
    half_t* v;
    const int32_t* page_table;
    int64_t stride_b, stride_h, stride_t;
    int32_t capacity, page_shift, page_mask, max_pages, last_page;
    const half_t* k_new;
    const half_t* v_new;
    const int32_t* seq_lens;
    int32_t batch, num_kv_heads, head_dim;
};

// Arguments of the bulk KV write (prefill side): rows start[b] .. start[b]+count[b]-1.
struct WriteArgs {
    KvView kv;
    const half_t* k_src;   // [B][Hkv][max_new][D]
    const half_t* v_src;
    const int32_t* start;
    const int32_t* count;
    int32_t batch, num_kv_heads, head_dim, max_new;
};

// Launchers (one per kernel family); each returns hipGetLastError() of its launch.
hipError_t launch_decode_mha(const DecodeArgs& a, int batch, int head_dim, hipStream_t stream);
hipError_t launch_decode_gqa(const DecodeArgs& a, int batch, int head_dim, hipStream_t stream);
hipError_t launch_list_units(const DecodeArgs& a, int batch, hipStream_t stream);
hipError_t launch_merge(const MergeArgs& a, int batch, int head_dim, hipStream_t stream);
hipError_t launch_kv_append(const AppendArgs& a, hipStream_t stream);
hipError_t launch_kv_write(const WriteArgs& a, hipStream_t stream);
hipError_t launch_probe_read(const void* src, size_t bytes, void* sink, hipStream_t stream);
hipError_t launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t stream);
hipError_t launch_probe_columns(const void* base, size_t row_stride, size_t col_stride, int rows, int dims, int r,
                                int positions, void* sink, hipStream_t stream);

__device__ __forceinline__ int clamp_len(int L, int max_len) {
    L = L < 0 ? 0 : L;
    return L > max_len ? max_len : L;
}

// Which (sequence, split, head) a block of the split pass works on: its grid coordinates,
// or, with the unit list, an entry of the list.  The list's grid is one-dimensional and a
// unit's `heads` blocks are 8 apart in it: consecutive block ids go round-robin over the 8
// XCDs, so the blocks of a unit run on one XCD and walk the same pages of a paged pool
// together (one address translation serves all of them), while the list's order deals the
// units out evenly over the XCDs.  False: no unit (the list's tail).
__device__ __forceinline__ bool unit_of_block(const DecodeArgs& a, int heads, int& b, int& split, int& h) {
    if (a.unit_list == nullptr) {
        h = blockIdx.x;
        split = blockIdx.y;
        b = blockIdx.z;
        return true;
    }
    const uint32_t i = blockIdx.x, s = i >> 3, u = s / (uint32_t)heads;
    const int j = (int)(u * 8 + (i & 7));
    h = (int)(s - u * (uint32_t)heads);
    if (j >= a.list_len) return false;
    const int e = a.unit_list[j];
    b = (int)((uint32_t)e >> 16);
    split = e & 0xFFFF;
    return e >= 0;
}

// A page id as read from a page table: the table lives on the device and cannot be
// checked by the host, so an entry outside [0, num_pages) (a caller's mistake) is read as
// the pool's last page and costs a wrong result, never an access outside the pool.
__device__ __forceinline__ int pool_page(int id, int last_page) {
    return (int)min((uint32_t)id, (uint32_t)last_page);     // one unsigned minimum: a negative id goes to the last page
}

// The same for the split passes, which fetch a wave's page id with a vector load and keep
// the address arithmetic behind it on the vector ALU: the minimum is taken there too.
__device__ __forceinline__ int pool_page_valu(int id, int last_page) {
    int r;
    asm("v_min_u32 %0, %1, %2" : "=v"(r) : "s"(last_page), "v"(id));
    return r;
}

// Element offset of row t of (sequence b, KV head hk).
__device__ __forceinline__ int64_t row_offset(const KvView& kv, int b, int hk, int t) {
    if (kv.page_table == nullptr)
        return (int64_t)b * kv.stride_b + (int64_t)hk * kv.stride_h + (int64_t)t * kv.stride_t;
    const int page = pool_page(kv.page_table[(int64_t)b * kv.max_pages + (t >> kv.page_shift)], kv.last_page);
    return (int64_t)page * kv.stride_b + (int64_t)hk * kv.stride_h +
           (int64_t)(t & kv.page_mask) * kv.stride_t;
}

// Fused append: the unit whose range holds position seq_lens[b] - 1 (the last
// unit if the caller's bound was too small) copies the new K and V rows of KV
// head hk into the cache, 16 bytes per thread, then the whole block synchronises
// so that its own later loads of that row see the new bits.  Exactly one block per
// (b, hk) may call this with owner == true.
template <int D>
__device__ __forceinline__ void fused_append(const DecodeArgs& a, int b, int hk, int split, int tid) {
    if (a.k_new == nullptr) return;
    const int La = a.seq_lens[b];
    if (La < 1 || La > a.kv.capacity) return;
    const int ta = La - 1;
    if (split != min(ta / a.chunk, a.num_splits - 1)) return;   // block-uniform
    constexpr int LPR = D / 8;
    if (tid < 2 * LPR) {
        const int c = tid % LPR;
        const int64_t src = ((int64_t)b * a.num_kv_heads + hk) * D + c * 8;
        const int64_t dst = row_offset(a.kv, b, hk, ta) + c * 8;
        if (tid < LPR) *(u32x4*)(const_cast<half_t*>(a.kv.k) + dst) = *(const u32x4*)(a.k_new + src);
        else *(u32x4*)(const_cast<half_t*>(a.kv.v) + dst) = *(const u32x4*)(a.v_new + src);
    }
    __syncthreads();
}

// Cross-lane exchange inside a row of 16 lanes with DPP (no LDS traffic).
template <int Ctrl>
__device__ __forceinline__ float dpp_f32(float x) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), Ctrl, 0xF, 0xF, true));
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i within 8
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i within 16

// Sum over groups of `Lanes` (8 or 16) adjacent lanes; every lane gets the total.
template <int Lanes>
__device__ __forceinline__ float group_sum(float x) {
    x += dpp_f32<kDppXor1>(x);
    x += dpp_f32<kDppXor2>(x);
    x += dpp_f32<kDppHalfMirror>(x);
    if (Lanes == 16) x += dpp_f32<kDppMirror>(x);
    return x;
}

// fp32 dot product of 8 fp16 pairs (v_dot2_f32_f16: exact products, fp32 sums).
// Pairs are taken with shufflevector: bit-casting a single element of a vector
// lvalue reads element 0 with this compiler.
__device__ __forceinline__ float dot8(half8_t a, half8_t b, float acc) {
    acc = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 0, 1), __builtin_shufflevector(b, b, 0, 1), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 2, 3), __builtin_shufflevector(b, b, 2, 3), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 4, 5), __builtin_shufflevector(b, b, 4, 5), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_shufflevector(a, a, 6, 7), __builtin_shufflevector(b, b, 6, 7), acc, false);
    return acc;
}

// Keeps the compiler from sinking the loads issued above this point down to
// their uses: they must stay in flight across the arithmetic that follows.
__device__ __forceinline__ void pin_order() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

}  // namespace instattn
