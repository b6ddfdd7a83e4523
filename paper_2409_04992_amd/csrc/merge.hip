// Log-sum-exp merge of the split pass's units, the list of units of a ragged batch, the
// KV append, and two measurement kernels.
#include "common.h"

namespace instattn {

// ---------------------------------------------------------------------------
// List of the units that hold rows, for the split pass over a paged cache: of the
// sequences x splits grid only the pairs with rows, the full units first (in sequence
// order), behind them the partly filled ones from long to short (in sixteenths of a
// unit), -1 in the rest of the list (with a single split an empty sequence stays in the
// list, at its end: the pass writes its zero row).  The pass deals the list out over the XCDs in this
// order, has no empty blocks and ends on its shortest units.  One block; wave w places
// class w in order (ballot + popcount), so the same lengths give the same list.
constexpr int kListClasses = 18;        // 0: full, 1..16: partly filled, long to short, 17: no rows
constexpr int kListMaxBatch = 4096;     // sequences whose lengths the block keeps in LDS

__global__ __launch_bounds__(1024) void list_units_kernel(DecodeArgs a, int batch)
{
    __shared__ int s_len[kListMaxBatch];
    __shared__ int s_count[kListClasses];
    __shared__ int s_base[kListClasses + 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, E = a.list_len;
    for (int b = tid; b < batch; b += 1024) s_len[b] = clamp_len(a.seq_lens[b], a.max_len);
    if (tid < kListClasses) s_count[tid] = 0;
    __syncthreads();
    auto klass = [&](int e, int& packed) {
        const int b = e / a.num_splits, split = e - b * a.num_splits;
        packed = b << 16 | split;
        const int rows = min(s_len[b] - split * a.chunk, a.chunk);
        // with a single split the pass itself writes the zero row of an empty sequence: listed, last
        if (rows <= 0) return a.num_splits == 1 ? kListClasses - 2 : kListClasses - 1;
        if (rows == a.chunk) return 0;
        return 16 - (int)((int64_t)rows * 16 / a.chunk);
    };
    int packed;
    for (int e = tid; e < E; e += 1024) atomicAdd(&s_count[klass(e, packed)], 1);
    __syncthreads();
    if (tid == 0) {
        int at = 0;
        for (int c = 0; c < kListClasses; ++c) {
            s_base[c] = at;
            at += s_count[c];
        }
        s_base[kListClasses] = at;
    }
    __syncthreads();
    for (int cls = wave; cls < kListClasses - 1; cls += 16) {
        if (s_count[cls] == 0) continue;                        // wave-uniform
        int pos = s_base[cls];
        for (int e0 = 0; e0 < E; e0 += 64) {
            const int e = e0 + lane;
            const bool mine = e < E && klass(e, packed) == cls;
            const uint64_t m = __ballot(mine);
            if (mine) a.unit_list[pos + __popcll(m & ((1ull << lane) - 1))] = packed;
            pos += __popcll(m);
        }
    }
    for (int e = s_base[kListClasses - 1] + tid; e < E; e += 1024) a.unit_list[e] = -1;
}

hipError_t launch_list_units(const DecodeArgs& a, int batch, hipStream_t stream)
{
    if (batch > kListMaxBatch || a.list_len != batch * a.num_splits) return hipErrorInvalidValue;
    hipLaunchKernelGGL(list_units_kernel, dim3(1), dim3(1024), 0, stream, a, batch);
    return hipGetLastError();
}

// One block per (b, h).  Unit i of a row holds the attention over positions
// [i*chunk, (i+1)*chunk) and 2^lse_i = sum of exp(score) there, so the whole row is
// sum_i 2^lse_i o_i / sum_i 2^lse_i.  Only the ceil(L_b / chunk) units that contain
// positions are read.  GROUPS groups of D threads (one thread per output dim) share
// the units of a row (a long sequence of a small batch has a hundred of them: four
// groups then), four loads in flight each; the groups' sums are added in a fixed
// order.
template <int D, int GROUPS>
__global__ __launch_bounds__(GROUPS * D) void merge_kernel(MergeArgs a)
{
    constexpr int NT = GROUPS * D, NW = NT / 64;
    const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int d = tid % D, g = tid / D;
    const int64_t row = (int64_t)b * a.num_q_heads + h;
    const int L = clamp_len(a.seq_lens[b], a.max_len);
    const int n = (L + a.chunk - 1) / a.chunk;
    const float* lp = a.lse_part + row * a.num_splits;
    const float* op = a.o_part + row * a.num_splits * D + d;
    __shared__ float s_max[NW];
    __shared__ float s_o[GROUPS][D];
    __shared__ float s_w[GROUPS];

    // reference maximum over the units' lse
    float m = -__builtin_inff();
    for (int i = tid; i < n; i += NT) m = fmaxf(m, lp[i]);
#pragma unroll
    for (int sft = 32; sft > 0; sft >>= 1) m = fmaxf(m, __shfl_xor(m, sft, 64));
    if ((tid & 63) == 0) s_max[tid >> 6] = m;
    __syncthreads();
    float M = s_max[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) M = fmaxf(M, s_max[w]);

    float o = 0.f, wsum = 0.f;
    int i = g;
    for (; i + 3 * GROUPS < n; i += 4 * GROUPS) {
        float l4[4], o4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            l4[j] = lp[i + j * GROUPS];
            o4[j] = op[(int64_t)(i + j * GROUPS) * D];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float w = fast_exp2(l4[j] - M);
            wsum += w;
            o += w * o4[j];
        }
    }
    for (; i < n; i += GROUPS) {
        const float w = fast_exp2(lp[i] - M);
        wsum += w;
        o += w * op[(int64_t)i * D];
    }
    s_o[g][d] = o;
    if (d == 0) s_w[g] = wsum;
    __syncthreads();
    if (g != 0) return;
    float lse = -__builtin_inff();
    o = 0.f;
    if (n > 0) {
        wsum = 0.f;
#pragma unroll
        for (int j = 0; j < GROUPS; ++j) {
            o += s_o[j][d];
            wsum += s_w[j];
        }
        o /= wsum;
        lse = (M + fast_log2(wsum)) * kLn2;
    }
    if (a.out_f32) ((float*)a.out)[row * D + d] = o;
    else ((half_t*)a.out)[row * D + d] = (half_t)o;
    if (a.lse && d == 0) a.lse[row] = lse;
}

hipError_t launch_merge(const MergeArgs& a, int batch, int head_dim, hipStream_t stream)
{
    dim3 grid(a.num_q_heads, batch);
    // one group of D threads is enough for a handful of units
    if (a.num_splits <= 16) {
        if (head_dim == 128) hipLaunchKernelGGL((merge_kernel<128, 1>), grid, dim3(128), 0, stream, a);
        else hipLaunchKernelGGL((merge_kernel<64, 1>), grid, dim3(64), 0, stream, a);
    } else {
        if (head_dim == 128) hipLaunchKernelGGL((merge_kernel<128, 4>), grid, dim3(512), 0, stream, a);
        else hipLaunchKernelGGL((merge_kernel<64, 4>), grid, dim3(256), 0, stream, a);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// KV append: one thread moves 16 bytes of k_new and of v_new into row L_b - 1.
__global__ __launch_bounds__(256) void kv_append_kernel(AppendArgs a)
{
    const int cols = a.head_dim / 8;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)a.batch * a.num_kv_heads * cols;
    if (i >= total) return;
    const int c = (int)(i % cols);
    const int hk = (int)((i / cols) % a.num_kv_heads);
    const int b = (int)(i / ((int64_t)cols * a.num_kv_heads));
    const int L = a.seq_lens[b];
    if (L < 1 || L > a.capacity) return;
    const int t = L - 1;
    int64_t off;
    if (a.page_table == nullptr) {
        off = (int64_t)b * a.stride_b + (int64_t)t * a.stride_t;
    } else {
        const int page = pool_page(a.page_table[(int64_t)b * a.max_pages + (t >> a.page_shift)], a.last_page);
        off = (int64_t)page * a.stride_b + (int64_t)(t & a.page_mask) * a.stride_t;
    }
    off += (int64_t)hk * a.stride_h + c * 8;
    const int64_t src = ((int64_t)b * a.num_kv_heads + hk) * a.head_dim + c * 8;
    *(u32x4*)(a.k + off) = *(const u32x4*)(a.k_new + src);
    *(u32x4*)(a.v + off) = *(const u32x4*)(a.v_new + src);
}

hipError_t launch_kv_append(const AppendArgs& a, hipStream_t stream)
{
    const int64_t total = (int64_t)a.batch * a.num_kv_heads * (a.head_dim / 8);
    const int blocks = (int)((total + 255) / 256);
    hipLaunchKernelGGL(kv_append_kernel, dim3(blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Bulk KV write: one thread moves 16 bytes of K and of V; a block covers 16 rows of
// one (sequence, KV head), i.e. one 4 KB page-sized group of each tensor.
__global__ __launch_bounds__(256) void kv_write_kernel(WriteArgs a)
{
    const int cols = a.head_dim / 8;
    const int rows_per_block = 256 / cols;
    const int hk = blockIdx.y, b = blockIdx.z;
    const int i = blockIdx.x * rows_per_block + threadIdx.x / cols;   // row inside the source run
    const int c = threadIdx.x % cols;
    if (i >= a.max_new || i >= a.count[b]) return;
    const int t = a.start[b] + i;
    if (t < 0 || t >= a.kv.capacity) return;
    const int64_t src = (((int64_t)b * a.num_kv_heads + hk) * a.max_new + i) * a.head_dim + c * 8;
    const int64_t dst = row_offset(a.kv, b, hk, t) + c * 8;
    *(u32x4*)(const_cast<half_t*>(a.kv.k) + dst) = __builtin_nontemporal_load((const u32x4*)(a.k_src + src));
    *(u32x4*)(const_cast<half_t*>(a.kv.v) + dst) = __builtin_nontemporal_load((const u32x4*)(a.v_src + src));
}

hipError_t launch_kv_write(const WriteArgs& a, hipStream_t stream)
{
    const int rows_per_block = 256 / (a.head_dim / 8);
    dim3 grid((a.max_new + rows_per_block - 1) / rows_per_block, a.num_kv_heads, a.batch);
    hipLaunchKernelGGL(kv_write_kernel, grid, dim3(256), 0, stream, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Measurement kernels: a pure streaming read and a plain copy.
constexpr int kProbeBlocks = 4096;
constexpr size_t kProbeSeg16 = 16384;   // 16-byte words per block segment (256 KiB)

// Each block streams its own contiguous 256 KiB segments with eight 128-bit
// loads per lane in flight -- the access shape of the attention split pass
// without its arithmetic.
__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4* src, size_t n16, uint32_t* sink)
{
    uint32_t x = 0;
    const size_t nseg = (n16 + kProbeSeg16 - 1) / kProbeSeg16;
    for (size_t seg = blockIdx.x; seg < nseg; seg += gridDim.x) {
        const size_t lo = seg * kProbeSeg16;
        const size_t hi = lo + kProbeSeg16 < n16 ? lo + kProbeSeg16 : n16;
        size_t i = lo + threadIdx.x;
        for (; i + 7 * 256 < hi; i += 8 * 256) {
            u32x4 a[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) a[j] = __builtin_nontemporal_load(src + i + j * 256);
#pragma unroll
            for (int j = 0; j < 8; ++j) x ^= a[j].x ^ a[j].y ^ a[j].z ^ a[j].w;
        }
        for (; i < hi; i += 256) {
            u32x4 a0 = __builtin_nontemporal_load(src + i);
            x ^= a0.x ^ a0.y ^ a0.z ^ a0.w;
        }
    }
    // Fold the wave so that one small store per wave keeps the loads alive.
    for (int s = 32; s > 0; s >>= 1) x ^= __shfl_xor(x, s);
    if ((threadIdx.x & 63) == 0) atomicXor(&sink[blockIdx.x % kProbeBlocks], x);
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const u32x4* src, u32x4* dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        dst[i] = src[i];
}

// A bare read of the addresses the SparF score pass reads: r of the `dims` columns of every
// row of a component-major array (row n at n * row_stride, column d of it d * col_stride
// further on, strides in bytes), the first `positions` fp16 of each (a multiple of 8).  A block takes a row
// and a unit of 2048 positions; a lane reads 16 bytes per column, 8 columns per step, the
// next step's loads in flight while one is folded: the score pass without its arithmetic,
// its ranking and its stores.  Which columns: (7 n + 5 j) mod dims, j < r - spread over the
// row like the columns a query picks.
__global__ __launch_bounds__(256) void probe_columns_kernel(const char* base, size_t row_stride, size_t col_stride,
                                                            int dims, int r, int positions, uint32_t* sink)
{
    constexpr int CG = 8, UNIT = 2048;
    const int n = blockIdx.x, tid = threadIdx.x;
    const int t = min((int)blockIdx.y * UNIT + tid * 8, positions - 8);
    const char* p = base + (size_t)n * row_stride + (size_t)t * 2;
    const int groups = (r + CG - 1) / CG;
    auto load = [&](u32x4 (&T)[CG], int g) {
#pragma unroll
        for (int j = 0; j < CG; ++j) {
            const int col = (7 * n + 5 * min(g * CG + j, r - 1)) % dims;
            T[j] = __builtin_nontemporal_load((const u32x4*)(p + (size_t)col * col_stride));
        }
    };
    uint32_t x = 0;
    u32x4 A[CG], B[CG];
    load(A, 0);
    for (int g = 0; g < groups; g += 2) {
        if (g + 1 < groups) load(B, g + 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < CG; ++j) x ^= A[j].x ^ A[j].y ^ A[j].z ^ A[j].w;
        if (g + 2 < groups) load(A, g + 2);
        __builtin_amdgcn_sched_barrier(0);
        if (g + 1 < groups) {
#pragma unroll
            for (int j = 0; j < CG; ++j) x ^= B[j].x ^ B[j].y ^ B[j].z ^ B[j].w;
        }
    }
    for (int s = 32; s > 0; s >>= 1) x ^= __shfl_xor(x, s);
    if ((tid & 63) == 0) atomicXor(&sink[(blockIdx.x + blockIdx.y) % kProbeBlocks], x);
}

hipError_t launch_probe_columns(const void* base, size_t row_stride, size_t col_stride, int rows, int dims, int r,
                                int positions, void* sink, hipStream_t stream)
{
    const dim3 grid((unsigned)rows, (unsigned)((positions + 2047) / 2048));
    hipLaunchKernelGGL(probe_columns_kernel, grid, dim3(256), 0, stream, (const char*)base, row_stride, col_stride,
                       dims, r, positions, (uint32_t*)sink);
    return hipGetLastError();
}

hipError_t launch_probe_read(const void* src, size_t bytes, void* sink, hipStream_t stream)
{
    const size_t nseg = (bytes / 16 + kProbeSeg16 - 1) / kProbeSeg16;
    // as many blocks as are resident at once (5 per compute unit); each walks its segments
    const unsigned blocks = (unsigned)(nseg < 1280 ? nseg : 1280);
    hipLaunchKernelGGL(probe_read_kernel, dim3(blocks), dim3(256), 0, stream,
                       (const u32x4*)src, bytes / 16, (uint32_t*)sink);
    return hipGetLastError();
}

hipError_t launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t stream)
{
    hipLaunchKernelGGL(probe_copy_kernel, dim3(kProbeBlocks), dim3(256), 0, stream,
                       (const u32x4*)src, (u32x4*)dst, bytes / 16);
    return hipGetLastError();
}

}  // namespace instattn
