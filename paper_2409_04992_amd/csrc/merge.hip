// Log-sum-exp merge of the split pass's units, the KV append, and two
// measurement kernels.
#include "common.h"

namespace instattn {

// One block per (b, h), one thread per output dim.  Unit i of a row holds the
// attention over positions [i*chunk, (i+1)*chunk) and 2^lse_i = sum of exp(score)
// there, so the whole row is sum_i 2^lse_i o_i / sum_i 2^lse_i.  Only the
// ceil(L_b / chunk) units that contain positions are read.
template <int D>
__global__ __launch_bounds__(D) void merge_kernel(MergeArgs a)
{
    const int h = blockIdx.x, b = blockIdx.y, d = threadIdx.x;
    const int64_t row = (int64_t)b * a.num_q_heads + h;
    const int L = clamp_len(a.seq_lens[b], a.max_len);
    const int n = (L + a.chunk - 1) / a.chunk;
    const float* lp = a.lse_part + row * a.num_splits;
    const float* op = a.o_part + row * a.num_splits * D + d;
    float o = 0.f, lse = -__builtin_inff();
    if (n > 0) {
        float M = lp[0];
        for (int i = 1; i < n; ++i) M = fmaxf(M, lp[i]);
        float wsum = 0.f;
        for (int i = 0; i < n; ++i) {
            const float w = fast_exp2(lp[i] - M);
            wsum += w;
            o += w * op[(int64_t)i * D];
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
    if (head_dim == 128) hipLaunchKernelGGL(merge_kernel<128>, grid, dim3(128), 0, stream, a);
    else hipLaunchKernelGGL(merge_kernel<64>, grid, dim3(64), 0, stream, a);
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
        const int page = a.page_table[(int64_t)b * a.max_pages + (t >> a.page_shift)];
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

hipError_t launch_probe_read(const void* src, size_t bytes, void* sink, hipStream_t stream)
{
    const size_t nseg = (bytes / 16 + kProbeSeg16 - 1) / kProbeSeg16;
    const unsigned blocks = (unsigned)(nseg < 65536 ? nseg : 65536);
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
