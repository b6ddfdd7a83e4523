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
//                         2048 positions of one query head; reads the component-
//                         major K copy, writes fp32 scores (log2 domain) and the
//                         block's max / sum.
//   sparf_select_kernel   steps 4 (normaliser), 5-7: one block per query head; an
//                         exact radix select over the scores, ordered compaction
//                         (ties towards the lower position), alpha.
//   sparf_attend_kernel   steps 10-11: one block per query head gathers the
//                         selected rows of K and V (online softmax as in the dense
//                         vector-ALU kernel) and blends with the mean of V.
//   sparf_build_kernel    builds the component-major K copy and the running sum
//                         of V from an existing cache (prefill side).
//   sparf_append_kernel   kv_append plus the new column entry and sum update.
#include "sparf.h"

namespace instattn {

namespace {

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) x = fmaxf(x, __shfl_xor(x, s, 64));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) x += __shfl_xor(x, s, 64);
    return x;
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

}  // namespace

// ---------------------------------------------------------------------------
// Steps 1-4 (without the normaliser).
__global__ __launch_bounds__(256) void sparf_logits_kernel(SparfArgs a)
{
    const int h = blockIdx.x, chunk = blockIdx.y, b = blockIdx.z;
    const int D = a.head_dim;
    const int G = a.num_q_heads / a.num_kv_heads;
    const int hk = h / G;
    const int tid = threadIdx.x;
    const int64_t row = (int64_t)b * a.num_q_heads + h;
    const int L = clamp_len(a.seq_lens[b], a.max_len);
    const int t0 = chunk * kSparfChunk;
    float* stats = a.stats + (row * a.nchunk + chunk) * 2;
    if (t0 >= L) {
        if (tid == 0) {
            stats[0] = kNegBig;
            stats[1] = 0.f;
        }
        return;
    }

    __shared__ float s_q[128];
    __shared__ float s_abs[128];
    __shared__ int s_dim[128];       // component with magnitude rank j
    __shared__ float s_red[4];
    if (tid < D) {
        const float qd = (float)a.q[row * D + tid];
        s_q[tid] = qd;
        s_abs[tid] = fabsf(qd);
    }
    __syncthreads();
    // Step 1: rank of |q_d| (larger first, ties towards the lower index).
    if (tid < D) {
        const float mine = s_abs[tid];
        int rank = 0;
        for (int d = 0; d < D; ++d) {
            const float o = s_abs[d];
            rank += (o > mine) || (o == mine && d < tid);
        }
        s_dim[rank] = tid;
    }
    __syncthreads();
    // Step 4 temperature: sqrt(d_h * |q_kept|_1 / |q|_1); 1/sqrt(d_h) is in `scale`.
    float tot = 0.f, kept = 0.f;
    for (int j = 0; j < D; ++j) {
        const float v = s_abs[s_dim[j]];
        tot += v;
        if (j < a.r) kept += v;
    }
    const float rho = tot > 0.f ? kept / tot : 1.f;
    const float factor = rho > 0.f ? a.scale_log2 / sqrtf(rho) : 0.f;

    // Eight consecutive positions per thread, one 128-bit load per kept component.
    const int t = t0 + tid * 8;
    float x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = 0.f;
    if (t < L) {
        const half_t* base = a.aux.kt + (int64_t)b * a.aux.stride_b + (int64_t)hk * a.aux.stride_h + t;
#pragma unroll 8
        for (int j = 0; j < a.r; ++j) {
            const int d = s_dim[j];
            const float qd = s_q[d];
            const half8_t kc = __builtin_nontemporal_load((const half8_t*)(base + (int64_t)d * a.aux.stride_d));
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = __builtin_fmaf(qd, (float)kc[e], x[e]);
        }
    }
    float mx = kNegBig;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        x[e] = (t + e < L) ? x[e] * factor : -__builtin_inff();
        mx = fmaxf(mx, x[e]);
    }
    float* dst = a.logits + row * a.lpad + t;
    *(float4_t*)dst = float4_t{x[0], x[1], x[2], x[3]};
    *(float4_t*)(dst + 4) = float4_t{x[4], x[5], x[6], x[7]};

    const float M = block_max(mx, s_red);
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) s += fast_exp2(x[e] - M);
    s = block_sum(s, s_red);
    if (tid == 0) {
        stats[0] = M;
        stats[1] = s;
    }
}

// ---------------------------------------------------------------------------
// Steps 4 (normaliser) to 7.  NT threads per block: 256 for short rows (more blocks
// per CU, cheaper barriers), 1024 for long ones.
template <int NT>
__global__ __launch_bounds__(NT) void sparf_select_kernel(SparfArgs a)
{
    constexpr int NW = NT / 64;
    const int h = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int64_t row = (int64_t)b * a.num_q_heads + h;
    const int L = clamp_len(a.seq_lens[b], a.max_len);
    if (L == 0) {
        if (tid == 0) a.alpha[row] = 0.f;
        return;
    }
    const int keff = min(a.k, L);
    const int leff = min(a.l, keff);
    const int want = keff - leff;          // rows to pick among the candidates
    const int ncand = L - leff;            // candidates: positions [0, ncand)
    const float* x = a.logits + row * a.lpad;
    int32_t* sel = a.sel + row * a.k;

    __shared__ uint32_t s_hist[256];
    __shared__ uint32_t s_prefix, s_remaining;
    __shared__ uint32_t s_wtot[2][NW];
    __shared__ float s_red[NW];

    // Normaliser of step 4 from the per-block statistics.
    const int nc = (L + kSparfChunk - 1) / kSparfChunk;
    const float* st = a.stats + row * a.nchunk * 2;
    float M = kNegBig;
    for (int c = 0; c < nc; ++c) M = fmaxf(M, st[2 * c]);
    float Z = 0.f;
    for (int c = 0; c < nc; ++c) Z += st[2 * c + 1] * fast_exp2(st[2 * c] - M);

    // Radix select, most significant byte first: after the four passes `prefix` is
    // the key of the want-th largest candidate and `remaining` says how many rows
    // with exactly that key are still to be taken.
    uint32_t prefix = 0, remaining = (uint32_t)want;
    if (want > 0) {
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (tid < 256) s_hist[tid] = 0;
            __syncthreads();
            const uint32_t hi_mask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
            for (int t = tid; t < ncand; t += NT) {
                const uint32_t key = order_key(x[t]);
                if ((key & hi_mask) == (prefix & hi_mask)) atomicAdd(&s_hist[(key >> shift) & 255u], 1u);
            }
            __syncthreads();
            if (wave == 0) {
                // lane i owns bins 4i .. 4i+3; suffix sums over the lanes find the bin
                // that holds the remaining-th largest key
                const uint32_t c0 = s_hist[4 * lane], c1 = s_hist[4 * lane + 1];
                const uint32_t c2 = s_hist[4 * lane + 2], c3 = s_hist[4 * lane + 3];
                const uint32_t mine = c0 + c1 + c2 + c3;
                uint32_t suffix = mine;                       // inclusive, over lanes >= this one
#pragma unroll
                for (int d = 1; d < 64; d <<= 1) {
                    const uint32_t o = __shfl_down(suffix, d, 64);
                    if (lane + d < 64) suffix += o;
                }
                uint32_t above = suffix - mine;               // keys in bins above this lane's
                if (above < remaining && remaining <= suffix) {
                    int bin = 4 * lane + 3;
                    const uint32_t cs[4] = {c0, c1, c2, c3};
#pragma unroll
                    for (int j = 3; j > 0; --j) {
                        if (above + cs[j] >= remaining) break;
                        above += cs[j];
                        --bin;
                    }
                    s_prefix = prefix | ((uint32_t)bin << shift);
                    s_remaining = remaining - above;
                }
            }
            __syncthreads();
            prefix = s_prefix;
            remaining = s_remaining;
        }
    }

    // Ordered compaction: rows above the threshold key, plus the first `remaining`
    // rows with the threshold key, in ascending position.
    float mass = 0.f;
    uint32_t eq_base = 0, out_base = 0;
    const uint64_t lt_mask = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    for (int t0 = 0; t0 < ncand && want > 0; t0 += NT) {
        const int t = t0 + tid;
        const bool valid = t < ncand;
        const float xv = valid ? x[t] : 0.f;
        const uint32_t key = valid ? order_key(xv) : 0u;
        const bool gt = valid && key > prefix;
        const bool eq = valid && key == prefix;
        const uint64_t eq_bal = __ballot(eq);
        if (lane == 0) s_wtot[0][wave] = (uint32_t)__popcll(eq_bal);
        __syncthreads();
        uint32_t eq_before = eq_base, eq_tile = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const uint32_t c = s_wtot[0][w];
            if (w < wave) eq_before += c;
            eq_tile += c;
        }
        eq_before += (uint32_t)__popcll(eq_bal & lt_mask);
        const bool take = gt || (eq && eq_before < remaining);
        const uint64_t tk_bal = __ballot(take);
        if (lane == 0) s_wtot[1][wave] = (uint32_t)__popcll(tk_bal);
        __syncthreads();
        uint32_t pos = out_base, tk_tile = 0;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const uint32_t c = s_wtot[1][w];
            if (w < wave) pos += c;
            tk_tile += c;
        }
        pos += (uint32_t)__popcll(tk_bal & lt_mask);
        if (take) {
            sel[pos] = t;
            mass += fast_exp2(xv - M);
        }
        eq_base += eq_tile;
        out_base += tk_tile;
    }
    // Step 5: the l most recent positions are always kept.
    for (int i = tid; i < leff; i += NT) {
        const int t = ncand + i;
        sel[want + i] = t;
        mass += fast_exp2(x[t] - M);
    }
    mass = block_sum(mass, s_red);
    if (tid == 0) a.alpha[row] = mass / Z;     // step 7
}

// ---------------------------------------------------------------------------
// Steps 10-11 over the selected rows.
template <int D>
__global__ __launch_bounds__(kSparfAttendWaves * 64) void sparf_attend_kernel(SparfArgs a)
{
    constexpr int LPR = D / 8;
    constexpr int RPW = kWave / LPR;
    constexpr int WAVES = kSparfAttendWaves;
    constexpr int U = 16 / RPW;            // 16 rows per wave and iteration
    constexpr int TILE = WAVES * 16;
    constexpr int NG = WAVES * RPW;

    const int h = blockIdx.x, b = blockIdx.y;
    const int G = a.num_q_heads / a.num_kv_heads;
    const int hk = h / G;
    const int tid = threadIdx.x;
    const int64_t row = (int64_t)b * a.num_q_heads + h;
    const int L = clamp_len(a.seq_lens[b], a.max_len);
    if (L == 0) {
        if (tid < D) {
            if (a.out_f32) ((float*)a.out)[row * D + tid] = 0.f;
            else ((half_t*)a.out)[row * D + tid] = (half_t)0.f;
        }
        return;
    }
    const int n = min(a.k, L);
    const int32_t* sel = a.sel + row * a.k;

    const int wave = tid >> 6, lane = tid & 63;
    const int r = lane / LPR, c = lane % LPR;
    const half8_t q8 = *(const half8_t*)(a.q + row * D + c * 8);
    const int64_t head_base = (int64_t)b * a.kv.stride_b + (int64_t)hk * a.kv.stride_h + c * 8;

    float m = kNegBig, l = 0.f;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;

    for (int p0 = 0; p0 < n; p0 += TILE) {
        u32x4 kr[U], vr[U];
        bool ok[U];
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const int p = p0 + wave * 16 + j * RPW + r;
            ok[j] = p < n;
            const int t = sel[min(p, n - 1)];
            const int64_t off = head_base + (int64_t)t * a.kv.stride_t;
            kr[j] = *(const u32x4*)(a.kv.k + off);
            vr[j] = *(const u32x4*)(a.kv.v + off);
        }
        float s[U];
        float mx = m;
#pragma unroll
        for (int j = 0; j < U; ++j) {
            float d = dot8(__builtin_bit_cast(half8_t, kr[j]), q8, 0.f);
            d = group_sum<LPR>(d);
            s[j] = ok[j] ? d * a.scale_log2 : -__builtin_inff();
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
            const half8_t vh = __builtin_bit_cast(half8_t, vr[j]);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = __builtin_fmaf((float)vh[e], p, acc[e]);
        }
    }

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
        // Step 11: alpha * (attention over the kept rows) + (1 - alpha) * mean of V.
        const float alpha = a.alpha[row];
        const float vbar = a.aux.vsum[((int64_t)b * a.num_kv_heads + hk) * D + tid] / (float)L;
        o = alpha * o + (1.f - alpha) * vbar;
        if (a.out_f32) ((float*)a.out)[row * D + tid] = o;
        else ((half_t*)a.out)[row * D + tid] = (half_t)o;
    }
}

// ---------------------------------------------------------------------------
// Component-major copy of K and column sums of V for rows [0, L_b).
__global__ __launch_bounds__(256) void sparf_build_kernel(SparfArgs a)
{
    const int hk = blockIdx.x, b = blockIdx.y;
    const int D = a.head_dim;
    const int tid = threadIdx.x;
    const int L = clamp_len(a.seq_lens[b], min(a.kv.capacity, a.aux.capacity));
    const half_t* kb = a.kv.k + (int64_t)b * a.kv.stride_b + (int64_t)hk * a.kv.stride_h;
    const half_t* vb = a.kv.v + (int64_t)b * a.kv.stride_b + (int64_t)hk * a.kv.stride_h;
    half_t* ktb = a.aux.kt + (int64_t)b * a.aux.stride_b + (int64_t)hk * a.aux.stride_h;

    __shared__ half_t s_tile[64][128 + 2];   // +2: odd word stride for the column reads
    const int cols8 = D / 8;
    for (int t0 = 0; t0 < L; t0 += 64) {
        // rows t0 .. t0+63 (rows at or behind L are not read; their slots become 0)
        for (int i = tid; i < 64 * cols8; i += 256) {
            const int tr = i / cols8, c8 = i % cols8;
            half8_t v = {0, 0, 0, 0, 0, 0, 0, 0};
            if (t0 + tr < L) v = *(const half8_t*)(kb + (int64_t)(t0 + tr) * a.kv.stride_t + c8 * 8);
#pragma unroll
            for (int e = 0; e < 8; ++e) s_tile[tr][c8 * 8 + e] = v[e];
        }
        __syncthreads();
        for (int i = tid; i < D * 8; i += 256) {
            const int d = i / 8, t8 = i % 8;
            half8_t v;
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = s_tile[t8 * 8 + e][d];
            if (t0 + t8 * 8 < L) *(half8_t*)(ktb + (int64_t)d * a.aux.stride_d + t0 + t8 * 8) = v;
        }
        __syncthreads();
    }
    if (tid < D) {
        float s = 0.f;
        for (int t = 0; t < L; ++t) s += (float)vb[(int64_t)t * a.kv.stride_t + tid];
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
    const int L = a.seq_lens[b];
    if (L < 1 || L > a.kv.capacity || L > a.aux.capacity) return;
    const int t = L - 1;
    const half_t kn = a.k_new[i], vn = a.v_new[i];
    const int64_t off = (int64_t)b * a.kv.stride_b + (int64_t)hk * a.kv.stride_h + (int64_t)t * a.kv.stride_t + d;
    const_cast<half_t*>(a.kv.k)[off] = kn;
    const_cast<half_t*>(a.kv.v)[off] = vn;
    a.aux.kt[(int64_t)b * a.aux.stride_b + (int64_t)hk * a.aux.stride_h + (int64_t)d * a.aux.stride_d + t] = kn;
    a.aux.vsum[i] += (float)vn;
}

// ---------------------------------------------------------------------------
hipError_t launch_sparf_build(const SparfArgs& a, hipStream_t stream)
{
    hipLaunchKernelGGL(sparf_build_kernel, dim3(a.num_kv_heads, a.batch), dim3(256), 0, stream, a);
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
    hipLaunchKernelGGL(sparf_logits_kernel, dim3(a.num_q_heads, a.nchunk, a.batch), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_sparf_select(const SparfArgs& a, hipStream_t stream)
{
    dim3 grid(a.num_q_heads, a.batch);
    if (a.max_len <= 8192) hipLaunchKernelGGL(sparf_select_kernel<256>, grid, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(sparf_select_kernel<1024>, grid, dim3(1024), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_sparf_attend(const SparfArgs& a, hipStream_t stream)
{
    dim3 grid(a.num_q_heads, a.batch), block(kSparfAttendWaves * 64);
    if (a.head_dim == 128) hipLaunchKernelGGL(sparf_attend_kernel<128>, grid, block, 0, stream, a);
    else hipLaunchKernelGGL(sparf_attend_kernel<64>, grid, block, 0, stream, a);
    return hipGetLastError();
}

}  // namespace instattn
