// Host-side checks of the cache descriptor shared by the dense and the SparF
// entry points, and its translation into the view the kernels take.
#pragma once

#include <stdint.h>

#include "../../include/instattn.h"
#include "common.h"

namespace instattn {

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }
inline bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }
inline int ilog2(int x) { int s = 0; while ((1 << s) < x) ++s; return s; }

// The kernels address the rows of one tile as a 64-bit base plus a 32-bit byte
// offset of at most 15 rows: the row stride must leave room for that.
constexpr int64_t kMaxRowStride = (int64_t)1 << 24;   // elements

inline int check_kv(const instattn_kv_desc* kv, int head_dim)
{
    if (!kv || !kv->k || !kv->v) return INSTATTN_ERR_INVALID_ARG;
    if (!aligned16(kv->k) || !aligned16(kv->v)) return INSTATTN_ERR_INVALID_ARG;
    if (kv->reserved != 0) return INSTATTN_ERR_INVALID_ARG;
    if (kv->stride_b <= 0 || kv->stride_h <= 0 || kv->stride_t < head_dim)
        return INSTATTN_ERR_INVALID_ARG;
    if (kv->stride_t > kMaxRowStride) return INSTATTN_ERR_UNSUPPORTED;
    if (kv->stride_b % 8 || kv->stride_h % 8 || kv->stride_t % 8) return INSTATTN_ERR_INVALID_ARG;
    if (kv->capacity <= 0) return INSTATTN_ERR_INVALID_ARG;
    if (kv->layout == INSTATTN_KV_CONTIGUOUS) {
        if (kv->page_table != nullptr) return INSTATTN_ERR_INVALID_ARG;
    } else if (kv->layout == INSTATTN_KV_PAGED) {
        if (!kv->page_table) return INSTATTN_ERR_INVALID_ARG;
        if (!pow2(kv->page_size) || kv->page_size < 16) return INSTATTN_ERR_INVALID_ARG;
        if (kv->max_pages_per_seq <= 0 || kv->num_pages <= 0) return INSTATTN_ERR_INVALID_ARG;
        if ((int64_t)kv->capacity != (int64_t)kv->page_size * kv->max_pages_per_seq)
            return INSTATTN_ERR_INVALID_ARG;
    } else {
        return INSTATTN_ERR_INVALID_ARG;
    }
    return INSTATTN_OK;
}

inline KvView make_view(const instattn_kv_desc* kv)
{
    KvView w;
    w.k = (const half_t*)kv->k;
    w.v = (const half_t*)kv->v;
    w.page_table = kv->layout == INSTATTN_KV_PAGED ? kv->page_table : nullptr;
    w.stride_b = kv->stride_b;
    w.stride_h = kv->stride_h;
    w.stride_t = kv->stride_t;
    w.capacity = kv->capacity;
    w.page_shift = kv->layout == INSTATTN_KV_PAGED ? ilog2(kv->page_size) : 0;
    w.page_mask = kv->layout == INSTATTN_KV_PAGED ? kv->page_size - 1 : 0;
    w.max_pages = kv->max_pages_per_seq;
    w.last_page = kv->layout == INSTATTN_KV_PAGED ? kv->num_pages - 1 : 0;
    return w;
}

}  // namespace instattn
