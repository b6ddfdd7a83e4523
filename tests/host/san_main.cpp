// Driver of the sanitizer build of the library's host side (see stub_launch.hip): calls the
// public entry points over a sweep of shapes and of the implementation switches, with a
// workspace that is a host allocation of exactly the size the library asked for.  Prints
// the number of calls and stub launches; any sanitizer report or failed check aborts.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/instattn.h"

namespace instattn {
int stub_launch_count();
}

static int g_calls = 0;

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            fprintf(stderr, "san_main: %s failed at line %d\n", #cond, __LINE__); \
            abort();                                                       \
        }                                                                  \
    } while (0)

static void* dummy(size_t bytes)
{
    void* p = nullptr;
    CHECK(posix_memalign(&p, 256, bytes ? bytes : 256) == 0);
    return p;
}

static void set_all(int chunk, int compact, int rotate, int dist, int three, int wide, int split_tail, int ring = -1)
{
    CHECK(instattn_set_option("INSTATTN_MHA_RING", ring) == INSTATTN_OK);
    CHECK(instattn_set_option("INSTATTN_CHUNK", chunk) == INSTATTN_OK);
    CHECK(instattn_set_option("INSTATTN_COMPACT", compact) == INSTATTN_OK);
    CHECK(instattn_set_option("INSTATTN_ROTATE", rotate) == INSTATTN_OK);
    CHECK(instattn_set_option("INSTATTN_SPARF_DISTRIBUTED", dist) == INSTATTN_OK);
    CHECK(instattn_set_option("INSTATTN_SPARF_THREE_LAUNCHES", three) == INSTATTN_OK);
    CHECK(instattn_set_option("INSTATTN_SPARF_WIDE", wide) == INSTATTN_OK);
    CHECK(instattn_set_option("INSTATTN_SPARF_SPLIT_TAIL", split_tail) == INSTATTN_OK);
}

static instattn_kv_desc make_desc(void* k, void* v, bool paged, int hkv, int dim, int max_len, const int32_t* table)
{
    instattn_kv_desc d;
    memset(&d, 0, sizeof d);
    d.k = k;
    d.v = v;
    if (paged) {
        d.layout = INSTATTN_KV_PAGED;
        d.page_size = 16;
        d.max_pages_per_seq = (max_len + 15) / 16;
        d.num_pages = 1000;
        d.capacity = 16 * d.max_pages_per_seq;
        d.stride_t = dim;
        d.stride_h = 16 * dim;
        d.stride_b = (int64_t)hkv * 16 * dim;
        d.page_table = table;
    } else {
        d.layout = INSTATTN_KV_CONTIGUOUS;
        d.capacity = (max_len + 15) / 16 * 16;
        d.stride_t = dim;
        d.stride_h = (int64_t)d.capacity * dim;
        d.stride_b = d.stride_h * hkv;
    }
    return d;
}

int main()
{
    void* q = dummy(1 << 16);
    void* kbuf = dummy(1 << 16);
    void* vbuf = dummy(1 << 16);
    void* outbuf = dummy(1 << 16);
    void* newrow = dummy(1 << 16);
    int32_t* lens = (int32_t*)dummy(1 << 16);
    int32_t* table = (int32_t*)dummy(1 << 16);
    const size_t kMostWorkspace = (size_t)24 << 20;     // larger shapes are skipped: the sweep stays within seconds

    const int batches[] = {1, 3, 64, 300};
    const int heads[][2] = {{1, 1}, {4, 4}, {8, 2}, {40, 40}, {64, 8}, {48, 1}, {34, 2}};
    const int dims[] = {64, 128};
    const int lengths[] = {1, 128, 385, 4097, 8192, 8193, 18432, 18433, 36865, 70000, 140000};
    const int chunks[] = {-1, 128, 1000, 1 << 20};

    // ---- dense path: every unit length, with and without the unit list, both layouts
    for (int b : batches)
        for (auto& h : heads)
            for (int dim : dims)
                for (int len : lengths)
                    for (int chunk : chunks)
                        for (int compact = -1; compact <= 1; ++compact)
                            for (int paged = 0; paged <= 1; ++paged) {
                                set_all(chunk, compact, compact == 1, -1, -1, -1, -1, (b + len + paged) % 3 - 1);
                                const size_t need = instattn_decode_workspace_size(b, h[0], h[1], dim, len);
                                CHECK(need > 0 && need % 256 == 0);
                                if (need > kMostWorkspace) continue;
                                int c = 0, n = 0;
                                CHECK(instattn_decode_plan(b, h[0], h[1], dim, len, &c, &n) == INSTATTN_OK);
                                CHECK(c % 128 == 0 && (int64_t)c * n >= len && (int64_t)c * (n - 1) < len);
                                void* ws = dummy(need);
                                const instattn_kv_desc d = make_desc(kbuf, vbuf, paged, h[1], dim, len, table);
                                const int before = instattn::stub_launch_count();
                                int st = instattn_append_decode(q, newrow, newrow, &d, lens, b, h[0], h[1], dim, 0.1f, outbuf,
                                                                INSTATTN_F16, nullptr, ws, need, len, nullptr);
                                CHECK(st == INSTATTN_OK);
                                int32_t launches[4];
                                CHECK(instattn_decode_launches(b, h[0], h[1], dim, len, d.layout, 1, launches) == INSTATTN_OK);
                                CHECK(instattn::stub_launch_count() - before == launches[0] + launches[1] + launches[2] + launches[3]);
                                st = instattn_decode(q, &d, lens, b, h[0], h[1], dim, 0.1f, outbuf, INSTATTN_F32, (float*)outbuf,
                                                     ws, need, len, nullptr);
                                CHECK(st == INSTATTN_OK);
                                // one byte less is refused
                                st = instattn_decode(q, &d, lens, b, h[0], h[1], dim, 0.1f, outbuf, INSTATTN_F32, nullptr, ws,
                                                     need - 1, len, nullptr);
                                CHECK(st == INSTATTN_ERR_WORKSPACE);
                                free(ws);
                                g_calls += 3;
                            }

    // ---- SparF: every combination of the switches that force a form of the decode
    const int ks[] = {1, 256, 2048, 1 << 30};
    const int sparf_heads[][2] = {{1, 1}, {8, 2}, {40, 40}, {34, 2}};
    for (int b : {1, 3, 16})
        for (auto& h : sparf_heads)
            for (int dim : dims)
                for (int len : lengths)
                    for (int k : ks)
                        for (int sw = 0; sw < 36; ++sw) {
                            const int dist = sw % 3 - 1, wide = sw / 3 % 3 - 1, three = sw / 9 % 2 ? 1 : -1, tail = sw / 18 ? 1 : -1;
                            set_all(-1, -1, -1, dist, three, wide, tail);
                            const size_t need = instattn_sparf_workspace_size(b, h[0], dim, len, k);
                            CHECK(need > 0 && need % 256 == 0);
                            if (need > kMostWorkspace) continue;
                            void* ws = dummy(need);
                            const instattn_kv_desc d = make_desc(kbuf, vbuf, sw & 1, h[1], dim, len, table);
                            instattn_sparf_aux aux;
                            memset(&aux, 0, sizeof aux);
                            aux.kt = kbuf;
                            aux.vsum = (float*)vbuf;
                            aux.capacity = (len + 7) / 8 * 8;
                            aux.stride_d = aux.capacity;
                            aux.stride_h = (int64_t)aux.capacity * dim;
                            aux.stride_b = aux.stride_h * h[1];
                            int32_t plan[6];
                            CHECK(instattn_sparf_plan(b, h[0], h[1], dim, len, k, 1, plan) == INSTATTN_OK);
                            int st = instattn_sparf_append_decode(q, newrow, newrow, &d, &aux, lens, b, h[0], h[1], dim, 0.1f,
                                                                  dim / 8, k, 16, outbuf, INSTATTN_F16, nullptr, nullptr, ws, need,
                                                                  len, nullptr);
                            CHECK(st == INSTATTN_OK);
                            st = instattn_sparf_decode(q, &d, &aux, lens, b, h[0], h[1], dim, 0.1f, dim / 8, k, 16, outbuf,
                                                       INSTATTN_F32, nullptr, nullptr, ws, need - 1, len, nullptr);
                            CHECK(st == INSTATTN_ERR_WORKSPACE);
                            free(ws);
                            g_calls += 2;
                        }

    // ---- the set-up's scratch
    set_all(-1, -1, -1, -1, -1, -1, -1);
    for (int b : {1, 2, 16, 64})
        for (int hkv : {1, 8, 40})
            for (int dim : dims) {
                const size_t need = instattn_sparf_build_workspace_size(b, hkv, dim);
                const instattn_kv_desc d = make_desc(kbuf, vbuf, false, hkv, dim, 4097, table);
                instattn_sparf_aux aux;
                memset(&aux, 0, sizeof aux);
                aux.kt = kbuf;
                aux.vsum = (float*)vbuf;
                aux.capacity = 4104;
                aux.stride_d = aux.capacity;
                aux.stride_h = (int64_t)aux.capacity * dim;
                aux.stride_b = aux.stride_h * hkv;
                void* ws = need ? dummy(need) : nullptr;
                CHECK(instattn_sparf_build(&d, &aux, lens, b, hkv, dim, ws, need, nullptr) == INSTATTN_OK);
                free(ws);
                ++g_calls;
            }

    printf("san_main: %d calls, %d stub launches, no report\n", g_calls, instattn::stub_launch_count());
    return 0;
}
