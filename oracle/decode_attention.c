/*
 * Oracle, C form: decode-phase attention and KV append as plain fp64 loops.
 *
 * TEST INFRASTRUCTURE ONLY.  Not part of the product path; shares no code,
 * header or table with the HIP library.  Same definition and conventions as the
 * numpy form next to it (paper Sec. II-A: softmax(Q K^T / sqrt(d_k)) V per head;
 * Sec. II-B: one query row per step over the cached K, V; Sec. IV-C/IV-D: the new
 * k, v are stored, the output row is returned):
 *
 *   s_t   = scale * sum_d q[d] * K[t][d]            t = 0 .. L-1
 *   w_t   = exp(s_t - max s) / sum_t' exp(s_t' - max s)
 *   out_d = sum_t w_t * V[t][d]
 *   lse   = max s + log sum_t exp(s_t - max s)
 *
 * fp16 values arrive as their 16-bit patterns and are widened exactly.
 * Layouts: contiguous cache [B][Hkv][capacity][D]; paged pool
 * [num_pages][Hkv][page_size][D] with page_table [B][max_pages] (int32).
 * seq_lens[b] = L_b counts the token appended in this step.  L_b <= 0 gives a
 * zero row and lse = -inf; L_b is cut off at the capacity.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC decode_attention.c -o liboracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* IEEE binary16 -> double, exact (subnormals, infinities, NaN included). */
double oracle_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double x;
    if (expo == 0)
        x = ldexp((double)frac, -24);                 /* zero / subnormal: frac * 2^-24 */
    else if (expo == 31)
        x = frac ? NAN : INFINITY;
    else
        x = ldexp((double)(frac + 1024), expo - 25);  /* (1 + frac/1024) * 2^(expo-15) */
    return sign ? -x : x;
}

typedef struct {
    const uint16_t *base;
    const int32_t *page_table; /* NULL: contiguous */
    int Hkv, D;
    int capacity;              /* contiguous: rows per (b, hk) */
    int page_size, max_pages;  /* paged */
} cache_view;

static const uint16_t *row_ptr(const cache_view *c, int b, int hk, int t)
{
    if (!c->page_table)
        return c->base + (((size_t)b * c->Hkv + hk) * c->capacity + t) * c->D;
    int page = c->page_table[(size_t)b * c->max_pages + t / c->page_size];
    return c->base + (((size_t)page * c->Hkv + hk) * c->page_size + t % c->page_size) * c->D;
}

/* One (sequence, query head): scratch s[] holds L doubles. */
static void attend_one(const uint16_t *q, const cache_view *kc, const cache_view *vc,
                       int b, int hk, int L, int D, double scale,
                       double *s, double *out, double *lse)
{
    double m = -INFINITY;
    for (int t = 0; t < L; ++t) {
        const uint16_t *krow = row_ptr(kc, b, hk, t);
        double dot = 0.0;
        for (int d = 0; d < D; ++d)
            dot += oracle_half_to_double(q[d]) * oracle_half_to_double(krow[d]);
        s[t] = scale * dot;
        if (s[t] > m) m = s[t];
    }
    double Z = 0.0;
    for (int t = 0; t < L; ++t) {
        s[t] = exp(s[t] - m);
        Z += s[t];
    }
    for (int d = 0; d < D; ++d) out[d] = 0.0;
    for (int t = 0; t < L; ++t) {
        const uint16_t *vrow = row_ptr(vc, b, hk, t);
        double w = s[t] / Z;
        for (int d = 0; d < D; ++d)
            out[d] += w * oracle_half_to_double(vrow[d]);
    }
    *lse = m + log(Z);
}

/*
 * out [B][Hq][D] doubles, lse [B][Hq] doubles.  page_table == NULL selects the
 * contiguous layout (capacity rows); otherwise page_size/max_pages apply.
 * Only pairs p = b*Hq + h with p % pair_stride == pair_offset are computed (the
 * others are left untouched), so a caller can time or check a stated sample.
 * nthreads > 1 spreads the independent (b, h) pairs over OpenMP threads.
 * Returns the number of (b, h) pairs computed.
 */
long oracle_decode(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                   const int32_t *seq_lens, const int32_t *page_table,
                   int B, int Hq, int Hkv, int D,
                   int capacity, int page_size, int max_pages,
                   float scale, double *out, double *lse,
                   int pair_stride, int pair_offset, int nthreads)
{
    cache_view kc = {k, page_table, Hkv, D, capacity, page_size, max_pages};
    cache_view vc = {v, page_table, Hkv, D, capacity, page_size, max_pages};
    int cap = page_table ? page_size * max_pages : capacity;
    int G = Hq / Hkv;
    long done = 0;
    if (pair_stride < 1) pair_stride = 1;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads) reduction(+ : done)
    for (long p = pair_offset; p < (long)B * Hq; p += pair_stride) {
        int b = (int)(p / Hq), h = (int)(p % Hq);
        int L = seq_lens[b] < cap ? seq_lens[b] : cap;
        double *o = out + (size_t)p * D;
        if (L <= 0) {
            for (int d = 0; d < D; ++d) o[d] = 0.0;
            lse[p] = -INFINITY;
        } else {
            double *s = (double *)malloc((size_t)L * sizeof(double));
            attend_one(q + (size_t)p * D, &kc, &vc, b, h / G, L, D, (double)scale, s, o, &lse[p]);
            free(s);
        }
        done += 1;
    }
    return done;
}

/* Bit copy of the new token's k, v into position L_b - 1; lengths outside [1, cap] skip. */
void oracle_kv_append(uint16_t *k, uint16_t *v, const uint16_t *k_new, const uint16_t *v_new,
                      const int32_t *seq_lens, const int32_t *page_table,
                      int B, int Hkv, int D, int capacity, int page_size, int max_pages)
{
    cache_view kc = {k, page_table, Hkv, D, capacity, page_size, max_pages};
    cache_view vc = {v, page_table, Hkv, D, capacity, page_size, max_pages};
    int cap = page_table ? page_size * max_pages : capacity;
    for (int b = 0; b < B; ++b) {
        int L = seq_lens[b];
        if (L < 1 || L > cap) continue;
        for (int hk = 0; hk < Hkv; ++hk) {
            size_t src = ((size_t)b * Hkv + hk) * D;
            memcpy((uint16_t *)row_ptr(&kc, b, hk, L - 1), k_new + src, (size_t)D * 2);
            memcpy((uint16_t *)row_ptr(&vc, b, hk, L - 1), v_new + src, (size_t)D * 2);
        }
    }
}
