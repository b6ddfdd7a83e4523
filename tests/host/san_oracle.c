/* Driver for the sanitizer build of the C oracle (tests/test_sanitizers.py): reads one case
 * from a file, runs oracle_kv_append and oracle_decode on heap copies of exactly the stated
 * sizes (so AddressSanitizer sees any access outside a tensor), writes the caches, the
 * output rows and the lse back.  File: 8 int32 (B, Hq, Hkv, D, capacity, page_size,
 * max_pages, rows of the cache's first axis), one float (scale), then q, k, v, k_new,
 * v_new (fp16 bit patterns), seq_lens and, if page_size > 0, the page table (int32). */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

long oracle_decode(const uint16_t *q, const uint16_t *k, const uint16_t *v, const int32_t *seq_lens,
                   const int32_t *page_table, int B, int Hq, int Hkv, int D, int capacity, int page_size,
                   int max_pages, float scale, double *out, double *lse, int pair_stride, int pair_offset,
                   int nthreads);
void oracle_kv_append(uint16_t *k, uint16_t *v, const uint16_t *k_new, const uint16_t *v_new,
                      const int32_t *seq_lens, const int32_t *page_table, int B, int Hkv, int D, int capacity,
                      int page_size, int max_pages);

static void *slurp(FILE *f, size_t bytes)
{
    void *p = malloc(bytes ? bytes : 1);
    if (!p || fread(p, 1, bytes, f) != bytes) {
        fprintf(stderr, "san_oracle: short read\n");
        exit(2);
    }
    return p;
}

int main(int argc, char **argv)
{
    if (argc != 3) return 2;
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 2;
    int32_t h[8];
    float scale;
    if (fread(h, 4, 8, f) != 8 || fread(&scale, 4, 1, f) != 1) return 2;
    const int B = h[0], Hq = h[1], Hkv = h[2], D = h[3], cap = h[4], ps = h[5], mp = h[6], first = h[7];
    const size_t cache = (size_t)first * Hkv * (ps ? ps : cap) * D;
    uint16_t *q = slurp(f, (size_t)B * Hq * D * 2);
    uint16_t *k = slurp(f, cache * 2), *v = slurp(f, cache * 2);
    uint16_t *kn = slurp(f, (size_t)B * Hkv * D * 2), *vn = slurp(f, (size_t)B * Hkv * D * 2);
    int32_t *lens = slurp(f, (size_t)B * 4);
    int32_t *table = ps ? slurp(f, (size_t)B * mp * 4) : NULL;
    fclose(f);
    double *out = malloc((size_t)B * Hq * D * sizeof(double)), *lse = malloc((size_t)B * Hq * sizeof(double));
    oracle_kv_append(k, v, kn, vn, lens, table, B, Hkv, D, cap, ps, mp);
    const long done = oracle_decode(q, k, v, lens, table, B, Hq, Hkv, D, cap, ps, mp, scale, out, lse, 1, 0, 2);
    if (done != (long)B * Hq) return 3;
    f = fopen(argv[2], "wb");
    if (!f) return 2;
    fwrite(k, 2, cache, f);
    fwrite(v, 2, cache, f);
    fwrite(out, sizeof(double), (size_t)B * Hq * D, f);
    fwrite(lse, sizeof(double), (size_t)B * Hq, f);
    fclose(f);
    free(q); free(k); free(v); free(kn); free(vn); free(lens); free(table); free(out); free(lse);
    return 0;
}
