/*
 * instattn -- decode-phase attention over a long fp16 KV cache, for one MI355X (gfx950).
 *
 * C ABI of the shared library built from paper_2409_04992_amd/csrc.  The operation
 * is the one the paper moves next to the stored KV cache: per sequence and head,
 * one new query row attends over all cached keys and values
 * (softmax(q K^T * scale) V, Sec. II-A; matrix-vector form of the decode phase,
 * Sec. II-B), after the new token's k and v have been stored behind the cached
 * ones (Sec. IV-C "Batch Writing Requests", Sec. IV-D "GPU-CSD coordination": the
 * device receives q, k, v, keeps k, v, returns the output row).
 *
 * General rules of every entry point
 *   - Pointers marked "device" are HIP device pointers owned by the caller; the
 *     library allocates no device memory, frees nothing, and keeps no pointer
 *     after the call returns.  Pointers marked "host" are ordinary host memory.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without synchronising.
 *   - The return value is an instattn_status.  Arguments are checked on the host
 *     before anything is launched; a rejected call launches nothing.
 *   - Lengths live on the device and cannot be checked by the host, so kernels
 *     clamp them: L_b is read as min(max(seq_lens[b], 0), capacity, max_seq_len).
 *   - fp16 is IEEE binary16; all accumulation is fp32.  NaN and infinities in q, K or V
 *     spread through the arithmetic into the output rows that read them (under SparF the
 *     kept positions of such a head are then arbitrary positions of its row); no address
 *     computed from them leaves the caller's buffers.
 *   - Query head h reads KV head h / (num_q_heads / num_kv_heads).
 */
#ifndef INSTATTN_H
#define INSTATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    INSTATTN_OK = 0,
    INSTATTN_ERR_INVALID_ARG = 1, /* NULL pointer, non-positive size, bad stride/alignment, bad enum */
    INSTATTN_ERR_UNSUPPORTED = 2, /* valid request outside what the kernels cover (see decode) */
    INSTATTN_ERR_WORKSPACE = 3,   /* workspace NULL, misaligned or smaller than decode_workspace_size */
    INSTATTN_ERR_RUNTIME = 4      /* a HIP launch failed */
} instattn_status;

typedef enum { INSTATTN_KV_CONTIGUOUS = 0, INSTATTN_KV_PAGED = 1 } instattn_kv_layout;
typedef enum { INSTATTN_F16 = 0, INSTATTN_F32 = 1 } instattn_dtype;

/*
 * Where the cached keys and values live.  k and v have the same geometry.
 * Strides are in fp16 elements; the head dimension is unit-stride; every stride
 * must be a multiple of 8 elements and k, v 16-byte aligned (rows are moved with
 * 128-bit accesses).  stride_t may not exceed 2^24 elements
 * (INSTATTN_ERR_UNSUPPORTED beyond).
 *
 *   contiguous: element (b, hk, t, d) at  b*stride_b    + hk*stride_h + t*stride_t + d
 *               capacity = rows available per (b, hk); page_table = NULL.
 *   paged:      position t of sequence b is row t % page_size of pool page
 *               p = page_table[b*max_pages_per_seq + t / page_size]; element at
 *               p*stride_b + hk*stride_h + (t % page_size)*stride_t + d.
 *               page_size is a power of two >= 16 (the paper's 16-token, 4 KB group of
 *               Sec. IV-C "Token-Indexed Mapping" is page_size 16 with head_dim 128);
 *               capacity = page_size*max_pages_per_seq.  k and v may point into one
 *               pool that keeps the K and the V block of a (page, head) adjacent
 *               ([num_pages][Hkv][2][page_size][D]: same strides, v = k + page_size*D);
 *               the split pass reads it about 1 % faster than two pools at page_size 16.
 *               Entries behind the last
 *               used page are never read.  Pool ids must lie in [0, num_pages); the
 *               table is device data the host cannot check, so the kernels read an id
 *               outside that range as the pool's last page: such a table costs a
 *               meaningless result, never an access outside the pool.
 */
typedef struct {
    void* k;                   /* device, fp16 */
    void* v;                   /* device, fp16 */
    int32_t layout;            /* instattn_kv_layout */
    int32_t page_size;         /* paged only */
    int64_t stride_b;          /* contiguous: per sequence; paged: per pool page */
    int64_t stride_h;          /* per KV head */
    int64_t stride_t;          /* per position (row) */
    int32_t capacity;          /* max positions per sequence */
    int32_t max_pages_per_seq; /* paged only: row length of page_table */
    int32_t num_pages;         /* paged only: pool size */
    int32_t reserved;          /* must be 0 */
    const int32_t* page_table; /* device [batch][max_pages_per_seq]; NULL if contiguous */
} instattn_kv_desc;

/* Library version: major*10000 + minor*100 + patch. */
int instattn_version(void);

/* Static, NUL-terminated description of a status value (host memory, never freed). */
const char* instattn_status_string(int status);

/*
 * Implementation switches, for experiments and tests (host only; no effect on what is
 * computed beyond the order of floating-point sums).  Each forces one choice the host
 * otherwise makes from the sizes of a call; value < 0 hands the choice back to the host.
 * They are process-wide: a call reads them once when it starts; setting one while calls
 * run in other threads is safe and affects calls that start later.  On first use every
 * switch takes the integer value of the environment variable of the same name, if set.
 *   "INSTATTN_CHUNK"                n > 0: positions per unit of the dense split pass (rounded up to 128)
 *   "INSTATTN_ROTATE"               1: every unit starts its walk over its rows at a tile of its own
 *   "INSTATTN_COMPACT"              1 / 0: the dense split pass walks a device-built list of the units
 *                                   that hold rows (one small launch in front; the host's choice for
 *                                   large paged caches), or never does
 *   "INSTATTN_MHA_RING"             1 / 0: the vector-ALU split pass stages its tiles through its LDS ring
 *                                   (the host's choice for launches of 2^20 rows or more of sequences of
 *                                   2048 rows or more whose units fill their rounds over the compute
 *                                   units), or holds two tiles in registers; the unit length follows the form
 *   "INSTATTN_SPARF_DISTRIBUTED"    1 / 0: SparF selection spread over one block per 8192 scores, or never
 *   "INSTATTN_SPARF_THREE_LAUNCHES" 1: SparF never takes its one-launch kernel
 *   "INSTATTN_SPARF_WIDE"           1 / 0: the one-launch kernel's 512/1024-thread forms whenever they fit, or never
 *   "INSTATTN_SPARF_SPLIT_TAIL"     1: SparF selection and gather never share a launch
 * An unknown name (or a NULL pointer) is INSTATTN_ERR_INVALID_ARG.  name, value: host.
 */
int instattn_set_option(const char* name, int value);
int instattn_get_option(const char* name, int* value);

/*
 * Store the new token's key and value (Sec. IV-C "Batch Writing Requests").
 * For every sequence b and KV head hk, copies the head_dim fp16 values
 * k_new[b][hk][:] and v_new[b][hk][:] bit for bit into position seq_lens[b] - 1
 * of the cache.  seq_lens[b] is the length INCLUDING the token being stored.  A
 * length outside [1, capacity] stores nothing for that sequence.
 *   k_new, v_new : device, [batch][num_kv_heads][head_dim] fp16, dense, 16-byte aligned
 *   seq_lens     : device, [batch] int32, not modified
 * head_dim must be a multiple of 8.  One kernel launch.
 */
int instattn_kv_append(const instattn_kv_desc* kv, const void* k_new, const void* v_new,
                       const int32_t* seq_lens, int batch, int num_kv_heads, int head_dim,
                       void* stream);

/*
 * Store a run of rows per sequence: the prefill side of Sec. IV-D, where a layer's
 * K and V for all prompt tokens are handed over at once.  For every b, hk and
 * i < min(count[b], max_new), copies k_src[b][hk][i][:] and v_src[b][hk][i][:] bit
 * for bit into position start[b] + i; positions outside [0, capacity) are
 * skipped.  Equivalent to calling instattn_kv_append once per row.
 *   k_src, v_src : device, [batch][num_kv_heads][max_new][head_dim] fp16, dense, 16-byte aligned
 *   start, count : device, [batch] int32, not modified
 * head_dim 64 or 128.  One launch.
 */
int instattn_kv_write(const instattn_kv_desc* kv, const void* k_src, const void* v_src,
                      const int32_t* start, const int32_t* count, int batch, int num_kv_heads,
                      int head_dim, int max_new, void* stream);

/*
 * How decode cuts the sequence axis (host arithmetic only; no device access).
 * Work is split into units of `chunk_tokens` consecutive positions so that a
 * single long sequence still fills the chip; unit i of sequence b covers
 * positions [i*chunk, (i+1)*chunk) cut off at L_b, and num_splits =
 * ceil(max_seq_len / chunk).  The plan depends only on the arguments given here
 * (and the "INSTATTN_CHUNK" switch, which forces chunk_tokens for experiments).
 * Either output pointer may be NULL.  host pointers.  More than 65535 splits are
 * INSTATTN_ERR_UNSUPPORTED (here and in every call that uses the plan).
 */
int instattn_decode_plan(int batch, int num_q_heads, int num_kv_heads, int head_dim,
                         int max_seq_len, int* chunk_tokens, int* num_splits);

/*
 * Which kernels instattn_decode (with_append = 0) or instattn_append_decode
 * (with_append = 1) launches for these sizes on a cache of the given layout
 * (an instattn_kv_layout): host arithmetic only.  launches: host, 4 int32, each 0 or 1:
 *   [0] the store of the new token as a launch of its own (groups of more than 16 query heads)
 *   [1] the list of the units that hold rows: paged caches with 2 to 4096 sequences, at
 *       most 8192 (sequence, split) pairs and max_seq_len x KV streams >= 2^21 rows; the
 *       split pass then walks that list with the blocks of a unit on one XCD
 *   [2] the split pass
 *   [3] the merge (plans with more than one split)
 */
int instattn_decode_launches(int batch, int num_q_heads, int num_kv_heads, int head_dim, int max_seq_len,
                             int kv_layout, int with_append, int32_t* launches);

/* Bytes of device workspace decode needs for these arguments (0 if they are invalid). */
size_t instattn_decode_workspace_size(int batch, int num_q_heads, int num_kv_heads,
                                      int head_dim, int max_seq_len);

/*
 * Decode attention (Sec. II-A, II-B): for every sequence b and query head h
 *     s_t  = scale * sum_d q[b][h][d] * K[b][hk][t][d]        t = 0 .. L_b-1
 *     out[b][h][:] = sum_t softmax(s)_t * V[b][hk][t][:]
 *     lse[b][h]    = log sum_t exp(s_t)                         (natural log)
 * over exactly the first L_b = seq_lens[b] positions; rows at or behind L_b are
 * never read.  L_b <= 0 gives a zero output row and lse = -inf.
 *   q         : device, [batch][num_q_heads][head_dim] fp16, dense, 16-byte aligned
 *   out       : device, [batch][num_q_heads][head_dim], fp16 (round to nearest even,
 *               once, at the end) or fp32 according to out_dtype
 *   lse       : device, [batch][num_q_heads] fp32, or NULL
 *   workspace : device, >= instattn_decode_workspace_size(...) bytes, 256-byte aligned;
 *               contents on entry are ignored, contents on return are unspecified
 *   max_seq_len : host-known upper bound of every L_b (<= capacity); it fixes the
 *               split plan, so no device value is read back
 * Supported: head_dim 64 or 128; num_q_heads a multiple of num_kv_heads with a
 * ratio of 1 (vector-ALU path) or more (MFMA group path: up to 16 query heads of a
 * group share one pass over their KV head; a larger group, as in multi-query
 * models, takes one pass per 16 of its heads); both layouts; both output types.
 * One to three kernel launches (instattn_decode_launches tells which): the split pass,
 * the merge unless the plan has a single split, and for large paged caches a small
 * launch in front that lists the units that hold rows.
 */
int instattn_decode(const void* q, const instattn_kv_desc* kv, const int32_t* seq_lens,
                    int batch, int num_q_heads, int num_kv_heads, int head_dim, float scale,
                    void* out, int out_dtype, float* lse, void* workspace,
                    size_t workspace_bytes, int max_seq_len, void* stream);

/*
 * instattn_kv_append followed by instattn_decode in one call (Sec. IV-D: q, k, v
 * of the new token arrive together).  Same arguments, checks and results as the
 * two calls in that order: the caches end up bit-identical and out/lse are those
 * of instattn_decode on the updated caches.  The store of the new row is done
 * inside the split pass by the unit that owns position seq_lens[b] - 1, which
 * saves a kernel launch (groups of more than 16 query heads: a launch of its own).
 *   k_new, v_new : device, [batch][num_kv_heads][head_dim] fp16, dense, 16-byte aligned
 */
int instattn_append_decode(const void* q, const void* k_new, const void* v_new,
                           const instattn_kv_desc* kv, const int32_t* seq_lens, int batch,
                           int num_q_heads, int num_kv_heads, int head_dim, float scale, void* out,
                           int out_dtype, float* lse, void* workspace, size_t workspace_bytes,
                           int max_seq_len, void* stream);

/*
 * The two halves of instattn_decode, callable on their own (same arguments, same
 * checks) so that each can be timed or composed separately.  decode_partial
 * runs the split pass: per unit an online-softmax pass over its positions,
 * leaving a normalised partial output row and its log-sum-exp in the workspace
 * (when the plan has one split it writes out/lse directly).  decode_merge
 * combines the units of each (b, h) by their log-sum-exp weights into out/lse;
 * with a single split it launches nothing.  append_decode_partial is the split pass of
 * instattn_append_decode: it stores the new token as well (calling it twice with the same
 * arguments stores the same bits twice).
 */
int instattn_decode_partial(const void* q, const instattn_kv_desc* kv, const int32_t* seq_lens,
                            int batch, int num_q_heads, int num_kv_heads, int head_dim,
                            float scale, void* out, int out_dtype, float* lse, void* workspace,
                            size_t workspace_bytes, int max_seq_len, void* stream);
int instattn_append_decode_partial(const void* q, const void* k_new, const void* v_new,
                                   const instattn_kv_desc* kv, const int32_t* seq_lens, int batch,
                                   int num_q_heads, int num_kv_heads, int head_dim, float scale, void* out,
                                   int out_dtype, float* lse, void* workspace, size_t workspace_bytes,
                                   int max_seq_len, void* stream);
int instattn_decode_merge(const int32_t* seq_lens, int batch, int num_q_heads, int num_kv_heads,
                          int head_dim, int capacity, void* out, int out_dtype, float* lse,
                          const void* workspace, size_t workspace_bytes, int max_seq_len,
                          void* stream);

/*
 * instattn_decode for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments minus
 * the workspace, same checks, same kernels and bit for bit the same out/lse.  The
 * partial rows of the split pass go to a scratch array of INSTATTN_STATIC_SCRATCH_BYTES
 * that is part of the library's device code: every GPU the library runs on holds its
 * own copy until the process ends.  The call allocates and frees nothing.  Its first
 * call on a device looks up that device's copy (make that call before a graph capture).
 * A shape whose instattn_decode_workspace_size exceeds INSTATTN_STATIC_SCRATCH_BYTES is
 * rejected with INSTATTN_ERR_WORKSPACE and launches nothing (the five measured
 * configurations need 0.5 KB to 16 MB).  All calls on one GPU share that GPU's array:
 * calls that overlap there - on different streams, or from several threads - race;
 * order them.  Nothing in the array has to start at zero (the merge reads only what
 * the split pass of the same call wrote), so nothing is cleared.
 */
#define INSTATTN_STATIC_SCRATCH_BYTES (32u << 20)
int instattn_decode_static(const void* q, const instattn_kv_desc* kv, const int32_t* seq_lens,
                           int batch, int num_q_heads, int num_kv_heads, int head_dim, float scale,
                           void* out, int out_dtype, float* lse, int max_seq_len, void* stream);

/* ------------------------------------------------------------------------
 * SparF attention (Algorithm 1): decode attention from a fraction of the cache.
 *
 * Per query head: keep the r components of q with the largest magnitude, score
 * every position from those r columns of K alone (softmax with the algorithm's
 * temperature), keep the k best-scored positions, the l most recent always among
 * them, let alpha be their share of the approximate softmax, run exact softmax
 * attention over the kept rows and return
 *     out = alpha * attention_over_kept_rows + (1 - alpha) * mean(V[0:L_b]).
 * 1/sqrt(d_h) enters through `scale` as in the dense path.  Ties in either top-k
 * go to the lower index.  k and l are cut off at L_b, l at k.  With k >= L_b the
 * result equals instattn_decode.  Both cache layouts, head_dim 64 or 128.
 *
 * The column reads need K stored a second time, component-major (the paper's
 * hidden-embedding-indexed copy, Sec. IV-C), and the blend needs the running sum
 * of V; both live in caller-owned device memory described by instattn_sparf_aux:
 *   kt   : fp16, 16-byte aligned, strides multiples of 8.
 *          contiguous (page_size 0, page_table NULL): element (b, hk, d, t) at
 *            b*stride_b + hk*stride_h + d*stride_d + t; capacity (a multiple of 8)
 *            positions per (b, hk, d) row.
 *          paged (page_size > 0): position t of sequence b is entry t % page_size of
 *            pool page p = page_table[b*max_pages_per_seq + t / page_size]; element
 *            (d, t) at p*stride_b + hk*stride_h + d*stride_d + t % page_size;
 *            capacity = page_size*max_pages_per_seq.  page_size is a power of two
 *            >= 8 and independent of the cache's own page size: a column is read in
 *            runs along t, so this copy wants long pages (Sec. IV-C puts the
 *            granularity of the hidden-embedding-indexed copy at 256 to 1K tokens),
 *            while the row-major cache is fine with 16-token pages.  Entries of
 *            page_table behind the last used page are never read; ids outside
 *            [0, num_pages) are read as the pool's last page, as for the cache's own table.
 *   vsum : fp32 [batch][num_kv_heads][head_dim], sum of rows 0 .. L_b-1 of V
 * The layout of kt is independent of the layout of the cache itself.
 */
typedef struct {
    void* kt;
    int64_t stride_b, stride_h, stride_d;
    float* vsum;
    int32_t capacity;          /* max positions per sequence in kt */
    int32_t page_size;         /* 0: contiguous kt; else positions per kt page */
    const int32_t* page_table; /* device [batch][max_pages_per_seq]; NULL if contiguous */
    int32_t max_pages_per_seq; /* paged only */
    int32_t num_pages;         /* paged only: pool size */
} instattn_sparf_aux;

/*
 * Bytes of device scratch with which instattn_sparf_build spreads the sum of V of
 * one (sequence, KV head) over several blocks: worth it when there are few such
 * pairs with long rows (0: there are pairs enough, or the arguments are invalid).
 */
size_t instattn_sparf_build_workspace_size(int batch, int num_kv_heads, int head_dim);

/*
 * Fill aux (kt and vsum) from the rows 0 .. seq_lens[b]-1 of an existing cache:
 * what the storage side does when the prefill phase hands over a layer's K and V
 * (Sec. IV-D).  Rows at or behind the length are not read.
 *   workspace : device scratch of at least instattn_sparf_build_workspace_size
 *               bytes, 256-byte aligned, or NULL (then one block sums the V rows of
 *               a pair: same result to fp32 rounding, slow for few pairs with long
 *               rows); a non-NULL workspace that is too small is
 *               INSTATTN_ERR_WORKSPACE.  Contents on entry are ignored.
 * Two launches, three with the workspace in use.  The sums are taken in a fixed
 * order: the same inputs give the same bits.
 */
int instattn_sparf_build(const instattn_kv_desc* kv, const instattn_sparf_aux* aux,
                         const int32_t* seq_lens, int batch, int num_kv_heads, int head_dim,
                         void* workspace, size_t workspace_bytes, void* stream);

/*
 * instattn_kv_append that also keeps aux current: stores k_new as entry
 * seq_lens[b]-1 of every K column and adds v_new to vsum.  Unlike kv_append it is
 * not idempotent (vsum is a running sum): call it once per new token.  A length
 * outside [1, capacity] changes nothing for that sequence.  One launch.
 */
int instattn_sparf_append(const instattn_kv_desc* kv, const instattn_sparf_aux* aux,
                          const void* k_new, const void* v_new, const int32_t* seq_lens,
                          int batch, int num_kv_heads, int head_dim, void* stream);

/*
 * Which kernels instattn_sparf_decode (with_append = 0) or
 * instattn_sparf_append_decode (with_append = 1) launches for these sizes: host
 * arithmetic only, no device access (the choices are the implementation's, not
 * the paper's; they depend on the arguments and on the "INSTATTN_SPARF_*"
 * switches that force a form for tests).  plan: host, 6 int32:
 *   [0] kernel launches in all
 *   [1] threads per block of the one-launch kernel (256, 512 or 1024), 0 if the
 *       pipeline runs instead
 *   [2] 1 if the decode's first launch stores the new token itself
 *   [3] pipeline only: 1 = one block per head selects, 2 = one block per 8192 scores
 *   [4] pipeline only: 1 if the block that selects also gathers the kept rows
 *   [5] slices a head's kept rows are gathered in
 */
int instattn_sparf_plan(int batch, int num_q_heads, int num_kv_heads, int head_dim, int max_seq_len,
                        int k, int with_append, int32_t* plan);

/* Bytes of device workspace instattn_sparf_decode needs (0 if the arguments are invalid). */
size_t instattn_sparf_workspace_size(int batch, int num_q_heads, int head_dim, int max_seq_len,
                                     int k);

/*
 * SparF decode as described above.  Arguments as for instattn_decode, plus
 *   r, k, l   : Algorithm 1's inputs; 1 <= r <= head_dim, k >= 1, l >= 0
 *   sel_rows  : device [batch][num_q_heads][k] int32 or NULL: receives the kept
 *               positions of every head in ascending order (min(k, L_b) entries
 *               are written per head)
 *   alpha     : device [batch][num_q_heads] fp32 or NULL: receives alpha, the kept share
 * L_b <= 0 gives a zero row (alpha 0).  One launch when max_seq_len <= 8192, or
 * <= 18432 with at least 96 (sequence, query head) pairs, or <= 36864 with 96 to
 * 256 of them (one block per query head keeps the scores in LDS; 256, 512 or 1024
 * threads), otherwise two to six: column
 * scores; then either one launch in which a block per head selects and gathers
 * (many heads, rows below 65536), or selection (one launch with a block per head,
 * or three with a block per 8192 scores for rows of 96K positions or more and, from
 * 40K on, for at most 128 or more than 512 heads),
 * attention over the kept rows, and a launch that combines the slices when a
 * head's kept rows are cut up.
 * A paged cache is limited to num_pages*page_size < 2^31 rows here, max_seq_len to
 * 65535 x 8192 (INSTATTN_ERR_UNSUPPORTED beyond).  max_seq_len must bound every L_b: a longer
 * sequence is cut off at max_seq_len as everywhere (memory-safe), but aux.vsum still
 * holds the sum of all its rows, so the mean of V that is blended in is then not
 * the mean of the rows attended.
 */
int instattn_sparf_decode(const void* q, const instattn_kv_desc* kv, const instattn_sparf_aux* aux,
                          const int32_t* seq_lens, int batch, int num_q_heads, int num_kv_heads,
                          int head_dim, float scale, int r, int k, int l, void* out, int out_dtype,
                          int32_t* sel_rows, float* alpha, void* workspace, size_t workspace_bytes,
                          int max_seq_len, void* stream);

/*
 * instattn_sparf_append followed by instattn_sparf_decode, as the storage side sees
 * a decode step (the new token's q, k, v arrive together, Sec. IV-D): same results
 * in the cache, in aux and in out/sel_rows/alpha as the two calls in that order.
 * When every KV head has one query head the decode's first launch (the one-launch
 * kernel, or the column-score pass) stores the new token itself; otherwise the
 * append is a launch of its own in front.  Like instattn_sparf_append it must be called once per new token.
 *   k_new, v_new : device, [batch][num_kv_heads][head_dim] fp16, dense, 16-byte aligned
 */
int instattn_sparf_append_decode(const void* q, const void* k_new, const void* v_new,
                                 const instattn_kv_desc* kv, const instattn_sparf_aux* aux,
                                 const int32_t* seq_lens, int batch, int num_q_heads, int num_kv_heads,
                                 int head_dim, float scale, int r, int k, int l, void* out, int out_dtype,
                                 int32_t* sel_rows, float* alpha, void* workspace, size_t workspace_bytes,
                                 int max_seq_len, void* stream);

/*
 * Measurement aids, not part of the attention path.  probe_read streams `bytes`
 * (a multiple of 16) from src with 128-bit loads and folds them into 4 bytes per
 * workgroup written to sink (device, >= 16 KiB): the read ceiling a streaming
 * kernel can reach.  probe_copy copies `bytes` from src to dst (device, disjoint):
 * a kernel of known traffic for scaling hardware counters.  probe_read_columns reads
 * what the SparF score pass (Algorithm 1, the approximate scores) reads of a contiguous
 * component-major copy and nothing else: of each of `rows` rows (row n at
 * base + n * row_stride bytes, 16-byte aligned) r of its `dims` columns (column d
 * d * col_stride bytes further on), the first `positions` fp16 (a multiple of 8) of
 * each; the columns are a fixed spread, the same for every call.  It gives the rate the
 * memory system reaches on those addresses, the ceiling of that pass.  sink as for
 * probe_read.  positions <= 65535 x 2048 (INSTATTN_ERR_UNSUPPORTED beyond).
 */
int instattn_probe_read(const void* src, size_t bytes, void* sink, void* stream);
int instattn_probe_read_columns(const void* base, size_t row_stride, size_t col_stride, int rows, int dims, int r,
                                int positions, void* sink, void* stream);
int instattn_probe_copy(const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* INSTATTN_H */
