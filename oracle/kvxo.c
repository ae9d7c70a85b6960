/*
 * kvxo -- CPU oracle for block-free KV-cache transfer.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the GPU library is checked
 * against.  Only tests, the smoke check and the benchmark's CPU-baseline leg
 * may call it; the product path never does.  It shares no code, header or
 * table with the GPU library: the structs below are declared here on their own.
 *
 * What it computes (paper section 3.6, "Block-free D2D KVCache Transfer"):
 *
 *   pack     "Contiguous Buffer at Sender": the K and V of every layer of a
 *            request are laid one after another in a contiguous byte buffer,
 *            gathered out of the sender's discrete fixed-size blocks.
 *   unpack   "RecvScatter at Receiver": the discrete blocks of the receiver's
 *            pool are restored from those bytes.
 *   convert  both in one step, pool to pool (the bytes on the wire carry no
 *            block structure, so sender and receiver block geometry are
 *            independent; section 2.2.3 "Opportunity"/"Challenge").
 *   segment  offset and length of one layer of one request inside the buffer,
 *            a function of the layer index, the prompt length, the hidden size
 *            and the precision only (section 3.6, first paragraph).
 *   total    the KV size formula of section 2.1: bytes per layer =
 *            elem_bytes * hidden * 2 (K and V) * tokens.
 *
 * Readings where the paper is silent:
 *   - a token row [head][dim] is contiguous, row = heads*dim*elem_bytes;
 *   - inside a request's buffer: layers ascending, per layer all K rows then
 *     all V rows, tokens ascending;
 *   - several requests are concatenated in batch order with no padding;
 *   - a layer range [l0,l1) yields a compact buffer relative to l0;
 *   - slots of a request's last page beyond its length are neither read nor
 *     written; block-table entries beyond ceil(n/P) are ignored;
 *   - inside one page (one layer, K or V) a pool keeps its P tokens in one of
 *     three arrangements, the "desired discrete blocks" of the receiver:
 *       0  [token][head][dim]           a token row is contiguous
 *       1  [head][token][dim]           head-major
 *       2  [head][dim/x][token][x]      x = 16/elem_bytes elements: the token
 *                                       axis sits inside every 16-byte group of
 *                                       the head dimension
 *       3  [head][dim][token]           the token axis innermost, element by
 *                                       element (a transposed page)
 *     the buffer is always [token][head][dim].
 *
 * Loops are in the order of the definition; one memcpy per token row where
 * rows are contiguous on both sides, one per element otherwise.  The
 * optional thread count splits the outermost loop over requests (OpenMP) and
 * changes nothing else.
 */
#include <stdint.h>
#include <string.h>

typedef struct {
    uint32_t num_layers, num_kv_heads, head_dim, elem_bytes;
    uint32_t page_tokens, num_pages;
    uint32_t layout;             /* 0: [layer][K,V][page]{page}  1: [page][layer][K,V]{page} */
    uint32_t inner;              /* arrangement inside {page}: 0, 1, 2 or 3 as listed above */
    uint64_t stride_layer, stride_kv, stride_page, stride_token; /* bytes; all 0 = derive from layout */
} kvxo_pool;

typedef struct {
    uint32_t num_requests;
    uint32_t reserved;
    const uint32_t *seq_lens;      /* [R] tokens per request */
    const uint32_t *block_ids;     /* CSR values: physical page ids */
    const uint64_t *block_offsets; /* CSR offsets [R+1] */
} kvxo_batch;

static uint64_t row_bytes(const kvxo_pool *p)
{
    return (uint64_t)p->num_kv_heads * p->head_dim * p->elem_bytes;
}

/* Byte strides of the two named layouts, or the caller's own. */
static void strides(const kvxo_pool *p, uint64_t *sl, uint64_t *sk, uint64_t *sp, uint64_t *st)
{
    uint64_t row = row_bytes(p);
    if (p->stride_layer | p->stride_kv | p->stride_page | p->stride_token) {
        *sl = p->stride_layer; *sk = p->stride_kv; *sp = p->stride_page; *st = p->stride_token;
        return;
    }
    *st = row;
    if (p->layout == 0) {
        *sp = (uint64_t)p->page_tokens * row;
        *sk = (uint64_t)p->num_pages * *sp;
        *sl = 2 * *sk;
    } else {
        *sk = (uint64_t)p->page_tokens * row;
        *sl = 2 * *sk;
        *sp = (uint64_t)p->num_layers * *sl;
    }
}

/* Where one token (one layer, K or V) lives: the start of its page and its
 * slot there, or, for the buffer, the start of its row (pool == NULL). */
typedef struct {
    const kvxo_pool *pool;
    uint64_t base;
    uint64_t slot;
} place;

/* Token t of request r, layer l, c in {0:K, 1:V}, in a paged pool.  Returns -1
 * when the block table does not cover the token or names a page outside the
 * pool. */
static int pool_place(const kvxo_pool *p, const kvxo_batch *b, uint32_t r,
                      uint32_t l, uint32_t c, uint32_t t, place *w)
{
    uint64_t sl, sk, sp, st;
    strides(p, &sl, &sk, &sp, &st);
    uint64_t logical = t / p->page_tokens;
    uint64_t slot = t % p->page_tokens;
    uint64_t have = b->block_offsets[r + 1] - b->block_offsets[r];
    if (logical >= have) return -1;
    uint32_t page = b->block_ids[b->block_offsets[r] + logical];
    if (page >= p->num_pages) return -1;
    w->pool = p;
    w->base = l * sl + c * sk + page * sp;
    w->slot = slot;
    return 0;
}

/* Byte offset of element (head h, dim d) of the token at `w`; g gives H, D, e. */
static uint64_t elem_addr(const place *w, const kvxo_pool *g, uint32_t h, uint32_t d)
{
    uint64_t e = g->elem_bytes, D = g->head_dim;
    if (!w->pool)                                        /* buffer row [head][dim] */
        return w->base + (h * D + d) * e;
    uint64_t P = w->pool->page_tokens;
    if (w->pool->inner == 1)                             /* [head][token][dim] */
        return w->base + (h * P + w->slot) * D * e + d * e;
    if (w->pool->inner == 2) {                           /* [head][dim/x][token][x] */
        uint64_t x = 16 / e;
        return w->base + ((h * (D / x) + d / x) * P + w->slot) * 16 + (d % x) * e;
    }
    if (w->pool->inner == 3)                             /* [head][dim][token] */
        return w->base + ((h * D + d) * P + w->slot) * e;
    uint64_t sl, sk, sp, st;                             /* [token][head][dim] */
    strides(w->pool, &sl, &sk, &sp, &st);
    return w->base + w->slot * st + (h * D + d) * e;
}

static int row_contiguous(const place *w) { return !w->pool || w->pool->inner == 0; }

/* Copies one token (one layer, K or V) from `src` to `dst`. */
static void copy_token(const kvxo_pool *g, uint8_t *dst_mem, const place *dst,
                       const uint8_t *src_mem, const place *src)
{
    if (row_contiguous(dst) && row_contiguous(src)) {
        memcpy(dst_mem + elem_addr(dst, g, 0, 0), src_mem + elem_addr(src, g, 0, 0), row_bytes(g));
        return;
    }
    for (uint32_t h = 0; h < g->num_kv_heads; ++h)
        for (uint32_t d = 0; d < g->head_dim; ++d)
            memcpy(dst_mem + elem_addr(dst, g, h, d), src_mem + elem_addr(src, g, h, d), g->elem_bytes);
}

/* Tokens of all requests before r. */
static uint64_t tokens_before(const kvxo_batch *b, uint32_t r)
{
    uint64_t s = 0;
    for (uint32_t q = 0; q < r; ++q) s += b->seq_lens[q];
    return s;
}

/* The same token's row in the contiguous buffer of layers [l0,l1);
 * T_r = tokens_before(b, r), passed in so it is summed once per request. */
static uint64_t buf_addr(const kvxo_pool *p, const kvxo_batch *b, uint32_t l0, uint32_t l1,
                         uint64_t T_r, uint32_t r, uint32_t l, uint32_t c, uint32_t t)
{
    uint64_t row = row_bytes(p);
    uint64_t bytes_per_token = (uint64_t)(l1 - l0) * 2 * row;
    uint64_t n = b->seq_lens[r];
    return T_r * bytes_per_token + (((uint64_t)(l - l0) * 2 + c) * n + t) * row;
}

static int inner_ok(const kvxo_pool *p)
{
    if (p->inner > 3) return 0;
    if (p->inner && (p->stride_layer | p->stride_kv | p->stride_page | p->stride_token)) return 0;
    if (p->inner == 2 && (16 % p->elem_bytes || (p->head_dim * p->elem_bytes) % 16)) return 0;
    return 1;
}

int kvxo_total_bytes(const kvxo_pool *p, const kvxo_batch *b, uint32_t l0, uint32_t l1,
                     uint64_t *out)
{
    if (l0 > l1 || l1 > p->num_layers) return -1;
    uint64_t total = 0;
    for (uint32_t l = l0; l < l1; ++l)                 /* per layer: e * hidden * 2 * tokens */
        total += (uint64_t)p->elem_bytes * ((uint64_t)p->num_kv_heads * p->head_dim) * 2
                 * tokens_before(b, b->num_requests);
    *out = total;
    return 0;
}

int kvxo_segment(const kvxo_pool *p, const kvxo_batch *b, uint32_t l0, uint32_t l1,
                 uint32_t r, uint32_t l, uint64_t *off, uint64_t *len)
{
    if (l0 > l1 || l1 > p->num_layers || r >= b->num_requests || l < l0 || l >= l1) return -1;
    *off = buf_addr(p, b, l0, l1, tokens_before(b, r), r, l, 0, 0);
    *len = 2 * (uint64_t)b->seq_lens[r] * row_bytes(p);
    return 0;
}

int kvxo_pack(const kvxo_pool *p, const kvxo_batch *b, uint32_t l0, uint32_t l1,
              const uint8_t *pool, uint8_t *buf, int threads)
{
    if (l0 > l1 || l1 > p->num_layers || !inner_ok(p)) return -1;
    int bad = 0;
    (void)threads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads > 0 ? threads : 1) reduction(| : bad)
    for (int64_t r = 0; r < (int64_t)b->num_requests; ++r) {
        uint64_t T_r = tokens_before(b, (uint32_t)r);
        for (uint32_t l = l0; l < l1; ++l)
            for (uint32_t c = 0; c < 2; ++c)
                for (uint32_t t = 0; t < b->seq_lens[r]; ++t) {
                    place from, to = { 0, buf_addr(p, b, l0, l1, T_r, (uint32_t)r, l, c, t), 0 };
                    if (pool_place(p, b, (uint32_t)r, l, c, t, &from)) { bad = 1; continue; }
                    copy_token(p, buf, &to, pool, &from);
                }
    }
    return bad ? -1 : 0;
}

int kvxo_unpack(const kvxo_pool *p, const kvxo_batch *b, uint32_t l0, uint32_t l1,
                const uint8_t *buf, uint8_t *pool, int threads)
{
    if (l0 > l1 || l1 > p->num_layers || !inner_ok(p)) return -1;
    int bad = 0;
    (void)threads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads > 0 ? threads : 1) reduction(| : bad)
    for (int64_t r = 0; r < (int64_t)b->num_requests; ++r) {
        uint64_t T_r = tokens_before(b, (uint32_t)r);
        for (uint32_t l = l0; l < l1; ++l)
            for (uint32_t c = 0; c < 2; ++c)
                for (uint32_t t = 0; t < b->seq_lens[r]; ++t) {
                    place to, from = { 0, buf_addr(p, b, l0, l1, T_r, (uint32_t)r, l, c, t), 0 };
                    if (pool_place(p, b, (uint32_t)r, l, c, t, &to)) { bad = 1; continue; }
                    copy_token(p, pool, &to, buf, &from);
                }
    }
    return bad ? -1 : 0;
}

int kvxo_convert(const kvxo_pool *ps, const kvxo_batch *bs, const kvxo_pool *pd, const kvxo_batch *bd,
                 uint32_t l0, uint32_t l1, const uint8_t *src, uint8_t *dst, int threads)
{
    if (l0 > l1 || l1 > ps->num_layers || l1 > pd->num_layers || !inner_ok(ps) || !inner_ok(pd)) return -1;
    if (bs->num_requests != bd->num_requests || ps->num_kv_heads != pd->num_kv_heads ||
        ps->head_dim != pd->head_dim || ps->elem_bytes != pd->elem_bytes) return -1;
    int bad = 0;
    (void)threads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads > 0 ? threads : 1) reduction(| : bad)
    for (int64_t r = 0; r < (int64_t)bs->num_requests; ++r) {
        if (bs->seq_lens[r] != bd->seq_lens[r]) { bad = 1; continue; }
        for (uint32_t l = l0; l < l1; ++l)
            for (uint32_t c = 0; c < 2; ++c)
                for (uint32_t t = 0; t < bs->seq_lens[r]; ++t) {
                    place from, to;
                    if (pool_place(ps, bs, (uint32_t)r, l, c, t, &from)) { bad = 1; continue; }
                    if (pool_place(pd, bd, (uint32_t)r, l, c, t, &to)) { bad = 1; continue; }
                    copy_token(ps, dst, &to, src, &from);
                }
    }
    return bad ? -1 : 0;
}
