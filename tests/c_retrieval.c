/* Asynchronous retrieval (paper section 3.6) driven from plain C, no Python in the loop: requests arrive one
 * after another (or a few at a time), each is gathered out of the sender's pool into a free receive slot
 * (sender plan + kvx_pack on the slot's stream, standing in for the bytes arriving), scattered from there
 * into the receiver's pool (kvx_retriever_scatter), and reported by kvx_retriever_poll.  Arrivals of at most
 * KVX_INLINE_RUNS pages are planned on the host on both sides: one launch to gather, one to scatter.  Prints the host
 * wall time per request for every (slots, requests per arrival) pair asked for, and checks rows of the
 * receiver's pool against the sender's through both block tables.
 *
 *   c_retrieval R L H D E P  k1,k2,...  g1,g2,...  [check_every]
 *
 * R requests of 32..512 tokens, L layers, H heads, D head_dim, E elem_bytes, P tokens per page.
 * Built and run by tests/test_gpu_c_retrieval.py. */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

#include "kvx.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP: %s (line %d)\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define CHECK_KVX(x) do { kvx_status s_ = (x); if (s_ != KVX_OK) { printf("kvx: %s (line %d)\n", kvx_status_string(s_), __LINE__); return 3; } } while (0)

static uint64_t rng_state = 0x2408081470000001ull;
static uint32_t rnd(void) {
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 16);
}
static double now_us(void) {
    struct timespec t;
    clock_gettime(CLOCK_MONOTONIC, &t);
    return t.tv_sec * 1e6 + t.tv_nsec * 1e-3;
}
static void shuffle(uint32_t *a, uint32_t n) {
    for (uint32_t i = n; i > 1; --i) {
        uint32_t j = rnd() % i, t = a[i - 1];
        a[i - 1] = a[j];
        a[j] = t;
    }
}
static int parse_list(const char *s, uint32_t *out, int cap) {
    int n = 0;
    while (*s && n < cap) {
        out[n++] = (uint32_t)strtoul(s, (char **)&s, 10);
        if (*s == ',') ++s;
    }
    return n;
}

enum { PATTERN_BYTES = 64u << 20 };

int main(int argc, char **argv) {
    if (argc < 9) { printf("usage: c_retrieval R L H D E P k-list g-list [check_every]\n"); return 64; }
    const uint32_t R = atoi(argv[1]), L = atoi(argv[2]), H = atoi(argv[3]), D = atoi(argv[4]), E = atoi(argv[5]),
                   P = atoi(argv[6]);
    uint32_t ks[8], gs[8];
    const int nk = parse_list(argv[7], ks, 8), ng = parse_list(argv[8], gs, 8);
    const uint32_t check_every = argc > 9 ? atoi(argv[9]) : 1;
    const uint64_t row = (uint64_t)H * D * E;

    uint32_t *lens = malloc(4 * R);
    uint64_t *offs = malloc(8 * (R + 1));
    uint64_t used = 0, tokens = 0;
    offs[0] = 0;
    for (uint32_t r = 0; r < R; ++r) {
        lens[r] = 32 + rnd() % 481;
        used += (lens[r] + P - 1) / P;
        tokens += lens[r];
        offs[r + 1] = used;
    }
    const uint32_t NP = (uint32_t)(2 * used);
    uint32_t *perm_s = malloc(4 * NP), *perm_d = malloc(4 * NP);
    for (uint32_t i = 0; i < NP; ++i) perm_s[i] = perm_d[i] = i;
    shuffle(perm_s, NP);
    shuffle(perm_d, NP); /* the first `used` entries are the block tables, dealt to the requests in order */
    kvx_pool_desc pool;
    memset(&pool, 0, sizeof pool);
    pool.num_layers = L; pool.num_kv_heads = H; pool.head_dim = D; pool.elem_bytes = E;
    pool.page_tokens = P; pool.num_pages = NP; pool.layout = KVX_LAYOUT_LAYER_MAJOR; pool.inner = KVX_INNER_TOKEN_ROWS;
    const uint64_t pool_bytes = (uint64_t)L * 2 * NP * P * row;
    const uint64_t bpt = (uint64_t)L * 2 * row;
    printf("retrieval from C: %u requests, %llu tokens, %.2f GB payload, pools of %.2f GB\n", R,
           (unsigned long long)tokens, tokens * bpt / 1e9, pool_bytes / 1e9);

    /* sender pool: a host pattern repeated, so that a row's bytes depend on where it lives */
    unsigned char *pattern = malloc(PATTERN_BYTES);
    for (uint64_t i = 0; i < PATTERN_BYTES; i += 4) { uint32_t v = rnd(); memcpy(pattern + i, &v, 4); }
    char *d_src, *d_dst;
    CHECK_HIP(hipMalloc((void **)&d_src, pool_bytes));
    CHECK_HIP(hipMalloc((void **)&d_dst, pool_bytes));
    for (uint64_t o = 0; o < pool_bytes; o += PATTERN_BYTES)
        CHECK_HIP(hipMemcpy(d_src + o, pattern, pool_bytes - o < PATTERN_BYTES ? pool_bytes - o : PATTERN_BYTES,
                            hipMemcpyHostToDevice));

    for (int gi = 0; gi < ng; ++gi)
        for (int ki = 0; ki < nk; ++ki) {
            const uint32_t k = ks[ki], g = gs[gi];
            /* arrivals: groups of g consecutive requests; a slot must hold the largest group */
            const uint32_t arrivals = (R + g - 1) / g;
            uint64_t slot_buf = 0, slot_ws = 0;
            for (uint32_t a = 0; a < arrivals; ++a) {
                const uint32_t r0 = a * g, r1 = r0 + g < R ? r0 + g : R;
                uint64_t t = 0;
                for (uint32_t r = r0; r < r1; ++r) t += lens[r];
                if (t * bpt > slot_buf) slot_buf = t * bpt;
                kvx_batch_desc b = {r1 - r0, 0, lens + r0, perm_d + offs[r0], NULL};
                uint64_t *o = malloc(8 * (r1 - r0 + 1));
                for (uint32_t r = r0; r <= r1; ++r) o[r - r0] = offs[r] - offs[r0];
                b.block_offsets = o;
                size_t ws = 0;
                CHECK_KVX(kvx_plan_workspace_bytes(&pool, &b, &pool, &b, &ws));
                if (ws > slot_ws) slot_ws = ws;
                free(o);
            }
            uint64_t arena_bytes = 0;
            CHECK_KVX(kvx_retriever_arena_bytes(k, slot_buf, slot_ws, &arena_bytes));
            char *d_arena, *d_send_ws;
            CHECK_HIP(hipMalloc((void **)&d_arena, arena_bytes));
            CHECK_HIP(hipMalloc((void **)&d_send_ws, (uint64_t)k * ((slot_ws + 255) / 256 * 256)));
            CHECK_HIP(hipMemset(d_dst, 0xC3, pool_bytes));
            CHECK_HIP(hipDeviceSynchronize());
            kvx_retriever_t *ret = NULL;
            CHECK_KVX(kvx_retriever_create(k, slot_buf, slot_ws, d_arena, arena_bytes, &ret));
            uint64_t *group_offs = malloc(8 * (g + 1));
            uint64_t tickets[64];
            double wall = 0;
            for (int timed = 0; timed < 2; ++timed) { /* the first pass warms up; results are the same bytes */
                uint32_t next = 0, done = 0;
                const double t0 = now_us();
                while (done < arrivals) {
                    uint32_t n = 0;
                    CHECK_KVX(kvx_retriever_poll(ret, tickets, 64, &n));
                    done += n;
                    while (next < arrivals) {
                        const uint32_t r0 = next * g, r1 = r0 + g < R ? r0 + g : R;
                        uint64_t t = 0;
                        for (uint32_t r = r0; r < r1; ++r) t += lens[r];
                        uint32_t slot;
                        void *buf, *stream;
                        kvx_status st = kvx_retriever_acquire(ret, next, t * bpt, &slot, &buf, &stream);
                        if (st == KVX_ERR_BUSY) break;
                        CHECK_KVX(st);
                        for (uint32_t r = r0; r <= r1; ++r) group_offs[r - r0] = offs[r] - offs[r0];
                        kvx_batch_desc sb = {r1 - r0, 0, lens + r0, perm_s + offs[r0], group_offs};
                        kvx_batch_desc db = {r1 - r0, 0, lens + r0, perm_d + offs[r0], group_offs};
                        kvx_plan_t *plan = NULL;
                        uint64_t pages = offs[r1] - offs[r0];
                        int runs_inline = 0;
                        if (pages <= KVX_INLINE_RUNS) { /* planned on the host: the pack is the only launch */
                            CHECK_KVX(kvx_plan(&pool, &sb, NULL, NULL, 0, L, NULL, 0, stream, &plan));
                            CHECK_KVX(kvx_plan_can_launch(plan, &runs_inline));
                            if (!runs_inline) kvx_plan_destroy(plan);
                        }
                        if (!runs_inline)
                            CHECK_KVX(kvx_plan(&pool, &sb, NULL, NULL, 0, L,
                                               d_send_ws + (uint64_t)slot * ((slot_ws + 255) / 256 * 256), slot_ws, stream,
                                               &plan));
                        CHECK_KVX(kvx_pack(plan, d_src, buf, slot_buf, stream));
                        kvx_plan_destroy(plan);
                        CHECK_KVX(kvx_retriever_scatter(ret, slot, &pool, &db, 0, L, d_dst, NULL));
                        ++next;
                    }
                }
                CHECK_KVX(kvx_retriever_drain(ret));
                CHECK_HIP(hipDeviceSynchronize());
                wall = now_us() - t0;
            }
            kvx_retriever_destroy(ret);
            free(group_offs);
            printf("slots %2u, requests per arrival %3u: %8.2f us per request, %7.1f GB/s moved (pack + unpack)\n", k, g,
                   wall / R, 2.0 * tokens * bpt / wall / 1e3);
            CHECK_HIP(hipFree(d_arena));
            CHECK_HIP(hipFree(d_send_ws));
        }

    /* rows of the receiver against rows of the sender, through both block tables: for every check_every-th
     * request, its first and last token, in the first and last layer, K and V */
    unsigned char *a = malloc(row), *b = malloc(row);
    uint64_t checked = 0;
    for (uint32_t r = 0; r < R; r += check_every) {
        const uint32_t ts[2] = {0, lens[r] - 1}, ls[2] = {0, L - 1};
        for (int ti = 0; ti < 2; ++ti)
            for (int li = 0; li < 2; ++li)
                for (uint32_t c = 0; c < 2; ++c) {
                    const uint32_t t = ts[ti], l = ls[li];
                    const uint64_t ps = perm_s[offs[r] + t / P], pd = perm_d[offs[r] + t / P];
                    const uint64_t os = (((uint64_t)(l * 2 + c) * NP + ps) * P + t % P) * row;
                    const uint64_t od = (((uint64_t)(l * 2 + c) * NP + pd) * P + t % P) * row;
                    CHECK_HIP(hipMemcpy(b, d_dst + od, row, hipMemcpyDeviceToHost));
                    for (uint64_t i = 0; i < row; ++i) a[i] = pattern[(os + i) % PATTERN_BYTES];
                    if (memcmp(a, b, row)) { printf("row mismatch r=%u l=%u c=%u t=%u\n", r, l, c, t); return 1; }
                    ++checked;
                }
    }
    /* pages no request was given keep their canary */
    for (uint32_t i = used; i < NP && i < used + 64; ++i) {
        CHECK_HIP(hipMemcpy(b, d_dst + (uint64_t)perm_d[i] * P * row, row, hipMemcpyDeviceToHost));
        for (uint64_t j = 0; j < row; ++j)
            if (b[j] != 0xC3) { printf("an unlisted page was written\n"); return 1; }
    }
    printf("retrieval ok: %llu rows checked\n", (unsigned long long)checked);
    return 0;
}
