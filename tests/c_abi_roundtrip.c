/* A plain C caller of libkvx: builds a plan for a few requests, packs a paged pool into the contiguous
 * buffer, unpacks it into a second pool with other page ids, and checks on the host that every live token
 * row arrived where the receiver's block table says, and that nothing else was written.
 * Built and run by tests/test_gpu_c_abi.py.  Also prints what one kvx_plan / kvx_pack / kvx_unpack call
 * costs the host thread, measured without any Python in the way. */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <time.h>

#include "kvx.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP: %s (line %d)\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define CHECK_KVX(x) do { kvx_status s_ = (x); if (s_ != KVX_OK) { printf("kvx: %s (line %d)\n", kvx_status_string(s_), __LINE__); return 3; } } while (0)

static double now_us(void) {
    struct timespec t;
    clock_gettime(CLOCK_MONOTONIC, &t);
    return t.tv_sec * 1e6 + t.tv_nsec * 1e-3;
}

int main(void) {
    enum { L = 4, H = 8, D = 128, E = 2, P = 16, R = 5, NP = 200 };
    const uint32_t lens[R] = {100, 1, 0, 333, 48};
    const uint64_t row = (uint64_t)H * D * E;
    uint32_t ids_s[64], ids_d[64];
    uint64_t offs[R + 1];
    uint32_t n_ids = 0;
    offs[0] = 0;
    for (int r = 0; r < R; ++r) {
        uint32_t need = (lens[r] + P - 1) / P;
        for (uint32_t j = 0; j < need; ++j, ++n_ids) {
            ids_s[n_ids] = (n_ids * 37u + 11u) % NP; /* two different one-to-one maps into the pools */
            ids_d[n_ids] = (n_ids * 53u + 7u) % NP;
        }
        offs[r + 1] = n_ids;
    }
    kvx_pool_desc pool;
    memset(&pool, 0, sizeof pool);
    pool.num_layers = L; pool.num_kv_heads = H; pool.head_dim = D; pool.elem_bytes = E;
    pool.page_tokens = P; pool.num_pages = NP; pool.layout = KVX_LAYOUT_LAYER_MAJOR; pool.inner = KVX_INNER_TOKEN_ROWS;
    kvx_batch_desc sb = {R, 0, lens, ids_s, offs}, db = {R, 0, lens, ids_d, offs};
    const uint64_t pool_bytes = (uint64_t)L * 2 * NP * P * row;

    size_t ws_bytes = 0;
    CHECK_KVX(kvx_plan_workspace_bytes(&pool, &sb, &pool, &db, &ws_bytes));
    unsigned char *h_src = malloc(pool_bytes), *h_dst = malloc(pool_bytes);
    for (uint64_t i = 0; i < pool_bytes; ++i) h_src[i] = (unsigned char)((i * 2654435761u) >> 13);
    void *d_src, *d_dst, *d_buf, *d_ws;
    hipStream_t stream;
    CHECK_HIP(hipMalloc(&d_src, pool_bytes));
    CHECK_HIP(hipMalloc(&d_dst, pool_bytes));
    CHECK_HIP(hipMalloc(&d_ws, ws_bytes));
    CHECK_HIP(hipStreamCreate(&stream));
    CHECK_HIP(hipMemcpy(d_src, h_src, pool_bytes, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemset(d_dst, 0xC3, pool_bytes));

    kvx_plan_t *plan = NULL;
    CHECK_KVX(kvx_plan(&pool, &sb, &pool, &db, 0, L, d_ws, ws_bytes, stream, &plan));
    uint64_t total = 0;
    CHECK_KVX(kvx_plan_total_bytes(plan, &total));
    uint64_t tokens = 0;
    for (int r = 0; r < R; ++r) tokens += lens[r];
    if (total != tokens * L * 2 * row) { printf("total bytes do not follow the closed form\n"); return 1; }
    CHECK_HIP(hipMalloc(&d_buf, total));
    CHECK_KVX(kvx_pack(plan, d_src, d_buf, total, stream));
    CHECK_KVX(kvx_unpack(plan, d_buf, total, d_dst, stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    CHECK_HIP(hipMemcpy(h_dst, d_dst, pool_bytes, hipMemcpyDeviceToHost));

    /* every live row: receiver's (page, slot) holds the sender's (page, slot); count them */
    unsigned char *live = calloc(pool_bytes / row, 1);
    uint64_t checked = 0;
    for (int r = 0; r < R; ++r)
        for (uint32_t l = 0; l < L; ++l)
            for (uint32_t c = 0; c < 2; ++c)
                for (uint32_t t = 0; t < lens[r]; ++t) {
                    uint64_t ps = ids_s[offs[r] + t / P], pd = ids_d[offs[r] + t / P];
                    uint64_t rs = ((uint64_t)(l * 2 + c) * NP + ps) * P + t % P;
                    uint64_t rd = ((uint64_t)(l * 2 + c) * NP + pd) * P + t % P;
                    if (memcmp(h_dst + rd * row, h_src + rs * row, row)) { printf("row mismatch r=%d l=%u c=%u t=%u\n", r, l, c, t); return 1; }
                    live[rd] = 1;
                    ++checked;
                }
    for (uint64_t i = 0; i < pool_bytes / row; ++i)
        if (!live[i])
            for (uint64_t j = 0; j < row; ++j)
                if (h_dst[i * row + j] != 0xC3) { printf("a row outside the live slots was written\n"); return 1; }
    printf("C ABI round trip ok: %llu rows checked, %llu payload bytes\n", (unsigned long long)checked, (unsigned long long)total);

    /* host cost per call, no Python involved */
    const int iters = 2000;
    double t0 = now_us();
    for (int i = 0; i < iters; ++i) {
        kvx_plan_t *p2 = NULL;
        CHECK_KVX(kvx_plan(&pool, &sb, &pool, &db, 0, L, d_ws, ws_bytes, stream, &p2));
        kvx_plan_destroy(p2);
    }
    double t1 = now_us();
    CHECK_HIP(hipStreamSynchronize(stream));
    double t2 = now_us();
    for (int i = 0; i < iters; ++i) CHECK_KVX(kvx_pack(plan, d_src, d_buf, total, stream));
    double t3 = now_us();
    CHECK_HIP(hipStreamSynchronize(stream));
    printf("host cost per call: kvx_plan+destroy %.2f us, kvx_pack launch %.2f us\n", (t1 - t0) / iters, (t3 - t2) / iters);
    kvx_plan_destroy(plan);
    return 0;
}
