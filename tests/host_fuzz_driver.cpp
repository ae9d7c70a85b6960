// Host-only fuzz driver for the validation and plan arithmetic of libkvx, built with
// AddressSanitizer and UndefinedBehaviorSanitizer on the host side (tests/test_host_sanitizers.py).
// It never launches a kernel: every plan is host-only (no device workspace), and the ones that could launch
// all the same (small one-sided plans, whose run records the host builds) are only inspected.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "kvx.h"
#include "kvx_internal.h"

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd() {
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return state;
}
static uint32_t below(uint32_t n) { return n ? (uint32_t)(rnd() % n) : 0; }

// The multiply-shift division the data movers use for their tile indices, against the plain quotient.
static int check_fast_div() {
    const uint32_t edge[] = {0u, 1u, 2u, 3u, 7u, 8u, 9u, 255u, 256u, 65535u, 65536u, 0x7FFFFFFFu, 0x80000000u,
                             0x80000001u, 0xFFFFFFFEu, 0xFFFFFFFFu};
    for (uint32_t d : edge) {
        if (!d) continue;
        const kvx::FastDiv f = kvx::make_fast_div(d);
        for (uint32_t n : edge)
            if (kvx::fast_div(n, f) != n / d) { printf("fast_div(%u, %u) is wrong\n", n, d); return 1; }
    }
    for (int i = 0; i < 2000000; ++i) {
        uint32_t d = (uint32_t)rnd() >> below(32), n = (uint32_t)rnd() >> below(32);
        if (!d) d = 1;
        const kvx::FastDiv f = kvx::make_fast_div(d);
        if (kvx::fast_div(n, f) != n / d || kvx::fast_div(n - n % d, f) != n / d ||
            (n / d && kvx::fast_div(n - n % d - 1, f) != n / d - 1)) {
            printf("fast_div(%u, %u) is wrong\n", n, d);
            return 1;
        }
    }
    return 0;
}

int main(int argc, char **argv) {
    const int iters = argc > 1 ? atoi(argv[1]) : 20000;
    int devices = 0;
    if (hipGetDeviceCount(&devices) == hipSuccess && devices > 0) {
        // the calls below hand host addresses to entry points that would launch with them
        printf("a GPU is present: this driver only runs where nothing can be launched\n");
        return 77;
    }
    if (check_fast_div()) return 1;
    long ok = 0, rejected = 0, inline_plans = 0;
    for (int it = 0; it < iters; ++it) {
        kvx_pool_desc s{}, d{};
        const uint32_t elems[] = {1, 2, 4, 3, 8};
        s.num_layers = 1 + below(8);
        s.num_kv_heads = below(20) == 0 ? 0 : 1 + below(8);
        s.head_dim = 8u << below(5);
        s.elem_bytes = elems[below(5)];
        s.page_tokens = below(30) == 0 ? 0 : 1 + below(40);
        s.num_pages = 1 + below(300);
        s.layout = below(12) == 0 ? 5 : below(2);
        s.inner = below(15) == 0 ? 4 : below(4);
        d = s;
        d.page_tokens = 1 + below(40);
        d.num_pages = 1 + below(300);
        d.layout = below(2);
        d.inner = below(4);
        if (below(10) == 0) d.head_dim *= 2;
        if (below(10) == 0) { // explicit strides, sometimes inconsistent
            const uint64_t row = (uint64_t)s.num_kv_heads * s.head_dim * s.elem_bytes;
            s.stride_token = row + 16 * below(3) - (below(8) == 0 ? 8 : 0);
            s.stride_page = s.stride_token * s.page_tokens + 32 * below(2);
            s.stride_kv = s.stride_page * s.num_pages;
            s.stride_layer = below(9) == 0 ? 0 : 2 * s.stride_kv;
        }
        if (below(10) == 0) { // a receiver with explicit strides, nested or (now and then) aliasing
            const uint64_t row = (uint64_t)d.num_kv_heads * d.head_dim * d.elem_bytes;
            d.inner = 0;
            d.stride_token = row + 16 * below(3);
            d.stride_page = d.stride_token * d.page_tokens + 32 * below(2) - (below(6) == 0 ? 16 : 0);
            d.stride_kv = d.stride_page * (d.num_pages - (below(6) == 0 ? 1 : 0));
            d.stride_layer = (below(6) == 0 ? 1 : 2) * d.stride_kv;
            if (!d.stride_kv) d.stride_kv = d.stride_layer = 16;
        }
        const uint32_t R = below(7);
        std::vector<uint32_t> lens(R), ids_s, ids_d;
        std::vector<uint64_t> offs_s(R + 1, 0), offs_d(R + 1, 0);
        for (uint32_t r = 0; r < R; ++r) {
            lens[r] = below(5) == 0 ? 0 : below(400);
            const uint32_t ps = s.page_tokens ? s.page_tokens : 1, pd = d.page_tokens;
            uint32_t ns = (lens[r] + ps - 1) / ps + below(3), nd = (lens[r] + pd - 1) / pd + below(3);
            if (below(25) == 0 && ns) --ns; // too short now and then
            if (below(25) == 0 && nd) --nd;
            for (uint32_t j = 0; j < ns; ++j) ids_s.push_back(below(s.num_pages + (below(40) == 0 ? 3 : 0)));
            for (uint32_t j = 0; j < nd; ++j) ids_d.push_back(below(d.num_pages + (below(40) == 0 ? 3 : 0)));
            offs_s[r + 1] = ids_s.size();
            offs_d[r + 1] = ids_d.size();
        }
        kvx_batch_desc sb{R, 0, lens.data(), ids_s.data(), offs_s.data()};
        kvx_batch_desc db{R, 0, lens.data(), ids_d.data(), offs_d.data()};
        const uint32_t l0 = below(s.num_layers + 1), l1 = below(s.num_layers + 2);
        const int mode = below(3);
        size_t ws = 0;
        (void)kvx_plan_workspace_bytes(mode != 1 ? &s : nullptr, mode != 1 ? &sb : nullptr,
                                       mode != 0 ? &d : nullptr, mode != 0 ? &db : nullptr, &ws);
        kvx_plan_t *plan = nullptr;
        kvx_status st = kvx_plan(mode != 1 ? &s : nullptr, mode != 1 ? &sb : nullptr, mode != 0 ? &d : nullptr,
                                 mode != 0 ? &db : nullptr, l0, l1, nullptr, 0, nullptr, &plan);
        if (mode == 1) {
            // The entry point that allocates nothing runs the same checks on a code path of its own.  What
            // kvx_plan refuses for a receiver it must refuse too; what kvx_plan accepts it may only turn
            // down for its own limits, or (with no device here) at its first HIP call.
            const kvx_status sn = kvx_unpack_noalloc(&d, &db, l0, l1, lens.data(), 1ull << 40, &d, nullptr);
            if (st != KVX_OK && (sn == KVX_OK || sn == KVX_ERR_DEVICE)) {
                printf("noalloc got past what kvx_plan refused (%d vs %d)\n", (int)st, (int)sn);
                return 1;
            }
            if (st == KVX_OK && sn != KVX_OK && sn != KVX_ERR_DEVICE && sn != KVX_ERR_ALIGNMENT &&
                sn != KVX_ERR_CAPACITY && sn != KVX_ERR_INVALID_ARG) {
                printf("noalloc refused what kvx_plan accepted (%d)\n", (int)sn);
                return 1;
            }
        }
        if (st != KVX_OK) {
            if (plan) { printf("plan returned on failure\n"); return 1; }
            (void)kvx_status_string(st);
            ++rejected;
            continue;
        }
        ++ok;
        uint64_t total = 0, off = 0, len = 0, sum = 0;
        if (kvx_plan_total_bytes(plan, &total) != KVX_OK) return 1;
        for (uint32_t r = 0; r < R; ++r) {
            if (kvx_plan_request_segment(plan, r, &off, &len) != KVX_OK || off != sum) {
                printf("request segments do not tile the buffer\n");
                return 1;
            }
            uint64_t inner = off;
            for (uint32_t l = l0; l < l1; ++l) {
                uint64_t o2, n2;
                if (kvx_plan_segment(plan, r, l, &o2, &n2) != KVX_OK || o2 != inner) {
                    printf("layer segments do not tile the request\n");
                    return 1;
                }
                inner += n2;
            }
            if (inner != off + len) { printf("layer segments do not fill the request\n"); return 1; }
            sum += len;
        }
        if (sum != total) { printf("segments do not add up to the total\n"); return 1; }
        (void)kvx_plan_segment(plan, R, l0, &off, &len);
        kvx_launch_cfg cfg{};
        cfg.unroll = below(10);
        cfg.threads = 64u << below(6);
        (void)kvx_plan_set_launch(plan, &cfg);
        int can = 0;
        if (kvx_plan_can_launch(plan, &can) != KVX_OK) return 1;
        if (can) {
            // one side, token rows, few pages: the host worked the run records out itself.  Every token of every
            // request must lie in exactly the record its page gives it, at the addresses the geometry defines.
            if (mode == 2 || !plan->inline_runs) { printf("a plan without run records says it can launch\n"); return 1; }
            ++inline_plans;
            const kvx::Geometry &g = mode == 0 ? plan->s : plan->d;
            const std::vector<uint32_t> &ids = mode == 0 ? ids_s : ids_d;
            const std::vector<uint64_t> &offs = mode == 0 ? offs_s : offs_d;
            const uint32_t P = g.desc.page_tokens;
            const uint64_t row = plan->row, bpt = 2ull * (l1 - l0) * row;
            uint64_t first = 0, tokens_before = 0;
            for (uint32_t r = 0; r < R; ++r) {
                for (uint32_t t = 0; t < lens[r]; ++t) {
                    const kvx_run &run = plan->inline_runs->run[first + t / P];
                    const uint64_t pool = mode == 0 ? run.src_off : run.dst_off, buf = mode == 0 ? run.dst_off : run.src_off;
                    const uint64_t in_run = (uint64_t)(t - run.token) * row;
                    if (run.request != r || run.seq_len != lens[r] || run.token > t || in_run + row > run.bytes ||
                        run.token / P != t / P ||
                        pool + in_run != ids[offs[r] + t / P] * g.sp + (uint64_t)(t % P) * g.token_step ||
                        buf + in_run != tokens_before * bpt + (uint64_t)t * row) {
                        printf("host-built run record is wrong (request %u token %u)\n", r, t);
                        return 1;
                    }
                }
                first += (lens[r] + P - 1) / P;
                tokens_before += lens[r];
            }
            if (first == 0 || first > KVX_INLINE_RUNS) { printf("run records for %llu pages\n", (unsigned long long)first); return 1; }
            // a run ends with its page or its request: no two records may claim the same token
            for (uint64_t i = 0; i < first; ++i) {
                const kvx_run &run = plan->inline_runs->run[i];
                if (run.bytes == 0 || run.bytes % row || run.token % P || run.token + run.bytes / row > run.seq_len ||
                    run.bytes / row > P) { printf("host-built run %llu has a bad extent\n", (unsigned long long)i); return 1; }
            }
        } else if (kvx_pack(plan, &s, &d, total, nullptr) == KVX_OK && total) {
            // (a plan that can launch is never handed these host addresses)
            printf("host-only plan launched\n");
            return 1;
        }
        kvx_plan_destroy(plan);
    }
    printf("fuzz done: %ld plans accepted (%ld with host-built runs), %ld rejected\n", ok, inline_plans, rejected);
    return ok > 100 && rejected > 100 && inline_plans > 20 ? 0 : 2;
}
