// Host side of libkvx: argument validation, plan construction, launches.
// The operations and their layout conventions are stated in include/kvx.h
// (paper section 3.6, "Block-free D2D KVCache Transfer").
#include <algorithm>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <numeric>
#include <vector>

#include "kvx_internal.h"

using namespace kvx;

namespace {
thread_local int g_last_hip_error = 0;
thread_local const char *g_last_hip_where = "";
} // namespace

void kvx::note_device_error(hipError_t e, const char *where) {
    g_last_hip_error = (int)e;
    g_last_hip_where = where;
}

namespace {

// Pinned staging blocks are costly to create, so destroyed plans hand theirs
// back to a small free list instead of freeing them.  A block carries an event
// recorded behind the H2D copy that reads it; it is handed out again, or freed,
// only once that event has completed, so a plan destroyed with work still
// queued never has its staged tables overwritten or unmapped before they were
// copied.  Freeing and re-creating a block costs about a millisecond, so the
// list is trimmed with hysteresis: once it holds more than 2 * kPinnedKeep
// blocks, those whose copies are done are freed down to kPinnedKeep.
// kvx_release_cached frees every idle block on request.
constexpr size_t kPinnedKeep = 32;
std::mutex g_pinned_mu;
std::vector<PinnedBlock> g_pinned_free;

void pinned_free_block(const PinnedBlock &b) {
    (void)hipHostFree(b.ptr);
    (void)hipEventDestroy(b.copied);
}

hipError_t pinned_acquire(size_t bytes, PinnedBlock *out) {
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    {
        std::lock_guard<std::mutex> lk(g_pinned_mu);
        for (size_t i = 0; i < g_pinned_free.size(); ++i) {
            if (g_pinned_free[i].device == device && g_pinned_free[i].bytes >= bytes &&
                g_pinned_free[i].bytes <= 4 * bytes + 4096 &&
                hipEventQuery(g_pinned_free[i].copied) == hipSuccess) {
                *out = g_pinned_free[i];
                g_pinned_free.erase(g_pinned_free.begin() + i);
                return hipSuccess;
            }
        }
    }
    size_t cap = std::max<size_t>(align_up(bytes, 4096), 4096);
    void *p = nullptr;
    e = hipHostMalloc(&p, cap, hipHostMallocDefault);
    if (e != hipSuccess) return e;
    hipEvent_t ev = nullptr;
    e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
    if (e != hipSuccess) {
        (void)hipHostFree(p);
        return e;
    }
    out->ptr = p;
    out->bytes = cap;
    out->copied = ev;
    out->device = device;
    return hipSuccess;
}

// Frees listed blocks whose copies have completed, oldest first, until at most `keep` such blocks are left.
// Blocks still being read stay listed whatever `keep` says.  Returns the bytes freed.  Caller holds the lock.
uint64_t pinned_trim(size_t keep) {
    size_t done = 0;
    for (const PinnedBlock &b : g_pinned_free)
        if (hipEventQuery(b.copied) == hipSuccess) ++done;
    uint64_t freed = 0;
    size_t w = 0;
    for (size_t i = 0; i < g_pinned_free.size(); ++i) {
        // a block that completed between the two queries is only kept a little longer
        if (done > keep && hipEventQuery(g_pinned_free[i].copied) == hipSuccess) {
            freed += g_pinned_free[i].bytes;
            pinned_free_block(g_pinned_free[i]);
            --done;
        } else {
            g_pinned_free[w++] = g_pinned_free[i];
        }
    }
    g_pinned_free.resize(w);
    return freed;
}

void pinned_release(PinnedBlock b) {
    if (!b.ptr) return;
    std::lock_guard<std::mutex> lk(g_pinned_mu);
    g_pinned_free.push_back(b);
    if (g_pinned_free.size() > 2 * kPinnedKeep) (void)pinned_trim(kPinnedKeep);
}

} // namespace

namespace kvx {

// Explicit strides of a pool that is written: the four axes (token, page, K|V, layer) must nest, every
// stride at least the extent of everything that lies inside it, so that no two rows share a byte.  An axis
// of extent 1 has no say.
static bool strides_nest(const kvx_pool_desc *d, uint64_t row) {
    struct Axis { uint64_t stride, extent; };
    Axis ax[4] = {{d->stride_token, d->page_tokens}, {d->stride_page, d->num_pages}, {d->stride_kv, 2},
                  {d->stride_layer, d->num_layers}};
    std::sort(ax, ax + 4, [](const Axis &a, const Axis &b) { return a.stride < b.stride; });
    unsigned __int128 inner = row; // bytes covered by everything inside the axis being looked at
    for (const Axis &a : ax) {
        if (a.extent == 1) continue;
        if ((unsigned __int128)a.stride < inner) return false;
        inner = (unsigned __int128)a.stride * (a.extent - 1) + inner;
    }
    return true;
}

kvx_status resolve_pool(const kvx_pool_desc *d, bool receiver, Geometry *g) {
    if (!d->num_layers || !d->num_kv_heads || !d->head_dim || !d->elem_bytes || !d->page_tokens ||
        !d->num_pages || d->inner > KVX_INNER_TOKEN_INNERMOST)
        return KVX_ERR_INVALID_ARG;
    g->present = true;
    g->desc = *d;
    const uint64_t row = (uint64_t)d->num_kv_heads * d->head_dim * d->elem_bytes;
    if (row % 16) return KVX_ERR_ALIGNMENT;
    if (row * d->page_tokens >= (1ull << 32)) return KVX_ERR_UNSUPPORTED;
    g->row = row;
    const bool any = d->stride_layer || d->stride_kv || d->stride_page || d->stride_token;
    if (d->inner != KVX_INNER_TOKEN_ROWS) {
        const uint64_t head_bytes = (uint64_t)d->head_dim * d->elem_bytes;
        if (any) return KVX_ERR_INVALID_ARG;
        if (d->inner == KVX_INNER_TOKEN_INNERMOST) {
            if (d->elem_bytes != 1 && d->elem_bytes != 2 && d->elem_bytes != 4 && d->elem_bytes != 8)
                return KVX_ERR_INVALID_ARG;
        } else if (head_bytes % 16) {
            return KVX_ERR_ALIGNMENT;
        }
        if (d->inner == KVX_INNER_DIM_SPLIT_TOKEN && 16 % d->elem_bytes) return KVX_ERR_INVALID_ARG;
    }
    if (any) {
        if (!d->stride_layer || !d->stride_kv || !d->stride_page || !d->stride_token)
            return KVX_ERR_INVALID_ARG;
        if ((d->stride_layer | d->stride_kv | d->stride_page | d->stride_token) % 16)
            return KVX_ERR_ALIGNMENT;
        if (d->stride_token < row) return KVX_ERR_INVALID_ARG;
        if (receiver && !strides_nest(d, row)) return KVX_ERR_INVALID_ARG;
        g->custom_strides = true;
        g->sl = d->stride_layer;
        g->sk = d->stride_kv;
        g->sp = d->stride_page;
        g->st = d->stride_token;
    } else if (d->layout == KVX_LAYOUT_LAYER_MAJOR) {
        g->st = row;
        g->sp = row * d->page_tokens;
        g->sk = g->sp * d->num_pages;
        g->sl = 2 * g->sk;
    } else if (d->layout == KVX_LAYOUT_PAGE_MAJOR) {
        g->st = row;
        g->sk = row * d->page_tokens;
        g->sl = 2 * g->sk;
        g->sp = g->sl * d->num_layers;
    } else {
        return KVX_ERR_INVALID_ARG;
    }
    // Inside a page every arrangement is affine in the slot, so a run may span a whole page; only pages
    // whose rows are back to back can be moved as flat bytes, the others go through the tile kernel.
    g->quantum = d->page_tokens;
    g->dense_rows = (d->inner == KVX_INNER_TOKEN_ROWS && g->st == row);
    if (!g->dense_rows && row / 16 >= 65536) return KVX_ERR_UNSUPPORTED;
    g->token_step = g->st;
    g->upg = (uint32_t)(row / 16);
    if (d->inner == KVX_INNER_HEAD_MAJOR) {
        const uint64_t head_bytes = (uint64_t)d->head_dim * d->elem_bytes;
        g->token_step = head_bytes;
        g->upg = (uint32_t)(head_bytes / 16);
        g->granule_step = head_bytes * d->page_tokens;
    } else if (d->inner == KVX_INNER_DIM_SPLIT_TOKEN) {
        g->token_step = 16;
        g->upg = 1;
        g->granule_step = 16ull * d->page_tokens;
        g->token_fast = true;
    } else if (d->inner == KVX_INNER_TOKEN_INNERMOST) {
        g->token_step = d->elem_bytes;
        g->token_innermost = true;
        g->column_step = d->page_tokens * d->elem_bytes; // below 2^32: page_tokens * row is
    }
    // last byte of the last row, one past: pages of every arrangement hold page_tokens * row bytes
    {
        const unsigned __int128 span = (unsigned __int128)(d->num_layers - 1) * g->sl + g->sk +
                                       (unsigned __int128)(d->num_pages - 1) * g->sp +
                                       (g->custom_strides ? (unsigned __int128)(d->page_tokens - 1) * g->st + row
                                                          : (unsigned __int128)d->page_tokens * row);
        if (span >> 63) return KVX_ERR_UNSUPPORTED;
        g->span = (uint64_t)span;
    }
    return KVX_OK;
}

kvx_status check_batch_shape(const kvx_batch_desc *b) {
    if (b->reserved) return KVX_ERR_INVALID_ARG;
    if (!b->block_offsets) return KVX_ERR_INVALID_ARG;
    if (b->num_requests && !b->seq_lens) return KVX_ERR_INVALID_ARG;
    if (b->block_offsets[0] != 0) return KVX_ERR_BLOCK_TABLE;
    for (uint32_t r = 0; r < b->num_requests; ++r)
        if (b->block_offsets[r + 1] < b->block_offsets[r]) return KVX_ERR_BLOCK_TABLE;
    if (b->block_offsets[b->num_requests] && !b->block_ids) return KVX_ERR_INVALID_ARG;
    return KVX_OK;
}

} // namespace kvx

namespace {

// Checks one side's block tables against its pool and gathers the ids that
// are actually used (the first ceil(n/P) of each request) into `compact`.
kvx_status check_tables(const Geometry &g, const kvx_batch_desc *b, bool receiver,
                        std::vector<uint32_t> *compact, uint64_t *used_pages) {
    const uint32_t P = g.desc.page_tokens;
    uint64_t used = 0;
    for (uint32_t r = 0; r < b->num_requests; ++r) {
        const uint64_t need = ((uint64_t)b->seq_lens[r] + P - 1) / P;
        if (need > b->block_offsets[r + 1] - b->block_offsets[r]) return KVX_ERR_BLOCK_TABLE;
        used += need;
    }
    if (compact) compact->reserve(used);
    std::vector<uint64_t> seen;
    if (receiver) seen.assign(((uint64_t)g.desc.num_pages + 63) / 64, 0);
    for (uint32_t r = 0; r < b->num_requests; ++r) {
        const uint64_t need = ((uint64_t)b->seq_lens[r] + P - 1) / P;
        const uint32_t *ids = b->block_ids + b->block_offsets[r];
        for (uint64_t j = 0; j < need; ++j) {
            const uint32_t id = ids[j];
            if (id >= g.desc.num_pages) return KVX_ERR_BLOCK_TABLE;
            if (receiver) {
                uint64_t &w = seen[id >> 6];
                const uint64_t bit = 1ull << (id & 63);
                if (w & bit) return KVX_ERR_BLOCK_TABLE;
                w |= bit;
            }
            if (compact) compact->push_back(id);
        }
    }
    *used_pages = used;
    return KVX_OK;
}

uint64_t ceil_div_q(uint64_t x, uint64_t q) {
    if (q == 0) return x ? 1 : 0;
    return (x + q - 1) / q;
}

uint64_t lcm_q(uint32_t a, uint32_t b) {
    if (a == 0 || b == 0) return 0;
    return (uint64_t)a / std::gcd(a, b) * b;
}

} // namespace

void kvx::shape_ops(const Geometry &s, const Geometry &d, const uint32_t *seq_lens, uint32_t R,
                    OpShape ops[NUM_OPS]) {
    if (s.present) {
        ops[OP_PACK].planned = true;
        ops[OP_PACK].qa = s.quantum;
        ops[OP_PACK].qb = 0;
    }
    if (d.present) {
        ops[OP_UNPACK].planned = true;
        ops[OP_UNPACK].qa = 0;
        ops[OP_UNPACK].qb = d.quantum;
    }
    if (s.present && d.present) {
        ops[OP_CONVERT].planned = true;
        ops[OP_CONVERT].qa = s.quantum;
        ops[OP_CONVERT].qb = d.quantum;
    }
    const uint64_t row = s.present ? s.row : d.row;
    for (int op = 0; op < (int)NUM_OPS; ++op) {
        OpShape &o = ops[op];
        if (!o.planned) continue;
        o.lcm = lcm_q(o.qa, o.qb);
        uint64_t q = o.qa && o.qb ? std::min(o.qa, o.qb) : std::max(o.qa, o.qb);
        o.max_run_bytes = (uint32_t)(q * row);
        uint64_t runs = 0;
        if (op == OP_CONVERT) {
            // One group per page of the coarser side, each with room for the most runs a group can hold.
            const uint32_t coarse = std::max(o.qa, o.qb), fine = std::min(o.qa, o.qb);
            o.group_quantum = coarse;
            o.group_slots = coarse % fine == 0 ? coarse / fine : coarse / fine + 2;
            for (uint32_t r = 0; r < R; ++r)
                runs += ((uint64_t)seq_lens[r] + coarse - 1) / coarse * o.group_slots;
        } else {
            for (uint32_t r = 0; r < R; ++r) {
                const uint64_t n = seq_lens[r];
                if (n) runs += ceil_div_q(n, o.qa) + ceil_div_q(n, o.qb) - ceil_div_q(n, o.lcm);
            }
        }
        o.num_runs = runs;
    }
}

void kvx::layout_workspace(Sizing *z, uint64_t used_s, uint64_t used_d) {
    uint64_t off = 0;
    z->off_lens = off;
    off = align_up(off + 4ull * z->R);
    z->off_ids_s = off;
    off = align_up(off + 4ull * used_s);
    z->off_ids_d = off;
    off = align_up(off + 4ull * used_d);
    z->staging_bytes = off;
    for (int k = 0; k < kNumScans; ++k) {
        z->off_prefix[k] = off;
        off = align_up(off + 8ull * (z->R + 1ull));
    }
    for (int op = 0; op < (int)NUM_OPS; ++op) {
        z->off_runs[op] = off;
        off = align_up(off + sizeof(kvx_run) * z->ops[op].num_runs);
    }
    z->total_bytes = std::max<uint64_t>(off, kAlign);
}

namespace {

kvx_status check_sides(const kvx_pool_desc *s, const kvx_batch_desc *sb, const kvx_pool_desc *d,
                       const kvx_batch_desc *db, Geometry *gs, Geometry *gd) {
    if ((!s) != (!sb) || (!d) != (!db) || (!s && !d)) return KVX_ERR_INVALID_ARG;
    kvx_status st;
    if (s) {
        if ((st = resolve_pool(s, false, gs)) != KVX_OK) return st;
        if ((st = check_batch_shape(sb)) != KVX_OK) return st;
    }
    if (d) {
        if ((st = resolve_pool(d, true, gd)) != KVX_OK) return st;
        if ((st = check_batch_shape(db)) != KVX_OK) return st;
    }
    if (s && d) {
        if (s->num_kv_heads != d->num_kv_heads || s->head_dim != d->head_dim ||
            s->elem_bytes != d->elem_bytes || sb->num_requests != db->num_requests)
            return KVX_ERR_INVALID_ARG;
        if (sb->num_requests && sb->seq_lens != db->seq_lens &&
            std::memcmp(sb->seq_lens, db->seq_lens, 4ull * sb->num_requests) != 0)
            return KVX_ERR_INVALID_ARG;
    }
    return KVX_OK;
}

} // namespace

// Fields the library fills at once; order, threads, unroll and nontemporal stay 0 (= chosen per operation
// at launch).
void kvx::default_launch(kvx_launch_cfg *c) {
    if (!c->xcd_swizzle) c->xcd_swizzle = 2;
    if (!c->max_workgroups) c->max_workgroups = 1u << 24;
}

namespace {

// Tile shape when the caller left it open.  Measured on MI355X: with (layer,kv) outermost the smallest
// tile (256 lanes x 16 B) with the largest grid is fastest; with the run outermost (page-major receiver)
// 128 lanes x 4 loads each = 8 KiB tiles, four workgroups to a compute unit (run_op caps them), are: against
// one 32 KiB tile of 512 lanes per compute unit +2 % on workload 4, +7 % into a page-major pool of workload
// 2's shape, +2 % of workload 3's, +6 % on an unpack into 128-token pages; four loads per lane matter more
// than the lanes (one or two loads per lane: 4.6-5.5 TB/s where four give 6.3-6.6).
// Cache policy when the caller left it open (values as in kvx_launch_cfg, minus one for the kernels).
// Measured on MI355X: agent-scope stores gain 1-2 % wherever the runs are long (128 KiB and more), into a
// pool or into the buffer alike, and on a plain copy; they lose up to 8 % where the runs are short.
// Non-temporal loads and stores are the safe choice there.  `flat_copy`: the kernel for [token][head][dim]
// pages; the tile kernels gather a run's bytes in pieces, so for a pack they keep the non-temporal stores.
// One more case takes the agent-scope stores: a pack of at most kSmallPackBytes.  What it writes is read
// again at once (by the network, here by the unpack that stands in for it), and written through it is where
// that reader finds it when the kernel ends, instead of waiting in the L2 for the write-back at the kernel's
// end.  Measured with short runs (16 KiB) through the receive slots: a request (22 MB) at a time 18-21 ->
// 15.5-19 us per request, 355 MB at a time 15.9 -> 14.5, 1.4 GB 16.3 -> 14.8, 5.7 GB no difference; a
// 23 GB pack + unpack loses 3.6 % with them.
constexpr uint64_t kSmallPackBytes = 2ull << 30;
int resolve_policy(uint32_t nontemporal, bool flat_copy, bool writes_pool, uint64_t max_run_bytes,
                   uint64_t launch_bytes) {
    if (nontemporal) return (int)nontemporal - 1;
    if (flat_copy && !writes_pool && launch_bytes <= kSmallPackBytes) return 2;
    return ((writes_pool || flat_copy) && max_run_bytes >= 128u * 1024u) ? 2 : 1;
}

void resolve_tile(uint32_t order, uint32_t max_run_bytes, uint32_t *threads, uint32_t *unroll) {
    if (*threads && *unroll) return;
    uint32_t t = 256, u = 1;
    if (order == 2) {
        t = 128;
        while (u < 4 && tile_bytes(t, u * 2) <= max_run_bytes) u *= 2;
    }
    if (!*threads) *threads = t;
    if (!*unroll) *unroll = u;
}
} // namespace

void kvx::planner_params(const kvx_plan_s &p, ScanParams *scan, FillParams *fill) {
    const Sizing &z = p.z;
    ScanParams sp{};
    FillParams fp{};
    sp.seq_lens = reinterpret_cast<const uint32_t *>(p.ws + z.off_lens);
    sp.num_requests = p.R;
    sp.page_s = p.s.present ? p.s.desc.page_tokens : 0;
    sp.page_d = p.d.present ? p.d.desc.page_tokens : 0;
    fp.seq_lens = sp.seq_lens;
    fp.token_prefix = reinterpret_cast<const uint64_t *>(p.ws + z.off_prefix[SCAN_TOKENS]);
    fp.num_requests = p.R;
    fp.row = (uint32_t)p.row;
    fp.bytes_per_token = p.bpt;
    for (int k = 0; k < kNumScans; ++k) sp.prefix[k] = reinterpret_cast<uint64_t *>(p.ws + z.off_prefix[k]);
    SideGeom src_side{}, dst_side{}, buf_side{};
    if (p.s.present) {
        src_side.ids = reinterpret_cast<const uint32_t *>(p.ws + z.off_ids_s);
        src_side.page_prefix = sp.prefix[SCAN_PAGES_S];
        src_side.stride_page = p.s.sp;
        src_side.stride_token = p.s.token_step;
        src_side.page_tokens = p.s.desc.page_tokens;
        src_side.quantum = p.s.quantum;
        src_side.which = 1;
    }
    if (p.d.present) {
        dst_side.ids = reinterpret_cast<const uint32_t *>(p.ws + z.off_ids_d);
        dst_side.page_prefix = sp.prefix[SCAN_PAGES_D];
        dst_side.stride_page = p.d.sp;
        dst_side.stride_token = p.d.token_step;
        dst_side.page_tokens = p.d.desc.page_tokens;
        dst_side.quantum = p.d.quantum;
        dst_side.which = 2;
    }
    fp.src[OP_PACK] = src_side;   fp.dst[OP_PACK] = buf_side;
    fp.src[OP_UNPACK] = buf_side; fp.dst[OP_UNPACK] = dst_side;
    fp.src[OP_CONVERT] = src_side; fp.dst[OP_CONVERT] = dst_side;
    for (int op = 0; op < (int)NUM_OPS; ++op) {
        sp.qa[op] = z.ops[op].qa;
        sp.qb[op] = z.ops[op].qb;
        sp.lcm[op] = z.ops[op].lcm;
        sp.planned[op] = z.ops[op].planned;
        fp.lcm[op] = z.ops[op].lcm;
        fp.planned[op] = z.ops[op].planned;
        if (op == OP_CONVERT) {
            sp.group_quantum = fp.group_quantum = z.ops[op].group_quantum;
            sp.group_slots = fp.group_slots = z.ops[op].group_slots;
        }
        fp.run_prefix[op] = sp.prefix[SCAN_RUNS0 + op];
        fp.runs[op] = reinterpret_cast<kvx_run *>(p.ws + z.off_runs[op]);
    }
    *scan = sp;
    *fill = fp;
}

extern "C" {

const char *kvx_status_string(kvx_status st) {
    switch (st) {
    case KVX_OK: return "ok";
    case KVX_ERR_INVALID_ARG: return "invalid argument";
    case KVX_ERR_ALIGNMENT: return "row, stride or pointer not a multiple of 16 bytes";
    case KVX_ERR_BLOCK_TABLE: return "bad block table";
    case KVX_ERR_CAPACITY: return "buffer or workspace too small";
    case KVX_ERR_UNSUPPORTED: return "size not supported";
    case KVX_ERR_DEVICE: return "HIP error";
    case KVX_ERR_BUSY: return "every receive slot is in flight";
    case KVX_ERR_HOST_MEMORY: return "out of host memory";
    }
    return "unknown status";
}

kvx_status kvx_plan_workspace_bytes(const kvx_pool_desc *s, const kvx_batch_desc *sb,
                                    const kvx_pool_desc *d, const kvx_batch_desc *db,
                                    size_t *out_bytes) {
    if (!out_bytes) return KVX_ERR_INVALID_ARG;
    Geometry gs, gd;
    kvx_status st = check_sides(s, sb, d, db, &gs, &gd);
    if (st != KVX_OK) return st;
    const kvx_batch_desc *b = sb ? sb : db;
    uint64_t used_s = 0, used_d = 0;
    if (s && (st = check_tables(gs, sb, false, nullptr, &used_s)) != KVX_OK) return st;
    if (d && (st = check_tables(gd, db, false, nullptr, &used_d)) != KVX_OK) return st;
    Sizing z;
    z.R = b->num_requests;
    shape_ops(gs, gd, b->seq_lens, z.R, z.ops);
    layout_workspace(&z, used_s, used_d);
    *out_bytes = (size_t)z.total_bytes;
    return KVX_OK;
}

kvx_status kvx_plan(const kvx_pool_desc *s, const kvx_batch_desc *sb, const kvx_pool_desc *d,
                    const kvx_batch_desc *db, uint32_t layer_begin, uint32_t layer_end,
                    void *dev_workspace, size_t workspace_bytes, void *stream,
                    kvx_plan_t **out_plan) try {
    if (!out_plan) return KVX_ERR_INVALID_ARG;
    *out_plan = nullptr;
    std::unique_ptr<kvx_plan_s> owner(new kvx_plan_s);
    kvx_plan_s *p = owner.get();
    kvx_status st = check_sides(s, sb, d, db, &p->s, &p->d);
    if (st != KVX_OK) return st;
    if (layer_begin > layer_end || (s && layer_end > s->num_layers) || (d && layer_end > d->num_layers)) return KVX_ERR_INVALID_ARG;
    if ((dev_workspace == nullptr) != (workspace_bytes == 0)) return KVX_ERR_INVALID_ARG;
    if ((uintptr_t)dev_workspace % kAlign) return KVX_ERR_ALIGNMENT;

    const kvx_batch_desc *b = sb ? sb : db;
    const uint32_t R = b->num_requests;
    std::vector<uint32_t> &ids_s = p->ids_s;
    std::vector<uint32_t> ids_d;
    if (s && (st = check_tables(p->s, sb, false, &ids_s, &p->s.used_pages)) != KVX_OK) return st;
    if (d && (st = check_tables(p->d, db, true, &ids_d, &p->d.used_pages)) != KVX_OK) return st;

    p->R = R;
    p->l0 = layer_begin;
    p->l1 = layer_end;
    p->row = s ? p->s.row : p->d.row;
    p->bpt = (uint64_t)(layer_end - layer_begin) * 2 * p->row;
    p->seq_lens.assign(b->seq_lens, b->seq_lens + R);
    p->token_prefix.resize((size_t)R + 1);
    p->token_prefix[0] = 0;
    for (uint32_t r = 0; r < R; ++r) p->token_prefix[r + 1] = p->token_prefix[r] + p->seq_lens[r];
    p->total = p->token_prefix[R] * p->bpt;

    Sizing &z = p->z;
    z.R = R;
    shape_ops(p->s, p->d, p->seq_lens.data(), R, z.ops);
    layout_workspace(&z, p->s.used_pages, p->d.used_pages);
    default_launch(&p->launch);
    const uint64_t num_lc = 2ull * (layer_end - layer_begin);
    for (int op = 0; op < (int)NUM_OPS; ++op) {
        // even the smallest tile (one 16-byte load per lane) must give a 32-bit tile count
        const uint64_t tpr = (z.ops[op].max_run_bytes + tile_bytes(64, 1) - 1) / tile_bytes(64, 1);
        if (z.ops[op].planned && z.ops[op].num_runs * tpr * num_lc >= (1ull << 32)) return KVX_ERR_UNSUPPORTED;
    }

    if (dev_workspace) {
        if (workspace_bytes < z.total_bytes) return KVX_ERR_CAPACITY;
        p->ws = static_cast<char *>(dev_workspace);
        hipStream_t hs = static_cast<hipStream_t>(stream);
        // Tables of a small batch ride in the scan kernel's arguments; larger ones are staged in pinned
        // memory and copied.
        const uint64_t table_words = (uint64_t)R + ids_s.size() + ids_d.size();
        const bool tables_inline = table_words <= kInlineWords;
        bool ok = true;
        InlineTables it{}; // zeroed: the whole struct travels as a launch argument
        if (tables_inline) {
            const uint32_t *seg[3] = {p->seq_lens.data(), ids_s.data(), ids_d.data()};
            const uint64_t off[3] = {z.off_lens, z.off_ids_s, z.off_ids_d};
            uint32_t at = 0;
            it.count[0] = R;
            it.count[1] = (uint32_t)ids_s.size();
            it.count[2] = (uint32_t)ids_d.size();
            for (int k = 0; k < 3; ++k) {
                it.dst_word[k] = (uint32_t)(off[k] / 4);
                if (it.count[k]) std::memcpy(it.words + at, seg[k], 4ull * it.count[k]);
                at += it.count[k];
            }
        } else {
            if (!hip_ok(pinned_acquire((size_t)z.staging_bytes, &p->staging), "pinned staging block"))
                return KVX_ERR_DEVICE;
            char *h = static_cast<char *>(p->staging.ptr);
            if (R) std::memcpy(h + z.off_lens, p->seq_lens.data(), 4ull * R);
            if (!ids_s.empty()) std::memcpy(h + z.off_ids_s, ids_s.data(), 4ull * ids_s.size());
            if (!ids_d.empty()) std::memcpy(h + z.off_ids_d, ids_d.data(), 4ull * ids_d.size());
            ok = hip_ok(hipMemcpyAsync(p->ws, h, z.staging_bytes, hipMemcpyHostToDevice, hs), "copy of the tables");
            ok = ok && hip_ok(hipEventRecord(p->staging.copied, hs), "event behind the copy");
        }

        ScanParams sp{};
        FillParams fp{};
        planner_params(*p, &sp, &fp);
        if (tables_inline) {
            // one launch for the whole plan: a single workgroup scans and writes the runs
            ok = ok && hip_ok(launch_plan_small(sp, fp, it, reinterpret_cast<uint32_t *>(p->ws), hs),
                              "plan_small_kernel launch");
        } else {
            ok = ok && hip_ok(launch_scan(sp, hs), "scan_kernel launch");
            ok = ok && hip_ok(launch_fill(fp, hs), "fill_kernel launch");
        }
        if (!ok) {
            pinned_release(p->staging);
            return KVX_ERR_DEVICE;
        }
    } else if (s == nullptr || d == nullptr) {
        // No workspace: a plan for the size and segment queries.  It can still run when it is small and
        // simple enough for its run records to ride in the copy kernel's launch arguments: one side, pages
        // that hold token rows, at most kInlineRuns used pages.  A run of a one-sided plan is the part of a
        // request inside one page, so the records follow from the block table directly.
        const Geometry &g = s ? p->s : p->d;
        const Op op = s ? OP_PACK : OP_UNPACK;
        const std::vector<uint32_t> &ids = s ? ids_s : ids_d;
        if (g.dense_rows && !g.token_innermost && z.ops[op].num_runs > 0 && z.ops[op].num_runs <= kInlineRuns &&
            z.ops[op].num_runs == ids.size()) {
            p->inline_runs.reset(new InlineRuns());
            const uint32_t P = g.desc.page_tokens;
            size_t at = 0;
            for (uint32_t r = 0; r < R; ++r) {
                const uint32_t n = p->seq_lens[r];
                for (uint32_t x = 0; x < n; x += P, ++at) {
                    kvx_run &run = p->inline_runs->run[at];
                    const uint64_t in_pool = (uint64_t)ids[at] * g.sp;
                    const uint64_t in_buf = p->token_prefix[r] * p->bpt + (uint64_t)x * p->row;
                    run.src_off = s ? in_pool : in_buf;
                    run.dst_off = s ? in_buf : in_pool;
                    run.bytes = (uint32_t)(std::min<uint64_t>(n - x, P) * p->row);
                    run.seq_len = n;
                    run.request = r;
                    run.token = x;
                    if (n - x <= P) { ++at; break; } // also keeps x += P from wrapping near 2^32
                }
            }
        }
    }
    *out_plan = owner.release();
    return KVX_OK;
} catch (...) { // the host tables could not be allocated; nothing was enqueued yet
    return KVX_ERR_HOST_MEMORY;
}

kvx_status kvx_release_cached(uint64_t *freed_bytes) {
    std::lock_guard<std::mutex> lk(g_pinned_mu);
    const uint64_t freed = pinned_trim(0);
    if (freed_bytes) *freed_bytes = freed;
    return KVX_OK;
}

#ifndef KVX_BUILD_ID
#define KVX_BUILD_ID "unknown"
#endif
const char *kvx_build_id(void) { return KVX_BUILD_ID; }

void kvx_plan_destroy(kvx_plan_t *plan) {
    if (!plan) return;
    // Work already enqueued with this plan keeps running: launches carry their
    // arguments, and the staging block is recycled only after its copy is done.
    pinned_release(plan->staging);
    delete plan;
}

kvx_status kvx_plan_total_bytes(const kvx_plan_t *plan, uint64_t *payload_bytes) {
    if (!plan || !payload_bytes) return KVX_ERR_INVALID_ARG;
    *payload_bytes = plan->total;
    return KVX_OK;
}

kvx_status kvx_plan_segment(const kvx_plan_t *plan, uint32_t request, uint32_t layer, uint64_t *offset,
                            uint64_t *length) {
    if (!plan || !offset || !length) return KVX_ERR_INVALID_ARG;
    if (request >= plan->R || layer < plan->l0 || layer >= plan->l1) return KVX_ERR_INVALID_ARG;
    const uint64_t n = plan->seq_lens[request];
    *offset = plan->token_prefix[request] * plan->bpt + (uint64_t)(layer - plan->l0) * 2 * n * plan->row;
    *length = 2 * n * plan->row;
    return KVX_OK;
}

kvx_status kvx_plan_request_segment(const kvx_plan_t *plan, uint32_t request, uint64_t *offset,
                                    uint64_t *length) {
    if (!plan || !offset || !length || request >= plan->R) return KVX_ERR_INVALID_ARG;
    *offset = plan->token_prefix[request] * plan->bpt;
    *length = (uint64_t)plan->seq_lens[request] * plan->bpt;
    return KVX_OK;
}

kvx_status kvx_plan_get_tables(const kvx_plan_t *plan, kvx_plan_tables *out) {
    if (!plan || !out || !plan->ws) return KVX_ERR_INVALID_ARG;
    out->token_prefix_off = plan->z.off_prefix[SCAN_TOKENS];
    for (int op = 0; op < (int)NUM_OPS; ++op) {
        out->run_prefix_off[op] = plan->z.off_prefix[SCAN_RUNS0 + op];
        out->runs_off[op] = plan->z.off_runs[op];
        out->num_runs[op] = plan->z.ops[op].planned ? plan->z.ops[op].num_runs : 0;
    }
    return KVX_OK;
}

kvx_status kvx_plan_can_launch(const kvx_plan_t *plan, int *out) {
    if (!plan || !out) return KVX_ERR_INVALID_ARG;
    *out = (plan->ws || plan->inline_runs) ? 1 : 0;
    return KVX_OK;
}

kvx_status kvx_plan_set_launch(kvx_plan_t *plan, const kvx_launch_cfg *cfg) {
    if (!plan || !cfg) return KVX_ERR_INVALID_ARG;
    kvx_launch_cfg c = *cfg;
    default_launch(&c);
    if ((c.unroll && !valid_unroll(c.unroll)) || (c.threads && !valid_threads(c.threads)))
        return KVX_ERR_INVALID_ARG;
    if (c.nontemporal > 3 || c.order > 3 || c.xcd_swizzle > 2 || c.workgroups_per_cu > 8)
        return KVX_ERR_INVALID_ARG;
    if (c.xcd_block_tiles & (c.xcd_block_tiles - 1u) || c.xcd_block_tiles > 4096u) return KVX_ERR_INVALID_ARG;
    plan->launch = c;
    return KVX_OK;
}

kvx_status kvx_plan_get_launch(const kvx_plan_t *plan, kvx_launch_cfg *out) {
    if (!plan || !out) return KVX_ERR_INVALID_ARG;
    *out = plan->launch;
    return KVX_OK;
}

} // extern "C"

namespace {

XposeSide xpose_side(const Geometry &g, bool is_buf, uint64_t row) {
    XposeSide x{};
    x.is_buf = is_buf;
    if (is_buf) { // the buffer: plain [token][head][dim] rows
        x.token_step = row;
        x.units_per_granule = (uint32_t)(row / 16);
    } else {
        x.stride_layer = g.sl;
        x.stride_kv = g.sk;
        x.token_step = g.token_step;
        x.granule_step = g.granule_step;
        x.units_per_granule = g.upg;
    }
    x.granule_magic = x.units_per_granule > 1 ? (uint32_t)((1ull << 32) / x.units_per_granule) + 1u : 0u;
    return x;
}

// The same as run_op's launch, for pools whose pages are not [token][head][dim] inside.
kvx_status run_xpose(const kvx_plan_t *plan, Op op, uint32_t lb, uint32_t le, const void *src, void *dst,
                     void *stream) {
    const OpShape &o = plan->z.ops[op];
    const kvx_launch_cfg &c = plan->launch;
    XposeParams xp{};
    xp.runs = reinterpret_cast<const kvx_run *>(plan->ws + plan->z.off_runs[op]);
    xp.src = static_cast<const char *>(src);
    xp.dst = static_cast<char *>(dst);
    xp.s = xpose_side(plan->s, op == OP_UNPACK, plan->row);
    xp.d = xpose_side(plan->d, op == OP_PACK, plan->row);
    const bool src_tf = op != OP_UNPACK && plan->s.token_fast;
    const bool dst_tf = op != OP_PACK && plan->d.token_fast;
    xp.row = (uint32_t)plan->row;
    xp.units_per_row = (uint32_t)(plan->row / 16);
    xp.layer_begin = plan->l0;
    xp.lc_first = 2 * (lb - plan->l0);
    xp.num_lc = 2 * (le - lb);
    xp.num_runs = (uint32_t)o.num_runs;
    // 1024 units per tile: as wide along the row as the row allows (up to 64 units = 1 KiB), the rest in tokens
    xp.log2_uu = xp.units_per_row >= 64 ? 6 : (xp.units_per_row >= 32 ? 5 : 4);
    xp.log2_tt = 10 - xp.log2_uu;
    const uint32_t max_tokens = o.max_run_bytes / xp.row;
    xp.tiles_t = (max_tokens + (1u << xp.log2_tt) - 1) >> xp.log2_tt;
    xp.tiles_u = (xp.units_per_row + (1u << xp.log2_uu) - 1) >> xp.log2_uu;
    const uint64_t total = (uint64_t)xp.num_lc * xp.num_runs * xp.tiles_t * xp.tiles_u;
    if (total >= (1ull << 32)) return KVX_ERR_UNSUPPORTED;
    xp.total_tiles = (uint32_t)total;
    xp.order = c.order == 3 ? 1u : c.order; // an eighth of the runs per XCD exists in the flat kernel only
    if (!xp.order)
        xp.order = (op != OP_PACK && !plan->d.custom_strides && plan->d.desc.layout == KVX_LAYOUT_PAGE_MAJOR) ? 2 : 1;
    // as in run_op: with the receiver's pages the finer ones, one run goes through all its (layer,kv) pieces
    xp.group = (op == OP_CONVERT && plan->d.desc.page_tokens < plan->s.desc.page_tokens) ? 1u : o.group_slots;
    const uint32_t grid_cap = std::min<uint32_t>(c.max_workgroups, (1u << 31) / kXposeThreads - 8u);
    uint32_t grid = std::min(xp.total_tiles, grid_cap);
    if (c.xcd_swizzle == 2) {
        grid = (grid + 7u) / 8u * 8u;
        xp.swizzle_chunk = grid / 8u;
    }
    hipError_t e = launch_xpose(xp, src_tf, dst_tf, resolve_policy(c.nontemporal, false, op != OP_PACK, o.max_run_bytes, 0), grid,
                                static_cast<hipStream_t>(stream));
    return hip_ok(e, "xpose_kernel launch") ? KVX_OK : KVX_ERR_DEVICE;
}

ElemSide elem_side(const Geometry &g, bool is_buf, uint64_t row) {
    ElemSide x{};
    x.is_buf = is_buf;
    if (is_buf) {
        x.token_step = row;
        x.units_per_granule = (uint32_t)(row / 16);
    } else {
        x.stride_layer = g.sl;
        x.stride_kv = g.sk;
        x.token_step = g.token_step;
        x.granule_step = g.granule_step;
        x.units_per_granule = g.upg;
        x.column_step = g.column_step;
    }
    x.granule_magic = x.units_per_granule > 1 ? (uint32_t)((1ull << 32) / x.units_per_granule) + 1u : 0u;
    return x;
}

// The same again for a pool with the token axis innermost on either side: tiles transposed at element
// granularity through LDS.
kvx_status run_xpose_elem(const kvx_plan_t *plan, Op op, uint32_t lb, uint32_t le, const void *src, void *dst,
                          void *stream) {
    const OpShape &o = plan->z.ops[op];
    const kvx_launch_cfg &c = plan->launch;
    const Geometry &gs = plan->s, &gd = plan->d;
    ElemParams ep{};
    ep.runs = reinterpret_cast<const kvx_run *>(plan->ws + plan->z.off_runs[op]);
    ep.src = static_cast<const char *>(src);
    ep.dst = static_cast<char *>(dst);
    ep.s = elem_side(gs, op == OP_UNPACK, plan->row);
    ep.d = elem_side(gd, op == OP_PACK, plan->row);
    const int sk = op == OP_UNPACK ? 0 : (gs.token_innermost ? 2 : (gs.token_fast ? 1 : 0));
    const int dk = op == OP_PACK ? 0 : (gd.token_innermost ? 2 : (gd.token_fast ? 1 : 0));
    const uint32_t elem = (op == OP_UNPACK ? gd : gs).desc.elem_bytes; // the two sides agree
    ep.row = (uint32_t)plan->row;
    ep.units_per_row = (uint32_t)(plan->row / 16);
    ep.layer_begin = plan->l0;
    ep.lc_first = 2 * (lb - plan->l0);
    ep.num_lc = 2 * (le - lb);
    ep.num_runs = (uint32_t)o.num_runs;
    // A convert whose token-innermost side has the coarser pages, a whole number of the other side's: tiles
    // span a group of runs (one coarse page), so that the pieces of its columns are as long as the page
    // allows instead of as short as a run.  A finer side that is token-innermost too must not have a
    // 16-byte piece straddle two of its pages.
    uint32_t max_tokens = o.max_run_bytes / ep.row;
    if (op == OP_CONVERT && o.group_slots > 1 && o.group_slots <= kElemMaxGroup) {
        const uint32_t ps = gs.desc.page_tokens, pd = gd.desc.page_tokens;
        const bool src_coarse = ps > pd;
        const Geometry &coarse = src_coarse ? gs : gd, &fine = src_coarse ? gd : gs;
        const uint32_t pc = coarse.desc.page_tokens, pf = fine.desc.page_tokens;
        if (coarse.token_innermost && pc % pf == 0 && (!fine.token_innermost || (pf * elem) % 16 == 0)) {
            ep.group_mode = src_coarse ? 1 : 2;
            ep.num_groups = ep.num_runs / o.group_slots;
            ep.coarse_tokens = pc;
            ep.fine_tokens = pf;
            ep.by_fine = make_fast_div(pf);
            max_tokens = pc;
        }
    }
    // A tile is 16 KiB: as many tokens as a run (or group) can have (long pieces along the token axis are
    // what the token-innermost side moves contiguously), between 16 and 256, and the rest along the row.
    ep.log2_tt = 4;
    while (ep.log2_tt < 8 && (1u << ep.log2_tt) < max_tokens) ++ep.log2_tt;
    ep.log2_wu = 10 - ep.log2_tt;
    ep.tiles_t = (max_tokens + (1u << ep.log2_tt) - 1) >> ep.log2_tt;
    ep.tiles_w = (ep.units_per_row + (1u << ep.log2_wu) - 1) >> ep.log2_wu;
    const uint64_t total = (uint64_t)ep.num_lc * (ep.group_mode ? ep.num_groups : ep.num_runs) * ep.tiles_t * ep.tiles_w;
    if (total >= (1ull << 32)) return KVX_ERR_UNSUPPORTED;
    ep.total_tiles = (uint32_t)total;
    ep.order = c.order == 3 ? 1u : c.order;
    if (!ep.order)
        ep.order = (op != OP_PACK && !gd.custom_strides && gd.desc.layout == KVX_LAYOUT_PAGE_MAJOR) ? 2 : 1;
    ep.group = o.group_slots; // the runs of one coarse page stay together: their pieces share 128-byte lines
    const uint32_t grid_cap = std::min<uint32_t>(c.max_workgroups, (1u << 31) / kElemThreads - 8u);
    uint32_t grid = std::min(ep.total_tiles, grid_cap);
    if (c.xcd_swizzle == 2) {
        grid = (grid + 7u) / 8u * 8u;
        ep.swizzle_chunk = grid / 8u;
    }
    const int nt = c.nontemporal == 1 ? 0 : 1; // default policy only on request; agent-scope stores are not offered here
    // A token-innermost side whose runs are shorter than its pages (the other side's pages are finer) hands
    // every tile pieces of a column that are shorter than a 128-byte line; the rest of each line belongs to
    // the neighbouring runs of the same page, whose tiles come next.  Accesses that may stay in the L2 let
    // those find the line there: a line is fetched once instead of once per piece, and written back whole
    // instead of piece by piece (measured on 128 <-> 16 tokens: reads 4.1 -> 5.2 TB/s, writes 1.4 -> ?).
    ep.cached_loads = (sk == 2 && (uint64_t)max_tokens * elem < 128u && max_tokens < gs.desc.page_tokens) ? 1u : 0u;
    ep.cached_stores = (dk == 2 && (uint64_t)max_tokens * elem < 128u && max_tokens < gd.desc.page_tokens) ? 1u : 0u;
    if (ep.group_mode) ep.cached_loads = ep.cached_stores = 0; // whole pieces: nothing to share through the L2
    hipError_t e = launch_xpose_elem(ep, elem, sk, dk, nt, grid, static_cast<hipStream_t>(stream));
    return hip_ok(e, "xpose_elem_kernel launch") ? KVX_OK : KVX_ERR_DEVICE;
}

// Launches one operation over layers [lb, le) of the plan's range.  Buffer offsets stay those of the
// plan's whole range, so a sub-range touches exactly its own segments of the same buffer.
} // namespace

kvx_status kvx::run_op(const kvx_plan_s *plan, Op op, uint32_t lb, uint32_t le, const void *src, void *dst,
                       void *stream) {
    const OpShape &o = plan->z.ops[op];
    if ((!plan->ws && !plan->inline_runs) || !o.planned) return KVX_ERR_INVALID_ARG;
    if (lb > le || lb < plan->l0 || le > plan->l1) return KVX_ERR_INVALID_ARG;
    if (plan->total == 0 || lb == le) return KVX_OK;
    if (!src || !dst) return KVX_ERR_INVALID_ARG;
    if (((uintptr_t)src | (uintptr_t)dst) % 16) return KVX_ERR_ALIGNMENT;
    if (op == OP_CONVERT && !plan->s.custom_strides && !plan->d.custom_strides) {
        // two dense pools: their extents are known, so an overlap can be refused
        const uintptr_t a = (uintptr_t)src, b = (uintptr_t)dst;
        if (a < b + plan->d.span && b < a + plan->s.span) return KVX_ERR_INVALID_ARG;
    }
    const kvx_launch_cfg &c = plan->launch;
    const bool src_rows = (op == OP_UNPACK) || plan->s.dense_rows;
    const bool dst_rows = (op == OP_PACK) || plan->d.dense_rows;
    if ((op != OP_UNPACK && plan->s.token_innermost) || (op != OP_PACK && plan->d.token_innermost))
        return run_xpose_elem(plan, op, lb, le, src, dst, stream);
    if (!src_rows || !dst_rows) return run_xpose(plan, op, lb, le, src, dst, stream);
    CopyParams cp{};
    cp.runs = plan->ws ? reinterpret_cast<const kvx_run *>(plan->ws + plan->z.off_runs[op]) : nullptr;
    cp.src = static_cast<const char *>(src);
    cp.dst = static_cast<char *>(dst);
    cp.src_is_buf = (op == OP_UNPACK);
    cp.dst_is_buf = (op == OP_PACK);
    cp.src_stride_layer = plan->s.sl;
    cp.src_stride_kv = plan->s.sk;
    cp.dst_stride_layer = plan->d.sl;
    cp.dst_stride_kv = plan->d.sk;
    cp.row = (uint32_t)plan->row;
    cp.layer_begin = plan->l0;
    cp.lc_first = 2 * (lb - plan->l0);
    cp.num_lc = 2 * (le - lb);
    cp.num_runs = (uint32_t)o.num_runs;
    // Order of the tile space.  Unless the caller fixed it: keep the write side contiguous.  A page-major
    // receiver holds all (layer,kv) of a page side by side, so there the run group goes outermost;
    // everywhere else consecutive runs of a request are what is contiguous (in the buffer).  Which part of
    // that space an XCD works on is then a measured choice: for pack an eighth of the runs through all
    // (layer,kv), so that the eight XCDs gather from different pages at any moment (never slower than an
    // eighth of the (layer,kv) range each, up to 8 % faster); for unpack and convert the latter, which is
    // the faster one there.
    // Eight parts want runs to deal out: below kRunsForParts of them the parts come out uneven (17 runs make
    // parts of 3, 3, 3, 3, 3, 2, 0, 0), and a pack of so few is faster with (layer,kv) outermost (a request at
    // a time through the receive slots: 19.3 -> 18.6 us per request).
    constexpr uint64_t kRunsForParts = 64;
    cp.order = c.order;
    if (!cp.order) {
        if (op != OP_PACK && !plan->d.custom_strides && plan->d.desc.layout == KVX_LAYOUT_PAGE_MAJOR) cp.order = 2;
        else cp.order = (op == OP_PACK && o.num_runs >= kRunsForParts) ? 3 : 1;
    }
    // Order 2 keeps `group` consecutive runs together inside one (layer,kv) before it moves to the next.  With
    // the receiver's pages the coarser ones the runs of a group fill one receiver page, side by side for every
    // (layer,kv): the whole group it is.  With the receiver's pages the finer ones every run is a receiver page
    // of its own, whose (layer,kv) pieces lie one behind the other: walking one run through all of them writes
    // that page front to back (workload 4, 128 -> 16 tokens: 25.1 -> 24.4 ms, three processes).
    cp.group = (op == OP_CONVERT && plan->d.desc.page_tokens < plan->s.desc.page_tokens) ? 1u : o.group_slots;
    uint32_t threads = c.threads, unroll = c.unroll;
    resolve_tile(cp.order, o.max_run_bytes, &threads, &unroll);
    const uint32_t tile = tile_bytes(threads, unroll);
    cp.tiles_per_run = (o.max_run_bytes + tile - 1) / tile;
    cp.total_tiles = (uint32_t)((uint64_t)cp.num_lc * cp.num_runs * cp.tiles_per_run);
    if (cp.order == 3) {
        // eight parts of ceil(num_runs/8) runs each; where that would not index in 32 bits, order 1 serves
        cp.runs_per_part = (cp.num_runs + 7u) / 8u;
        const uint64_t tiles = 8ull * cp.num_lc * cp.runs_per_part * cp.tiles_per_run;
        if (tiles < (1ull << 32)) cp.total_tiles = (uint32_t)tiles;
        else cp.order = 1;
    }
    // keep grid * threads below 2^31 work-items; the kernel's grid-stride loop takes the rest
    const uint32_t grid_cap = std::min<uint32_t>(c.max_workgroups, (1u << 31) / threads - 8u);
    uint32_t grid = std::min(cp.total_tiles, grid_cap);
    if (c.xcd_swizzle == 2) {
        const uint32_t unit = 8u * std::max(c.xcd_block_tiles, 1u);
        grid = (grid + unit - 1u) / unit * unit; // the tile map is a bijection on a grid of whole units
        const uint32_t limit = (1u << 31) / threads;
        if (grid > limit) grid = limit / unit * unit;
        cp.swizzle_chunk = grid / 8u;
        cp.swizzle_block = c.xcd_block_tiles;
    }
    cp.by_tiles_per_run = make_fast_div(cp.tiles_per_run);
    cp.by_num_runs = make_fast_div(cp.num_runs);
    cp.by_runs_per_part = make_fast_div(cp.runs_per_part);
    cp.by_group = make_fast_div(cp.group);
    cp.by_num_lc = make_fast_div(cp.num_lc);
    cp.by_swizzle_block = make_fast_div(cp.swizzle_block);
    // Bytes in flight: the tiles of order 2 (four loads per lane) fill a compute unit with 128 KiB of loads
    // when as many workgroups as fit are resident; measured, 32 KiB per compute unit (8 MB over the device,
    // what the small tiles of the other orders have anyway) is 3 % faster.  Unless the caller chose a tile or
    // a cap.
    uint32_t per_cu = c.workgroups_per_cu;
    if (!per_cu && cp.order == 2 && !c.threads && !c.unroll) per_cu = std::min(16u, std::max(1u, 32768u / tile));
    const uint64_t launch_bytes = plan->total / (plan->l1 - plan->l0) * (le - lb);
    // What counts as a long run for the cache policy: in a page-major receiver the (layer,kv) pieces of a
    // page lie one behind the other, and order 2 writes them in that order, so the stretch written front to
    // back is all of them (workload 4: 80 x 32 KiB).
    uint64_t stretch = o.max_run_bytes;
    if (cp.order == 2 && op != OP_PACK && !plan->d.custom_strides && plan->d.desc.layout == KVX_LAYOUT_PAGE_MAJOR)
        stretch *= cp.num_lc;
    // with a workspace the table in it is what the kernel reads, as kvx_plan_get_tables promises
    const InlineRuns *inline_runs = plan->ws ? nullptr : plan->inline_runs.get();
    hipError_t e = launch_copy(cp, inline_runs, threads, unroll,
                               resolve_policy(c.nontemporal, true, op != OP_PACK, stretch, launch_bytes), grid,
                               occupancy_lds(per_cu), static_cast<hipStream_t>(stream));
    return hip_ok(e, "copy_kernel launch") ? KVX_OK : KVX_ERR_DEVICE;
}

extern "C" {

kvx_status kvx_pack(const kvx_plan_t *plan, const void *src_pool, void *buf, uint64_t buf_bytes,
                    void *stream) {
    if (!plan) return KVX_ERR_INVALID_ARG;
    if (buf_bytes < plan->total) return KVX_ERR_CAPACITY;
    return run_op(plan, OP_PACK, plan->l0, plan->l1, src_pool, buf, stream);
}

kvx_status kvx_unpack(const kvx_plan_t *plan, const void *buf, uint64_t buf_bytes, void *dst_pool,
                      void *stream) {
    if (!plan) return KVX_ERR_INVALID_ARG;
    if (buf_bytes < plan->total) return KVX_ERR_CAPACITY;
    return run_op(plan, OP_UNPACK, plan->l0, plan->l1, buf, dst_pool, stream);
}

kvx_status kvx_convert(const kvx_plan_t *plan, const void *src_pool, void *dst_pool, void *stream) {
    if (!plan) return KVX_ERR_INVALID_ARG;
    return run_op(plan, OP_CONVERT, plan->l0, plan->l1, src_pool, dst_pool, stream);
}

kvx_status kvx_pack_layers(const kvx_plan_t *plan, uint32_t layer_begin, uint32_t layer_end,
                           const void *src_pool, void *buf, uint64_t buf_bytes, void *stream) {
    if (!plan) return KVX_ERR_INVALID_ARG;
    if (buf_bytes < plan->total) return KVX_ERR_CAPACITY;
    return run_op(plan, OP_PACK, layer_begin, layer_end, src_pool, buf, stream);
}

kvx_status kvx_unpack_layers(const kvx_plan_t *plan, uint32_t layer_begin, uint32_t layer_end, const void *buf,
                             uint64_t buf_bytes, void *dst_pool, void *stream) {
    if (!plan) return KVX_ERR_INVALID_ARG;
    if (buf_bytes < plan->total) return KVX_ERR_CAPACITY;
    return run_op(plan, OP_UNPACK, layer_begin, layer_end, buf, dst_pool, stream);
}

kvx_status kvx_convert_layers(const kvx_plan_t *plan, uint32_t layer_begin, uint32_t layer_end,
                              const void *src_pool, void *dst_pool, void *stream) {
    if (!plan) return KVX_ERR_INVALID_ARG;
    return run_op(plan, OP_CONVERT, layer_begin, layer_end, src_pool, dst_pool, stream);
}

kvx_status kvx_pack_blockwise(const kvx_plan_t *plan, const void *src_pool, void *buf, uint64_t buf_bytes,
                              uint32_t confirm_every, void *stream) {
    if (!plan || !plan->s.present) return KVX_ERR_INVALID_ARG;
    if (plan->s.desc.inner != KVX_INNER_TOKEN_ROWS) return KVX_ERR_UNSUPPORTED; // blocks would not be contiguous
    if (buf_bytes < plan->total) return KVX_ERR_CAPACITY;
    if (plan->total == 0) return KVX_OK;
    if (!src_pool || !buf) return KVX_ERR_INVALID_ARG;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const char *src = static_cast<const char *>(src_pool);
    char *dst = static_cast<char *>(buf);
    const Geometry &g = plan->s;
    const uint32_t P = g.desc.page_tokens;
    const uint64_t row = plan->row;
    uint64_t first_id = 0, issued = 0;
    for (uint32_t r = 0; r < plan->R; ++r) {
        const uint64_t n = plan->seq_lens[r];
        const uint64_t pages = (n + P - 1) / P;
        for (uint32_t l = plan->l0; l < plan->l1; ++l)
            for (uint32_t kv = 0; kv < 2; ++kv)
                for (uint64_t j = 0; j < pages; ++j) {
                    const uint64_t tokens = std::min<uint64_t>(P, n - j * P);
                    const uint64_t so = l * g.sl + kv * g.sk + (uint64_t)plan->ids_s[first_id + j] * g.sp;
                    const uint64_t bo = plan->token_prefix[r] * plan->bpt +
                                        (((uint64_t)(l - plan->l0) * 2 + kv) * n + j * P) * row;
                    hipError_t e;
                    if (g.st == row) { // a page's tokens are contiguous: the block moves as one copy
                        e = hipMemcpyAsync(dst + bo, src + so, tokens * row, hipMemcpyDeviceToDevice, hs);
                    } else {
                        e = hipMemcpy2DAsync(dst + bo, row, src + so, g.st, row, tokens, hipMemcpyDeviceToDevice, hs);
                    }
                    if (!hip_ok(e, "block copy")) return KVX_ERR_DEVICE;
                    if (confirm_every && ++issued % confirm_every == 0 &&
                        !hip_ok(hipStreamSynchronize(hs), "wait for a block"))
                        return KVX_ERR_DEVICE;
                }
        first_id += pages;
    }
    return KVX_OK;
}

kvx_status kvx_copy_yardstick(void *dst, const void *src, uint64_t bytes, const kvx_launch_cfg *cfg,
                              void *stream) {
    if (!dst || !src) return KVX_ERR_INVALID_ARG;
    if ((((uintptr_t)dst | (uintptr_t)src) % 16) || bytes % 16) return KVX_ERR_ALIGNMENT;
    kvx_launch_cfg c{};
    if (cfg) c = *cfg;
    default_launch(&c);
    resolve_tile(1, 0, &c.threads, &c.unroll);
    if (!valid_unroll(c.unroll) || !valid_threads(c.threads)) return KVX_ERR_INVALID_ARG;
    hipError_t e = launch_plain_copy(static_cast<char *>(dst), static_cast<const char *>(src), bytes, c.threads,
                                     c.unroll, c.nontemporal ? (int)c.nontemporal - 1 : 2, c.max_workgroups,
                                     static_cast<hipStream_t>(stream));
    return hip_ok(e, "plain_copy_kernel launch") ? KVX_OK : KVX_ERR_DEVICE;
}

int kvx_last_device_error(const char **where) {
    if (where) *where = g_last_hip_where;
    return g_last_hip_error;
}

} // extern "C"
