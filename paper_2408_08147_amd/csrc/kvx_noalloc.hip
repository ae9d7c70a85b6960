// RecvScatter for callers that cannot allocate (code under HIP graph capture, tight serving loops,
// harnesses that forbid hipMalloc): kvx_plan for a receiver side and kvx_unpack in one call that creates
// no plan object, stages nothing in pinned memory and takes no workspace from the caller.  The plan's
// device tables live in a fixed array inside the library's device image, one copy per GPU.
#include <algorithm>
#include <atomic>
#include <cstring>

#include "kvx_internal.h"

using namespace kvx;

namespace {

// The plan workspace of every kvx_unpack_noalloc call on a GPU.  Each GPU that loads the library's code
// object holds its own copy at its own address until the process ends.
static __device__ __align__(256) unsigned char scratch[KVX_NOALLOC_SCRATCH_BYTES];

// In host code `scratch` is only a handle for the runtime's symbol table, not a device address: the
// address of a GPU's copy is asked for once per device, with that device current, and kept here.  Host
// code uses these pointers, never the array's name, wherever the array's memory is meant.
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

hipError_t scratch_of_current_device(char **out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(p, std::memory_order_release); // two threads racing here store the same value
    }
    *out = static_cast<char *>(p);
    return hipSuccess;
}

} // namespace

extern "C" kvx_status kvx_unpack_noalloc(const kvx_pool_desc *d, const kvx_batch_desc *db, uint32_t layer_begin,
                                         uint32_t layer_end, const void *buf, uint64_t buf_bytes, void *dst_pool,
                                         void *stream) {
    if (!d || !db) return KVX_ERR_INVALID_ARG;
    // A plan object on the stack: its vectors stay empty (the launches below read the caller's arrays and
    // the scratch array only), so constructing and destroying it touches no heap.
    kvx_plan_s plan;
    kvx_status st = resolve_pool(d, true, &plan.d);
    if (st != KVX_OK) return st;
    if ((st = check_batch_shape(db)) != KVX_OK) return st;
    if (layer_begin > layer_end || layer_end > d->num_layers) return KVX_ERR_INVALID_ARG;

    // Block tables: enough pages per request, ids inside the pool, no receiver page used twice.  The ids that
    // are used go straight into the launch arguments; a sorted copy on the stack finds repeats.
    const uint32_t R = db->num_requests, P = d->page_tokens;
    if (R > KVX_NOALLOC_MAX_TABLE_WORDS) return KVX_ERR_CAPACITY;
    InlineTables it{}; // zeroed: the whole struct travels as a launch argument
    uint32_t sorted[kInlineWords];
    static_assert(KVX_NOALLOC_MAX_TABLE_WORDS <= kInlineWords, "the tables must fit one launch");
    uint64_t used = 0, tokens = 0;
    for (uint32_t r = 0; r < R; ++r) {
        const uint64_t need = ((uint64_t)db->seq_lens[r] + P - 1) / P;
        if (need > db->block_offsets[r + 1] - db->block_offsets[r]) return KVX_ERR_BLOCK_TABLE;
        if (R + used + need > KVX_NOALLOC_MAX_TABLE_WORDS) return KVX_ERR_CAPACITY;
        const uint32_t *ids = db->block_ids + db->block_offsets[r];
        for (uint64_t j = 0; j < need; ++j) {
            if (ids[j] >= d->num_pages) return KVX_ERR_BLOCK_TABLE;
            it.words[R + used + j] = sorted[used + j] = ids[j];
        }
        it.words[r] = db->seq_lens[r];
        used += need;
        tokens += db->seq_lens[r];
    }
    std::sort(sorted, sorted + used);
    if (std::adjacent_find(sorted, sorted + used) != sorted + used) return KVX_ERR_BLOCK_TABLE;

    plan.R = R;
    plan.l0 = layer_begin;
    plan.l1 = layer_end;
    plan.row = plan.d.row;
    plan.bpt = (uint64_t)(layer_end - layer_begin) * 2 * plan.row;
    plan.total = tokens * plan.bpt;
    plan.d.used_pages = used;
    if (buf_bytes < plan.total) return KVX_ERR_CAPACITY;
    Sizing &z = plan.z;
    z.R = R;
    shape_ops(plan.s, plan.d, db->seq_lens, R, z.ops);
    layout_workspace(&z, 0, used);
    default_launch(&plan.launch);
    {
        const OpShape &o = z.ops[OP_UNPACK];
        const uint64_t tpr = (o.max_run_bytes + tile_bytes(64, 1) - 1) / tile_bytes(64, 1);
        if (o.num_runs * tpr * 2ull * (layer_end - layer_begin) >= (1ull << 32)) return KVX_ERR_UNSUPPORTED;
    }
    if (z.total_bytes > KVX_NOALLOC_SCRATCH_BYTES) return KVX_ERR_CAPACITY;
    if (plan.total == 0) return KVX_OK; // nothing to move: nothing is enqueued
    if (!buf || !dst_pool) return KVX_ERR_INVALID_ARG;
    if (((uintptr_t)buf | (uintptr_t)dst_pool) % 16) return KVX_ERR_ALIGNMENT;

    char *ws = nullptr;
    if (!hip_ok(scratch_of_current_device(&ws), "address of the scratch array")) return KVX_ERR_DEVICE;
    plan.ws = ws;
    it.count[0] = R;
    it.count[1] = 0;
    it.count[2] = (uint32_t)used;
    it.dst_word[0] = (uint32_t)(z.off_lens / 4);
    it.dst_word[1] = (uint32_t)(z.off_ids_s / 4);
    it.dst_word[2] = (uint32_t)(z.off_ids_d / 4);
    ScanParams sp{};
    FillParams fp{};
    planner_params(plan, &sp, &fp);
    hipStream_t hs = static_cast<hipStream_t>(stream);
    // Every table the unpack kernel reads is rewritten by this launch, so whatever the previous call left
    // in the array does not matter and nothing has to be cleared first.
    if (!hip_ok(launch_plan_small(sp, fp, it, reinterpret_cast<uint32_t *>(ws), hs), "plan_small_kernel launch"))
        return KVX_ERR_DEVICE;
    return run_op(&plan, OP_UNPACK, layer_begin, layer_end, buf, dst_pool, stream);
}
