// Receive slots for asynchronous retrieval (paper section 3.6, "Asynchronous Retrieval"): a small,
// fixed number of in-flight transfers on the decoding side, each on a stream of its own, completion found
// by polling events.  Host code only; the data moves through kvx_plan + kvx_unpack.
#include <new>
#include <vector>

#include "kvx_internal.h"

using kvx::hip_ok;

namespace {
constexpr uint64_t kAlign = 256;
inline uint64_t align_up(uint64_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

enum SlotState : uint32_t { SLOT_FREE = 0, SLOT_ACQUIRED = 1, SLOT_SCATTERING = 2 };

struct Slot {
    SlotState state = SLOT_FREE;
    uint64_t ticket = 0;
    char *buf = nullptr;
    char *ws = nullptr;
    hipStream_t stream = nullptr;
    hipEvent_t done = nullptr;
};
} // namespace

struct kvx_retriever_s {
    std::vector<Slot> slots;
    uint64_t buf_bytes = 0, ws_bytes = 0;
};

extern "C" {

kvx_status kvx_retriever_arena_bytes(uint32_t num_slots, uint64_t slot_buf_bytes, uint64_t slot_ws_bytes,
                                     uint64_t *out_bytes) {
    if (!num_slots || !slot_buf_bytes || !slot_ws_bytes || !out_bytes) return KVX_ERR_INVALID_ARG;
    if (slot_buf_bytes > (1ull << 48) || slot_ws_bytes > (1ull << 48) || num_slots > 1024) return KVX_ERR_UNSUPPORTED;
    *out_bytes = num_slots * (align_up(slot_buf_bytes) + align_up(slot_ws_bytes));
    return KVX_OK;
}

kvx_status kvx_retriever_create(uint32_t num_slots, uint64_t slot_buf_bytes, uint64_t slot_ws_bytes,
                                void *dev_arena, uint64_t arena_bytes, kvx_retriever_t **out) try {
    if (!out) return KVX_ERR_INVALID_ARG;
    *out = nullptr;
    uint64_t need = 0;
    kvx_status st = kvx_retriever_arena_bytes(num_slots, slot_buf_bytes, slot_ws_bytes, &need);
    if (st != KVX_OK) return st;
    if (!dev_arena) return KVX_ERR_INVALID_ARG;
    if ((uintptr_t)dev_arena % kAlign) return KVX_ERR_ALIGNMENT;
    if (arena_bytes < need) return KVX_ERR_CAPACITY;
    kvx_retriever_s *r = new (std::nothrow) kvx_retriever_s;
    if (!r) return KVX_ERR_HOST_MEMORY;
    r->buf_bytes = align_up(slot_buf_bytes);
    r->ws_bytes = align_up(slot_ws_bytes);
    try {
        r->slots.resize(num_slots);
    } catch (...) {
        delete r;
        return KVX_ERR_HOST_MEMORY;
    }
    char *base = static_cast<char *>(dev_arena);
    for (uint32_t i = 0; i < num_slots; ++i) {
        Slot &s = r->slots[i];
        s.buf = base + i * (r->buf_bytes + r->ws_bytes);
        s.ws = s.buf + r->buf_bytes;
        // default priority on purpose: streams of mixed priorities are not used anywhere in this library
        if (!hip_ok(hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking), "stream of a receive slot") ||
            !hip_ok(hipEventCreateWithFlags(&s.done, hipEventDisableTiming), "event of a receive slot")) {
            kvx_retriever_destroy(r);
            return KVX_ERR_DEVICE;
        }
    }
    *out = r;
    return KVX_OK;
} catch (...) {
    return KVX_ERR_HOST_MEMORY;
}

void kvx_retriever_destroy(kvx_retriever_t *ret) {
    if (!ret) return;
    for (Slot &s : ret->slots) {
        if (s.stream) {
            (void)hipStreamSynchronize(s.stream);
            (void)hipStreamDestroy(s.stream);
        }
        if (s.done) (void)hipEventDestroy(s.done);
    }
    delete ret;
}

kvx_status kvx_retriever_acquire(kvx_retriever_t *ret, uint64_t ticket, uint64_t need_bytes, uint32_t *slot,
                                 void **slot_buf, void **slot_stream) {
    if (!ret || !slot || !slot_buf || !slot_stream) return KVX_ERR_INVALID_ARG;
    if (need_bytes > ret->buf_bytes) return KVX_ERR_CAPACITY;
    for (uint32_t i = 0; i < ret->slots.size(); ++i) {
        Slot &s = ret->slots[i];
        if (s.state != SLOT_FREE) continue;
        s.state = SLOT_ACQUIRED;
        s.ticket = ticket;
        *slot = i;
        *slot_buf = s.buf;
        *slot_stream = s.stream;
        return KVX_OK;
    }
    return KVX_ERR_BUSY;
}

kvx_status kvx_retriever_scatter(kvx_retriever_t *ret, uint32_t slot, const kvx_pool_desc *d,
                                 const kvx_batch_desc *db, uint32_t layer_begin, uint32_t layer_end,
                                 void *dst_pool, const kvx_launch_cfg *launch) {
    if (!ret || slot >= ret->slots.size() || !d || !db || !dst_pool) return KVX_ERR_INVALID_ARG;
    Slot &s = ret->slots[slot];
    if (s.state != SLOT_ACQUIRED) return KVX_ERR_INVALID_ARG;
    kvx_status st = KVX_OK;
    kvx_plan_t *plan = nullptr;
    // A small arrival (a request or a few) is planned on the host, without the slot's workspace: its run
    // records ride in the launch arguments, and the scatter below is the only launch.
    uint64_t pages = db->num_requests;
    if (db->seq_lens && d->page_tokens)
        for (uint32_t r = 0; r < db->num_requests && pages <= KVX_INLINE_RUNS; ++r)
            pages += db->seq_lens[r] / d->page_tokens; // ceil(len/P) <= 1 + len/P, the 1 counted above
    if (pages <= KVX_INLINE_RUNS) {
        st = kvx_plan(nullptr, nullptr, d, db, layer_begin, layer_end, nullptr, 0, s.stream, &plan);
        if (st != KVX_OK) return st;
        int runs = 0;
        (void)kvx_plan_can_launch(plan, &runs);
        if (!runs) { // pages that are not token rows inside: planned on the device like any larger arrival
            kvx_plan_destroy(plan);
            plan = nullptr;
        }
    }
    if (!plan) {
        size_t ws_need = 0;
        st = kvx_plan_workspace_bytes(nullptr, nullptr, d, db, &ws_need);
        if (st != KVX_OK) return st;
        if (ws_need > ret->ws_bytes) return KVX_ERR_CAPACITY;
        st = kvx_plan(nullptr, nullptr, d, db, layer_begin, layer_end, s.ws, ret->ws_bytes, s.stream, &plan);
        if (st != KVX_OK) return st;
    }
    uint64_t total = 0;
    (void)kvx_plan_total_bytes(plan, &total);
    if (total > ret->buf_bytes) {
        kvx_plan_destroy(plan);
        return KVX_ERR_CAPACITY;
    }
    if (launch) st = kvx_plan_set_launch(plan, launch);
    if (st == KVX_OK) st = kvx_unpack(plan, s.buf, ret->buf_bytes, dst_pool, s.stream);
    kvx_plan_destroy(plan); // the launch carries its arguments; the workspace stays with the slot
    if (st != KVX_OK) return st;
    if (!hip_ok(hipEventRecord(s.done, s.stream), "event behind a scatter")) return KVX_ERR_DEVICE;
    s.state = SLOT_SCATTERING;
    return KVX_OK;
}

kvx_status kvx_retriever_abandon(kvx_retriever_t *ret, uint32_t slot) {
    if (!ret || slot >= ret->slots.size()) return KVX_ERR_INVALID_ARG;
    Slot &s = ret->slots[slot];
    if (s.state != SLOT_ACQUIRED) return KVX_ERR_INVALID_ARG;
    if (!hip_ok(hipStreamSynchronize(s.stream), "wait for an abandoned slot")) return KVX_ERR_DEVICE;
    s.state = SLOT_FREE;
    return KVX_OK;
}

kvx_status kvx_retriever_poll(kvx_retriever_t *ret, uint64_t *tickets, uint32_t capacity, uint32_t *count) {
    if (!ret || !count || (capacity && !tickets)) return KVX_ERR_INVALID_ARG;
    uint32_t n = 0;
    *count = 0;
    for (Slot &s : ret->slots) {
        if (n >= capacity) break;
        if (s.state != SLOT_SCATTERING) continue;
        const hipError_t e = hipEventQuery(s.done);
        if (e == hipErrorNotReady) continue;
        if (!hip_ok(e, "query of a slot's event")) return KVX_ERR_DEVICE; // *count already names the slots freed
        tickets[n++] = s.ticket;
        s.state = SLOT_FREE;
        *count = n;
    }
    return KVX_OK;
}

kvx_status kvx_retriever_drain(kvx_retriever_t *ret) {
    if (!ret) return KVX_ERR_INVALID_ARG;
    for (Slot &s : ret->slots)
        if (s.state == SLOT_SCATTERING && !hip_ok(hipEventSynchronize(s.done), "wait for a slot's event"))
            return KVX_ERR_DEVICE;
    return KVX_OK;
}

} // extern "C"
