// HIP kernels of libkvx for gfx950 (CDNA4, 64-wide wavefronts).
//
//   scan_kernel  exclusive prefix sums over the variable request lengths
//                (tokens, pages per side, copy runs per operation), done with
//                wavefront-level sums and one LDS hop across the waves of
//                a single workgroup.  These are the offsets section 3.6 of the
//                paper derives from prompt length, hidden size and precision.
//   fill_kernel  writes the flat copy plan: one kvx_run per maximal span of
//                tokens that stays inside one page on both sides of an
//                operation.  For
//                convert the runs are laid out in groups of a fixed number of
//                slots, one group per page of the coarser side, so that the
//                data mover can keep a group together.
//   plan_small_kernel  scan and fill in one launch of one workgroup, for a
//                batch whose lengths and block tables fit the launch arguments.
//   copy_kernel  the pack / unpack / convert data mover for pages that are
//                [token][head][dim] with rows back to back (a run is then one
//                flat byte range on both sides): every workgroup takes tiles
//                of (run, layer, K|V) and moves them with 16-byte loads and
//                stores, all loads of a tile in flight before its first store.
//                No LDS: no byte changes its position inside a 16-byte unit.
//   copy_inline_kernel  the same data mover with the run records inside its
//                launch arguments, for a small one-sided plan whose runs the
//                host worked out: nothing is planned on the device.
//   xpose_kernel the same three operations for every other page arrangement
//                (head-major, token axis inside 16-byte dim groups, padded or
//                sliced rows): tiles of tokens x 16-byte units, staged through
//                LDS when one side is contiguous along the row and the other
//                along the tokens.
//   xpose_elem_kernel  the same once more for pages that keep the token axis
//                innermost element by element ([head][dim][token]): there bytes
//                change place below the 16-byte grain, and the tile is
//                transposed in LDS one element at a time.
#include <algorithm>
#include <atomic>

#include "kvx_internal.h"

namespace kvx {

using u32x4 = uint32_t __attribute__((ext_vector_type(4)));

// Lengths, page sizes and token positions are all below 2^32, so every division of the planner is a 32-bit
// one (the 64-bit kind is a long dependent instruction sequence here, and it was most of the planner's time).
__device__ __forceinline__ uint32_t ceil_div_q(uint32_t x, uint32_t q) {
    // q == 0 stands for an infinite quantum: only x == 0 has no multiple below it.
    if (q == 0) return x ? 1u : 0u;
    return x ? (x - 1u) / q + 1u : 0u;
}

// lcm(qa, qb) may not fit 32 bits; any value of 2^32 - 1 or more divides like 2^32 - 1 does, since x < 2^32.
__device__ __forceinline__ uint32_t clamp_lcm(uint64_t l) { return l > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)l; }

// Number of cut points in [0, x) at multiples of qa and of qb (l = their lcm): the rank of a run that starts at x.
__device__ __forceinline__ uint64_t cuts_below(uint32_t x, uint32_t qa, uint32_t qb, uint32_t l) {
    return (uint64_t)ceil_div_q(x, qa) + ceil_div_q(x, qb) - ceil_div_q(x, l);
}

// Number of maximal runs of n tokens cut at multiples of qa and of qb.
__device__ __forceinline__ uint64_t count_runs(uint32_t n, uint32_t qa, uint32_t qb, uint32_t l) {
    return n ? cuts_below(n, qa, qb, l) : 0;
}

// ---------------------------------------------------------------------------
// scan
// ---------------------------------------------------------------------------
constexpr int kScanThreads = 1024;
constexpr int kScanWaves = kScanThreads / 64;

// x + (x of another lane), the other lane picked by a data-parallel-primitive control word: the value moves
// inside the vector ALU, not through the LDS crossbar that shuffles use (sixteen waves of shuffles on one
// compute unit were most of this kernel's time).  Lanes the control leaves without a source add 0.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint64_t dpp_add(uint64_t x) {
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)x, CTRL, ROW_MASK, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)(x >> 32), CTRL, ROW_MASK, 0xF, true);
    return x + (((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}
// Inclusive sum over each row of 16 lanes: shifts by 1, 2, 4 and 8 lanes that stop at the row's first lane.
__device__ __forceinline__ uint64_t row_inclusive_sum(uint64_t x) {
    x = dpp_add<0x111, 0xF>(x); // row_shr:1
    x = dpp_add<0x112, 0xF>(x); // row_shr:2
    x = dpp_add<0x114, 0xF>(x); // row_shr:4
    x = dpp_add<0x118, 0xF>(x); // row_shr:8
    return x;
}
// Inclusive sum over the 64 lanes: rows first, then lane 15 of rows 0 and 2 into rows 1 and 3
// (row_bcast:15), then lane 31 into rows 2 and 3 (row_bcast:31).
__device__ __forceinline__ uint64_t wave_inclusive_sum(uint64_t x) {
    x = row_inclusive_sum(x);
    x = dpp_add<0x142, 0xA>(x);
    x = dpp_add<0x143, 0xC>(x);
    return x;
}
__device__ __forceinline__ uint64_t read_lane(uint64_t x, int lane) { // lane is the same for the whole wave
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, lane);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), lane);
    return ((uint64_t)hi << 32) | lo;
}

// `length_of(r)` reads request r's length: from the workspace, or straight from the launch arguments.
// `keep(k, r, value)` sees every prefix sum as it is written (the fused planner keeps them in LDS).
template <typename Lengths, typename Keep>
__device__ __forceinline__ void scan_body(const ScanParams &p, Lengths length_of, Keep keep) {
    __shared__ uint64_t wave_tot[kNumScans][kScanWaves];
    const uint32_t tid = threadIdx.x;
    const uint32_t lane = tid & 63u;
    const uint32_t wave = tid >> 6;
    const uint32_t num_waves = blockDim.x >> 6; // the launch sizes the workgroup to the batch, up to kScanThreads
    uint64_t carry[kNumScans]; // sums over all earlier passes; every lane keeps the same copy
#pragma unroll
    for (int k = 0; k < kNumScans; ++k) carry[k] = 0;

    for (uint32_t base = 0; base < p.num_requests; base += blockDim.x) {
        const uint32_t r = base + tid;
        uint64_t v[kNumScans];
#pragma unroll
        for (int k = 0; k < kNumScans; ++k) v[k] = 0;
        if (r < p.num_requests) {
            const uint32_t n = length_of(r);
            v[SCAN_TOKENS] = n;
            v[SCAN_PAGES_S] = p.page_s ? ceil_div_q(n, p.page_s) : 0;
            v[SCAN_PAGES_D] = p.page_d ? ceil_div_q(n, p.page_d) : 0;
#pragma unroll
            for (int op = 0; op < (int)NUM_OPS; ++op)
                v[SCAN_RUNS0 + op] = p.planned[op] ? count_runs(n, p.qa[op], p.qb[op], clamp_lcm(p.lcm[op])) : 0;
            if (p.planned[OP_CONVERT]) // slots, not runs: a fixed number per group
                v[(int)SCAN_RUNS0 + (int)OP_CONVERT] = (uint64_t)ceil_div_q(n, p.group_quantum) * p.group_slots;
        }
        uint64_t inc[kNumScans];
#pragma unroll
        for (int k = 0; k < kNumScans; ++k) inc[k] = wave_inclusive_sum(v[k]);
        if (lane == 63) {
#pragma unroll
            for (int k = 0; k < kNumScans; ++k) wave_tot[k][wave] = inc[k];
        }
        __syncthreads();
        // second level inside every wave: its lanes 0..15 (one row) scan the at most sixteen wave totals
        const int my_wave = __builtin_amdgcn_readfirstlane((int)wave);
#pragma unroll
        for (int k = 0; k < kNumScans; ++k) {
            const uint64_t t = lane < num_waves ? wave_tot[k][lane] : 0;
            const uint64_t x = row_inclusive_sum(t);
            const uint64_t before = read_lane(x - t, my_wave);
            const uint64_t all = read_lane(x, kScanWaves - 1);
            if (r < p.num_requests) {
                const uint64_t ex = carry[k] + before + inc[k] - v[k];
                p.prefix[k][r] = ex;
                keep(k, r, ex);
            }
            carry[k] += all;
        }
        __syncthreads(); // the next pass overwrites the wave totals
    }
    if (tid < kNumScans) {
        // carry is indexed by a run-time value here: pick it without spilling the array
        uint64_t total = 0;
#pragma unroll
        for (int k = 0; k < kNumScans; ++k) total = (int)tid == k ? carry[k] : total;
        p.prefix[tid][p.num_requests] = total;
        keep((int)tid, p.num_requests, total);
    }
}

__global__ __launch_bounds__(kScanThreads) void scan_kernel(ScanParams p) {
    scan_body(p, [&](uint32_t r) { return p.seq_lens[r]; }, [](int, uint32_t, uint64_t) {});
}

// ---------------------------------------------------------------------------
// fill
// ---------------------------------------------------------------------------
// Where the run-building code reads its inputs: the workspace in global memory (the scan kernel wrote them
// there), or, in the fused planner, LDS and the launch arguments.
struct FillFromWorkspace {
    const FillParams &p;
    __device__ uint32_t len(uint32_t r) const { return p.seq_lens[r]; }
    __device__ uint64_t token_prefix(uint32_t r) const { return p.token_prefix[r]; }
    __device__ uint64_t run_prefix(uint32_t op, uint32_t r) const { return p.run_prefix[op][r]; }
    __device__ uint64_t page(const SideGeom &g, uint32_t r, uint32_t logical) const {
        return g.ids[g.page_prefix[r] + logical];
    }
};

template <typename In>
__device__ __forceinline__ uint64_t side_offset(const SideGeom &g, const In &in, uint32_t r, uint32_t x,
                                                uint64_t buf_base, uint32_t row) {
    if (g.quantum == 0) return buf_base + (uint64_t)x * row;
    const uint32_t logical = x / g.page_tokens;
    const uint32_t slot = x - logical * g.page_tokens;
    return in.page(g, r, logical) * g.stride_page + slot * g.stride_token;
}

// The runs of request r for operation op, written by `nlanes` lanes of which this is lane `lane`.  `between`
// is what separates clearing a request's convert slots from claiming them (a barrier over those lanes).
template <typename In, typename Between>
__device__ __forceinline__ void fill_request(const FillParams &p, const In &in, uint32_t op, uint32_t r,
                                             uint32_t lane, uint32_t nlanes, Between between) {
    const SideGeom &a = p.src[op];
    const SideGeom &b = p.dst[op];
    const uint32_t l = clamp_lcm(p.lcm[op]);
    const uint32_t n = in.len(r);
    if (n == 0) return; // the same for every lane that works on r
    const uint64_t ca = ceil_div_q(n, a.quantum);
    const uint64_t cb = ceil_div_q(n, b.quantum);
    const uint64_t buf_base = in.token_prefix(r) * p.bytes_per_token;
    kvx_run *out = p.runs[op] + in.run_prefix(op, r);
    const bool grouped = (op == OP_CONVERT);
    if (grouped) {
        // slots that no run claims must read as empty (bytes == 0)
        const uint64_t slots = in.run_prefix(op, r + 1) - in.run_prefix(op, r);
        kvx_run none{};
        for (uint64_t i = lane; i < slots; i += nlanes) out[i] = none;
        between();
    }
    // one lane per cut point: the ca multiples of a's quantum, then the cb multiples of b's (all below n)
    for (uint64_t i = lane; i < ca + cb; i += nlanes) {
        uint32_t x;
        if (i < ca) {
            x = (uint32_t)i * a.quantum; // quantum 0 -> ca == 1 -> x == 0
        } else {
            x = (uint32_t)(i - ca) * b.quantum;
            const bool also_a = a.quantum ? (x % a.quantum == 0) : (x == 0);
            if (also_a) continue; // that boundary belongs to the other side's lane
        }
        uint64_t rank = cuts_below(x, a.quantum, b.quantum, l);
        if (grouped) {
            // position = group * slots + rank among the boundaries inside the group
            const uint32_t g = x / p.group_quantum;
            const uint32_t g0 = g * p.group_quantum;
            rank = (uint64_t)g * p.group_slots + rank - cuts_below(g0, a.quantum, b.quantum, l);
        }
        uint64_t end = n;
        if (a.quantum) end = min(end, (uint64_t)(x / a.quantum + 1u) * a.quantum);
        if (b.quantum) end = min(end, (uint64_t)(x / b.quantum + 1u) * b.quantum);
        kvx_run run;
        run.src_off = side_offset(a, in, r, x, buf_base, p.row);
        run.dst_off = side_offset(b, in, r, x, buf_base, p.row);
        run.bytes = (uint32_t)((end - x) * p.row);
        run.seq_len = n;
        run.request = r;
        run.token = x;
        out[rank] = run;
    }
}

constexpr int kFillThreads = 256;

// grid: x = request, y = operation
__global__ __launch_bounds__(kFillThreads) void fill_kernel(FillParams p) {
    const uint32_t op = blockIdx.y;
    if (!p.planned[op]) return;
    const FillFromWorkspace in{p};
    for (uint32_t r = blockIdx.x; r < p.num_requests; r += gridDim.x)
        fill_request(p, in, op, r, threadIdx.x, kFillThreads, [] { __syncthreads(); });
}

// The whole plan of a small batch in one launch: one workgroup stores the tables that came in the launch
// arguments, scans, and writes the runs, the prefix sums going from the scan to the run-building code through
// LDS (nothing a lane wrote to global memory is read back by another inside this kernel).  A wave takes a
// (request, operation) pair at a time.
template <int MAXR>
struct FillFromLds {
    const uint32_t *words;                       // the launch's tables, copied to LDS
    const uint64_t (*prefix)[MAXR + 1];          // [kNumScans][R+1] in LDS
    uint32_t first_id[3];                        // where a side's page ids start in `words` (index = SideGeom::which)
    __device__ uint32_t len(uint32_t r) const { return words[r]; }
    __device__ uint64_t token_prefix(uint32_t r) const { return prefix[SCAN_TOKENS][r]; }
    __device__ uint64_t run_prefix(uint32_t op, uint32_t r) const { return prefix[SCAN_RUNS0 + op][r]; }
    __device__ uint64_t page(const SideGeom &g, uint32_t r, uint32_t logical) const {
        const uint64_t at = prefix[g.which == 1 ? SCAN_PAGES_S : SCAN_PAGES_D][r] + logical;
        return words[first_id[g.which] + (uint32_t)at];
    }
};

// What the fused planner needs beyond the scan's own parameters; everything else of FillParams follows from
// the two (a launch carries at most 4 KiB of arguments, and the tables take most of that).
struct PlanSmallExtra {
    SideGeom sender, receiver;
    kvx_run *runs[NUM_OPS];
    uint64_t bytes_per_token;
    uint32_t row;
    uint32_t pad;
};
static_assert(sizeof(ScanParams) + sizeof(PlanSmallExtra) + sizeof(InlineTables) + sizeof(void *) <= 4096,
              "the fused planner's arguments must fit one launch");

// THREADS lanes for batches of at most MAXR requests: a batch of a few requests (one request arriving at a
// receive slot) gets a single wave and a few KiB of LDS, which finds a place on a device that is busy copying
// far sooner than sixteen waves and their LDS on one compute unit do.
template <int THREADS, int MAXR>
__global__ __launch_bounds__(THREADS) void plan_small_kernel(ScanParams sp, PlanSmallExtra x, InlineTables t,
                                                             uint32_t *__restrict__ workspace_words) {
    __shared__ uint64_t prefix[kNumScans][MAXR + 1];
    __shared__ uint32_t words[kInlineWords];
    FillParams fp{};
    fp.num_requests = sp.num_requests;
    fp.row = x.row;
    fp.bytes_per_token = x.bytes_per_token;
    fp.src[OP_PACK] = x.sender;    // the buffer side of pack and unpack stays all zero
    fp.dst[OP_UNPACK] = x.receiver;
    fp.src[OP_CONVERT] = x.sender;
    fp.dst[OP_CONVERT] = x.receiver;
    fp.group_quantum = sp.group_quantum;
    fp.group_slots = sp.group_slots;
#pragma unroll
    for (int op = 0; op < (int)NUM_OPS; ++op) {
        fp.lcm[op] = sp.lcm[op];
        fp.planned[op] = sp.planned[op];
        fp.runs[op] = x.runs[op];
    }
    const uint32_t c0 = t.count[0], c01 = c0 + t.count[1], total = c01 + t.count[2];
    // The launch arguments live in host memory: every read of them is a trip over the bus.  So they are read
    // once, all of a lane's words in flight together, into LDS (what the scan and the run-building code read)
    // and into the workspace (where inspection finds them).
    constexpr int kPerLane = (kInlineWords + THREADS - 1) / THREADS;
    uint32_t mine[kPerLane];
#pragma unroll
    for (int k = 0; k < kPerLane; ++k) {
        const uint32_t i = k * THREADS + threadIdx.x;
        if (i < total) mine[k] = t.words[i];
    }
#pragma unroll
    for (int k = 0; k < kPerLane; ++k) {
        const uint32_t i = k * THREADS + threadIdx.x;
        if (i >= total) continue;
        const uint32_t seg = i < c0 ? 0u : (i < c01 ? 1u : 2u);
        const uint32_t j = i - (seg == 0u ? 0u : (seg == 1u ? c0 : c01));
        words[i] = mine[k];
        workspace_words[t.dst_word[seg] + j] = mine[k];
    }
    __syncthreads();
    scan_body(sp, [&](uint32_t r) { return words[r]; },
              [&](int k, uint32_t r, uint64_t v) { prefix[k][r] = v; });
    __syncthreads();
    const FillFromLds<MAXR> in{words, prefix, {0u, c0, c01}};
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6, waves = blockDim.x >> 6;
    // The operations one after another (unrolled: the parameters of each are then picked at compile time and
    // stay in registers), the requests of each dealt to the waves; the waves start at different requests per
    // operation so that a batch of one or two requests still spreads over three waves.
#pragma unroll
    for (int op = 0; op < (int)NUM_OPS; ++op) {
        if (!fp.planned[op]) continue;
        for (uint32_t r = (wave + waves - (uint32_t)op % waves) % waves; r < sp.num_requests; r += waves)
            // one wave clears and then claims the slots: its stores to one address keep their order
            fill_request(fp, in, (uint32_t)op, r, lane, 64u, [] { __builtin_amdgcn_wave_barrier(); });
    }
}

// ---------------------------------------------------------------------------
// copy
// ---------------------------------------------------------------------------
// Cache policy of the 16-byte accesses.  0: default.  1: non-temporal loads and stores.  2: non-temporal
// loads, stores at agent scope (sc1), which the L2 writes through at once instead of keeping the line until
// it is evicted; on a streaming copy this measured 6.8 instead of 6.6 TB/s.  The sc1 store has no builtin
// for 16-byte vectors, hence the one-instruction inline asm; the s_nop keeps the following instruction from
// rewriting the four data registers while the store still reads them.
template <int POLICY>
__device__ __forceinline__ u32x4 ld16(const char *p) {
    if (POLICY != 0) return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return *reinterpret_cast<const u32x4 *>(p);
}
// The compiler cannot see that the inline-asm store below joins the queue of outstanding vector memory
// operations.  Making every loaded value "used" before the first such store puts the compiler's own wait
// for the loads in front of all the stores, so no wait of its choosing ever has to count operations it does
// not know about.
template <int POLICY, int N>
__device__ __forceinline__ void loads_done_before_asm_stores(u32x4 (&r)[N]) {
    if (POLICY == 2) {
#pragma unroll
        for (int k = 0; k < N; ++k) asm volatile("" : : "v"(r[k]));
    }
}

template <int POLICY>
__device__ __forceinline__ void st16(char *p, u32x4 v) {
    if (POLICY == 2) asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
    else if (POLICY == 1) __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(p));
    else *reinterpret_cast<u32x4 *>(p) = v;
}

// One run record, fetched as a single 32-byte load from a wave-uniform address.
__device__ __forceinline__ kvx_run load_run(const kvx_run *p) {
    using u32x8 = uint32_t __attribute__((ext_vector_type(8)));
    const u32x8 w = __builtin_nontemporal_load(reinterpret_cast<const u32x8 *>(p));
    kvx_run r;
    r.src_off = ((uint64_t)w[1] << 32) | w[0];
    r.dst_off = ((uint64_t)w[3] << 32) | w[2];
    r.bytes = w[4];
    r.seq_len = w[5];
    r.request = w[6];
    r.token = w[7];
    return r;
}

// The body of the two data movers below, which differ only in where run record e comes from (RUN_AT).  It is a
// macro, not a device function that both call: handed the parameters through a function (by reference or by
// value) the compiler orders the kernel's argument loads differently, and the plan-table kernel came out
// 1.5 % (workload 2) to 3 % (workload 4) slower than with the text in place.
#define KVX_COPY_TILES(RUN_AT) \
    constexpr uint32_t kStep = T * 16u; /* bytes one load instruction of the workgroup covers */                      \
    constexpr uint32_t kTile = kStep * U;                                                                             \
    const uint32_t lane_off = threadIdx.x * 16u;                                                                      \
                                                                                                                      \
    /* Workgroup b runs on XCD b mod 8 and is the (b div 8)-th one there. */                                          \
    uint32_t first = blockIdx.x;                                                                                      \
    if (p.swizzle_block) {                                                                                            \
        const uint32_t j = blockIdx.x >> 3, k = blockIdx.x & 7u;                                                      \
        const uint32_t jb = fast_div(j, p.by_swizzle_block);                                                          \
        first = jb * (8u * p.swizzle_block) + k * p.swizzle_block + (j - jb * p.swizzle_block);                       \
    } else if (p.swizzle_chunk) {                                                                                     \
        first = (blockIdx.x & 7u) * p.swizzle_chunk + (blockIdx.x >> 3);                                              \
    }                                                                                                                 \
                                                                                                                      \
    /* Order 3 deals the tiles out one by one: tile v belongs to part v mod 8 of the runs, and with a grid that is */ \
    /* a multiple of 8 a workgroup stays with its part, the one its XCD works on. */                                  \
    if (p.order == 3) first = blockIdx.x;                                                                             \
                                                                                                                      \
    for (uint64_t v64 = first; v64 < p.total_tiles; v64 += gridDim.x) {                                               \
        uint32_t v = (uint32_t)v64;                                                                                   \
        uint32_t lc, e;                                                                                               \
        uint32_t part = 0;                                                                                            \
        if (p.order == 3) {                                                                                           \
            part = v & 7u;                                                                                            \
            v >>= 3;                                                                                                  \
        }                                                                                                             \
        const uint32_t q = fast_div(v, p.by_tiles_per_run);                                                           \
        const uint32_t s = v - q * p.tiles_per_run;                                                                   \
        if (p.order == 3) {                                                                                           \
            lc = fast_div(q, p.by_runs_per_part);                                                                     \
            e = part * p.runs_per_part + (q - lc * p.runs_per_part);                                                  \
            if (e >= p.num_runs) continue; /* the last part may be short */                                           \
        } else if (p.order == 2) {                                                                                    \
            const uint32_t q2 = fast_div(q, p.by_group);                                                              \
            const uint32_t i = q - q2 * p.group;                                                                      \
            const uint32_t g = fast_div(q2, p.by_num_lc);                                                             \
            lc = q2 - g * p.num_lc;                                                                                   \
            e = g * p.group + i;                                                                                      \
        } else {                                                                                                      \
            lc = fast_div(q, p.by_num_runs);                                                                          \
            e = q - lc * p.num_runs;                                                                                  \
        }                                                                                                             \
        lc += p.lc_first;                                                                                             \
        /* the whole 32-byte record in one scalar load (field by field the compiler fetches it in three */            \
        /* dependent steps, each a round trip to the scalar cache or beyond) */                                       \
        const kvx_run run = RUN_AT(e);                                                                                \
        const uint32_t base = s * kTile;                                                                              \
        if (base >= run.bytes) continue;                                                                              \
        const uint32_t rem = run.bytes - base;                                                                        \
                                                                                                                      \
        const uint32_t layer = p.layer_begin + (lc >> 1);                                                             \
        const uint32_t kv = lc & 1u;                                                                                  \
        const uint64_t seg = (uint64_t)lc * run.seq_len * p.row; /* (layer,kv) step inside a request's buffer */      \
        const uint64_t so = run.src_off + base +                                                                      \
                            (p.src_is_buf ? seg : layer * p.src_stride_layer + kv * p.src_stride_kv);                 \
        const uint64_t dk = run.dst_off + base +                                                                      \
                            (p.dst_is_buf ? seg : layer * p.dst_stride_layer + kv * p.dst_stride_kv);                 \
        const char *sp = src + so + lane_off;                                                                         \
        char *dp = dst + dk + lane_off;                                                                               \
                                                                                                                      \
        if (rem >= kTile) {                                                                                           \
            u32x4 r[U];                                                                                               \
            _Pragma("unroll")                                                                                         \
            for (int k = 0; k < U; ++k) r[k] = ld16<NT>(sp + k * kStep);                                              \
            loads_done_before_asm_stores<NT>(r);                                                                      \
            _Pragma("unroll")                                                                                         \
            for (int k = 0; k < U; ++k) st16<NT>(dp + k * kStep, r[k]);                                               \
        } else {                                                                                                      \
            u32x4 r[U] = {}; /* lanes past the end load nothing, yet every register is handed to the asm below */     \
            _Pragma("unroll")                                                                                         \
            for (int k = 0; k < U; ++k)                                                                               \
                if (lane_off + k * kStep < rem) r[k] = ld16<NT>(sp + k * kStep);                                      \
            loads_done_before_asm_stores<NT>(r);                                                                      \
            _Pragma("unroll")                                                                                         \
            for (int k = 0; k < U; ++k)                                                                               \
                if (lane_off + k * kStep < rem) st16<NT>(dp + k * kStep, r[k]);                                       \
        }                                                                                                             \
    }

template <int T, int U, int NT>
__global__ __launch_bounds__(T) void copy_kernel(const kvx_run *__restrict__ runs, const char *__restrict__ src,
                                                 char *__restrict__ dst, CopyParams p) {
#define KVX_RUN_IN_TABLE(e) load_run(runs + (e))
    KVX_COPY_TILES(KVX_RUN_IN_TABLE)
#undef KVX_RUN_IN_TABLE
}

// The same with the run records inside the launch arguments (a small one-sided batch whose runs the host worked
// out): no table in device memory, no planning launch.
template <int T, int U, int NT>
__global__ __launch_bounds__(T) void copy_inline_kernel(InlineRuns runs, const char *__restrict__ src,
                                                        char *__restrict__ dst, CopyParams p) {
#define KVX_RUN_IN_ARGUMENTS(e) runs.run[e]
    KVX_COPY_TILES(KVX_RUN_IN_ARGUMENTS)
#undef KVX_RUN_IN_ARGUMENTS
}
#undef KVX_COPY_TILES
static_assert(sizeof(InlineRuns) + sizeof(CopyParams) + 2 * sizeof(void *) <= 4096, "launch arguments are limited to 4 KiB");

// ---------------------------------------------------------------------------
// xpose: pages that are not [token][head][dim] inside
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint64_t unit_offset(const XposeSide &g, uint32_t u) {
    // u < 65536 and units_per_granule < 65536 make the multiply-high division exact
    const uint32_t q = g.units_per_granule == 1u ? u : __umulhi(u, g.granule_magic);
    return (uint64_t)q * g.granule_step + (uint64_t)(u - q * g.units_per_granule) * 16u;
}

// Cell c of a tile -> (token, unit) inside the tile.  On a token-fast side consecutive lanes walk the
// tokens of one unit column, otherwise the units of one token.
template <bool TOKEN_FAST>
__device__ __forceinline__ void cell_to_tu(uint32_t c, uint32_t log2_tt, uint32_t log2_uu, uint32_t &t, uint32_t &u) {
    if (TOKEN_FAST) {
        t = c & ((1u << log2_tt) - 1u);
        u = c >> log2_tt;
    } else {
        u = c & ((1u << log2_uu) - 1u);
        t = c >> log2_uu;
    }
}

template <bool SRC_TF, bool DST_TF, int NT>
__global__ __launch_bounds__(kXposeThreads) void xpose_kernel(const kvx_run *__restrict__ runs,
                                                              const char *__restrict__ src,
                                                              char *__restrict__ dst, XposeParams p) {
    constexpr int kPerLane = kXposeCells / kXposeThreads;
    // [token][unit] with one unit of padding per token row, so that a column walk spreads over the banks
    __shared__ u32x4 stage[(SRC_TF != DST_TF) ? kXposeCells + 64 : 1];
    const uint32_t pitch = (1u << p.log2_uu) + 1u;
    const uint32_t tiles_per_run = p.tiles_t * p.tiles_u;

    uint32_t first = blockIdx.x;
    if (p.swizzle_chunk) first = (blockIdx.x & 7u) * p.swizzle_chunk + (blockIdx.x >> 3);

    for (uint64_t v64 = first; v64 < p.total_tiles; v64 += gridDim.x) {
        const uint32_t v = (uint32_t)v64;
        const uint32_t sidx = v % tiles_per_run;
        const uint32_t q = v / tiles_per_run;
        uint32_t lc, e;
        if (p.order == 2) {
            const uint32_t i = q % p.group;
            const uint32_t q2 = q / p.group;
            lc = q2 % p.num_lc;
            e = (q2 / p.num_lc) * p.group + i;
        } else {
            e = q % p.num_runs;
            lc = q / p.num_runs;
        }
        lc += p.lc_first;
        const kvx_run run = runs[e];
        const uint32_t tokens = run.bytes / p.row;
        const uint32_t t0 = (sidx / p.tiles_u) << p.log2_tt;
        const uint32_t u0 = (sidx % p.tiles_u) << p.log2_uu;
        if (t0 >= tokens) continue; // uniform over the workgroup: no barrier is skipped by part of it

        const uint32_t layer = p.layer_begin + (lc >> 1);
        const uint32_t kv = lc & 1u;
        const uint64_t seg = (uint64_t)lc * run.seq_len * p.row;
        const char *sp = src + run.src_off + (p.s.is_buf ? seg : layer * p.s.stride_layer + kv * p.s.stride_kv);
        char *dp = dst + run.dst_off + (p.d.is_buf ? seg : layer * p.d.stride_layer + kv * p.d.stride_kv);

        u32x4 r[kPerLane] = {}; // cells outside the run load nothing, yet every register is handed on below
        bool ok[kPerLane];
#pragma unroll
        for (int k = 0; k < kPerLane; ++k) {
            uint32_t t, u;
            cell_to_tu<SRC_TF>(k * kXposeThreads + threadIdx.x, p.log2_tt, p.log2_uu, t, u);
            ok[k] = (t0 + t < tokens) && (u0 + u < p.units_per_row);
            if (ok[k]) r[k] = ld16<NT>(sp + (uint64_t)(t0 + t) * p.s.token_step + unit_offset(p.s, u0 + u));
        }
        if (SRC_TF == DST_TF) {
            loads_done_before_asm_stores<NT>(r);
#pragma unroll
            for (int k = 0; k < kPerLane; ++k) {
                uint32_t t, u;
                cell_to_tu<DST_TF>(k * kXposeThreads + threadIdx.x, p.log2_tt, p.log2_uu, t, u);
                if (ok[k]) st16<NT>(dp + (uint64_t)(t0 + t) * p.d.token_step + unit_offset(p.d, u0 + u), r[k]);
            }
        } else {
#pragma unroll
            for (int k = 0; k < kPerLane; ++k) {
                uint32_t t, u;
                cell_to_tu<SRC_TF>(k * kXposeThreads + threadIdx.x, p.log2_tt, p.log2_uu, t, u);
                if (ok[k]) stage[t * pitch + u] = r[k];
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < kPerLane; ++k) {
                uint32_t t, u;
                cell_to_tu<DST_TF>(k * kXposeThreads + threadIdx.x, p.log2_tt, p.log2_uu, t, u);
                if ((t0 + t < tokens) && (u0 + u < p.units_per_row))
                    st16<NT>(dp + (uint64_t)(t0 + t) * p.d.token_step + unit_offset(p.d, u0 + u),
                             stage[t * pitch + u]);
            }
            __syncthreads(); // the next tile of this workgroup reuses the stage
        }
    }
}

// ---------------------------------------------------------------------------
// xpose_elem: a side whose pages keep the token axis innermost, element by element
// ---------------------------------------------------------------------------
// [head][dim][token] pages: element (column j of the row, token t) sits at j*column_step + t*E, so going to
// or from token rows moves every element, not whole 16-byte units.  A tile of 2^log2_tt tokens by
// 2^log2_wu units of the row (16 KiB) is staged in LDS as [token][row bytes of the tile]: the side that is
// addressed by units moves 16 bytes per lane along its contiguous axis, the token-innermost side moves 16
// bytes per lane along the tokens of one column (16/E tokens) and picks or drops them in LDS one element
// at a time.  Both sides see only whole, aligned 16-byte accesses in global memory whenever a column's
// piece starts on a 16-byte boundary and is wholly live; ragged ends, and pages whose columns are no
// multiple of 16 bytes, go element by element.  In LDS, row t starts 4 bytes after a multiple of the tile's
// width and is rotated by 8 bytes per group of 16/E tokens: a wave that walks down the columns (16 or more
// groups of tokens, a few neighbouring columns) then touches every bank once instead of four of them
// sixteen times.
template <int E> struct ElemType;
template <> struct ElemType<1> { using type = uint8_t; };
template <> struct ElemType<2> { using type = uint16_t; };
template <> struct ElemType<4> { using type = uint32_t; };
template <> struct ElemType<8> { using type = uint64_t; };

template <int E>
__device__ __forceinline__ typename ElemType<E>::type lds_get(const unsigned char *p) {
    if constexpr (E == 8) { // the rows of the stage are only 4-byte aligned
        const uint32_t *q = reinterpret_cast<const uint32_t *>(p);
        return (uint64_t)q[0] | ((uint64_t)q[1] << 32);
    } else {
        return *reinterpret_cast<const typename ElemType<E>::type *>(p);
    }
}
template <int E>
__device__ __forceinline__ void lds_put(unsigned char *p, typename ElemType<E>::type v) {
    if constexpr (E == 8) {
        uint32_t *q = reinterpret_cast<uint32_t *>(p);
        q[0] = (uint32_t)v;
        q[1] = (uint32_t)(v >> 32);
    } else {
        *reinterpret_cast<typename ElemType<E>::type *>(p) = v;
    }
}
template <int E, int NT>
__device__ __forceinline__ typename ElemType<E>::type ld_elem(const char *p) {
    using T = typename ElemType<E>::type;
    if (NT != 0) return __builtin_nontemporal_load(reinterpret_cast<const T *>(p));
    return *reinterpret_cast<const T *>(p);
}
template <int E, int NT>
__device__ __forceinline__ void st_elem(char *p, typename ElemType<E>::type v) {
    using T = typename ElemType<E>::type;
    if (NT != 0) __builtin_nontemporal_store(v, reinterpret_cast<T *>(p));
    else *reinterpret_cast<T *>(p) = v;
}

__device__ __forceinline__ uint64_t elem_unit_offset(const ElemSide &g, uint32_t u) {
    const uint32_t q = g.units_per_granule == 1u ? u : __umulhi(u, g.granule_magic);
    return (uint64_t)q * g.granule_step + (uint64_t)(u - q * g.units_per_granule) * 16u;
}

// GM (group mode), for a convert whose token-innermost side has the coarser pages: 0 = a tile belongs to one
// run; 1 / 2 = a tile spans the tokens of one whole group of runs, i.e. one page of the coarser side, which is
// the source (1) or the destination (2).  The coarser side is then addressed from the group's first record
// (its runs follow one another inside that one page), the finer side run by run through a small table of
// the group's offsets in LDS.  Per run, a fine receiver would hand each tile only a short piece of every
// column of the coarse page, a fraction of a 128-byte line; per group the pieces are whole.
template <int E, int SK, int DK, int NT, int GM>
__global__ __launch_bounds__(kElemThreads) void xpose_elem_kernel(const kvx_run *__restrict__ runs,
                                                                  const char *__restrict__ src,
                                                                  char *__restrict__ dst, ElemParams p) {
    using T = typename ElemType<E>::type;
    constexpr int kPerLane = kElemCells / kElemThreads;
    constexpr uint32_t X = 16u / E;                 // tokens in 16 bytes of a column
    constexpr uint32_t kLog2X = X == 16 ? 4 : (X == 8 ? 3 : (X == 4 ? 2 : 1));
    __shared__ __align__(16) unsigned char stage[kElemCells * 16 + 4 * kElemMaxTokens];
    __shared__ uint64_t fine_off[GM ? kElemMaxGroup : 1];
    union Unit {
        u32x4 v;
        T e[X];
    };
    const uint32_t width = 16u << p.log2_wu;        // bytes of the row per tile
    const uint32_t pitch = width + 4u;
    const uint32_t log2_gt = p.log2_tt - kLog2X;    // 16-byte pieces per column of the tile
    // byte `b` of the tile's row of token `t` in the stage (b and the rotation are multiples of the access size)
    auto at_stage = [&](uint32_t t, uint32_t b) -> uint32_t {
        return t * pitch + ((b + ((t >> kLog2X) << 3)) & (width - 1u));
    };
    const uint32_t tiles_per_run = p.tiles_t * p.tiles_w;
    const uint32_t num_units = GM ? p.num_groups : p.num_runs; // what the tile space counts: groups or runs

    uint32_t first = blockIdx.x;
    if (p.swizzle_chunk) first = (blockIdx.x & 7u) * p.swizzle_chunk + (blockIdx.x >> 3);

    for (uint64_t v64 = first; v64 < p.total_tiles; v64 += gridDim.x) {
        const uint32_t v = (uint32_t)v64;
        const uint32_t sidx = v % tiles_per_run;
        const uint32_t q = v / tiles_per_run;
        uint32_t lc, e;
        if (GM) {                       // one "run" per group: no inner group index to keep together
            if (p.order == 2) {
                lc = q % p.num_lc;
                e = q / p.num_lc;
            } else {
                e = q % num_units;
                lc = q / num_units;
            }
        } else if (p.order == 2) {
            const uint32_t i = q % p.group;
            const uint32_t q2 = q / p.group;
            lc = q2 % p.num_lc;
            e = (q2 / p.num_lc) * p.group + i;
        } else {
            e = q % num_units;
            lc = q / num_units;
        }
        lc += p.lc_first;
        const kvx_run run = runs[GM ? e * p.group : e];
        // tokens this tile space unit holds: those of the run, or those of the whole group (the group's first
        // run starts at a page boundary of the coarser side, and the request may end inside that page)
        const uint32_t tokens = GM ? min(p.coarse_tokens, run.seq_len - run.token) : run.bytes / p.row;
        const uint32_t t0 = (sidx / p.tiles_w) << p.log2_tt;
        const uint32_t w0 = (sidx % p.tiles_w) << p.log2_wu; // first unit of the row in this tile
        if (run.bytes == 0 || t0 >= tokens) continue; // uniform over the workgroup: no barrier is skipped by part of it
        const uint32_t live = tokens - t0;                   // tokens from the tile's first one on

        const uint32_t layer = p.layer_begin + (lc >> 1);
        const uint32_t kv = lc & 1u;
        const uint64_t seg = (uint64_t)lc * run.seq_len * p.row;
        const uint64_t s_lc = p.s.is_buf ? seg : layer * p.s.stride_layer + kv * p.s.stride_kv;
        const uint64_t d_lc = p.d.is_buf ? seg : layer * p.d.stride_layer + kv * p.d.stride_kv;
        if (GM) {
            if (threadIdx.x < p.group) {
                const kvx_run *r = runs + e * p.group + threadIdx.x;
                fine_off[threadIdx.x] = GM == 1 ? r->dst_off : r->src_off;
            }
            __syncthreads();
        }
        // Where token `t` of the tile lives on a side: the base its addressing starts from, and the token's
        // index from there.  The finer side of a group changes base with every run.
        auto src_at = [&](uint32_t t, uint32_t &tin) -> const char * {
            if (GM == 2) {
                const uint32_t i = fast_div(t0 + t, p.by_fine);
                tin = t0 + t - i * p.fine_tokens;
                return src + fine_off[i] + s_lc;
            }
            tin = t0 + t;
            return src + run.src_off + s_lc;
        };
        auto dst_at = [&](uint32_t t, uint32_t &tin) -> char * {
            if (GM == 1) {
                const uint32_t i = fast_div(t0 + t, p.by_fine);
                tin = t0 + t - i * p.fine_tokens;
                return dst + fine_off[i] + d_lc;
            }
            tin = t0 + t;
            return dst + run.dst_off + d_lc;
        };

        // ---- source -> stage
        if (SK != 2) {
            u32x4 r[kPerLane] = {};
            bool ok[kPerLane];
#pragma unroll
            for (int k = 0; k < kPerLane; ++k) {
                uint32_t t, u, tin;
                cell_to_tu<SK == 1>(k * kElemThreads + threadIdx.x, p.log2_tt, p.log2_wu, t, u);
                ok[k] = t < live && w0 + u < p.units_per_row;
                if (ok[k]) {
                    const char *a = src_at(t, tin);
                    a += (uint64_t)tin * p.s.token_step + elem_unit_offset(p.s, w0 + u);
                    r[k] = p.cached_loads ? ld16<0>(a) : ld16<NT>(a);
                }
            }
#pragma unroll
            for (int k = 0; k < kPerLane; ++k) {
                uint32_t t, u;
                cell_to_tu<SK == 1>(k * kElemThreads + threadIdx.x, p.log2_tt, p.log2_wu, t, u);
                if (ok[k]) {
                    const uint32_t d[4] = {r[k].x, r[k].y, r[k].z, r[k].w};
#pragma unroll
                    for (uint32_t i = 0; i < 4; ++i) // dword by dword: the rotation may wrap inside a unit
                        *reinterpret_cast<uint32_t *>(stage + at_stage(t, u * 16u + 4u * i)) = d[i];
                }
            }
        } else {
            Unit r[kPerLane];
            int how[kPerLane]; // 0 nothing, 1 a whole aligned piece (already loaded), 2 element by element
            const char *at[kPerLane];
#pragma unroll
            for (int k = 0; k < kPerLane; ++k) {
                const uint32_t c = k * kElemThreads + threadIdx.x;
                const uint32_t ta = (c & ((1u << log2_gt) - 1u)) << kLog2X, jl = c >> log2_gt;
                const uint32_t jb = w0 * 16u + jl * E;  // byte of the row this column starts at
                how[k] = 0;
                if (ta < live && jb < p.row) {
                    uint32_t tin;
                    const char *a = src_at(ta, tin);
                    at[k] = a += (uint64_t)(jb / E) * p.s.column_step + (uint64_t)tin * E;
                    how[k] = (ta + X <= live && ((uintptr_t)a & 15u) == 0) ? 1 : 2;
                    if (how[k] == 1) r[k].v = p.cached_loads ? ld16<0>(a) : ld16<NT>(a);
                }
            }
#pragma unroll
            for (int k = 0; k < kPerLane; ++k) {
                const uint32_t c = k * kElemThreads + threadIdx.x;
                const uint32_t ta = (c & ((1u << log2_gt) - 1u)) << kLog2X, jl = c >> log2_gt;
                unsigned char *w = stage + at_stage(ta, jl * E); // one group of tokens: the same rotation for all
                if (how[k] == 1) {
#pragma unroll
                    for (uint32_t i = 0; i < X; ++i) lds_put<E>(w + i * pitch, r[k].e[i]);
                } else if (how[k] == 2) {
                    // a ragged piece comes element by element out of one or two 64-byte sectors: loads that
                    // may stay in the cache, so that the sector is fetched once
                    for (uint32_t i = 0; i < X && ta + i < live; ++i) lds_put<E>(w + i * pitch, ld_elem<E, 0>(at[k] + i * E));
                }
            }
        }
        __syncthreads();
        // ---- stage -> destination
        if (DK != 2) {
#pragma unroll
            for (int k = 0; k < kPerLane; ++k) {
                uint32_t t, u, tin;
                cell_to_tu<DK == 1>(k * kElemThreads + threadIdx.x, p.log2_tt, p.log2_wu, t, u);
                if (t < live && w0 + u < p.units_per_row) {
                    uint32_t d[4];
#pragma unroll
                    for (uint32_t i = 0; i < 4; ++i)
                        d[i] = *reinterpret_cast<const uint32_t *>(stage + at_stage(t, u * 16u + 4u * i));
                    const u32x4 val = {d[0], d[1], d[2], d[3]};
                    char *a = dst_at(t, tin);
                    a += (uint64_t)tin * p.d.token_step + elem_unit_offset(p.d, w0 + u);
                    if (p.cached_stores) st16<0>(a, val);
                    else st16<NT>(a, val);
                }
            }
        } else {
#pragma unroll
            for (int k = 0; k < kPerLane; ++k) {
                const uint32_t c = k * kElemThreads + threadIdx.x;
                const uint32_t ta = (c & ((1u << log2_gt) - 1u)) << kLog2X, jl = c >> log2_gt;
                const uint32_t jb = w0 * 16u + jl * E;
                if (ta >= live || jb >= p.row) continue;
                uint32_t tin;
                char *a = dst_at(ta, tin);
                a += (uint64_t)(jb / E) * p.d.column_step + (uint64_t)tin * E;
                const unsigned char *w = stage + at_stage(ta, jl * E);
                if (ta + X <= live && ((uintptr_t)a & 15u) == 0) {
                    Unit val;
#pragma unroll
                    for (uint32_t i = 0; i < X; ++i) val.e[i] = lds_get<E>(w + i * pitch);
                    if (p.cached_stores) st16<0>(a, val.v);
                    else st16<NT>(a, val.v);
                } else {
                    for (uint32_t i = 0; i < X && ta + i < live; ++i) {
                        if (p.cached_stores) st_elem<E, 0>(a + i * E, lds_get<E>(w + i * pitch));
                        else st_elem<E, NT>(a + i * E, lds_get<E>(w + i * pitch));
                    }
                }
            }
        }
        __syncthreads(); // the next tile of this workgroup reuses the stage (and the table of offsets)
    }
}

// Plain contiguous copy with the data mover's access shape: the yardstick.
template <int T, int U, int NT>
__global__ __launch_bounds__(T) void plain_copy_kernel(const char *__restrict__ src, char *__restrict__ dst,
                                                       uint64_t bytes) {
    constexpr uint32_t kStep = T * 16u;
    constexpr uint64_t kTile = (uint64_t)kStep * U;
    const uint32_t lane_off = threadIdx.x * 16u;
    for (uint64_t base = (uint64_t)blockIdx.x * kTile; base < bytes; base += (uint64_t)gridDim.x * kTile) {
        const uint64_t rem = bytes - base;
        const char *sp = src + base + lane_off;
        char *dp = dst + base + lane_off;
        if (rem >= kTile) {
            u32x4 r[U];
#pragma unroll
            for (int k = 0; k < U; ++k) r[k] = ld16<NT>(sp + k * kStep);
            loads_done_before_asm_stores<NT>(r);
#pragma unroll
            for (int k = 0; k < U; ++k) st16<NT>(dp + k * kStep, r[k]);
        } else {
            u32x4 r[U] = {}; // lanes past the end load nothing, yet every register is handed to the asm below
#pragma unroll
            for (int k = 0; k < U; ++k)
                if (lane_off + k * kStep < rem) r[k] = ld16<NT>(sp + k * kStep);
            loads_done_before_asm_stores<NT>(r);
#pragma unroll
            for (int k = 0; k < U; ++k)
                if (lane_off + k * kStep < rem) st16<NT>(dp + k * kStep, r[k]);
        }
    }
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
// hipGetLastError reports the last error of ANY earlier runtime call of this thread (a caller's event
// query that was "not ready" is enough), so the slate is wiped before each launch and read right after it.
#define KVX_LAUNCH(...)                 \
    do {                                \
        (void)hipGetLastError();        \
        hipLaunchKernelGGL(__VA_ARGS__); \
    } while (0)
hipError_t launch_scan(const ScanParams &p, hipStream_t stream) {
    // whole waves, no more of them than the batch has requests for (a short batch then costs one wave's work)
    const uint32_t threads = std::min<uint32_t>(kScanThreads, std::max<uint32_t>(64u, (p.num_requests + 63u) / 64u * 64u));
    KVX_LAUNCH(scan_kernel, dim3(1), dim3(threads), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_plan_small(const ScanParams &sp, const FillParams &fp, const InlineTables &t,
                             uint32_t *workspace_words, hipStream_t stream) {
    if (sp.num_requests > kInlineWords) return hipErrorInvalidValue; // the prefix sums would not fit the LDS arrays
    PlanSmallExtra x{};
    x.sender = fp.src[OP_CONVERT].which == 1 ? fp.src[OP_CONVERT] : fp.src[OP_PACK];
    x.receiver = fp.dst[OP_CONVERT].which == 2 ? fp.dst[OP_CONVERT] : fp.dst[OP_UNPACK];
    for (int op = 0; op < (int)NUM_OPS; ++op) x.runs[op] = fp.runs[op];
    x.bytes_per_token = fp.bytes_per_token;
    x.row = fp.row;
    // A wave builds the runs of one request of one operation at a time: one wave for up to 4 requests, four
    // while that leaves a wave at most two turns, sixteen beyond.
    uint32_t ops = 0;
    for (int op = 0; op < (int)NUM_OPS; ++op) ops += sp.planned[op] ? 1u : 0u;
    if (sp.num_requests <= 4)
        KVX_LAUNCH((plan_small_kernel<64, 4>), dim3(1), dim3(64), 0, stream, sp, x, t, workspace_words);
    else if (sp.num_requests <= 64 && sp.num_requests * ops <= 8)
        KVX_LAUNCH((plan_small_kernel<256, 64>), dim3(1), dim3(256), 0, stream, sp, x, t, workspace_words);
    else if (sp.num_requests <= 64)
        KVX_LAUNCH((plan_small_kernel<kScanThreads, 64>), dim3(1), dim3(kScanThreads), 0, stream, sp, x, t,
                   workspace_words);
    else
        KVX_LAUNCH((plan_small_kernel<kScanThreads, (int)kInlineWords>), dim3(1), dim3(kScanThreads), 0, stream, sp, x, t,
                   workspace_words);
    return hipGetLastError();
}

hipError_t launch_fill(const FillParams &p, hipStream_t stream) {
    if (p.num_requests == 0) return hipSuccess;
    const uint32_t gx = p.num_requests < 65535u ? p.num_requests : 65535u;
    KVX_LAUNCH(fill_kernel, dim3(gx, NUM_OPS), dim3(kFillThreads), 0, stream, p);
    return hipGetLastError();
}

namespace {

// Lets kernel `fn` reserve all of a compute unit's LDS.  The attribute is sticky, per kernel instance and per
// device: `raised_on` (one per instance) remembers the devices where it has been set.
inline hipError_t raise_lds_limit(const void *fn, std::atomic<uint64_t> &raised_on) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = dev >= 0 && dev < 64 ? 1ull << dev : 0;
    if (!(raised_on.load(std::memory_order_relaxed) & bit) || !bit) {
        e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsPerCu);
        if (e != hipSuccess) return e;
        raised_on.fetch_or(bit, std::memory_order_relaxed);
    }
    return hipSuccess;
}

// Dispatch of the runtime (threads, unroll, nontemporal) triple to a template instance.
// `lds` bytes of dynamic LDS are reserved and never touched: they only cap the workgroups per compute unit.
template <int T, int U, int NT>
hipError_t copy_tun(const CopyParams &p, const InlineRuns *inline_runs, uint32_t grid, uint32_t lds,
                    hipStream_t stream) {
    if (inline_runs) {
        if (lds > 64u * 1024u) {
            static std::atomic<uint64_t> raised_on{0};
            const hipError_t e = raise_lds_limit(reinterpret_cast<const void *>(&copy_inline_kernel<T, U, NT>), raised_on);
            if (e != hipSuccess) return e;
        }
        KVX_LAUNCH((copy_inline_kernel<T, U, NT>), dim3(grid), dim3(T), lds, stream, *inline_runs, p.src, p.dst, p);
        return hipGetLastError();
    }
    if (lds > 64u * 1024u) {
        static std::atomic<uint64_t> raised_on{0};
        const hipError_t e = raise_lds_limit(reinterpret_cast<const void *>(&copy_kernel<T, U, NT>), raised_on);
        if (e != hipSuccess) return e;
    }
    KVX_LAUNCH((copy_kernel<T, U, NT>), dim3(grid), dim3(T), lds, stream, p.runs, p.src, p.dst, p);
    return hipGetLastError();
}

template <int T, int U>
hipError_t copy_tu(const CopyParams &p, const InlineRuns *ir, int nt, uint32_t grid, uint32_t lds, hipStream_t stream) {
    if (nt == 2) return copy_tun<T, U, 2>(p, ir, grid, lds, stream);
    return nt == 1 ? copy_tun<T, U, 1>(p, ir, grid, lds, stream) : copy_tun<T, U, 0>(p, ir, grid, lds, stream);
}

template <int T>
hipError_t copy_t(const CopyParams &p, const InlineRuns *ir, uint32_t unroll, int nt, uint32_t grid, uint32_t lds,
                  hipStream_t stream) {
    switch (unroll) {
    case 1: return copy_tu<T, 1>(p, ir, nt, grid, lds, stream);
    case 2: return copy_tu<T, 2>(p, ir, nt, grid, lds, stream);
    case 4: return copy_tu<T, 4>(p, ir, nt, grid, lds, stream);
    case 8: return copy_tu<T, 8>(p, ir, nt, grid, lds, stream);
    default: return hipErrorInvalidValue;
    }
}

template <int T, int U>
hipError_t plain_tu(char *dst, const char *src, uint64_t bytes, int nt, uint32_t max_wg, hipStream_t stream) {
    const uint64_t tile = (uint64_t)T * 16u * U;
    const uint64_t tiles = (bytes + tile - 1) / tile;
    const uint64_t cap = std::min<uint64_t>(max_wg, (1u << 31) / T);
    const uint32_t grid = (uint32_t)(tiles < cap ? tiles : cap);
    if (nt == 2) KVX_LAUNCH((plain_copy_kernel<T, U, 2>), dim3(grid), dim3(T), 0, stream, src, dst, bytes);
    else if (nt == 1) KVX_LAUNCH((plain_copy_kernel<T, U, 1>), dim3(grid), dim3(T), 0, stream, src, dst, bytes);
    else KVX_LAUNCH((plain_copy_kernel<T, U, 0>), dim3(grid), dim3(T), 0, stream, src, dst, bytes);
    return hipGetLastError();
}

template <int T>
hipError_t plain_t(char *dst, const char *src, uint64_t bytes, uint32_t unroll, int nt, uint32_t max_wg,
                   hipStream_t stream) {
    switch (unroll) {
    case 1: return plain_tu<T, 1>(dst, src, bytes, nt, max_wg, stream);
    case 2: return plain_tu<T, 2>(dst, src, bytes, nt, max_wg, stream);
    case 4: return plain_tu<T, 4>(dst, src, bytes, nt, max_wg, stream);
    case 8: return plain_tu<T, 8>(dst, src, bytes, nt, max_wg, stream);
    default: return hipErrorInvalidValue;
    }
}

} // namespace

hipError_t launch_copy(const CopyParams &p, const InlineRuns *inline_runs, uint32_t threads, uint32_t unroll,
                       int nontemporal, uint32_t grid, uint32_t lds_bytes, hipStream_t stream) {
    if (p.total_tiles == 0 || grid == 0) return hipSuccess;
    if (inline_runs && p.num_runs > kInlineRuns) return hipErrorInvalidValue;
    switch (threads) {
    case 64: return copy_t<64>(p, inline_runs, unroll, nontemporal, grid, lds_bytes, stream);
    case 128: return copy_t<128>(p, inline_runs, unroll, nontemporal, grid, lds_bytes, stream);
    case 256: return copy_t<256>(p, inline_runs, unroll, nontemporal, grid, lds_bytes, stream);
    case 512: return copy_t<512>(p, inline_runs, unroll, nontemporal, grid, lds_bytes, stream);
    case 1024: return copy_t<1024>(p, inline_runs, unroll, nontemporal, grid, lds_bytes, stream);
    default: return hipErrorInvalidValue;
    }
}

namespace {
template <bool S, bool D>
hipError_t xpose_sd(const XposeParams &p, int nt, uint32_t grid, hipStream_t stream) {
    if (nt == 2)
        KVX_LAUNCH((xpose_kernel<S, D, 2>), dim3(grid), dim3(kXposeThreads), 0, stream, p.runs, p.src,
                           p.dst, p);
    else if (nt == 1)
        KVX_LAUNCH((xpose_kernel<S, D, 1>), dim3(grid), dim3(kXposeThreads), 0, stream, p.runs, p.src,
                           p.dst, p);
    else
        KVX_LAUNCH((xpose_kernel<S, D, 0>), dim3(grid), dim3(kXposeThreads), 0, stream, p.runs, p.src,
                           p.dst, p);
    return hipGetLastError();
}
} // namespace

hipError_t launch_xpose(const XposeParams &p, bool src_token_fast, bool dst_token_fast, int nontemporal,
                        uint32_t grid, hipStream_t stream) {
    if (p.total_tiles == 0 || grid == 0) return hipSuccess;
    if (src_token_fast)
        return dst_token_fast ? xpose_sd<true, true>(p, nontemporal, grid, stream)
                              : xpose_sd<true, false>(p, nontemporal, grid, stream);
    return dst_token_fast ? xpose_sd<false, true>(p, nontemporal, grid, stream)
                          : xpose_sd<false, false>(p, nontemporal, grid, stream);
}

namespace {
template <int E, int SK, int DK, int GM>
hipError_t xpose_elem_esdg(const ElemParams &p, int nt, uint32_t grid, hipStream_t stream) {
    if (nt)
        KVX_LAUNCH((xpose_elem_kernel<E, SK, DK, 1, GM>), dim3(grid), dim3(kElemThreads), 0, stream, p.runs, p.src, p.dst, p);
    else
        KVX_LAUNCH((xpose_elem_kernel<E, SK, DK, 0, GM>), dim3(grid), dim3(kElemThreads), 0, stream, p.runs, p.src, p.dst, p);
    return hipGetLastError();
}
template <int E, int SK, int DK>
hipError_t xpose_elem_esd(const ElemParams &p, int nt, uint32_t grid, hipStream_t stream) {
    // a group's tile is addressed from the coarser side, which is the token-innermost one (kind 2)
    if (SK == 2 && p.group_mode == 1) return xpose_elem_esdg<E, SK, DK, (SK == 2 ? 1 : 0)>(p, nt, grid, stream);
    if (DK == 2 && p.group_mode == 2) return xpose_elem_esdg<E, SK, DK, (DK == 2 ? 2 : 0)>(p, nt, grid, stream);
    if (p.group_mode) return hipErrorInvalidValue;
    return xpose_elem_esdg<E, SK, DK, 0>(p, nt, grid, stream);
}
template <int E>
hipError_t xpose_elem_e(const ElemParams &p, int sk, int dk, int nt, uint32_t grid, hipStream_t stream) {
    switch (sk * 3 + dk) { // at least one side is token-innermost (kind 2)
    case 0 * 3 + 2: return xpose_elem_esd<E, 0, 2>(p, nt, grid, stream);
    case 1 * 3 + 2: return xpose_elem_esd<E, 1, 2>(p, nt, grid, stream);
    case 2 * 3 + 0: return xpose_elem_esd<E, 2, 0>(p, nt, grid, stream);
    case 2 * 3 + 1: return xpose_elem_esd<E, 2, 1>(p, nt, grid, stream);
    case 2 * 3 + 2: return xpose_elem_esd<E, 2, 2>(p, nt, grid, stream);
    default: return hipErrorInvalidValue;
    }
}
} // namespace

hipError_t launch_xpose_elem(const ElemParams &p, uint32_t elem_bytes, int src_kind, int dst_kind, int nontemporal,
                             uint32_t grid, hipStream_t stream) {
    if (p.total_tiles == 0 || grid == 0) return hipSuccess;
    if (p.log2_tt < 4 || (1u << p.log2_tt) > kElemMaxTokens || p.log2_tt + p.log2_wu != 10) return hipErrorInvalidValue;
    if (p.group_mode && (p.group == 0 || p.group > kElemMaxGroup || p.fine_tokens == 0)) return hipErrorInvalidValue;
    switch (elem_bytes) {
    case 1: return xpose_elem_e<1>(p, src_kind, dst_kind, nontemporal, grid, stream);
    case 2: return xpose_elem_e<2>(p, src_kind, dst_kind, nontemporal, grid, stream);
    case 4: return xpose_elem_e<4>(p, src_kind, dst_kind, nontemporal, grid, stream);
    case 8: return xpose_elem_e<8>(p, src_kind, dst_kind, nontemporal, grid, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_plain_copy(char *dst, const char *src, uint64_t bytes, uint32_t threads, uint32_t unroll,
                             int nontemporal, uint32_t max_wg, hipStream_t stream) {
    if (bytes == 0) return hipSuccess;
    switch (threads) {
    case 64: return plain_t<64>(dst, src, bytes, unroll, nontemporal, max_wg, stream);
    case 128: return plain_t<128>(dst, src, bytes, unroll, nontemporal, max_wg, stream);
    case 256: return plain_t<256>(dst, src, bytes, unroll, nontemporal, max_wg, stream);
    case 512: return plain_t<512>(dst, src, bytes, unroll, nontemporal, max_wg, stream);
    case 1024: return plain_t<1024>(dst, src, bytes, unroll, nontemporal, max_wg, stream);
    default: return hipErrorInvalidValue;
    }
}

} // namespace kvx
