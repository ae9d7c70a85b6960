// Internal interface between the host side of libkvx (plan construction and
// validation) and its HIP kernels.  Not installed; the public boundary is
// include/kvx.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <memory>
#include <vector>

#include "kvx.h"

namespace kvx {

// Remembers, per thread, the HIP error behind the last KVX_ERR_DEVICE and where it happened.
void note_device_error(hipError_t e, const char *where);
inline bool hip_ok(hipError_t e, const char *where) {
    if (e == hipSuccess) return true;
    note_device_error(e, where);
    return false;
}

enum Op : uint32_t { OP_PACK = 0, OP_UNPACK = 1, OP_CONVERT = 2, NUM_OPS = 3 };

// Number of prefix arrays the scan kernel produces, each uint64[R+1]:
// tokens, sender pages, receiver pages, runs of pack / unpack / convert.
constexpr int kNumScans = 6;
enum Scan : int { SCAN_TOKENS = 0, SCAN_PAGES_S = 1, SCAN_PAGES_D = 2, SCAN_RUNS0 = 3 };

// Division of any 32-bit n by a fixed divisor d >= 1 as a multiply-high and two shifts (Granlund and
// Montgomery's round-up method), the constants worked out once on the host: the data movers split a flat
// tile index by several run-time divisors per tile, and the hardware has no integer divide.
struct FastDiv {
    uint32_t d, mul, sh1, sh2;
};
inline FastDiv make_fast_div(uint32_t d) {
    FastDiv f{d ? d : 1u, 0, 0, 0};
    uint32_t l = 0;
    while (l < 32 && (1ull << l) < f.d) ++l;                       // l = ceil(log2 d)
    f.mul = (uint32_t)((((1ull << l) - f.d) << 32) / f.d + 1ull);
    f.sh1 = l < 1 ? l : 1;
    f.sh2 = l ? l - 1 : 0;
    return f;
}
__host__ __device__ inline uint32_t fast_div(uint32_t n, const FastDiv &f) {
#ifdef __HIP_DEVICE_COMPILE__
    const uint32_t t = __umulhi(f.mul, n);
#else
    const uint32_t t = (uint32_t)(((uint64_t)f.mul * n) >> 32);
#endif
    return (t + ((n - t) >> f.sh1)) >> f.sh2;
}

// One side of a copy as the run-building kernel sees it.  quantum == 0 means
// the contiguous buffer (no page boundary ever breaks a run).
struct SideGeom {
    const uint32_t *ids;         // compact block table: exactly ceil(n_r/page_tokens) ids per request
    const uint64_t *page_prefix; // uint64[R+1], first id of request r in `ids`
    uint64_t stride_page;
    uint64_t stride_token;
    uint32_t page_tokens;
    uint32_t quantum;            // tokens that are contiguous: page_tokens, 1 (padded rows) or 0 (buffer)
    uint32_t which;              // 0 the buffer, 1 the sender's pool, 2 the receiver's
    uint32_t pad;
};

struct ScanParams {
    const uint32_t *seq_lens;
    uint32_t num_requests;
    uint32_t page_s, page_d;     // 0 = side absent
    uint32_t qa[NUM_OPS], qb[NUM_OPS]; // contiguity quanta of source / destination per op (0 = buffer)
    uint64_t lcm[NUM_OPS];       // lcm(qa,qb); 0 = infinite
    uint32_t planned[NUM_OPS];
    uint32_t group_quantum;      // convert: tokens per group (the coarser side's quantum)
    uint32_t group_slots;        // convert: run slots reserved per group
    uint64_t *prefix[kNumScans]; // outputs
};

// Small batches hand their tables (lengths, then the sender's used page ids, then the receiver's) to the
// planning kernel inside its arguments: the launch itself carries them to the device, so there is no
// host-to-device copy to issue, no staging block to keep alive and no event to record.  The kernel stores the
// three segments at dst_word[] (32-bit words from the start of the workspace), where inspection finds them.
constexpr uint32_t kInlineWords = 896; // with the planner's own parameters this stays under the 4 KiB a launch may carry
struct InlineTables {
    uint32_t count[3];
    uint32_t dst_word[3];
    uint32_t words[kInlineWords];
};

struct FillParams {
    const uint32_t *seq_lens;
    const uint64_t *token_prefix;
    uint32_t num_requests;
    uint32_t row;
    uint64_t bytes_per_token;    // (l1-l0)*2*row
    SideGeom src[NUM_OPS], dst[NUM_OPS];
    uint64_t lcm[NUM_OPS];
    uint32_t planned[NUM_OPS];
    uint32_t group_quantum;      // convert only, as in ScanParams
    uint32_t group_slots;
    const uint64_t *run_prefix[NUM_OPS];
    kvx_run *runs[NUM_OPS];
};

// Run records that ride in a copy kernel's launch arguments: what a one-sided plan of at most this many
// used pages needs, worked out on the host, so that nothing has to be planned on the device.
constexpr uint32_t kInlineRuns = KVX_INLINE_RUNS;
struct InlineRuns {
    kvx_run run[kInlineRuns];
};

struct CopyParams {
    const kvx_run *runs;
    const char *src;
    char *dst;
    uint64_t src_stride_layer, src_stride_kv; // pool side only
    uint64_t dst_stride_layer, dst_stride_kv;
    uint32_t src_is_buf, dst_is_buf;
    uint32_t row;
    uint32_t layer_begin;     // first layer of the plan's range: buffer offsets are relative to it
    uint32_t lc_first;        // first (layer,kv) index of this launch inside the plan's range
    uint32_t num_lc;          // 2 * layers of this launch
    uint32_t num_runs;
    uint32_t tiles_per_run;
    uint32_t total_tiles;     // num_lc * num_runs * tiles_per_run
    uint32_t order;           // 1: (layer,kv) outermost   2: run group outermost   3: eighth of the runs outermost
    uint32_t runs_per_part;   // order 3: ceil(num_runs / 8); total_tiles then counts 8 * runs_per_part runs
    uint32_t group;           // order 2: consecutive runs that stay together inside one (layer,kv)
    uint32_t swizzle_chunk;   // 0 = off, else tiles per XCD (grid is a multiple of 8)
    uint32_t swizzle_block;   // 0 = eighths of the grid, else tiles per block dealt round-robin to the XCDs
    FastDiv by_tiles_per_run, by_num_runs, by_runs_per_part, by_group, by_num_lc, by_swizzle_block;
};

// One side of the tile-transposing kernel.  A row is row/16 units of 16 bytes; unit u of the token in
// slot s of a page lives at  page_base + s*token_step + (u / units_per_granule)*granule_step
// + (u % units_per_granule)*16.
struct XposeSide {
    uint64_t stride_layer, stride_kv; // pool side only
    uint64_t token_step;
    uint64_t granule_step;
    uint32_t units_per_granule;
    uint32_t granule_magic;           // floor(2^32 / units_per_granule) + 1; unused when units_per_granule == 1
    uint32_t is_buf;
    uint32_t pad;
};

struct XposeParams {
    const kvx_run *runs;
    const char *src;
    char *dst;
    XposeSide s, d;
    uint32_t row;
    uint32_t units_per_row;
    uint32_t layer_begin, lc_first, num_lc;
    uint32_t num_runs;
    uint32_t log2_tt, log2_uu;        // tile = 2^log2_tt tokens x 2^log2_uu units = 1024 units
    uint32_t tiles_t, tiles_u;        // tiles per run along tokens / along the row
    uint32_t total_tiles;
    uint32_t order, group;
    uint32_t swizzle_chunk;
};

// One side of the element-transposing kernel: either addressed by 16-byte units like XposeSide (kind 0:
// consecutive units of a token are nearest, kind 1: consecutive tokens of a unit are), or token-innermost
// (kind 2): element (column j of the row, token t of the run) at run_offset + j*column_step + t*elem_bytes.
struct ElemSide {
    uint64_t stride_layer, stride_kv; // pool side only
    uint64_t token_step;
    uint64_t granule_step;
    uint32_t units_per_granule;
    uint32_t granule_magic;
    uint32_t column_step;             // kind 2: page_tokens * elem_bytes
    uint32_t is_buf;
};

struct ElemParams {
    const kvx_run *runs;
    const char *src;
    char *dst;
    ElemSide s, d;
    uint32_t row;
    uint32_t units_per_row;
    uint32_t layer_begin, lc_first, num_lc;
    uint32_t num_runs;
    uint32_t log2_tt, log2_wu;        // tile = 2^log2_tt tokens x 2^log2_wu 16-byte units of the row = 16 KiB
    uint32_t tiles_t, tiles_w;
    uint32_t total_tiles;
    uint32_t order, group;
    uint32_t swizzle_chunk;
    uint32_t cached_loads;            // 1: loads keep the default cache policy whatever the kernel's own is
    uint32_t cached_stores;           // 1: the same for stores
    // Tiles that span a whole group of a convert's runs (one page of the coarser side): 0 = off, 1 = the
    // source is the coarser side, 2 = the destination is.
    uint32_t group_mode;
    uint32_t num_groups;              // num_runs / group
    uint32_t coarse_tokens;           // tokens per page of the coarser side
    uint32_t fine_tokens;             // tokens per page of the finer side (divides coarse_tokens)
    FastDiv by_fine;
};

constexpr uint32_t kElemThreads = 256;
constexpr uint32_t kElemCells = 1024;   // 16-byte units per tile
constexpr uint32_t kElemMaxTokens = 256; // tokens per tile at most (rows of 64 bytes per tile at least)
constexpr uint32_t kElemMaxGroup = 64;   // runs per group at most for tiles that span a group

// elem_bytes in {1,2,4,8}; kinds as in ElemSide, at least one of them 2; nontemporal 0 or 1.
hipError_t launch_xpose_elem(const ElemParams &p, uint32_t elem_bytes, int src_kind, int dst_kind, int nontemporal,
                             uint32_t grid, hipStream_t stream);

constexpr uint32_t kXposeThreads = 256;
constexpr uint32_t kXposeCells = 1024; // 16-byte units per tile (16 KiB)

hipError_t launch_xpose(const XposeParams &p, bool src_token_fast, bool dst_token_fast, int nontemporal,
                        uint32_t grid, hipStream_t stream);

inline uint32_t tile_bytes(uint32_t threads, uint32_t unroll) { return threads * 16u * unroll; }
inline bool valid_threads(uint32_t t) { return t == 64 || t == 128 || t == 256 || t == 512 || t == 1024; }
inline bool valid_unroll(uint32_t u) { return u == 1 || u == 2 || u == 4 || u == 8; }

hipError_t launch_scan(const ScanParams &p, hipStream_t stream);
hipError_t launch_fill(const FillParams &p, hipStream_t stream);
// Scan and fill of a batch whose tables ride in the launch arguments, in one launch of one workgroup.
hipError_t launch_plan_small(const ScanParams &sp, const FillParams &fp, const InlineTables &t,
                             uint32_t *workspace_words, hipStream_t stream);
// `inline_runs`: nullptr to read the records at p.runs, else the records themselves (p.runs is then unused).
hipError_t launch_copy(const CopyParams &p, const InlineRuns *inline_runs, uint32_t threads, uint32_t unroll,
                       int nontemporal, uint32_t grid, uint32_t lds_bytes, hipStream_t stream);

// LDS per compute unit on gfx950, and the unused dynamic LDS to reserve per workgroup so that at most
// `per_cu` workgroups are resident on a compute unit (0 = no cap).
constexpr uint32_t kLdsPerCu = 160u * 1024u;
inline uint32_t occupancy_lds(uint32_t per_cu) { return per_cu ? kLdsPerCu / per_cu / 1024u * 1024u : 0u; }

// `nontemporal` in these three: 0 default cache policy, 1 non-temporal loads and stores,
// 2 non-temporal loads with agent-scope (write-through) stores.
hipError_t launch_plain_copy(char *dst, const char *src, uint64_t bytes, uint32_t threads, uint32_t unroll,
                             int nontemporal, uint32_t max_wg, hipStream_t stream);

// ---------------------------------------------------------------------------
// Host side: what kvx_plan works out about a pool, an operation and the workspace
// ---------------------------------------------------------------------------
constexpr uint64_t kAlign = 256;
inline uint64_t align_up(uint64_t x, uint64_t a = kAlign) { return (x + a - 1) / a * a; }

struct Geometry {
    bool present = false;
    kvx_pool_desc desc{};
    uint64_t row = 0;
    uint64_t sl = 0, sk = 0, sp = 0, st = 0; // resolved byte strides
    bool custom_strides = false;
    bool dense_rows = true;                  // [token][head][dim] with rows back to back
    uint32_t quantum = 0;                    // tokens that form one affine span inside a page
    // 16-byte unit u of the token in slot s sits at s*token_step + (u/upg)*granule_step + (u%upg)*16
    uint64_t token_step = 0, granule_step = 0;
    uint32_t upg = 0;
    bool token_fast = false;                 // consecutive tokens are nearer than consecutive units
    bool token_innermost = false;            // [head][dim][token]: addressed by elements, not by 16-byte units
    uint32_t column_step = 0;                // then: bytes from one (head,dim) column to the next
    uint64_t span = 0;                       // bytes from the pool's base to the end of its last row
    uint64_t used_pages = 0;                 // sum over requests of ceil(n/P)
};

struct OpShape {
    bool planned = false;
    uint32_t qa = 0, qb = 0;
    uint64_t lcm = 0;
    uint64_t num_runs = 0;       // records in the device table (for convert: slots, some empty)
    uint32_t max_run_bytes = 0;
    uint32_t group_quantum = 0;  // convert: tokens per group = the coarser side's quantum
    uint32_t group_slots = 1;    // convert: slots per group
};

// Sizes shared by kvx_plan_workspace_bytes and kvx_plan.
struct Sizing {
    uint32_t R = 0;
    OpShape ops[NUM_OPS];
    uint64_t off_lens = 0, off_ids_s = 0, off_ids_d = 0, staging_bytes = 0;
    uint64_t off_prefix[kNumScans] = {};
    uint64_t off_runs[NUM_OPS] = {};
    uint64_t total_bytes = 0;
};

// A pinned staging block and the event recorded behind the copy that reads it.
struct PinnedBlock {
    void *ptr = nullptr;
    size_t bytes = 0;
    hipEvent_t copied = nullptr;
    int device = -1; // the event belongs to this device: a block serves plans of that device only
};

// `receiver`: the pool will be written, so its explicit strides must not let two rows share bytes.
kvx_status resolve_pool(const kvx_pool_desc *d, bool receiver, Geometry *g);
kvx_status check_batch_shape(const kvx_batch_desc *b);
void shape_ops(const Geometry &s, const Geometry &d, const uint32_t *seq_lens, uint32_t R, OpShape ops[NUM_OPS]);
void layout_workspace(Sizing *z, uint64_t used_s, uint64_t used_d);
void default_launch(kvx_launch_cfg *c);

} // namespace kvx

struct kvx_plan_s {
    kvx::Geometry s, d;
    uint32_t R = 0;
    uint32_t l0 = 0, l1 = 0;
    uint64_t row = 0;
    uint64_t bpt = 0;
    uint64_t total = 0;
    std::vector<uint32_t> seq_lens;
    std::vector<uint64_t> token_prefix; // T_r, host copy for segment queries
    std::vector<uint32_t> ids_s;        // sender's used page ids, request by request (for the block-by-block baseline)
    kvx::Sizing z;
    char *ws = nullptr; // device workspace (caller's), nullptr for a host-only plan
    std::unique_ptr<kvx::InlineRuns> inline_runs; // host-only plan of a small one-sided batch: its run records
    kvx::PinnedBlock staging;
    kvx_launch_cfg launch{};
};

namespace kvx {

// Fills the two planning kernels' parameters from a plan whose geometry, sizes and workspace are set.
void planner_params(const kvx_plan_s &p, ScanParams *sp, FillParams *fp);

// Launches one operation over layers [lb, le) of the plan's range.
kvx_status run_op(const kvx_plan_s *plan, Op op, uint32_t lb, uint32_t le, const void *src, void *dst, void *stream);

} // namespace kvx
