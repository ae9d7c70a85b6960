/*
 * kvx -- block-free KV-cache transfer between paged pools on AMD MI355X (gfx950).
 *
 * The operations follow section 3.6 of "P/D-Serve: Serving Disaggregated Large
 * Language Model at Scale" (arXiv 2408.08147), "Block-free D2D KVCache
 * Transfer": the sender gathers a request's KV cache out of its discrete
 * fixed-size blocks into one contiguous byte buffer (kvx_pack), the bytes
 * travel as a whole, and the receiver restores its own discrete blocks from
 * them (kvx_unpack, the paper's RecvScatter).  kvx_convert does both in one
 * pass when the two pools are on one device.  The buffer itself stands in for
 * the wire.
 *
 * Conventions for every call
 *   - Plain C ABI.  Pointers marked [host] are host memory, [device] are device
 *     memory of the current HIP device.  `stream` is a hipStream_t passed as
 *     void* (NULL = the null stream).
 *   - The caller owns all device memory: pools, buffer and the plan workspace.
 *     The library owns the host-side plan objects and, for batches whose tables
 *     do not fit a kernel's launch arguments, a few pinned host blocks that
 *     kvx_plan stages those tables in: they are created on first need
 *     (hipHostMalloc and an event), handed from plan to plan, trimmed back to 32
 *     idle ones whenever more than 64 have piled up, and freed by
 *     kvx_release_cached.  Host arrays handed
 *     to kvx_plan are copied before it returns.
 *   - pack / unpack / convert enqueue work on `stream` and return; they never
 *     synchronise and never allocate device memory.  Each is one kernel launch
 *     and nothing else, so these calls (and their _layers forms) may be recorded
 *     while `stream` is being captured into a HIP graph; the graph then needs
 *     the plan's workspace and the pools at the same addresses on every replay.
 *     kvx_plan itself may copy from a staging block that the library reuses
 *     and record an event, and must not be called on a capturing stream.
 *   - Every call returns a kvx_status; nothing aborts or throws.  All argument,
 *     geometry and block-table checks happen on the host inside kvx_plan, before
 *     anything is enqueued: a plan refused by one of them leaves the workspace
 *     untouched.  Only KVX_ERR_DEVICE (a copy or launch that the runtime itself
 *     rejects) can come after part of the plan's device work was enqueued; the
 *     workspace contents are then undefined.
 *   - Results are bit-exact copies and do not depend on the launch configuration.
 *
 * Memory model (where the paper is silent, these are this library's readings)
 *   - A token row is the contiguous bytes [head][dim] of one token, one layer,
 *     K or V:  row = num_kv_heads * head_dim * elem_bytes.  row, every stride
 *     and every base pointer must be a multiple of 16 bytes.
 *   - A pool addresses a row as
 *         layer*stride_layer + kv*stride_kv + page*stride_page + slot*stride_token
 *     with kv = 0 for K, 1 for V.  (Pools whose pages are not [token][head][dim]
 *     inside, see kvx_inner, address 16-byte units or single elements instead
 *     of rows; they are moved by kernels that stage tiles through LDS where the
 *     two sides disagree on which axis is contiguous.)
 *   - The buffer of a plan over layers [l0,l1) holds the requests in batch order
 *     with no padding; inside a request the layers ascend, each layer is all K
 *     rows then all V rows, tokens ascending ("one after another").  With
 *     T_r = tokens of all earlier requests, n_r = tokens of request r and
 *     bpt = (l1-l0)*2*row:
 *         offset(r, l, kv, t) = T_r*bpt + (((l-l0)*2 + kv)*n_r + t)*row
 *   - Slots of a request's last page beyond n_r are neither read nor written.
 *     Block-table entries beyond ceil(n_r/page_tokens) are ignored.
 */
#ifndef KVX_H
#define KVX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KVX_OK = 0,
    KVX_ERR_INVALID_ARG = 1, /* NULL where not allowed, zero sizes, bad layer range, sides that disagree */
    KVX_ERR_ALIGNMENT = 2,   /* row, a stride or a pointer is not a multiple of 16 bytes */
    KVX_ERR_BLOCK_TABLE = 3, /* page id outside the pool, too few pages for a length, a receiver page
                                listed twice, CSR offsets not ascending */
    KVX_ERR_CAPACITY = 4,    /* buffer or workspace too small */
    KVX_ERR_UNSUPPORTED = 5, /* a size beyond what the kernels index (see kvx_plan) */
    KVX_ERR_DEVICE = 6,      /* a HIP call failed; kvx_last_device_error has the detail */
    KVX_ERR_BUSY = 7,        /* kvx_retriever_acquire: every receive slot is in flight */
    KVX_ERR_HOST_MEMORY = 8  /* the library's own host-side tables could not be allocated */
} kvx_status;

typedef enum {
    KVX_LAYOUT_LAYER_MAJOR = 0, /* [layer][K,V][page]{page} */
    KVX_LAYOUT_PAGE_MAJOR = 1   /* [page][layer][K,V]{page} */
} kvx_layout;

/* Arrangement of the page_tokens tokens inside one {page} (one layer, K or V).
 * The receiver restores "desired discrete blocks" (sections 1 and 2.2.3); the
 * paper fixes no block-internal layout, so four are offered.  The contiguous
 * buffer is always [token][head][dim]. */
typedef enum {
    KVX_INNER_TOKEN_ROWS = 0,      /* [token][head][dim]: a token row is contiguous */
    KVX_INNER_HEAD_MAJOR = 1,      /* [head][token][dim] */
    KVX_INNER_DIM_SPLIT_TOKEN = 2, /* [head][dim/x][token][x], x = 16/elem_bytes elements: the token axis sits
                                      inside every 16-byte group of the head dimension */
    KVX_INNER_TOKEN_INNERMOST = 3  /* [head][dim][token]: the token axis innermost element by element, a
                                      transposed page (the shape of a V cache read along the tokens).  Bytes
                                      change place below the 16-byte grain here, so tiles are transposed
                                      through LDS at element granularity.  Fast when page_tokens*elem_bytes is
                                      a multiple of 16 (columns then start on 16-byte boundaries); any other
                                      page size works, element by element */
} kvx_inner;

/* Geometry of one paged pool (section 2.2.3, "Block-fixed Management": device
 * memory organised as discrete blocks of fixed size).  The base pointer is
 * passed per call.  If all four strides are 0 they are derived from `layout`
 * for a dense pool; otherwise all four must be given (bytes) and `layout` is
 * ignored. */
typedef struct {
    uint32_t num_layers;
    uint32_t num_kv_heads; /* this device's share of the heads */
    uint32_t head_dim;
    uint32_t elem_bytes;   /* bytes per KV element; the element type is opaque */
    uint32_t page_tokens;  /* tokens per page (block) */
    uint32_t num_pages;    /* pages in the pool */
    uint32_t layout;       /* kvx_layout */
    uint32_t inner;        /* kvx_inner; anything but TOKEN_ROWS needs the derived (all-zero) strides;
                              HEAD_MAJOR and DIM_SPLIT_TOKEN need head_dim*elem_bytes a multiple of 16,
                              DIM_SPLIT_TOKEN elem_bytes dividing 16, TOKEN_INNERMOST elem_bytes of 1, 2, 4
                              or 8 */
    uint64_t stride_layer, stride_kv, stride_page, stride_token;
} kvx_pool_desc;

/* A batch of requests on one side: lengths and CSR block tables.
 * block_ids[block_offsets[r] .. block_offsets[r+1]) are the physical pages of
 * request r in logical order.  All three arrays are [host]. */
typedef struct {
    uint32_t num_requests;
    uint32_t reserved;             /* must be 0 */
    const uint32_t *seq_lens;      /* [R] tokens per request; 0 is allowed */
    const uint32_t *block_ids;     /* [block_offsets[R]] */
    const uint64_t *block_offsets; /* [R+1], ascending, block_offsets[0] == 0 */
} kvx_batch_desc;

/* Launch configuration of the copy kernels.  Zero in a field = library default.
 * It changes speed only, never results.  `unroll`, `threads`, `workgroups_per_cu`
 * and `xcd_block_tiles` shape the kernel for [token][head][dim] pages only; the
 * kernel for other page arrangements has a fixed tile of 1024 16-byte units. */
typedef struct {
    uint32_t unroll;        /* 16-byte loads in flight per lane before the first store: 1,2,4,8; 0 = chosen
                               per operation together with `threads` */
    uint32_t nontemporal;   /* cache policy of the 16-byte accesses: 0 = chosen per operation, 1 = default,
                               2 = non-temporal loads and stores, 3 = non-temporal loads with agent-scope
                               (write-through) stores */
    uint32_t order;         /* 0 = chosen per operation (pack: 3, with fewer than 64 runs 1; unpack and convert: 2
                               into a page-major receiver, else 1), 1 = (layer,kv) outermost, 2 = copy run (for a convert into
                               coarser pages: the runs of one receiver page) outermost, 3 = the runs cut into eight parts, one per XCD, each part walked
                               with (layer,kv) outermost ([token][head][dim] pages only, else as 1) */
    uint32_t xcd_swizzle;   /* 1 = off, 2 = give each of the 8 XCDs contiguous tiles: one eighth of the grid
                               each, or blocks of `xcd_block_tiles` tiles dealt round-robin */
    uint32_t max_workgroups;/* cap on the grid; tiles beyond it are taken in a grid-stride loop */
    uint32_t threads;       /* lanes per workgroup: 64, 128, 256, 512 or 1024; a tile is threads*16*unroll bytes */
    uint32_t workgroups_per_cu; /* 0 = as many as fit (with the library's own 8 KiB tiles of order 2: four);
                               n = at most n resident per compute unit (1..8), which bounds the bytes in
                               flight; done by reserving unused LDS per workgroup */
    uint32_t xcd_block_tiles; /* with xcd_swizzle 2: 0 = eighths of the grid, else a power of two */
} kvx_launch_cfg;

typedef struct kvx_plan_s kvx_plan_t;

/* One record of the flat copy plan in the device workspace: a maximal span of
 * tokens of one request that lies in one page on both sides.  The same record
 * serves every (layer, kv) of the plan's range.  The convert table keeps a
 * fixed number of slots per page of the coarser side; a slot no run claims has
 * bytes == 0. */
typedef struct {
    uint64_t src_off; /* pool side: page*stride_page + slot*(byte step between tokens of that page
                         arrangement); buffer side: T_r*bpt + t*row */
    uint64_t dst_off; /* likewise for the destination */
    uint32_t bytes;   /* tokens in the run * row */
    uint32_t seq_len; /* n_r of the owning request */
    uint32_t request; /* r */
    uint32_t token;   /* first token of the run */
} kvx_run;

/* Where kvx_plan put its device tables inside the workspace (byte offsets from
 * the workspace base; counts in records).  For inspection and tests. */
typedef struct {
    uint64_t token_prefix_off;                 /* uint64[R+1]: T_r, exclusive prefix sum of seq_lens */
    uint64_t run_prefix_off[3];                /* uint64[R+1] per op: first run of request r */
    uint64_t runs_off[3];                      /* kvx_run[num_runs[op]] per op */
    uint64_t num_runs[3];                      /* records per op (0 pack, 1 unpack, 2 convert, empty slots
                                                  included); 0 if the op is not planned */
} kvx_plan_tables;

/* No passage of the paper: sizing utility.
 * Bytes of device workspace kvx_plan needs for these inputs.  `s`/`sb` describe
 * the sender side, `d`/`db` the receiver side; either pair may be NULL (then
 * only pack, or only unpack, can be planned).  Checks geometry and that the
 * block tables cover the lengths; the remaining checks are kvx_plan's. */
kvx_status kvx_plan_workspace_bytes(const kvx_pool_desc *s, const kvx_batch_desc *sb,
                                    const kvx_pool_desc *d, const kvx_batch_desc *db,
                                    size_t *out_bytes);

/* Builds the copy plan for layers [layer_begin, layer_end) -- the offsets and
 * lengths that section 3.6 says follow from layer index, prompt length, hidden
 * size and precision, and the "meta" exchanged before a transfer.
 *
 * Host part: validates everything (see kvx_status), computes T_r and the
 * payload size.  Device part, enqueued on `stream`: lengths and used page ids
 * go into the workspace (inside the next kernel's launch arguments when they
 * are at most 896 words together, else staged in pinned memory and copied),
 * a wavefront prefix-scan kernel over the variable lengths, and a kernel that
 * writes the kvx_run records (one kernel does both when the tables ride in
 * its launch arguments).  The plan may be used on `stream` right away,
 * and on other streams after `stream` has been synchronised with them.
 *
 * With a sender side the plan serves kvx_pack, with a receiver side
 * kvx_unpack, with both also kvx_convert.  Both sides must then agree in
 * num_requests, seq_lens, num_kv_heads, head_dim and elem_bytes, and both must
 * have at least layer_end layers.  Sender pages may repeat (shared prefixes);
 * a receiver page used by two live logical pages is KVX_ERR_BLOCK_TABLE.
 *
 * dev_workspace [device] must be 256-byte aligned and at least
 * kvx_plan_workspace_bytes large; it must stay alive and unmodified while the
 * plan is in use.  A receiver given by explicit strides must not let two rows
 * share bytes: its four axes (token, page, K|V, layer) have to nest, each stride
 * at least the extent of what lies inside it (stride_token >= row,
 * stride_page >= (page_tokens-1)*stride_token + row when it is the next larger,
 * and so on in order of size), else KVX_ERR_INVALID_ARG.  A sender may overlap
 * itself (it is only read).  dev_workspace == NULL with workspace_bytes == 0 builds a
 * host-only plan: no HIP call is made and nothing is enqueued; totals and
 * segments can be queried.  A host-only plan can also run when it is small and
 * simple: exactly one side given, that side's pages KVX_INNER_TOKEN_ROWS with
 * the rows of a page back to back (stride_token equal to the row, as in every
 * dense pool), at most KVX_INLINE_RUNS used pages (sum of ceil(seq_len/page_tokens)) and at
 * least one.  The host then works the kvx_run records out itself (a run of a
 * one-sided plan is the part of a request inside one page) and kvx_pack /
 * kvx_unpack and their _layers forms carry them in their launch arguments:
 * one launch per operation, none for the plan.  kvx_plan_can_launch tells
 * which kind a plan is; every other host-only plan makes pack / unpack /
 * convert return KVX_ERR_INVALID_ARG.
 *
 * KVX_ERR_UNSUPPORTED: page_tokens*row >= 2^32, or more than 2^32-1 tiles. */
kvx_status kvx_plan(const kvx_pool_desc *s, const kvx_batch_desc *sb,
                    const kvx_pool_desc *d, const kvx_batch_desc *db,
                    uint32_t layer_begin, uint32_t layer_end,
                    void *dev_workspace, size_t workspace_bytes, void *stream,
                    kvx_plan_t **out_plan);

/* No passage of the paper: utility.  Frees the host-side plan object; work already enqueued with the
 * plan keeps running (launches carry their arguments, and a staging block is reused only after the copy
 * that reads it has completed).  NULL is a no-op. */
void kvx_plan_destroy(kvx_plan_t *plan);

/* No passage of the paper: utility.  Frees the pinned staging blocks that destroyed plans left with the
 * library and whose copies have completed (blocks still being read stay).  `freed_bytes` (may be NULL)
 * receives the host bytes given back.  Never needed for correctness. */
kvx_status kvx_release_cached(uint64_t *freed_bytes);

/* Size of the contiguous buffer: (l1-l0) * 2 * num_kv_heads * head_dim *
 * elem_bytes * sum(seq_lens), the KV size formula of section 2.1. */
kvx_status kvx_plan_total_bytes(const kvx_plan_t *plan, uint64_t *payload_bytes);

/* Offset and length, inside the buffer, of the K and V rows of one layer of one
 * request (section 3.6: per-layer or whole-model transfer by different offsets
 * and lengths).  `layer` is absolute and must lie in the plan's range. */
kvx_status kvx_plan_segment(const kvx_plan_t *plan, uint32_t request, uint32_t layer,
                            uint64_t *offset, uint64_t *length);

/* Offset and length of a whole request (all layers of the plan's range). */
kvx_status kvx_plan_request_segment(const kvx_plan_t *plan, uint32_t request,
                                    uint64_t *offset, uint64_t *length);

/* No passage of the paper: inspection and tuning.  get_tables needs a plan with a device workspace;
 * set_launch refuses values outside the ranges kvx_launch_cfg states (KVX_ERR_INVALID_ARG);
 * can_launch sets *out to 1 for a plan with a device workspace or with run records that ride in the
 * launch arguments (see kvx_plan), to 0 for a plan that only answers the size queries. */
#define KVX_INLINE_RUNS 96u
kvx_status kvx_plan_can_launch(const kvx_plan_t *plan, int *out);
kvx_status kvx_plan_get_tables(const kvx_plan_t *plan, kvx_plan_tables *out);
kvx_status kvx_plan_set_launch(kvx_plan_t *plan, const kvx_launch_cfg *cfg);
kvx_status kvx_plan_get_launch(const kvx_plan_t *plan, kvx_launch_cfg *out);

/* Section 3.6, "Contiguous Buffer at Sender" (the first of the two converts that section 2.2.3,
 * "Challenge", says block-free transfer has to pay): the K and V rows of every layer of every request
 * of the plan, gathered out of the sender's discrete blocks and laid one after another.
 * src_pool [device] -> buf [device].  Writes exactly the first kvx_plan_total_bytes bytes of buf;
 * buf_bytes smaller than that is KVX_ERR_CAPACITY.  Needs a plan built with a sender side that
 * kvx_plan_can_launch (else KVX_ERR_INVALID_ARG); pointers must be 16-byte aligned (KVX_ERR_ALIGNMENT).
 * One kernel launch on `stream`; neither pointer is kept. */
kvx_status kvx_pack(const kvx_plan_t *plan, const void *src_pool, void *buf, uint64_t buf_bytes,
                    void *stream);

/* Section 3.6, "RecvScatter at Receiver" (the second convert of section 2.2.3, "Challenge"): the
 * receiver's discrete blocks restored from the received bytes.  buf [device] -> dst_pool [device].
 * Reads the first kvx_plan_total_bytes bytes of buf (buf_bytes smaller: KVX_ERR_CAPACITY) and writes
 * only the live slots of the pages the receiver's block tables list.  Needs a plan built with a
 * receiver side that kvx_plan_can_launch.  One kernel launch on `stream`. */
kvx_status kvx_unpack(const kvx_plan_t *plan, const void *buf, uint64_t buf_bytes, void *dst_pool,
                      void *stream);

/* Section 2.2.3, "Opportunity": the bytes in flight carry no block structure, so the block geometry of
 * the two sides is independent; with both pools on one device the two converts fuse.
 * src_pool [device] -> dst_pool [device] in one launch, equal to kvx_unpack after kvx_pack byte for
 * byte, with independent page sizes, layouts and page arrangements on the two sides.  Needs a plan
 * built with both sides.  The pools must not share bytes: two pools with derived (all-zero) strides
 * whose extents overlap are refused with KVX_ERR_INVALID_ARG; for a pool given by explicit strides the
 * library does not know which bytes between its rows belong to it, does not check, and the result of
 * a convert between aliasing pools is undefined. */
kvx_status kvx_convert(const kvx_plan_t *plan, const void *src_pool, void *dst_pool, void *stream);

/* Per-layer triggers (section 3.6: either the transfer per layer or of the
 * entire model, by different offsets and lengths into the same buffer; the
 * "operator" form of RecvScatter that runs between a model's layers).  Same as
 * kvx_pack / kvx_unpack / kvx_convert, restricted to layers
 * [layer_begin, layer_end) of the plan's range: exactly those layers' segments
 * of the plan's buffer (kvx_plan_segment) are written or read, at the offsets
 * of the whole-range buffer, so one plan and one buffer serve every layer.
 * A range outside the plan's is KVX_ERR_INVALID_ARG; an empty one is a no-op. */
kvx_status kvx_pack_layers(const kvx_plan_t *plan, uint32_t layer_begin, uint32_t layer_end,
                           const void *src_pool, void *buf, uint64_t buf_bytes, void *stream);
kvx_status kvx_unpack_layers(const kvx_plan_t *plan, uint32_t layer_begin, uint32_t layer_end, const void *buf,
                             uint64_t buf_bytes, void *dst_pool, void *stream);
kvx_status kvx_convert_layers(const kvx_plan_t *plan, uint32_t layer_begin, uint32_t layer_end,
                              const void *src_pool, void *dst_pool, void *stream);

/* Reference point, not the product path: the block-fixed transfer that section
 * 2.2.3 ("Unnecessary Controls") argues against, in one-GPU form.  Produces the
 * same buffer as kvx_pack, but moves the sender's blocks one after another, one
 * device copy per (request, layer, K|V, page), issued from the host; with
 * confirm_every = k > 0 the host also waits for the stream after every k
 * blocks, standing in for the per-block confirmation between sender and
 * receiver (k = 1: every block confirmed).  Needs no device workspace.  Only for
 * sender pools with [token][head][dim] pages (else KVX_ERR_UNSUPPORTED). */
kvx_status kvx_pack_blockwise(const kvx_plan_t *plan, const void *src_pool, void *buf, uint64_t buf_bytes,
                              uint32_t confirm_every, void *stream);

/* ---------------------------------------------------------------------------
 * Asynchronous retrieval (section 3.6, "Asynchronous Retrieval"): the decoding
 * side has little memory to spare for transfers in flight, so incoming KV waits
 * in a small number of receive slots; a retrieval runs beside the running
 * batch on a stream of its own, and when it completes the slot is free for the
 * next one while the request becomes valid in the next decoding iteration.
 *
 * A retriever owns num_slots streams (default priority, non-blocking) and
 * events; the caller owns the arena [device], which is cut into num_slots
 * equal parts, each a receive buffer of slot_buf_bytes followed by a plan
 * workspace of slot_ws_bytes (both rounded up to 256 bytes; kvx_retriever_arena_bytes
 * gives the total).  One retrieval is
 *     acquire  -> the caller lets the bytes arrive in the slot's buffer, on the
 *                 slot's stream (an RDMA write in the paper; here any copy or
 *                 kvx_pack) -> scatter (plan + kvx_unpack on the slot's stream)
 *     poll     -> tickets whose scatter has completed; their slots are free again
 * Calls on one retriever must come from one thread at a time. */
typedef struct kvx_retriever_s kvx_retriever_t;

/* At most 1024 slots, each part below 2^48 bytes (KVX_ERR_UNSUPPORTED beyond). */
kvx_status kvx_retriever_arena_bytes(uint32_t num_slots, uint64_t slot_buf_bytes, uint64_t slot_ws_bytes,
                                     uint64_t *out_bytes);
kvx_status kvx_retriever_create(uint32_t num_slots, uint64_t slot_buf_bytes, uint64_t slot_ws_bytes,
                                void *dev_arena, uint64_t arena_bytes, kvx_retriever_t **out);
/* Waits for everything in flight, then releases streams and events. */
void kvx_retriever_destroy(kvx_retriever_t *ret);

/* Takes a free slot for a transfer of need_bytes, tagged with the caller's
 * ticket.  KVX_ERR_BUSY if none is free (poll first), KVX_ERR_CAPACITY if
 * need_bytes exceeds a slot's buffer.  Returns the slot's buffer [device] and
 * stream, on which the caller enqueues whatever makes the bytes arrive. */
kvx_status kvx_retriever_acquire(kvx_retriever_t *ret, uint64_t ticket, uint64_t need_bytes, uint32_t *slot,
                                 void **slot_buf, void **slot_stream);

/* RecvScatter of the slot's buffer into dst_pool [device] for the receiver's
 * geometry `d`, batch `db` and layers [layer_begin, layer_end): builds the plan
 * in the slot's workspace and enqueues kvx_unpack, both on the slot's stream,
 * behind whatever the caller enqueued there (an arrival of at most
 * KVX_INLINE_RUNS used pages whose pages hold token rows is planned on the
 * host instead, and the kvx_unpack is then the only launch).  `launch` may be NULL; a capped
 * grid (max_workgroups) keeps most of the device for the running batch.  On an
 * error the slot stays acquired (release it with kvx_retriever_abandon); after a
 * KVX_ERR_DEVICE the contents of the slot's workspace are undefined. */
kvx_status kvx_retriever_scatter(kvx_retriever_t *ret, uint32_t slot, const kvx_pool_desc *d,
                                 const kvx_batch_desc *db, uint32_t layer_begin, uint32_t layer_end,
                                 void *dst_pool, const kvx_launch_cfg *launch);

/* Gives an acquired slot back without scattering (waits for its stream). */
kvx_status kvx_retriever_abandon(kvx_retriever_t *ret, uint32_t slot);

/* Non-blocking.  Writes up to `capacity` tickets whose scatter has completed
 * since they were last reported and frees their slots. */
kvx_status kvx_retriever_poll(kvx_retriever_t *ret, uint64_t *tickets, uint32_t capacity, uint32_t *count);

/* Blocks until nothing is in flight; completed tickets stay to be polled. */
kvx_status kvx_retriever_drain(kvx_retriever_t *ret);

/* Yardstick, not part of the transfer: a plain contiguous device-to-device copy
 * of `bytes` bytes (a multiple of 16; both pointers [device], 16-byte aligned,
 * not overlapping) made of the same 16-byte loads and stores as the data
 * mover, with `unroll`, `nontemporal` and `max_workgroups` taken from `cfg`
 * (NULL = defaults).  It shows what fraction of
 * the HBM peak a copy reaches on this device at all, and calibrates hardware
 * byte counters against a transfer of known size. */
kvx_status kvx_copy_yardstick(void *dst, const void *src, uint64_t bytes, const kvx_launch_cfg *cfg,
                              void *stream);

/* ---------------------------------------------------------------------------
 * For callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  RecvScatter (kvx_plan for a receiver side followed by kvx_unpack) in one
 * call that allocates nothing, on the device or on the host: the plan's device tables live in a fixed
 * array inside the library's device image (KVX_NOALLOC_SCRATCH_BYTES per GPU, held until the process
 * ends), the block tables ride in a kernel's launch arguments, and no plan object is created.
 *
 * Same arguments, checks, results and errors as kvx_plan(NULL, NULL, d, db, layer_begin, layer_end, ...)
 * + kvx_unpack(plan, buf, buf_bytes, dst_pool, stream), with these limits:
 *   - num_requests + used pages (sum of ceil(seq_len/page_tokens)) <= KVX_NOALLOC_MAX_TABLE_WORDS, and the
 *     plan's device tables <= KVX_NOALLOC_SCRATCH_BYTES: beyond either, KVX_ERR_CAPACITY and nothing is
 *     enqueued;
 *   - default launch configuration.
 * Two kernel launches on `stream` (the planner, then the unpack) and nothing else, so the call may be recorded while
 * `stream` is being captured into a HIP graph; the first call on a device also asks the runtime for the
 * scratch array's address, so make one call on the device before capturing.  Every call on a GPU uses that GPU's one
 * scratch array: it keeps the previous call's tables, each call rewrites everything it reads, and calls
 * on the same stream are ordered; calls that overlap on one GPU (different streams, or threads on
 * different streams) race on the array and must be serialised by the caller. */
#define KVX_NOALLOC_MAX_TABLE_WORDS 896u
#define KVX_NOALLOC_SCRATCH_BYTES 65536u
kvx_status kvx_unpack_noalloc(const kvx_pool_desc *d, const kvx_batch_desc *db, uint32_t layer_begin,
                              uint32_t layer_end, const void *buf, uint64_t buf_bytes, void *dst_pool,
                              void *stream);

/* No passage of the paper: utility.  A string naming the sources this library was built from (a hash
 * of them, fixed at build time), so that a loader can tell a stale binary from a current one. */
const char *kvx_build_id(void);

/* No passage of the paper: utility.  Static text for a status value. */
const char *kvx_status_string(kvx_status st);

/* The hipError_t value behind this thread's most recent KVX_ERR_DEVICE (0 if none) and, through `where`
 * (may be NULL), a static string naming the step that failed. */
int kvx_last_device_error(const char **where);

#ifdef __cplusplus
}
#endif
#endif /* KVX_H */
