/*
 * kvd - paged KV-cache pull for MI355X (gfx950).
 *
 * C ABI of the KV-cache transfer path of KVDirect (arXiv 2501.14743): one request's KV cache,
 * for every layer and for both K and V, is moved out of a source ("remote", prefill) paged
 * block pool addressed through its block table into a destination ("local", decode) paged
 * pool under a different block table.  The destination side initiates the copy (pull mode,
 * section 4.3) and the copies are described by block ids plus tensor metadata (section 4.1),
 * not by per-block messages.
 *
 * The three operations of section 4.1 map onto this interface as follows:
 *   Connect()   -> kvd_pool_create (x2) + kvd_plan_create : the tensor metadata of both sides
 *                  is registered once; the memory stays owned by the caller.
 *   Transfer()  -> kvd_build_descriptors : block ids are translated to byte ranges and queued;
 *                  queued ranges are coalesced (section 4.2);
 *                  kvd_pull : every (merged or unmerged) range is issued at once, no waiting
 *                  in between.
 *   Complete()  -> the caller's stream order / event after kvd_pull, or kvd_complete: a word in
 *                  memory that names the finished request; kvd_pull_notify gives every request
 *                  of a batched plan its own word, stored when its own reads are done (section 4.2).
 *
 * Conventions
 *   - Every call returns KVD_OK (0) or a negative kvd_status_t; kvd_last_error() gives a
 *     thread-local message for the last failure on the calling thread.  Nothing aborts or
 *     throws across this boundary.
 *   - Pointers are HOST pointers unless the comment says DEVICE.
 *   - `stream` arguments are hipStream_t values passed as void* (NULL = the null stream).
 *     Work is enqueued asynchronously; results are visible after the stream is synchronised.
 *   - Handles are not thread-safe: use one plan from one thread at a time.
 *   - The library never allocates, frees or writes the pools' memory except for the bytes a
 *     pull is defined to write.
 */
#ifndef KVD_H
#define KVD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KVD_OK = 0,
    KVD_ERR_INVALID = -1,  /* null pointer, zero dimension, empty layer range, misalignment       */
    KVD_ERR_RANGE = -2,    /* block id outside the pool, layer range outside a pool, table short  */
    KVD_ERR_MISMATCH = -3, /* the two pools do not hold the same kind of element / unsupported pair */
    KVD_ERR_ALIAS = -4,    /* a destination block is used twice in one plan, or the pools overlap  */
    KVD_ERR_CAPACITY = -5, /* plan is full                                                         */
    KVD_ERR_HIP = -6       /* a HIP runtime call failed (message holds the HIP error)              */
} kvd_status_t;

/* Order of the axes inside one block of one of K / V (section 4.1: the order of the
 * dimensions is free and part of the metadata). */
typedef enum {
    KVD_LAYOUT_BHTD = 0, /* [block][head][token][dim] */
    KVD_LAYOUT_BTHD = 1  /* [block][token][head][dim] */
} kvd_layout_t;

/*
 * Tensor metadata of one pool: Address, Shape and Stride of section 4.1, for all layers at
 * once.  Element (layer, kv, block, token, head, dim) lives at element offset
 *   layer*stride_layer + kv*stride_kv + block*stride_block + inner(token, head)*head_dim + dim
 * with inner = head*block_tokens + token (BHTD) or token*num_kv_heads + head (BTHD); the
 * axes inside a block are dense.  Strides count elements.
 * Requirements (else KVD_ERR_INVALID): base, stride_*xelem_bytes and head_dim*elem_bytes are
 * multiples of 16 bytes; elem_bytes is 1, 2, 4 or 8; stride_block >= elements of one block;
 * block_tokens <= 1024.  Every stride must be below 2^44 elements, stride_block below 64 GiB and
 * the block axis of one (layer, kv) slab below 2^50 bytes (KVD_ERR_RANGE); a plan accepts a block
 * axis above 64 GiB only for block-major pools on both sides (see kvd_plan_create).
 */
typedef struct {
    void *base; /* DEVICE pointer, borrowed for the pool's lifetime */
    uint32_t num_layers;
    uint32_t num_blocks;
    uint32_t block_tokens;
    uint32_t num_kv_heads;
    uint32_t head_dim;
    uint32_t elem_bytes;
    int32_t layout; /* kvd_layout_t */
    int64_t stride_layer;
    int64_t stride_kv;
    int64_t stride_block;
} kvd_pool_desc_t;

typedef struct kvd_pool kvd_pool_t;
typedef struct kvd_plan kvd_plan_t;

/* kvd_plan_create flags */
#define KVD_PLAN_NO_COALESCE 1u /* keep every read transaction separate (ablation of section 4.2) */
#define KVD_PLAN_WHOLE_BLOCKS 4u /* move every slot of a request's last block, not only the tokens below
                                   seq_len: the block-granular transfer of section 4.1 (needs equal
                                   block sizes, else KVD_ERR_MISMATCH)                              */
#define KVD_PLAN_QUEUE_ORDER 8u  /* never put the work items in the order of their destination: kvd_pull walks
                                   them in queue order whatever the plan looks like (ablation)      */
#define KVD_PLAN_DESTINATION_ORDER 64u /* put the work items of short transactions in the order of their
                                   destination (see kvd_pull) whatever the size of the transfer; by default
                                   that is done only from 0.5 to 1.5 GiB of payload on, where one pull earns
                                   the ordering launches back - a plan that is pulled many times (a recorded
                                   graph) earns them back at any size                                 */
#define KVD_PLAN_WIDE_OFFSETS 16u /* block-major plans: carry 48-bit offsets even where 32 bits reach the whole
                                   pool (the form pools above 64 GiB get by themselves); for testing  */
#define KVD_PLAN_COMPLETE_PER_REQUEST 32u /* every request of the plan is followed by its own completion
                                   transaction (section 4.2), so reads are merged inside a request only - merging stops
                                   at the first completion in the queue - and kvd_pull_notify can announce each request
                                   when its own reads are done                                        */
#define KVD_PLAN_PERSISTENT 2u  /* kvd_pull uses a persistent grid that stages the coalesced descriptors
                                   in LDS and walks them wave by wave, instead of one small workgroup
                                   per work item (for comparison; slower; one layer range per plan) */

/* A coalesced read transaction of the byte-copy path, relative to (layer 0, K): the copy for
 * (layer, kv) adds layer*stride_layer*elem_bytes + kv*stride_kv*elem_bytes of the respective
 * pool to both offsets.  In plans whose K and V are adjacent on both sides (see kvd_plan_create)
 * a transaction may span K and V and only the layer offset is added; in plans over block-major
 * pools a transaction spans the request's layers too and its offsets are final. */
typedef struct {
    uint64_t src_offset; /* bytes from the source pool's base       */
    uint64_t dst_offset; /* bytes from the destination pool's base  */
    uint64_t bytes;
} kvd_span_t;

/* A read transaction of the re-layout path: num_tokens tokens that sit in one source block
 * and one destination block. */
typedef struct {
    int32_t src_block;
    uint32_t src_token; /* first slot inside the source block      */
    int32_t dst_block;
    uint32_t dst_token; /* first slot inside the destination block */
    uint32_t num_tokens;
} kvd_piece_t;

typedef struct {
    uint32_t num_requests;
    uint32_t relayout;         /* 0: byte-copy path, 1: re-layout path                           */
    uint64_t num_src_blocks;   /* table entries consumed on the source side                      */
    uint64_t num_dst_blocks;   /* table entries consumed on the destination side                 */
    uint64_t num_transactions; /* read transactions before coalescing, per (layer, kv)           */
    uint64_t num_descriptors;  /* after coalescing, per (layer, kv)                              */
    uint64_t num_work_items;   /* 4 KiB pieces the descriptors expand to, per (layer, kv)        */
    uint64_t payload_bytes;    /* bytes one kvd_pull writes = bytes it reads                     */
    uint32_t work_order;       /* how kvd_pull walks the work items: KVD_ORDER_*                 */
    uint32_t reserved;
} kvd_stats_t;

#define KVD_ORDER_QUEUE 0u   /* as queued                                                           */
#define KVD_ORDER_REGIONS 1u /* grouped by 2 MiB region of the destination (transactions below four work items) */
#define KVD_ORDER_SORTED 2u  /* whole transactions sorted by destination address (four to eight work items)     */

/*
 * Register one pool's tensor metadata (section 4.1, what Connect() exchanges; the pool's
 * memory plays the role of the registered GPU memory region of section 4.2).
 * `desc` is copied.  No GPU call is made.  *out receives a handle to release with kvd_free.
 * Errors: KVD_ERR_INVALID, KVD_ERR_RANGE (see kvd_pool_desc_t).
 */
int kvd_pool_create(const kvd_pool_desc_t *desc, kvd_pool_t **out);

/*
 * Create a transfer plan from `src` to `dst`: the transaction queue of section 4.2.  A plan
 * holds the requests appended by kvd_build_descriptors until kvd_plan_reset.
 * max_requests / max_total_blocks bound the number of appended requests and the number of
 * block-table entries (per side) the plan can hold.  The pool metadata is copied, so the pool
 * handles may be freed before the plan.  Device and pinned scratch memory (a few bytes per
 * block) is allocated by the first kvd_build_descriptors that passes validation, on the
 * device that is current then.
 * When K and V of a block are neighbours in memory on both sides (stride_kv equals the elements
 * of one block) and the inner order is the same, a block's K and V are one byte range and merge
 * like any other contiguous ranges (section 4.1).
 * When, in addition, the layers of a block are neighbours on both sides (block-major pools:
 * stride_layer equals K plus V of one block, stride_block covers all layers), a request's layer
 * tensors are queued block by block, so that everything the request moves of a block is one byte
 * range (a ragged last block: one range per layer, K/V and head) and runs of adjacent blocks merge
 * over all layers.  Such plans count transactions, descriptors and work items (kvd_stats_t) for
 * the whole request, not per (layer, kv).  Offsets inside such a plan have 32 bits (of 16-byte
 * units) while both pools stay within 64 GiB and 48 bits beyond; with 48-bit offsets a descriptor
 * never continues across a multiple of 32 GiB from either pool's base (its length keeps 32 bits),
 * so a run that crosses one is two descriptors.
 * Errors: KVD_ERR_INVALID (null, zero capacity, unknown flag bits, KVD_PLAN_QUEUE_ORDER together with
 * KVD_PLAN_DESTINATION_ORDER), KVD_ERR_MISMATCH (num_kv_heads, head_dim or
 * elem_bytes differ; block sizes of which neither divides the other; KVD_PLAN_WIDE_OFFSETS or a
 * pool above 64 GiB with KVD_PLAN_PERSISTENT, KVD_PLAN_WIDE_OFFSETS without block-major pools),
 * KVD_ERR_RANGE (a block axis above 64 GiB in a plan that is not block-major on both sides with
 * the same inner order), KVD_ERR_ALIAS (the byte ranges of the two pools overlap).
 */
int kvd_plan_create(const kvd_pool_t *src, const kvd_pool_t *dst, uint32_t max_requests,
                    uint32_t max_total_blocks, uint32_t flags, kvd_plan_t **out);

/*
 * Append one request: Transfer() for each of its blocks (section 4.1), queued behind the
 * requests already in the plan, then coalesced with them (section 4.2: a transaction is
 * merged into its predecessor in the queue only when it continues it on both the source and
 * the destination side; merges may cross request boundaries when both requests move the same
 * layers).
 *
 * src_block_table[n_src], dst_block_table[n_dst]: HOST arrays of physical block ids in
 * logical order; token t of the request is in source block src_block_table[t / Tsrc] slot
 * t % Tsrc and goes to destination block dst_block_table[t / Tdst] slot t % Tdst.  Only the
 * first ceil(seq_len / T) entries of each table are used; both arrays may be reused by the
 * caller as soon as the call returns.  Only tokens below seq_len are moved: the unused slots
 * of the last destination block keep their contents.  Layers [layer_begin, layer_end) are
 * moved, K and V.  seq_len == 0 appends nothing and succeeds.
 *
 * Address translation and coalescing run in a kernel enqueued on `stream`; kvd_pull must be
 * enqueued on the same stream (or be ordered after it by the caller).  Builds of one plan normally
 * use one stream; a build on another stream than the plan's previous one first waits on the host
 * until that one has read its tables (the caller still orders the two streams' kernels).  `stream` must not be
 * recording a HIP graph (KVD_ERR_INVALID): the host part of the call happens at once.
 *
 * Errors (checked on the host before anything is enqueued; the plan is unchanged on error):
 * KVD_ERR_INVALID (null, layer_begin >= layer_end), KVD_ERR_RANGE (block id outside its pool,
 * layer range outside either pool, a table shorter than ceil(seq_len / T), seq_len above 2^30), KVD_ERR_ALIAS (a
 * destination block already used in this plan, or twice in this request; repeated source
 * blocks are allowed), KVD_ERR_CAPACITY, KVD_ERR_HIP.
 */
int kvd_build_descriptors(kvd_plan_t *plan, const int32_t *src_block_table, uint32_t n_src,
                          const int32_t *dst_block_table, uint32_t n_dst, uint32_t seq_len,
                          uint32_t layer_begin, uint32_t layer_end, void *stream);

/*
 * Append several requests that move the same layers with one call and one kernel launch per 512
 * requests: the same queue, in array order, as n_requests calls of kvd_build_descriptors.
 * src_block_tables[k] / dst_block_tables[k] (HOST arrays of n_src[k] / n_dst[k] ids) and
 * seq_lens[k] describe request k; requests with seq_lens[k] == 0 are skipped.  All requests are
 * validated before the plan is touched: on any error none of them is appended.
 * Errors: as kvd_build_descriptors; the message names the offending request.
 */
int kvd_build_descriptors_batch(kvd_plan_t *plan, uint32_t n_requests,
                                const int32_t *const *src_block_tables, const uint32_t *n_src,
                                const int32_t *const *dst_block_tables, const uint32_t *n_dst,
                                const uint32_t *seq_lens, uint32_t layer_begin, uint32_t layer_end,
                                void *stream);

/*
 * Issue every queued (merged or unmerged) read of the plan at once, for all its requests,
 * layers and K/V, as ONE kernel launch on `stream` (section 4.2: all reads are posted without
 * blocking; section 4.3: all layers in a single shot).  Every read is cut into work items of at
 * most 4 KiB and each (work item, layer, K/V) is moved by its own small workgroup, 16 bytes per
 * lane.  When the plan's merged transactions are short (at least three quarters of the work in
 * transactions of at most eight work items, as for lone blocks of 4 to 32 KiB; judged on the host from
 * the runs in the block tables) the first pull after an append is preceded by one or two small launches
 * that put the work items in the order of their destination (by 2 MiB region where transactions below
 * four items prevail, whole transactions sorted by address otherwise; a plan's first request of at
 * most 1024 transactions is sorted by kvd_build_descriptors itself, without those launches); which
 * bytes are moved does not depend on it.  Re-layout plans between two pools whose blocks are the outermost
 * axis are walked block by block (all slabs of a block together) instead of slab by slab.  May be
 * called repeatedly; a plan with no requests is a no-op.
 * May be recorded into a HIP graph (it allocates nothing and waits for nothing); the graph then
 * replays the pull of the plan as it was built at recording time and must not be replayed after
 * the plan has been reset or appended to.
 * Completion (section 4.1, Complete()) is the caller's synchronisation on `stream`.
 * Errors: KVD_ERR_INVALID, KVD_ERR_HIP, KVD_ERR_MISMATCH (KVD_PLAN_PERSISTENT with several layer
 * ranges in one plan).
 */
int kvd_pull(kvd_plan_t *plan, void *stream);

/*
 * The same as kvd_pull for layers [layer_begin, layer_end) of the pools only: of every request of
 * the plan, the layers of that range that the request was built for are moved (none, if the ranges
 * do not meet).  This is the layer-by-layer use that section 4.3 contrasts with the single shot: a
 * prefill worker that has just written layer l issues kvd_pull_layers(plan, l, l + 1) against the
 * plan built once for all layers, without another translation or coalescing pass.  Like kvd_pull it
 * may be recorded into a HIP graph.
 * Errors: KVD_ERR_INVALID (handle, empty range), KVD_ERR_RANGE (range outside a pool),
 * KVD_ERR_MISMATCH (plan over block-major pools, whose descriptors span the layers; KVD_PLAN_PERSISTENT),
 * KVD_ERR_HIP.
 */
int kvd_pull_layers(kvd_plan_t *plan, uint32_t layer_begin, uint32_t layer_end, void *stream);

/*
 * kvd_pull with a completion per request (section 4.2: a completion transaction is processed when the
 * reads of ITS request are done, while the reads of other requests go on): moves what kvd_pull moves,
 * and stores `value` into words[k] as soon as every byte of the plan's k-th request (in the order of
 * appending; requests of length 0 are not counted, see kvd_stats_t.num_requests) has arrived, with those
 * bytes visible to any reader of the word first (system-scope release).  `words` holds at least
 * num_requests 8-byte words owned by the caller, in device memory or in pinned host memory that a CPU
 * thread polls; the caller chooses `value` so that it differs from what the words held before.
 * The plan must have been created with KVD_PLAN_COMPLETE_PER_REQUEST.  Requests are moved in queue order,
 * one launch each (or per group, see kvd_plan_set_completion_granularity) on two library-owned side streams in turn (default priority), so that the next request's
 * reads are in flight while one request's last reads finish; `stream` is forked from and joined again:
 * work enqueued on `stream` after the call runs after the whole plan has been moved.  Work items are
 * walked in queue order (no grouping by destination region).  May be recorded into a HIP graph.
 * Errors: KVD_ERR_INVALID (handle, null or misaligned words, memory the GPU cannot reach),
 * KVD_ERR_MISMATCH (plan without KVD_PLAN_COMPLETE_PER_REQUEST, KVD_PLAN_PERSISTENT, re-layout plans between
 * block-major pools), KVD_ERR_HIP.
 */
int kvd_pull_notify(kvd_plan_t *plan, uint64_t *words, uint64_t value, void *stream);

/*
 * How finely kvd_pull_notify announces (a plan created with KVD_PLAN_COMPLETE_PER_REQUEST; else
 * KVD_ERR_MISMATCH).  0, the default: every request by itself, as soon as its own reads are done
 * (section 4.2).  min_tokens > 0: consecutive requests of the queue that move the same layer range
 * share a launch until it holds at least min_tokens tokens, and their words are stored together when
 * the launch's reads are done - a request is then announced no earlier than its own reads and no later
 * than those of the requests it shares the launch with.  A launch costs a few microseconds, so short
 * requests are announced more cheaply in company (64 requests of 16..16384 tokens, 10.5 GiB: 6 to 8 %
 * over kvd_pull one by one, 4.5 % with min_tokens = 1024, 3.9 % with 4096).  Takes effect at the next
 * kvd_pull_notify; host only.
 */
int kvd_plan_set_completion_granularity(kvd_plan_t *plan, uint32_t min_tokens);

/*
 * For callers that cannot allocate device memory - code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc: kvd_build_descriptors + kvd_pull for ONE request in one
 * call that allocates nothing, on the device or through any allocating runtime routine.  The pools
 * are described by their metadata directly (no handles), the block tables are HOST arrays as for
 * kvd_build_descriptors (they travel in kernel arguments, 448 ids per side and launch), and what a
 * plan keeps in allocated scratch lives in one array of about 19.6 MiB that is part of the library's
 * code object and that every GPU the call is used on holds until the process ends.
 * Limits (KVD_ERR_CAPACITY, nothing is enqueued): at most KVD_NOALLOC_MAX_BLOCKS block-table
 * entries per side, 2^17 read transactions before merging and KVD_NOALLOC_MAX_WORK_ITEMS work items
 * of 4 KiB (per (layer, K/V); for block-major pools over all layers of the request).
 * `flags`: KVD_PLAN_NO_COALESCE, KVD_PLAN_WHOLE_BLOCKS, KVD_PLAN_QUEUE_ORDER, KVD_PLAN_DESTINATION_ORDER or 0; anything else is
 * KVD_ERR_INVALID.  Moves exactly the bytes that kvd_plan_create(flags) + kvd_build_descriptors +
 * kvd_pull move for the same arguments, with the same kernels, enqueued on `stream`; may be
 * recorded into a HIP graph (the tables are captured by value).  seq_len == 0 enqueues nothing.
 * All calls on one GPU share that GPU's array: a call may follow another on the same stream, but
 * calls whose kernels could overlap on one GPU (different streams without ordering between them,
 * different threads) race and give undefined destination bytes.  The array needs no clearing
 * between calls: every part that is read is written first by the same call.
 * Errors: as kvd_pool_create, kvd_plan_create and kvd_build_descriptors for the same arguments,
 * all detected on the host before anything is enqueued.
 */
#define KVD_NOALLOC_MAX_BLOCKS 8192u
#define KVD_NOALLOC_MAX_WORK_ITEMS (1u << 19)
int kvd_pull_noalloc(const kvd_pool_desc_t *src, const kvd_pool_desc_t *dst,
                     const int32_t *src_block_table, uint32_t n_src,
                     const int32_t *dst_block_table, uint32_t n_dst, uint32_t seq_len,
                     uint32_t layer_begin, uint32_t layer_end, uint32_t flags, void *stream);

/*
 * Complete() of section 4.1 as the paper sends it, a message naming the finished request: stores
 * `value` (a request id, a sequence number) into *flag once everything enqueued on `stream`
 * before this call - the pulls - has finished, with the pulled bytes visible to any reader of the
 * flag first.  `flag` is 8-byte aligned and owned by the caller: device memory, or pinned host
 * memory (its host address) that a CPU thread polls; anything else is refused.  A caller that synchronises the stream or
 * records an event itself does not need this call.  May be recorded into a HIP graph.
 * Errors: KVD_ERR_INVALID (null or misaligned flag, memory the GPU cannot reach), KVD_ERR_HIP.
 */
int kvd_complete(uint64_t *flag, uint64_t value, void *stream);

/*
 * Reported baseline, not the product path: the buffer-based transfer the paper argues against
 * (section 4.1, message-based scheme).  Per iteration, as many 4 KiB work items of one (layer,
 * K/V) as `buffer_bytes` holds are gathered by a kernel into `send_buffer`, copied to
 * `recv_buffer` (standing in for the wire), waited for by the host, scattered by a second kernel
 * into the destination pool, and waited for again (the notification).  Both buffers are DEVICE
 * memory of at least buffer_bytes (>= 4096), owned by the caller.  Moves the same bytes as
 * kvd_pull with three times the memory traffic and two host waits per iteration.  Blocks the
 * calling thread until the transfer is complete.
 */
int kvd_pull_staged(kvd_plan_t *plan, void *send_buffer, void *recv_buffer, uint64_t buffer_bytes,
                    void *stream);

/*
 * Reported baseline, not the product path: the same transfer as one hipMemcpyAsync per
 * (request, layer, K/V, block) on `stream`, the way a per-block message scheme touches memory
 * (section 3, motivation 1).  Only for pools with equal layout and block size
 * (else KVD_ERR_MISMATCH).
 */
int kvd_pull_blockwise_memcpy(kvd_plan_t *plan, void *stream);

/* Forget all requests of the plan.  Waits (a short spin on a word in pinned host memory that the
 * build kernel sets) until the builds enqueued so far have read the plan's copy of the block
 * tables; it does not wait for pulls: the caller must not enqueue a new build of this plan on a
 * stream where it could overtake a pull of the old contents. */
int kvd_plan_reset(kvd_plan_t *plan);

/* Counters of the plan.  Synchronises `stream` (the one the builds were enqueued on) to read
 * the descriptor counts back. */
int kvd_plan_stats(kvd_plan_t *plan, void *stream, kvd_stats_t *out);

/*
 * Read the plan's descriptors back (synchronises `stream`).  Byte-copy plans fill `spans`
 * (pieces may be NULL), re-layout plans fill `pieces`.  At most `cap` entries are written;
 * *n_out receives the number available.  Order is queue order.
 */
int kvd_plan_get_descriptors(kvd_plan_t *plan, void *stream, kvd_span_t *spans,
                             kvd_piece_t *pieces, uint64_t cap, uint64_t *n_out);

/*
 * Plain streaming copy of `bytes` bytes (multiple of 16, DEVICE pointers 16-byte aligned) with
 * the same access width as the pull kernel.  Used to calibrate hardware byte counters and as
 * the practical copy ceiling next to which the pull is reported.
 */
int kvd_copy_plain(void *dst, const void *src, uint64_t bytes, void *stream);

/*
 * Calibration, not the product path: one pass over plain buffers of `bytes` bytes (a multiple of 4096;
 * DEVICE pointers, 16-byte aligned) with the pull kernel's access width and cache policies.  `mode`
 * selects a copy, a read-only or a write-only stream, each either with one access per lane and the
 * workgroups handed out by the hardware dispatcher in address order, or with a fixed grid of resident
 * workgroups striding over the buffer (the persistent form).  Shows what the memory system gives each
 * kind of stream, next to which the pull kernel's design is justified.  The write-only forms fill `dst`
 * with a constant; the read-only forms leave both buffers unchanged.
 */
#define KVD_PROBE_COPY 0u
#define KVD_PROBE_READ 1u
#define KVD_PROBE_WRITE 2u
#define KVD_PROBE_COPY_PERSISTENT 3u
#define KVD_PROBE_READ_PERSISTENT 4u
#define KVD_PROBE_WRITE_PERSISTENT 5u
int kvd_stream_probe(void *dst, const void *src, uint64_t bytes, uint32_t mode, void *stream);

/* Release a pool or a plan (NULL is allowed).  Frees the plan's own scratch, never pool memory.
 * The library keeps a list of the handles it has given out: a pointer that is not on it (released
 * before, or never a handle) is ignored here without being read, and refused with KVD_ERR_INVALID
 * by every other call. */
void kvd_free(void *handle);

/* Message for the last error on this thread ("" if none). */
const char *kvd_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* KVD_H */
