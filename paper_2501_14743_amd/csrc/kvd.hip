// kvd - paged KV-cache pull for MI355X (gfx950): host side of the C ABI declared in kvd.h.
//
// Validation, the plan object and its scratch memory, and the launches of the kernels in
// kvd_kernels.h (structures, device code and their description).

#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <exception>
#include <mutex>
#include <new>
#include <thread>
#include <unordered_set>
#include <vector>

#include "kvd.h"
#include "kvd_kernels.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define KVD_HIP(call)                                                                       \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess)                                                               \
            return fail(KVD_ERR_HIP, "%s failed: %s", #call, hipGetErrorString(e_));        \
    } while (0)

constexpr uint32_t kPoolTag = 0x6b76504fu;  // handle type tags
constexpr uint32_t kPlanTag = 0x6b76504cu;

// Every handle this library has given out and not yet released.  A pointer is looked up here
// before it is dereferenced, so a stale, foreign or already released handle is refused instead of
// being read.  Guarded by a mutex; a lookup costs some tens of nanoseconds per call.
// The list and its mutex are created at first use and never destroyed, so that a release
// that arrives while the process is shutting down still finds them.
struct HandleList {
    std::mutex mutex;
    std::unordered_set<const void *> live;
};

HandleList &handle_list()
{
    static HandleList *list = new HandleList;
    return *list;
}

void register_handle(const void *h)
{
    HandleList &l = handle_list();
    std::lock_guard<std::mutex> lock(l.mutex);
    l.live.insert(h);
}

bool is_live_handle(const void *h)
{
    HandleList &l = handle_list();
    std::lock_guard<std::mutex> lock(l.mutex);
    return l.live.count(h) != 0;
}

// True if h was live; it no longer is afterwards.
bool retire_handle(const void *h)
{
    HandleList &l = handle_list();
    std::lock_guard<std::mutex> lock(l.mutex);
    return l.live.erase(h) != 0;
}

struct ReqHost {
    uint32_t table_off_src, table_off_dst;  // into the plan's table mirrors
    uint32_t n_src, n_dst;                  // entries used
    uint32_t seq_len, layer_begin, layer_end;
    uint32_t item_bound;                    // work items per slab before merging (upper bound of what it has)
};

// What the block tables tell the host about how the plan's memory lies, for the decision in which
// order kvd_pull walks the work items (a hint for launch decisions only: what is done with the work
// items is decided on the device from the build kernel's own counts).
struct OrderHint {
    uint64_t items_below4;  // work items of pieces shorter than four work items (16 KiB)
    uint64_t items_4to8;    // ... of pieces of four to eight work items
    uint64_t src_descents, dst_descents;  // how often the queue steps back in either pool (0: it is in that pool's address order)
    bool rough;             // some request's pieces were not walked (block sizes differ): all taken as alike, of average size
};

}  // namespace

// Side streams that the per-request pulls of kvd_pull_notify take turns on.
#ifndef KVD_NOTIFY_STREAMS
#define KVD_NOTIFY_STREAMS 2
#endif
constexpr int kNotifyStreams = KVD_NOTIFY_STREAMS;

struct kvd_pool {
    uint32_t tag;
    kvd_pool_desc_t d;
    uint64_t extent_bytes;  // bytes from base that the metadata can reach
};

// Bytes the block axis of one (layer, K/V) slab spans.
static uint64_t block_axis_bytes(const kvd_pool_desc_t &d)
{
    return ((uint64_t)(d.num_blocks - 1) * d.stride_block + (uint64_t)d.block_tokens * d.num_kv_heads * d.head_dim) *
           d.elem_bytes;
}

struct kvd_plan {
    uint32_t tag;
    kvd_pool_desc_t src, dst;
    uint32_t max_requests, max_total_blocks, flags;
    Geo geo;
    // Block-major pools on both sides ([block][layer][K/V][...], every layer of a block adjacent):
    // the layers a request moves are folded into the head axis as well, so a whole block is one
    // byte range over all of them.  planes_per_layer = what one layer adds to that axis.
    bool fold_layers;
    uint32_t planes_per_layer;
    // Re-layout between two pools whose blocks are the outermost axis: pulled descriptor by
    // descriptor (kvd_pull_by_descriptor_kernel); items_per_desc = work items of a whole descriptor.
    bool by_descriptor;
    uint32_t items_per_desc;
    uint64_t max_txns, max_items;
    // host bookkeeping
    std::vector<ReqHost> reqs;
    std::vector<uint8_t> dst_used;  // one byte per destination block
    uint64_t used_src, used_dst, txns_total, item_bound, payload_bytes;
    OrderHint hint;                 // how the plan's memory lies, as far as the host can tell from the tables
    uint32_t max_layers;            // largest layer count of any request in the plan
    // device / pinned scratch (allocated on first use)
    bool allocated;
    int device;
    int num_cus;
    int32_t *tables_src, *tables_dst;  // pinned host, device-visible
    int32_t *tables_src_dev, *tables_dst_dev;
    ReqDev *reqs_pinned, *reqs_pinned_dev;  // one entry per request, same kind of memory
    Desc *desc_dev;
    uint32_t *desc_hi_dev;  // upper halves of the descriptors' offsets (used only when geo.wide)
    Item *items_dev;
    Item *ordered_dev;     // items in the order of their destination (plans of short descriptors)
    OrderEntry *order_dev; // per sorted descriptor: where its items go and come from (kvd_order_kernel -> kvd_order_copy_kernel)
    bool order_stale;      // requests were appended since ordered_dev was last written
    bool sorted_by_build;  // ordered_dev was written by the plan's only build launch (BuildArgs::sort_inline)
    uint32_t order_shift;  // log2 of the region size in 16-byte units
    Header *hdr_dev;
    // Completion of the build kernels, as far as the host's tables are concerned: every launch
    // carries a sequence number and stores it into a pinned host word when it has read them.
    // (An event recorded between the build and the pull would cost a few microseconds of every
    // step on the GPU's queue.)
    uint32_t *done_host, *done_dev;
    uint32_t build_seq;
    hipStream_t build_stream;
    // KVD_PLAN_COMPLETE_PER_REQUEST: where each request starts in the descriptor and work-item
    // tables (device), and the two streams its pulls alternate on with their fork / join events
    uint32_t *req_desc_dev, *req_item_dev;
    hipStream_t notify_stream[kNotifyStreams];
    hipEvent_t notify_fork, notify_join[kNotifyStreams];
    bool notify_ready;
    uint32_t notify_min_tokens;  // kvd_pull_notify: a launch takes requests until it holds this many tokens (0: one each)
};

namespace {

int check_pool_desc(const kvd_pool_desc_t &d, uint64_t *extent_out)
{
    if (!d.base) return fail(KVD_ERR_INVALID, "pool base is null");
    if (!d.num_layers || !d.num_blocks || !d.block_tokens || !d.num_kv_heads || !d.head_dim)
        return fail(KVD_ERR_INVALID, "pool has a zero dimension");
    if (d.elem_bytes != 1 && d.elem_bytes != 2 && d.elem_bytes != 4 && d.elem_bytes != 8)
        return fail(KVD_ERR_INVALID, "elem_bytes must be 1, 2, 4 or 8 (got %u)", d.elem_bytes);
    if (d.layout != KVD_LAYOUT_BHTD && d.layout != KVD_LAYOUT_BTHD)
        return fail(KVD_ERR_INVALID, "unknown layout %d", d.layout);
    if (d.block_tokens > 1024) return fail(KVD_ERR_INVALID, "block_tokens above 1024");
    if (d.num_layers > 32767) return fail(KVD_ERR_INVALID, "num_layers above 32767");
    if (d.stride_layer < 0 || d.stride_kv < 0 || d.stride_block < 0)
        return fail(KVD_ERR_INVALID, "negative stride");
    if (d.stride_layer >= (1ll << 44) || d.stride_kv >= (1ll << 44) || d.stride_block >= (1ll << 44))
        return fail(KVD_ERR_RANGE, "stride of 2^44 elements or more");
    const uint64_t e = d.elem_bytes;
    const uint64_t tile = (uint64_t)d.block_tokens * d.num_kv_heads * d.head_dim;
    if ((uint64_t)d.stride_block < tile)
        return fail(KVD_ERR_INVALID, "stride_block smaller than one block");
    if (((uintptr_t)d.base % 16) || ((uint64_t)d.stride_layer * e % 16) ||
        ((uint64_t)d.stride_kv * e % 16) || ((uint64_t)d.stride_block * e % 16) ||
        ((uint64_t)d.head_dim * e % 16))
        return fail(KVD_ERR_INVALID, "base, strides and head_dim*elem_bytes must be multiples of 16 bytes");
    if ((uint64_t)d.head_dim * e > 4096)
        return fail(KVD_ERR_INVALID, "head_dim*elem_bytes above 4096 bytes");
    if ((uint64_t)d.block_tokens * d.num_kv_heads > (1u << 20))
        return fail(KVD_ERR_INVALID, "block_tokens*num_kv_heads above 2^20");
    if ((uint64_t)d.stride_block * e >= (1ull << 36)) return fail(KVD_ERR_RANGE, "stride_block of 64 GiB or more");
    // in 128 bits: 2^32 blocks times a stride of up to 2^36 bytes does not fit 64
    const unsigned __int128 block_axis = ((unsigned __int128)(d.num_blocks - 1) * (uint64_t)d.stride_block + tile) * e;
    if (block_axis >= ((unsigned __int128)1 << 50))
        return fail(KVD_ERR_RANGE, "block axis spans more than 2^50 bytes");
    // the layer, K/V and block axes must nest without overlap, in whatever order the strides put them
    struct Axis { uint64_t n, stride; } ax[3] = {{d.num_layers, (uint64_t)d.stride_layer},
                                                 {2, (uint64_t)d.stride_kv},
                                                 {d.num_blocks, (uint64_t)d.stride_block}};
    std::sort(ax, ax + 3, [](const Axis &x, const Axis &y) { return x.stride < y.stride; });
    uint64_t extent = tile;
    for (const Axis &x : ax) {
        if (x.n > 1 && x.stride < extent)
            return fail(KVD_ERR_INVALID, "layer, K/V and block axes overlap (a stride of %llu elements is smaller than "
                        "the %llu elements nested inside it)", (unsigned long long)x.stride, (unsigned long long)extent);
        extent += (x.n - 1) * x.stride;
    }
    *extent_out = extent * e;
    return KVD_OK;
}

uint32_t ceil_div(uint32_t a, uint32_t b) { return (a + b - 1) / b; }

// Sizes of one request per (layer, kv): read transactions, and the work items they need before
// any merging (an upper bound of the number after merging).
void request_sizes(const Geo &g, uint32_t seq_len, uint32_t *n_txn, uint32_t *items)
{
    const uint32_t pieces = ceil_div(seq_len, g.piece_tokens);
    const uint32_t whole = seq_len / g.piece_tokens, tail = seq_len % g.piece_tokens;
    if (g.mode >= kRelayoutHT2TH) {
        *n_txn = pieces;
        *items = whole * ceil_div(g.piece_tokens * g.hk, g.rows_per_item) +
                 (tail ? ceil_div(tail * g.hk, g.rows_per_item) : 0);
    } else if (g.mode == kSpanTokenMajor) {
        *n_txn = pieces;
        *items = whole * ceil_div(g.piece_tokens * g.hk * g.du, kChunkUnits) +
                 (tail ? ceil_div(tail * g.hk * g.du, kChunkUnits) : 0);
    } else if (g.tb_src != g.tb_dst) {
        *n_txn = pieces * g.hk;
        *items = g.hk * (whole * ceil_div(g.piece_tokens * g.du, kChunkUnits) +
                         (tail ? ceil_div(tail * g.du, kChunkUnits) : 0));
    } else {
        *n_txn = whole + (tail ? g.hk : 0);
        *items = whole * ceil_div(g.piece_tokens * g.hk * g.du, kChunkUnits) +
                 (tail ? g.hk * ceil_div(tail * g.du, kChunkUnits) : 0);
    }
}

// Adds one request.  A piece is what the request's memory consists of on both sides at once as far as
// the adjacency of consecutive entries in the two block tables tells: the descriptors it merges into
// (with KVD_PLAN_NO_COALESCE the descriptors stay apart, but what matters for the order of the work is
// how the memory lies).
void add_order_hint(OrderHint *h, const Geo &g, const int32_t *st, const int32_t *dt, uint32_t seq_len, uint32_t n_txn,
                    uint32_t items)
{
    const uint32_t src_blocks = ceil_div(seq_len, g.tb_src), dst_blocks = ceil_div(seq_len, g.tb_dst);
    for (uint32_t i = 1; i < src_blocks; ++i) h->src_descents += st[i] < st[i - 1] ? 1u : 0u;
    for (uint32_t i = 1; i < dst_blocks; ++i) h->dst_descents += dt[i] < dt[i - 1] ? 1u : 0u;
    auto piece = [&](uint64_t units) {
        const uint64_t n = (units + kChunkUnits - 1) / kChunkUnits;
        if (n < 4) h->items_below4 += n;
        else if (n <= kSortItemsPerDesc) h->items_4to8 += n;
    };
    if (g.mode >= kRelayoutHT2TH || g.tb_src != g.tb_dst) {
        // pieces of min(block sizes) tokens; which of them merge is not looked at: all alike, of average size
        h->rough = true;
        const uint64_t per = n_txn ? (items + n_txn - 1) / n_txn : 0;
        if (per < 4) h->items_below4 += items;
        else if (per <= kSortItemsPerDesc) h->items_4to8 += items;
        return;
    }
    const uint32_t whole = seq_len / g.tb_src, tail = seq_len % g.tb_src;
    const uint64_t block_units = (uint64_t)g.tb_src * g.hk * g.du;
    const bool tail_per_head = g.mode == kSpanHeadMajor;  // a partial last block is then one piece per head
    const uint32_t in_runs = (tail && !tail_per_head) ? whole + 1 : whole;  // table entries that form runs
    uint64_t run_units = 0;
    for (uint32_t i = 0; i < in_runs; ++i) {
        if (i > 0 && (st[i] != st[i - 1] + 1 || dt[i] != dt[i - 1] + 1)) {
            piece(run_units);
            run_units = 0;
        }
        run_units += (i < whole) ? block_units : (uint64_t)tail * g.hk * g.du;
    }
    if (run_units) piece(run_units);
    if (tail && tail_per_head)
        for (uint32_t head = 0; head < g.hk; ++head) piece((uint64_t)tail * g.du);
}

// Frees whatever of the plan's scratch exists (pointers are null until allocated).
void free_scratch(kvd_plan *p)
{
    // the side streams of per-request pulls first: what is still running on them uses the memory below
    if (p->notify_ready) {
        for (int i = 0; i < kNotifyStreams; ++i) {
            (void)hipStreamSynchronize(p->notify_stream[i]);
            (void)hipStreamDestroy(p->notify_stream[i]);
        }
        for (int i = 0; i < kNotifyStreams; ++i) (void)hipEventDestroy(p->notify_join[i]);
        (void)hipEventDestroy(p->notify_fork);
        p->notify_ready = false;
    }
    if (p->done_host) (void)hipHostFree(p->done_host);
    if (p->tables_src) (void)hipHostFree(p->tables_src);
    if (p->tables_dst) (void)hipHostFree(p->tables_dst);
    if (p->reqs_pinned) (void)hipHostFree(p->reqs_pinned);
    if (p->desc_dev) (void)hipFree(p->desc_dev);
    if (p->desc_hi_dev) (void)hipFree(p->desc_hi_dev);
    if (p->items_dev) (void)hipFree(p->items_dev);
    if (p->ordered_dev) (void)hipFree(p->ordered_dev);
    if (p->order_dev) (void)hipFree(p->order_dev);
    if (p->hdr_dev) (void)hipFree(p->hdr_dev);
    if (p->req_desc_dev) (void)hipFree(p->req_desc_dev);
    if (p->req_item_dev) (void)hipFree(p->req_item_dev);
    p->req_desc_dev = p->req_item_dev = nullptr;
    p->done_host = nullptr;
    p->tables_src = p->tables_dst = nullptr;
    p->reqs_pinned = nullptr;
    p->desc_dev = nullptr;
    p->desc_hi_dev = nullptr;
    p->items_dev = p->ordered_dev = nullptr;
    p->order_dev = nullptr;
    p->hdr_dev = nullptr;
}

int allocate_scratch(kvd_plan *p)
{
    KVD_HIP(hipGetDevice(&p->device));
    hipDeviceProp_t prop;
    KVD_HIP(hipGetDeviceProperties(&prop, p->device));
    p->num_cus = prop.multiProcessorCount;
    const size_t tb = (size_t)p->max_total_blocks * sizeof(int32_t);
    KVD_HIP(hipHostMalloc((void **)&p->tables_src, tb, hipHostMallocMapped));
    KVD_HIP(hipHostMalloc((void **)&p->tables_dst, tb, hipHostMallocMapped));
    KVD_HIP(hipHostGetDevicePointer((void **)&p->tables_src_dev, p->tables_src, 0));
    KVD_HIP(hipHostGetDevicePointer((void **)&p->tables_dst_dev, p->tables_dst, 0));
    KVD_HIP(hipHostMalloc((void **)&p->reqs_pinned, (size_t)p->max_requests * sizeof(ReqDev), hipHostMallocMapped));
    KVD_HIP(hipHostGetDevicePointer((void **)&p->reqs_pinned_dev, p->reqs_pinned, 0));
    KVD_HIP(hipMalloc((void **)&p->desc_dev, (size_t)p->max_txns * sizeof(Desc)));
    KVD_HIP(hipMalloc((void **)&p->desc_hi_dev, (size_t)p->max_txns * sizeof(uint32_t)));
    KVD_HIP(hipMalloc((void **)&p->items_dev, (size_t)p->max_items * sizeof(Item)));
    KVD_HIP(hipMalloc((void **)&p->ordered_dev, (size_t)p->max_items * sizeof(Item)));
    KVD_HIP(hipMalloc((void **)&p->order_dev, (size_t)p->max_txns * sizeof(OrderEntry)));
    KVD_HIP(hipMalloc((void **)&p->hdr_dev, sizeof(Header)));
    if (p->flags & KVD_PLAN_COMPLETE_PER_REQUEST) {
        KVD_HIP(hipMalloc((void **)&p->req_desc_dev, (size_t)p->max_requests * sizeof(uint32_t)));
        KVD_HIP(hipMalloc((void **)&p->req_item_dev, (size_t)p->max_requests * sizeof(uint32_t)));
    }
    KVD_HIP(hipHostMalloc((void **)&p->done_host, 64, hipHostMallocMapped));
    KVD_HIP(hipHostGetDevicePointer((void **)&p->done_dev, p->done_host, 0));
    *p->done_host = 0;
    p->build_seq = 0;
    p->build_stream = nullptr;
    return KVD_OK;
}

// The plan's scratch, allocated at the first build that passes validation; all or nothing.
int ensure_allocated(kvd_plan *p)
{
    if (p->allocated) return KVD_OK;
    const int rc = allocate_scratch(p);
    if (rc != KVD_OK) {
        free_scratch(p);  // keeps the message of the failed call
        return rc;
    }
    p->allocated = true;
    return KVD_OK;
}

// Wait until the last build kernel of the plan has read the host's tables.  Normally a short spin
// on the pinned word; after two seconds without it, the stream is synchronised to see what happened.
int wait_for_builds(kvd_plan *p)
{
    if (!p->allocated) return KVD_OK;
    volatile uint32_t *done = p->done_host;
    if (*done == p->build_seq) return KVD_OK;
    const auto t0 = std::chrono::steady_clock::now();
    for (uint32_t spins = 1;; ++spins) {
        if (*done == p->build_seq) return KVD_OK;
        __builtin_ia32_pause();
        if (spins > 4096) std::this_thread::yield();  // a long pull is ahead of the build: let other threads run
        if ((spins & 0xFFF) == 0 && std::chrono::steady_clock::now() - t0 > std::chrono::seconds(2)) break;
    }
    KVD_HIP(hipStreamSynchronize(p->build_stream));
    if (*done != p->build_seq) return fail(KVD_ERR_HIP, "the build kernel did not report completion");
    return KVD_OK;
}

void release_plan(kvd_plan *p)
{
    if (p->allocated) {
        (void)wait_for_builds(p);
        free_scratch(p);
    }
    p->tag = 0;
    delete p;
}

// True while `stream` is recording a HIP graph (work enqueued now runs at replay, not now).
bool is_capturing(void *stream)
{
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing((hipStream_t)stream, &status) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return status == hipStreamCaptureStatusActive;
}

kvd_plan *as_plan(void *h)
{
    if (!h || !is_live_handle(h)) return nullptr;
    kvd_plan *p = (kvd_plan *)h;
    return p->tag == kPlanTag ? p : nullptr;
}

const kvd_pool *as_pool(const void *h)
{
    if (!h || !is_live_handle(h)) return nullptr;
    const kvd_pool *p = (const kvd_pool *)h;
    return p->tag == kPoolTag ? p : nullptr;
}

// How kvd_pull walks the plan's work items, as the host decides it from the block tables.  Scattered
// pieces of 4-32 KiB move faster in the order of their destination; longer ones do not (measured: runs of
// two 32 KiB blocks gain 1.5 points, about what the sort costs, the 1-8 block runs of the 8192-token
// configuration lose one, and a dense batch of 1024 short requests - lone blocks and runs mixed, six work
// items per descriptor on average - loses six).  So the work is reordered only if at least three quarters
// of it sits in pieces of at most eight work items.  If most of that is in pieces below four items, the
// items are grouped by region (one launch of about 8 us, which pays from half a GiB of payload on);
// otherwise whole descriptors are sorted (two launches, 18-50 us: level with the gain of one pull at a
// GiB, so from 1.5 GiB on).  Re-layout plans gain nothing from the sort (measured); a queue that never steps
// back in the destination pool is in that order already, and one that never steps back in the source pool
// reads in address order, which the sort would give up for about as much as it gains (measured: 70.4
// against 71.5 % of HBM peak for 512 lone destination blocks).
// `item_bound`: the plan's work items per slab; `by_build`: the sort costs no launches, because the build
// kernel does it on the way (a fresh plan's only launch, at most kBuildLdsDescs descriptors: about 5 us),
// and then pays from half a GiB on.
uint32_t work_order_for(const kvd_plan *p, uint64_t item_bound, bool by_build)
{
    if ((p->flags & (KVD_PLAN_QUEUE_ORDER | KVD_PLAN_PERSISTENT)) || p->by_descriptor) return KVD_ORDER_QUEUE;
    const OrderHint &h = p->hint;
    if (h.dst_descents == 0 || h.src_descents == 0) return KVD_ORDER_QUEUE;
    if ((h.items_below4 + h.items_4to8) * 4 < item_bound * 3) return KVD_ORDER_QUEUE;
    const uint64_t pieces = item_bound * ((uint64_t)p->max_layers << p->geo.kv_shift);  // 4 KiB each
    const bool always = (p->flags & KVD_PLAN_DESTINATION_ORDER) != 0;
    if (h.items_below4 >= h.items_4to8) return (always || pieces >= (1u << 17)) ? KVD_ORDER_REGIONS : KVD_ORDER_QUEUE;
    if (p->geo.mode < kRelayoutHT2TH)
        return (always || pieces >= (by_build ? (1u << 17) : (3u << 17))) ? KVD_ORDER_SORTED : KVD_ORDER_QUEUE;
    return KVD_ORDER_QUEUE;
}

uint32_t work_order(const kvd_plan *p) { return work_order_for(p, p->item_bound, p->sorted_by_build); }

// Whether the launch that is about to build `batch_txn` transactions and `batch_items` work items into
// a plan that holds nothing yet should sort its descriptors by destination itself (BuildArgs::sort_inline).
bool build_sorts(const kvd_plan *p, bool only_launch_of_a_fresh_plan, uint32_t batch_txn, uint32_t batch_items)
{
    return only_launch_of_a_fresh_plan && batch_txn <= kBuildLdsDescs && batch_items <= kInlineItems && !p->geo.wide &&
           !p->hint.rough && work_order_for(p, batch_items, true) == KVD_ORDER_SORTED;
}

// The launch(es) of a pull: the whole plan (whole = true), or layers [l0, l1) of the pools.
int launch_pull(kvd_plan *p, void *stream, bool whole, uint32_t l0, uint32_t l1)
{
    PullArgs a{};
    a.src_base = (const unsigned char *)p->src.base;
    a.dst_base = (unsigned char *)p->dst.base;
    a.items = p->items_dev;
    a.hdr = p->hdr_dev;
    a.slabs = (whole ? p->max_layers : l1 - l0) << p->geo.kv_shift;
    a.absolute_layers = whole ? 0u : 1u;
    a.layer0 = l0;
    a.req_item = nullptr;
    a.req = a.req_end = a.n_req = 0;
    a.announce = nullptr;
    a.announce_value = 0;
    a.announce_n = 0;
    a.flat_deal = 0;
    constexpr int T = 64;
    if (p->flags & KVD_PLAN_PERSISTENT) {
        for (const ReqHost &r : p->reqs)
            if (r.layer_begin != p->reqs[0].layer_begin || r.layer_end != p->reqs[0].layer_end)
                return fail(KVD_ERR_MISMATCH, "the persistent form needs one layer range for the whole plan");
        const uint32_t layers = p->fold_layers ? (1u << 16)
                                               : (p->reqs[0].layer_begin | ((p->reqs[0].layer_end - p->reqs[0].layer_begin) << 16));
        hipLaunchKernelGGL(kvd_pull_persistent_kernel, dim3((uint32_t)p->num_cus * 2), dim3(1024), 0,
                           (hipStream_t)stream, p->geo, a, p->desc_dev, layers);
    } else {
        if (p->by_descriptor) {
            const uint64_t gx = (uint64_t)p->items_per_desc * (kChunkUnits / T) * a.slabs;
            const uint64_t n = p->txns_total;  // descriptors of a re-layout plan = its transactions
            if (gx >= (1ull << 31) || n > 65535ull * 65535ull) return fail(KVD_ERR_CAPACITY, "too many work items for one launch");
            hipLaunchKernelGGL(kvd_pull_by_descriptor_kernel<T>,
                               dim3((uint32_t)gx, (uint32_t)std::min<uint64_t>(n, 65535), (uint32_t)((n + 65534) / 65535)),
                               dim3(T), 0, (hipStream_t)stream, p->geo, a, p->desc_dev, p->items_per_desc);
            KVD_HIP(hipGetLastError());
            return KVD_OK;
        }
        const uint32_t order = work_order(p);
        if (order != KVD_ORDER_QUEUE) {
            // recorded into a graph, the ordering runs at every replay and the plan still counts
            // as unordered for pulls outside the graph
            const bool capturing = is_capturing(stream);
            if ((p->order_stale || capturing) && !p->sorted_by_build) {
                const uint32_t guard = p->hint.rough ? 1u : 0u;
                hipLaunchKernelGGL(kvd_order_kernel, dim3(1), dim3(kBuildThreads), 0, (hipStream_t)stream, p->items_dev,
                                   p->ordered_dev, p->hdr_dev, p->desc_dev, p->desc_hi_dev, p->order_dev,
                                   order == KVD_ORDER_REGIONS ? 1u : 0u, guard, p->order_shift, p->geo.wide);
                KVD_HIP(hipGetLastError());
                if (order == KVD_ORDER_SORTED) {
                    hipLaunchKernelGGL(kvd_order_copy_kernel, dim3((uint32_t)(p->item_bound / 256 + 1)), dim3(256), 0,
                                       (hipStream_t)stream, p->items_dev, p->ordered_dev, p->hdr_dev, p->order_dev, guard);
                    KVD_HIP(hipGetLastError());
                }
                if (!capturing) p->order_stale = false;
            }
            a.items = p->ordered_dev;
            // sorted lone blocks that take an eighth of the destination pool or more: measured 73.3 against 71.2 %
            // of HBM peak (2048 lone 32 KiB blocks of 16384) and 75.9 against 73.7 % (4096) with the flat deal,
            // 64.7 against 67.2 % for 512 of them
            a.flat_deal = (order == KVD_ORDER_SORTED && !p->hint.rough && p->used_dst * 8 >= p->dst.num_blocks) ? 1u : 0u;
        }
        // sized from the host's pre-merge bound of the item count, rounded up to the 8 XCDs
        const uint64_t gx = (p->item_bound * (kChunkUnits / T) + 7) / 8 * 8;
        if (gx >= (1ull << 31)) return fail(KVD_ERR_CAPACITY, "too many work items for one launch");
        hipLaunchKernelGGL(kvd_pull_kernel<T>, dim3((uint32_t)gx, a.slabs), dim3(T), 0, (hipStream_t)stream,
                           p->geo, a);
    }
    KVD_HIP(hipGetLastError());
    return KVD_OK;
}

// The side streams (default priority) that the per-request pulls take turns on, and the events they
// fork from and join at.
int ensure_notify_streams(kvd_plan *p)
{
    if (p->notify_ready) return KVD_OK;
    KVD_HIP(hipEventCreateWithFlags(&p->notify_fork, hipEventDisableTiming));
    for (int i = 0; i < kNotifyStreams; ++i) {
        KVD_HIP(hipStreamCreateWithFlags(&p->notify_stream[i], hipStreamNonBlocking));
        KVD_HIP(hipEventCreateWithFlags(&p->notify_join[i], hipEventDisableTiming));
    }
    p->notify_ready = true;
    return KVD_OK;
}

// What every launch of the build kernel takes from the plan: where its scratch is, the layer range,
// the sizes of the batch.  The caller adds the batch itself (reqs, first, n_req) and how it joins
// the queue (fresh, may_merge_prev).
BuildArgs build_args(kvd_plan *p, const Geo &g, uint32_t layer_begin, uint32_t n_layers, uint32_t batch_txn,
                     uint32_t batch_items)
{
    BuildArgs a{};
    a.tables_src = p->tables_src_dev;
    a.tables_dst = p->tables_dst_dev;
    a.reqs = nullptr;
    a.desc = p->desc_dev;
    a.desc_hi = p->desc_hi_dev;
    a.items = p->items_dev;
    a.hdr = p->hdr_dev;
    a.n_req = 1;
    a.base_src16 = p->fold_layers ? (uint32_t)(layer_begin * g.src_layer_bytes / kUnitBytes) : 0u;
    a.base_dst16 = p->fold_layers ? (uint32_t)(layer_begin * g.dst_layer_bytes / kUnitBytes) : 0u;
    a.n_txn = batch_txn;
    a.layers = p->fold_layers ? (1u << 16) : (layer_begin | (n_layers << 16));
    a.fresh = 1;
    a.may_merge_prev = 0;
    a.no_coalesce = (p->flags & KVD_PLAN_NO_COALESCE) ? 1u : 0u;
    a.expand_inline = batch_items <= kInlineItems ? 1u : 0u;
    a.done = p->done_dev;
    a.seq = ++p->build_seq;
    a.req_desc = p->req_desc_dev;  // null unless the plan completes request by request
    a.req_item = p->req_item_dev;
    a.req_base = 0;
    a.sort_inline = 0;
    a.ordered = p->ordered_dev;
    return a;
}

// Everything of a plan that follows from the two pools' metadata and the flags: the geometry the
// kernels take, which axes fold into one byte range, capacity bounds.  Allocates nothing and leaves
// the plan's bookkeeping and scratch pointers alone.
int init_plan(kvd_plan *p, const kvd_pool_desc_t &s, uint64_t src_extent, const kvd_pool_desc_t &d, uint64_t dst_extent,
              uint32_t max_requests, uint32_t max_total_blocks, uint32_t flags)
{
    if (!max_requests || !max_total_blocks) return fail(KVD_ERR_INVALID, "zero capacity");
    constexpr uint32_t kKnownFlags = KVD_PLAN_NO_COALESCE | KVD_PLAN_PERSISTENT | KVD_PLAN_WHOLE_BLOCKS | KVD_PLAN_QUEUE_ORDER |
                                     KVD_PLAN_WIDE_OFFSETS | KVD_PLAN_COMPLETE_PER_REQUEST | KVD_PLAN_DESTINATION_ORDER;
    if (flags & ~kKnownFlags) return fail(KVD_ERR_INVALID, "flags 0x%x: unknown bits", flags);
    if ((flags & KVD_PLAN_QUEUE_ORDER) && (flags & KVD_PLAN_DESTINATION_ORDER))
        return fail(KVD_ERR_INVALID, "KVD_PLAN_QUEUE_ORDER and KVD_PLAN_DESTINATION_ORDER exclude each other");
    if (s.num_kv_heads != d.num_kv_heads || s.head_dim != d.head_dim || s.elem_bytes != d.elem_bytes)
        return fail(KVD_ERR_MISMATCH, "pools differ in num_kv_heads, head_dim or elem_bytes");
    const uint32_t tmin = std::min(s.block_tokens, d.block_tokens);
    const uint32_t tmax = std::max(s.block_tokens, d.block_tokens);
    if (tmax % tmin)
        return fail(KVD_ERR_MISMATCH, "block sizes %u and %u: neither divides the other",
                    s.block_tokens, d.block_tokens);
    const uintptr_t sb = (uintptr_t)s.base, db = (uintptr_t)d.base;
    if (sb < db + dst_extent && db < sb + src_extent)
        return fail(KVD_ERR_ALIAS, "source and destination pools overlap");
    p->src = s;
    p->dst = d;
    p->max_requests = max_requests;
    p->max_total_blocks = max_total_blocks;
    p->flags = flags;
    Geo &g = p->geo;
    const uint64_t e = s.elem_bytes;
    g.src_layer_bytes = (uint64_t)s.stride_layer * e;
    g.src_kv_bytes = (uint64_t)s.stride_kv * e;
    g.dst_layer_bytes = (uint64_t)d.stride_layer * e;
    g.dst_kv_bytes = (uint64_t)d.stride_kv * e;
    g.src_block16 = (uint32_t)((uint64_t)s.stride_block * e / kUnitBytes);
    g.dst_block16 = (uint32_t)((uint64_t)d.stride_block * e / kUnitBytes);
    g.tb_src = s.block_tokens;
    g.tb_dst = d.block_tokens;
    g.hk = s.num_kv_heads;
    g.du = (uint32_t)((uint64_t)s.head_dim * e / kUnitBytes);
    g.piece_tokens = tmin;
    g.kv_shift = 1;
    const bool same_inner = s.layout == d.layout || g.hk == 1;
    const bool kv_adjacent = (uint64_t)s.stride_kv == (uint64_t)s.block_tokens * s.num_kv_heads * s.head_dim &&
                             (uint64_t)d.stride_kv == (uint64_t)d.block_tokens * d.num_kv_heads * d.head_dim;
    if (same_inner && kv_adjacent) {
        // K and V of a block are neighbours on both sides: fold K/V into the head axis, so that a
        // block's K and V form one byte range and can merge (section 4.1: contiguity is a matter
        // of offsets).  [kv][head][token][dim] is 2*heads planes; [kv][token][head][dim] is 2
        // planes of (heads*dim)-wide rows.
        if (s.layout == KVD_LAYOUT_BTHD && g.hk > 1) {
            g.du *= g.hk;
            g.hk = 2;
        } else {
            g.hk *= 2;
        }
        g.kv_shift = 0;
        g.mode = kSpanHeadMajor;
    } else if (same_inner) {
        g.mode = (s.layout == KVD_LAYOUT_BTHD || g.hk == 1) ? kSpanTokenMajor : kSpanHeadMajor;
    } else {
        g.mode = (s.layout == KVD_LAYOUT_BHTD) ? kRelayoutHT2TH : kRelayoutTH2HT;
    }
    // layers adjacent too (stride_layer = K + V of one block) and the whole pool within reach of a
    // 32-bit unit offset: a block's layers form one range, in layer order
    p->planes_per_layer = g.hk;
    p->fold_layers = g.kv_shift == 0 &&
                     (uint64_t)s.stride_layer == 2 * (uint64_t)s.stride_kv && (uint64_t)d.stride_layer == 2 * (uint64_t)d.stride_kv &&
                     (uint64_t)g.hk * std::min(s.num_layers, d.num_layers) <= (1u << 20);
    // 32-bit unit offsets reach 64 GiB: enough for one slab of most pools.  A folded plan has one
    // slab, the whole pool; beyond 64 GiB (or when asked to) it carries 48-bit offsets.
    const bool beyond32 = (uint64_t)s.num_blocks * s.stride_block * e >= (1ull << 36) ||
                          (uint64_t)d.num_blocks * d.stride_block * e >= (1ull << 36);
    g.wide = (p->fold_layers && (beyond32 || (flags & KVD_PLAN_WIDE_OFFSETS))) ? 1u : 0u;
    if (!p->fold_layers && (block_axis_bytes(s) >= (1ull << 36) || block_axis_bytes(d) >= (1ull << 36)))
        return fail(KVD_ERR_RANGE, "a block axis that spans more than 64 GiB needs block-major pools with the same inner "
                                   "order on both sides");
    if ((flags & KVD_PLAN_WIDE_OFFSETS) && !p->fold_layers)
        return fail(KVD_ERR_MISMATCH, "48-bit offsets are for block-major pools with the same inner order on both sides");
    if ((flags & KVD_PLAN_PERSISTENT) && g.wide)
        return fail(KVD_ERR_MISMATCH, "the persistent form has 32-bit offsets only");
    const uint32_t hk_max = p->fold_layers ? g.hk * std::min(s.num_layers, d.num_layers) : g.hk;
    g.rows_per_item = g.du <= kChunkUnits ? kChunkUnits / g.du : 0;
    p->by_descriptor = g.mode >= kRelayoutHT2TH && !(flags & (KVD_PLAN_PERSISTENT | KVD_PLAN_QUEUE_ORDER)) &&
                       s.stride_block > s.stride_layer && s.stride_block > s.stride_kv &&
                       d.stride_block > d.stride_layer && d.stride_block > d.stride_kv;
    p->items_per_desc = g.rows_per_item ? ceil_div(tmin * g.hk, g.rows_per_item) : 0;
    if ((flags & KVD_PLAN_WHOLE_BLOCKS) && s.block_tokens != d.block_tokens)
        return fail(KVD_ERR_MISMATCH, "whole-block transfers need equal block sizes");
    g.div_du = make_fastdiv(g.du);
    g.div_hk = make_fastdiv(g.hk);
    g.div_tb_src = make_fastdiv(g.tb_src);
    g.div_tb_dst = make_fastdiv(g.tb_dst);

    // upper bounds of what the plan can hold: read transactions and work items (in 128 bits: the
    // products of caller-chosen capacities do not fit 64 for absurd arguments, which must be refused)
    typedef unsigned __int128 u128;
    const u128 pieces_max = (u128)max_total_blocks * (tmax / tmin);
    u128 max_txns = pieces_max;
    if (g.mode == kSpanHeadMajor)
        max_txns = (g.tb_src == g.tb_dst) ? pieces_max + (u128)max_requests * hk_max : pieces_max * hk_max;
    u128 max_items;
    if (g.mode >= kRelayoutHT2TH)
        max_items = pieces_max * tmin * g.hk / g.rows_per_item + max_txns + 1;
    else
        max_items = pieces_max * tmin * hk_max * g.du / kChunkUnits + max_txns + 1;
    if (max_items >= ((u128)1 << 31) || max_txns >= ((u128)1 << 31)) return fail(KVD_ERR_CAPACITY, "plan capacity too large");
    p->max_txns = (uint64_t)max_txns;
    p->max_items = (uint64_t)max_items;
    // destination regions for kvd_order_kernel: 2 MiB, or wider if the slab's block axis would
    // need more buckets than the kernel keeps
    const uint64_t dst_span16 = ((uint64_t)(d.num_blocks - 1) * d.stride_block +
                                 (uint64_t)d.block_tokens * d.num_kv_heads * d.head_dim) * e / kUnitBytes;
    p->order_shift = 17;
    while ((dst_span16 >> p->order_shift) >= kOrderBuckets) ++p->order_shift;
    p->order_stale = true;
    return KVD_OK;
}

// ------------------------------------------------------------------ the entry point that allocates nothing
//
// kvd_pull_noalloc serves callers that cannot allocate device memory.  What a plan keeps in
// hipMalloc / hipHostMalloc memory - the block tables, descriptors, work items, their region-ordered
// copy, the header - lives here in one array that is part of the code object, carved up at fixed
// offsets.  Every GPU the library is used on holds its own copy at its own address until the
// process ends; the name below is a host-side stand-in for it, so host code only ever uses the
// address hipGetSymbolAddress returns for the current device.
constexpr uint32_t kNaMaxBlocks = KVD_NOALLOC_MAX_BLOCKS;  // block-table entries per side
constexpr uint32_t kNaMaxTxns = 1u << 17;                  // read transactions before merging
constexpr uint32_t kNaMaxItems = KVD_NOALLOC_MAX_WORK_ITEMS;
constexpr size_t kNaOffTablesSrc = 0;
constexpr size_t kNaOffTablesDst = kNaOffTablesSrc + (size_t)kNaMaxBlocks * sizeof(int32_t);
constexpr size_t kNaOffHeader = kNaOffTablesDst + (size_t)kNaMaxBlocks * sizeof(int32_t);  // header, then the build's "done" word
constexpr size_t kNaOffDesc = kNaOffHeader + 256;
constexpr size_t kNaOffDescHi = kNaOffDesc + (size_t)kNaMaxTxns * sizeof(Desc);
constexpr size_t kNaOffItems = kNaOffDescHi + (size_t)kNaMaxTxns * sizeof(uint32_t);
constexpr size_t kNaOffOrdered = kNaOffItems + (size_t)kNaMaxItems * sizeof(Item);
constexpr size_t kNaOffOrder = kNaOffOrdered + (size_t)kNaMaxItems * sizeof(Item);
constexpr size_t kNaScratchBytes = kNaOffOrder + (size_t)kNaMaxTxns * sizeof(OrderEntry);
static_assert(kNaOffDesc % 256 == 0 && kNaOffDescHi % 256 == 0 && kNaOffItems % 256 == 0 && kNaOffOrdered % 256 == 0 &&
                  kNaOffOrder % 256 == 0,
              "every part of the scratch array starts on a 256-byte boundary");
static_assert(sizeof(Header) + sizeof(uint32_t) <= 128, "header and done word share the 256 bytes at kNaOffHeader");

}  // namespace

static __device__ __align__(256) unsigned char scratch[kNaScratchBytes];

namespace {

constexpr int kNaMaxDevices = 64;

// Per device: the address of that device's copy of the array.  Set up at the first call on the device.
struct NoAllocDevice {
    bool ready;
    unsigned char *ptr;
    int num_cus;
};
NoAllocDevice g_na[kNaMaxDevices];
std::mutex g_na_setup;
thread_local int32_t g_na_sorted[kNaMaxBlocks];  // host work space of the duplicate check

int noalloc_device(NoAllocDevice **out)
{
    int dev = 0;
    KVD_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kNaMaxDevices) return fail(KVD_ERR_INVALID, "device %d: only devices below %d are supported", dev, kNaMaxDevices);
    NoAllocDevice &nd = g_na[dev];
    std::lock_guard<std::mutex> lock(g_na_setup);
    if (!nd.ready) {
        unsigned char *ptr = nullptr;
        KVD_HIP(hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || ((uintptr_t)ptr % 256)) return fail(KVD_ERR_HIP, "the scratch array has no usable address on device %d", dev);
        hipDeviceProp_t prop;
        KVD_HIP(hipGetDeviceProperties(&prop, dev));
        nd.ptr = ptr;
        nd.num_cus = prop.multiProcessorCount;
        nd.ready = true;
    }
    *out = &nd;
    return KVD_OK;
}

}  // namespace

extern "C" {

const char *kvd_last_error(void) { return g_err; }

int kvd_pool_create(const kvd_pool_desc_t *desc, kvd_pool_t **out)
{
    if (!desc || !out) return fail(KVD_ERR_INVALID, "null argument");
    *out = nullptr;
    uint64_t extent = 0;
    int rc = check_pool_desc(*desc, &extent);
    if (rc != KVD_OK) return rc;
    kvd_pool *p = new (std::nothrow) kvd_pool;
    if (!p) return fail(KVD_ERR_INVALID, "out of host memory");
    p->tag = kPoolTag;
    p->d = *desc;
    p->extent_bytes = extent;
    try {
        register_handle(p);
    } catch (const std::exception &) {
        delete p;
        return fail(KVD_ERR_CAPACITY, "out of host memory");
    }
    *out = p;
    return KVD_OK;
}

int kvd_plan_create(const kvd_pool_t *src, const kvd_pool_t *dst, uint32_t max_requests,
                    uint32_t max_total_blocks, uint32_t flags, kvd_plan_t **out)
{
    if (!src || !dst || !out) return fail(KVD_ERR_INVALID, "null argument");
    *out = nullptr;
    if (!as_pool(src) || !as_pool(dst)) return fail(KVD_ERR_INVALID, "not a pool handle");
    kvd_plan *p = new (std::nothrow) kvd_plan();
    if (!p) return fail(KVD_ERR_INVALID, "out of host memory");
    const int rc = init_plan(p, src->d, src->extent_bytes, dst->d, dst->extent_bytes, max_requests, max_total_blocks, flags);
    if (rc != KVD_OK) {
        delete p;
        return rc;
    }
    p->tag = kPlanTag;
    try {  // no exception may cross this boundary: a pool or a capacity too large for the host is a refusal
        p->dst_used.assign(dst->d.num_blocks, 0);
        p->reqs.reserve(std::min<uint32_t>(max_requests, 4096));
        register_handle(p);
    } catch (const std::exception &) {
        delete p;
        return fail(KVD_ERR_CAPACITY, "out of host memory for a plan of %u requests over a pool of %u blocks", max_requests,
                    dst->d.num_blocks);
    }
    p->allocated = false;
    *out = p;
    return KVD_OK;
}

int kvd_plan_reset(kvd_plan_t *p)
{
    if (!as_plan(p)) return fail(KVD_ERR_INVALID, "not a plan handle");
    const int rc = wait_for_builds(p);
    if (rc != KVD_OK) return rc;
    for (const ReqHost &r : p->reqs)
        for (uint32_t i = 0; i < r.n_dst; ++i)
            p->dst_used[(uint32_t)p->tables_dst[r.table_off_dst + i]] = 0;
    p->reqs.clear();
    p->used_src = p->used_dst = p->txns_total = p->item_bound = p->payload_bytes = 0;
    p->hint = OrderHint{};
    p->max_layers = 0;
    p->sorted_by_build = false;
    p->order_stale = true;
    return KVD_OK;
}

int kvd_build_descriptors_batch(kvd_plan_t *p, uint32_t n_requests, const int32_t *const *src_tbls,
                                const uint32_t *n_src, const int32_t *const *dst_tbls, const uint32_t *n_dst,
                                const uint32_t *seq_lens, uint32_t layer_begin, uint32_t layer_end, void *stream)
{
    if (!as_plan(p)) return fail(KVD_ERR_INVALID, "not a plan handle");
    if (layer_begin >= layer_end) return fail(KVD_ERR_INVALID, "empty layer range [%u, %u)", layer_begin, layer_end);
    if (layer_end > p->src.num_layers || layer_end > p->dst.num_layers)
        return fail(KVD_ERR_RANGE, "layer range [%u, %u) outside a pool", layer_begin, layer_end);
    if (n_requests == 0) return KVD_OK;
    if (!src_tbls || !dst_tbls || !n_src || !n_dst || !seq_lens) return fail(KVD_ERR_INVALID, "null argument");
    // the host part of a build (checks, table copies, the wait for the kernel's completion word)
    // happens now, so its kernel cannot be deferred to a graph replay
    if (is_capturing(stream)) return fail(KVD_ERR_INVALID, "kvd_build_descriptors cannot be recorded into a HIP graph");
    // with the layers folded into the block, this call's layer range sets how many planes a block has
    const uint32_t n_layers = layer_end - layer_begin;
    Geo folded = p->geo;
    if (p->fold_layers) {
        folded.hk = p->planes_per_layer * n_layers;
        folded.div_hk = make_fastdiv(folded.hk);
    }
    const Geo &g = folded;
    const uint32_t slab_layers = p->fold_layers ? 1u : n_layers;  // layers left for the pull kernel to step through

    // whole-block mode moves every slot of the last block too (the block-granular transfer of
    // section 4.1); block sizes are equal then
    const bool whole = (p->flags & KVD_PLAN_WHOLE_BLOCKS) != 0;
    auto effective_len = [&](uint32_t seq_len) { return whole ? ceil_div(seq_len, g.tb_src) * g.tb_src : seq_len; };

    // 1. everything that can be checked without touching the plan
    uint64_t add_src = 0, add_dst = 0, add_txn = 0, add_items = 0, add_reqs = 0;
    for (uint32_t k = 0; k < n_requests; ++k) {
        if (seq_lens[k] > (1u << 30)) return fail(KVD_ERR_RANGE, "request %u: seq_len %u above 2^30", k, seq_lens[k]);
        const uint32_t seq_len = effective_len(seq_lens[k]);
        if (seq_len == 0) continue;
        const int32_t *st = src_tbls[k], *dt = dst_tbls[k];
        if (!st || !dt) return fail(KVD_ERR_INVALID, "request %u: null block table", k);
        const uint32_t need_src = ceil_div(seq_len, g.tb_src), need_dst = ceil_div(seq_len, g.tb_dst);
        if (n_src[k] < need_src || n_dst[k] < need_dst)
            return fail(KVD_ERR_RANGE, "request %u: block table too short for %u tokens (source %u of %u, destination %u of %u)",
                        k, seq_len, n_src[k], need_src, n_dst[k], need_dst);
        for (uint32_t i = 0; i < need_src; ++i)
            if (st[i] < 0 || (uint32_t)st[i] >= p->src.num_blocks)
                return fail(KVD_ERR_RANGE, "request %u: source block id %d at entry %u outside [0, %u)", k, st[i], i, p->src.num_blocks);
        for (uint32_t i = 0; i < need_dst; ++i)
            if (dt[i] < 0 || (uint32_t)dt[i] >= p->dst.num_blocks)
                return fail(KVD_ERR_RANGE, "request %u: destination block id %d at entry %u outside [0, %u)", k, dt[i], i, p->dst.num_blocks);
        uint32_t n_txn = 0, items = 0;
        request_sizes(g, seq_len, &n_txn, &items);
        add_src += need_src;
        add_dst += need_dst;
        add_txn += n_txn;
        add_items += items;
        ++add_reqs;
    }
    if (add_reqs == 0) return KVD_OK;
    if (p->reqs.size() + add_reqs > p->max_requests)
        return fail(KVD_ERR_CAPACITY, "plan holds at most %u requests", p->max_requests);
    if (p->used_src + add_src > p->max_total_blocks || p->used_dst + add_dst > p->max_total_blocks ||
        p->txns_total + add_txn > p->max_txns || p->item_bound + add_items > p->max_items)
        return fail(KVD_ERR_CAPACITY, "plan holds at most %u block-table entries per side", p->max_total_blocks);

    // 2. every destination byte is written at most once per plan: 2 marks this call's blocks
    //    until the call is sure to succeed, 1 marks blocks of accepted requests
    auto unmark_call = [&](uint32_t upto_req, uint32_t upto_entry) {
        for (uint32_t k = 0; k <= upto_req && k < n_requests; ++k) {
            if (seq_lens[k] == 0) continue;
            const uint32_t need = (k == upto_req) ? upto_entry : ceil_div(seq_lens[k], g.tb_dst);
            for (uint32_t i = 0; i < need; ++i)
                if (p->dst_used[(uint32_t)dst_tbls[k][i]] == 2) p->dst_used[(uint32_t)dst_tbls[k][i]] = 0;
        }
    };
    for (uint32_t k = 0; k < n_requests; ++k) {
        if (seq_lens[k] == 0) continue;
        const uint32_t need_dst = ceil_div(seq_lens[k], g.tb_dst);
        for (uint32_t i = 0; i < need_dst; ++i) {
            uint8_t &u = p->dst_used[(uint32_t)dst_tbls[k][i]];
            if (u) {
                unmark_call(k, i);
                return fail(KVD_ERR_ALIAS, "request %u: destination block %d (entry %u) is already a target in this plan",
                            k, dst_tbls[k][i], i);
            }
            u = 2;
        }
    }
    int rc = ensure_allocated(p);
    // Build kernels report through one word, in launch order.  Kernels on two streams could finish
    // in the other order and leave the older number in it, so a build on another stream than the
    // last one first waits until that one has reported.
    if (rc == KVD_OK && p->build_seq > 0 && (hipStream_t)stream != p->build_stream) rc = wait_for_builds(p);
    if (rc != KVD_OK) {
        unmark_call(n_requests, 0);
        return rc;
    }

    // 3. commit on the host, then one launch per kMaxBatch requests
    try {  // room for this call's requests first, so that nothing below can throw half-way
        p->reqs.reserve(p->reqs.size() + add_reqs);
    } catch (const std::exception &) {
        unmark_call(n_requests, 0);
        return fail(KVD_ERR_CAPACITY, "out of host memory");
    }
    const size_t first_new = p->reqs.size();
    const bool same_layers = first_new > 0 && p->reqs.back().layer_begin == layer_begin &&
                             p->reqs.back().layer_end == layer_end;
    for (uint32_t k = 0; k < n_requests; ++k) {
        const uint32_t seq_len = effective_len(seq_lens[k]);
        if (seq_len == 0) continue;
        ReqHost r;
        r.table_off_src = (uint32_t)p->used_src;
        r.table_off_dst = (uint32_t)p->used_dst;
        r.n_src = ceil_div(seq_len, g.tb_src);
        r.n_dst = ceil_div(seq_len, g.tb_dst);
        r.seq_len = seq_len;
        r.layer_begin = layer_begin;
        r.layer_end = layer_end;
        r.item_bound = 0;
        memcpy(p->tables_src + r.table_off_src, src_tbls[k], (size_t)r.n_src * sizeof(int32_t));
        memcpy(p->tables_dst + r.table_off_dst, dst_tbls[k], (size_t)r.n_dst * sizeof(int32_t));
        for (uint32_t i = 0; i < r.n_dst; ++i) p->dst_used[(uint32_t)dst_tbls[k][i]] = 1;
        p->used_src += r.n_src;
        p->used_dst += r.n_dst;
        p->payload_bytes += ((uint64_t)seq_len * slab_layers * g.hk * g.du * kUnitBytes) << g.kv_shift;
        uint32_t n_txn = 0, items = 0;
        request_sizes(g, seq_len, &n_txn, &items);
        if (!p->reqs.empty()) {
            const ReqHost &prev = p->reqs.back();
            if (src_tbls[k][0] < p->tables_src[prev.table_off_src + prev.n_src - 1]) ++p->hint.src_descents;
            if (dst_tbls[k][0] < p->tables_dst[prev.table_off_dst + prev.n_dst - 1]) ++p->hint.dst_descents;
        }
        add_order_hint(&p->hint, g, src_tbls[k], dst_tbls[k], seq_len, n_txn, items);
        p->reqs.push_back(r);
    }
    p->max_layers = std::max(p->max_layers, slab_layers);
    for (size_t b0 = first_new; b0 < p->reqs.size(); b0 += kMaxBatch) {
        const uint32_t nb = (uint32_t)std::min<size_t>(kMaxBatch, p->reqs.size() - b0);
        uint32_t batch_txn = 0, batch_items = 0;
        for (uint32_t i = 0; i < nb; ++i) {
            const ReqHost &r = p->reqs[b0 + i];
            uint32_t n_txn = 0, items = 0;
            request_sizes(g, r.seq_len, &n_txn, &items);
            p->reqs[b0 + i].item_bound = items;
            p->reqs_pinned[b0 + i] = ReqDev{r.table_off_src, r.table_off_dst, r.seq_len, batch_txn};
            batch_txn += n_txn;
            batch_items += items;
        }
        BuildArgs a = build_args(p, g, layer_begin, n_layers, batch_txn, batch_items);
        a.reqs = p->reqs_pinned_dev + b0;
        a.first = p->reqs_pinned[b0];
        a.n_req = nb;
        a.fresh = (b0 == 0) ? 1u : 0u;
        a.may_merge_prev = ((b0 > first_new || same_layers) && !(p->flags & KVD_PLAN_COMPLETE_PER_REQUEST)) ? 1u : 0u;
        a.req_base = (uint32_t)b0;
        p->sorted_by_build = build_sorts(p, b0 == 0 && nb == p->reqs.size(), batch_txn, batch_items);
        a.sort_inline = p->sorted_by_build ? 1u : 0u;
        p->build_stream = (hipStream_t)stream;
        hipLaunchKernelGGL(kvd_build_kernel, dim3(1), dim3(kBuildThreads), 0, (hipStream_t)stream, g, a);
        hipError_t launch = hipGetLastError();
        if (launch == hipSuccess && !a.expand_inline) {
            hipLaunchKernelGGL(kvd_expand_kernel, dim3(batch_items / 256 + 1), dim3(256), 0, (hipStream_t)stream, g,
                               p->desc_dev, p->desc_hi_dev, p->items_dev, p->hdr_dev, a.layers);
            launch = hipGetLastError();
        }
        if (launch != hipSuccess) {
            // the plan's device state no longer matches the host's: let what was queued before
            // finish, then drop everything (no kernel will report this sequence number)
            (void)hipStreamSynchronize((hipStream_t)stream);
            *p->done_host = p->build_seq;
            (void)kvd_plan_reset(p);
            return fail(KVD_ERR_HIP, "launch of the build kernel failed (plan was reset): %s", hipGetErrorString(launch));
        }
        p->order_stale = !p->sorted_by_build;
        p->txns_total += batch_txn;
        p->item_bound += batch_items;
    }
    return KVD_OK;
}

int kvd_build_descriptors(kvd_plan_t *p, const int32_t *src_tbl, uint32_t n_src,
                          const int32_t *dst_tbl, uint32_t n_dst, uint32_t seq_len,
                          uint32_t layer_begin, uint32_t layer_end, void *stream)
{
    return kvd_build_descriptors_batch(p, 1, &src_tbl, &n_src, &dst_tbl, &n_dst, &seq_len, layer_begin,
                                       layer_end, stream);
}

int kvd_pull(kvd_plan_t *p, void *stream)
{
    if (!as_plan(p)) return fail(KVD_ERR_INVALID, "not a plan handle");
    if (p->reqs.empty()) return KVD_OK;
    return launch_pull(p, stream, true, 0, 0);
}

int kvd_pull_layers(kvd_plan_t *p, uint32_t layer_begin, uint32_t layer_end, void *stream)
{
    if (!as_plan(p)) return fail(KVD_ERR_INVALID, "not a plan handle");
    if (layer_begin >= layer_end) return fail(KVD_ERR_INVALID, "empty layer range [%u, %u)", layer_begin, layer_end);
    if (layer_end > p->src.num_layers || layer_end > p->dst.num_layers)
        return fail(KVD_ERR_RANGE, "layer range [%u, %u) outside a pool", layer_begin, layer_end);
    if (p->fold_layers)
        return fail(KVD_ERR_MISMATCH, "plans over block-major pools move a block's layers as one range; build one plan "
                                      "per layer range instead");
    if (p->flags & KVD_PLAN_PERSISTENT) return fail(KVD_ERR_MISMATCH, "the persistent form moves whole plans only");
    if (p->reqs.empty()) return KVD_OK;
    return launch_pull(p, stream, false, layer_begin, layer_end);
}

int kvd_pull_notify(kvd_plan_t *p, uint64_t *words, uint64_t value, void *stream)
{
    if (!as_plan(p)) return fail(KVD_ERR_INVALID, "not a plan handle");
    if (!(p->flags & KVD_PLAN_COMPLETE_PER_REQUEST))
        return fail(KVD_ERR_MISMATCH, "the plan was not created with KVD_PLAN_COMPLETE_PER_REQUEST");
    if (p->by_descriptor || (p->flags & KVD_PLAN_PERSISTENT))
        return fail(KVD_ERR_MISMATCH, "per-request completion is not available for this kind of plan");
    if (p->reqs.empty()) return KVD_OK;
    if (!words) return fail(KVD_ERR_INVALID, "null completion words");
    if ((uintptr_t)words % 8) return fail(KVD_ERR_INVALID, "completion words must be 8-byte aligned");
    hipPointerAttribute_t at;
    if (hipPointerGetAttributes(&at, words) != hipSuccess) {
        (void)hipGetLastError();
        return fail(KVD_ERR_INVALID, "the completion words are not memory the GPU can reach (device memory or pinned host memory)");
    }
    if (!at.devicePointer) return fail(KVD_ERR_INVALID, "the completion words are host memory that is not mapped into the device");
    uint64_t *words_dev = (uint64_t *)at.devicePointer;
    int rc = ensure_notify_streams(p);
    if (rc != KVD_OK) return rc;

    // A group of requests' reads runs as one launch - one request per group unless the plan was given a
    // completion granularity; consecutive groups alternate between two side streams, so the next
    // group's reads are in flight while this one's last workgroups drain (section 4.2: reads of other
    // requests do not wait for a completion).  Stream order makes a group's launch complete before the
    // next launch on its side stream begins, and that launch's first workgroup stores the group's
    // words.  The side streams start behind everything enqueued on `stream` so far, and `stream`
    // continues behind both.
    constexpr int T = 64;
    const uint32_t n_req = (uint32_t)p->reqs.size();
    struct Group { uint32_t begin, end; uint64_t item_bound; };
    // where the group that starts at request k ends: requests are added while the group is below
    // the granularity and the next request moves the same layers (a launch has one number of slabs)
    auto group_at = [&](uint32_t k) {
        Group g{k, k + 1, p->reqs[k].item_bound};
        uint64_t tokens = p->reqs[k].seq_len;
        while (g.end < n_req && tokens < p->notify_min_tokens && p->reqs[g.end].layer_begin == p->reqs[k].layer_begin &&
               p->reqs[g.end].layer_end == p->reqs[k].layer_end) {
            tokens += p->reqs[g.end].seq_len;
            g.item_bound += p->reqs[g.end].item_bound;
            ++g.end;
        }
        return g;
    };
    for (uint32_t k = 0; k < n_req; k = group_at(k).end)
        if ((group_at(k).item_bound * (kChunkUnits / T) + 7) / 8 * 8 >= (1ull << 31))
            return fail(KVD_ERR_CAPACITY, "too many work items for one launch");
    hipStream_t st = (hipStream_t)stream;
    KVD_HIP(hipEventRecord(p->notify_fork, st));
    for (int i = 0; i < kNotifyStreams; ++i) KVD_HIP(hipStreamWaitEvent(p->notify_stream[i], p->notify_fork, 0));
    hipError_t launch = hipSuccess;
    Group before[kNotifyStreams] = {};  // the group that ran last on each side stream (empty: none yet)
    uint32_t turn = 0;
    for (uint32_t k = 0; k < n_req && launch == hipSuccess; ++turn) {
        const Group g = group_at(k);
        const ReqHost &r = p->reqs[k];
        const int side_i = (int)(turn % kNotifyStreams);
        hipStream_t side = p->notify_stream[side_i];
        PullArgs a{};
        a.src_base = (const unsigned char *)p->src.base;
        a.dst_base = (unsigned char *)p->dst.base;
        a.items = p->items_dev;  // queue order: a group's work items are one range of the table
        a.hdr = p->hdr_dev;
        a.slabs = (p->fold_layers ? 1u : r.layer_end - r.layer_begin) << p->geo.kv_shift;
        a.absolute_layers = 0;
        a.layer0 = 0;
        a.req_item = p->req_item_dev;
        a.req = g.begin;
        a.req_end = g.end;
        a.n_req = n_req;
        // the words of the group that ran on this side stream before this one are stored by this
        // launch's first workgroup; the last group of each side stream gets a launch for its words
        const Group &b = before[side_i];
        a.announce = b.end > b.begin ? words_dev + b.begin : nullptr;
        a.announce_n = b.end - b.begin;
        a.announce_value = value;
        const uint64_t gx = (g.item_bound * (kChunkUnits / T) + 7) / 8 * 8;
        hipLaunchKernelGGL(kvd_pull_kernel<T>, dim3((uint32_t)gx, a.slabs), dim3(T), 0, side, p->geo, a);
        launch = hipGetLastError();
        before[side_i] = g;
        k = g.end;
    }
    for (int i = 0; i < kNotifyStreams && launch == hipSuccess; ++i) {
        const Group &b = before[i];
        if (b.end == b.begin) continue;
        hipLaunchKernelGGL(kvd_complete_kernel, dim3(1), dim3(64), 0, p->notify_stream[i], words_dev + b.begin, b.end - b.begin, value);
        launch = hipGetLastError();
    }
    // also after a failed launch: whatever did reach the side streams stays ordered before `stream`
    for (int i = 0; i < kNotifyStreams; ++i) {
        KVD_HIP(hipEventRecord(p->notify_join[i], p->notify_stream[i]));
        KVD_HIP(hipStreamWaitEvent(st, p->notify_join[i], 0));
    }
    if (launch != hipSuccess)
        return fail(KVD_ERR_HIP, "launch of a per-request pull failed (some requests were not moved): %s", hipGetErrorString(launch));
    return KVD_OK;
}

int kvd_plan_set_completion_granularity(kvd_plan_t *p, uint32_t min_tokens)
{
    if (!as_plan(p)) return fail(KVD_ERR_INVALID, "not a plan handle");
    if (!(p->flags & KVD_PLAN_COMPLETE_PER_REQUEST))
        return fail(KVD_ERR_MISMATCH, "the plan was not created with KVD_PLAN_COMPLETE_PER_REQUEST");
    p->notify_min_tokens = min_tokens;
    return KVD_OK;
}

int kvd_pull_noalloc(const kvd_pool_desc_t *src, const kvd_pool_desc_t *dst, const int32_t *src_tbl, uint32_t n_src,
                     const int32_t *dst_tbl, uint32_t n_dst, uint32_t seq_len, uint32_t layer_begin,
                     uint32_t layer_end, uint32_t flags, void *stream)
{
    if (!src || !dst) return fail(KVD_ERR_INVALID, "null argument");
    if (flags & ~(uint32_t)(KVD_PLAN_NO_COALESCE | KVD_PLAN_WHOLE_BLOCKS | KVD_PLAN_QUEUE_ORDER | KVD_PLAN_DESTINATION_ORDER))
        return fail(KVD_ERR_INVALID, "flags 0x%x: only KVD_PLAN_NO_COALESCE, KVD_PLAN_WHOLE_BLOCKS, KVD_PLAN_QUEUE_ORDER and "
                                     "KVD_PLAN_DESTINATION_ORDER apply here", flags);
    uint64_t src_extent = 0, dst_extent = 0;
    int rc = check_pool_desc(*src, &src_extent);
    if (rc != KVD_OK) return rc;
    rc = check_pool_desc(*dst, &dst_extent);
    if (rc != KVD_OK) return rc;
    // a plan for this one call; it lives on the stack and its scratch pointers will point into the array
    kvd_plan plan{};
    kvd_plan *const p = &plan;
    rc = init_plan(p, *src, src_extent, *dst, dst_extent, 1, kNaMaxBlocks, flags);
    if (rc != KVD_OK) return rc;
    p->max_txns = kNaMaxTxns;  // what the array holds, not what the block count could need
    p->max_items = kNaMaxItems;
    if (layer_begin >= layer_end) return fail(KVD_ERR_INVALID, "empty layer range [%u, %u)", layer_begin, layer_end);
    if (layer_end > src->num_layers || layer_end > dst->num_layers)
        return fail(KVD_ERR_RANGE, "layer range [%u, %u) outside a pool", layer_begin, layer_end);
    if (seq_len > (1u << 30)) return fail(KVD_ERR_RANGE, "seq_len %u above 2^30", seq_len);
    if (seq_len == 0) return KVD_OK;
    if (!src_tbl || !dst_tbl) return fail(KVD_ERR_INVALID, "null block table");

    const uint32_t n_layers = layer_end - layer_begin;
    Geo g = p->geo;
    if (p->fold_layers) {  // block-major pools: this call's layers become planes of the block
        g.hk = p->planes_per_layer * n_layers;
        g.div_hk = make_fastdiv(g.hk);
    }
    const uint32_t slab_layers = p->fold_layers ? 1u : n_layers;
    const uint32_t len = (flags & KVD_PLAN_WHOLE_BLOCKS) ? ceil_div(seq_len, g.tb_src) * g.tb_src : seq_len;
    const uint32_t need_src = ceil_div(len, g.tb_src), need_dst = ceil_div(len, g.tb_dst);
    if (need_src > kNaMaxBlocks || need_dst > kNaMaxBlocks)
        return fail(KVD_ERR_CAPACITY, "%u tokens need %u source and %u destination blocks; this entry point takes at most %u per side",
                    len, need_src, need_dst, kNaMaxBlocks);
    if (n_src < need_src || n_dst < need_dst)
        return fail(KVD_ERR_RANGE, "block table too short for %u tokens (source %u of %u, destination %u of %u)", len, n_src,
                    need_src, n_dst, need_dst);
    uint32_t n_txn = 0, items = 0;
    request_sizes(g, len, &n_txn, &items);
    if (n_txn > kNaMaxTxns || items > kNaMaxItems)
        return fail(KVD_ERR_CAPACITY, "the request needs %u read transactions and %u work items; this entry point takes at most %u and %u",
                    n_txn, items, kNaMaxTxns, kNaMaxItems);
    for (uint32_t i = 0; i < need_src; ++i)
        if (src_tbl[i] < 0 || (uint32_t)src_tbl[i] >= src->num_blocks)
            return fail(KVD_ERR_RANGE, "source block id %d at entry %u outside [0, %u)", src_tbl[i], i, src->num_blocks);
    for (uint32_t i = 0; i < need_dst; ++i)
        if (dst_tbl[i] < 0 || (uint32_t)dst_tbl[i] >= dst->num_blocks)
            return fail(KVD_ERR_RANGE, "destination block id %d at entry %u outside [0, %u)", dst_tbl[i], i, dst->num_blocks);
    // every destination byte is written at most once: no destination block twice
    std::copy(dst_tbl, dst_tbl + need_dst, g_na_sorted);
    std::sort(g_na_sorted, g_na_sorted + need_dst);
    for (uint32_t i = 1; i < need_dst; ++i)
        if (g_na_sorted[i] == g_na_sorted[i - 1])
            return fail(KVD_ERR_ALIAS, "destination block %d appears twice in the table", g_na_sorted[i]);

    NoAllocDevice *nd = nullptr;
    rc = noalloc_device(&nd);
    if (rc != KVD_OK) return rc;
    unsigned char *const ptr = nd->ptr;  // this device's copy of the array
    p->num_cus = nd->num_cus;
    p->tables_src_dev = (int32_t *)(ptr + kNaOffTablesSrc);
    p->tables_dst_dev = (int32_t *)(ptr + kNaOffTablesDst);
    p->hdr_dev = (Header *)(ptr + kNaOffHeader);
    p->done_dev = (uint32_t *)(ptr + kNaOffHeader + 128);  // nobody waits for it: the tables were passed by value
    p->desc_dev = (Desc *)(ptr + kNaOffDesc);
    p->desc_hi_dev = (uint32_t *)(ptr + kNaOffDescHi);
    p->items_dev = (Item *)(ptr + kNaOffItems);
    p->ordered_dev = (Item *)(ptr + kNaOffOrdered);
    p->order_dev = (OrderEntry *)(ptr + kNaOffOrder);
    // the host's bookkeeping of a plan that holds this one request
    p->txns_total = n_txn;
    p->item_bound = items;
    add_order_hint(&p->hint, g, src_tbl, dst_tbl, len, n_txn, items);
    p->payload_bytes = ((uint64_t)len * slab_layers * g.hk * g.du * kUnitBytes) << g.kv_shift;
    p->max_layers = slab_layers;
    p->order_stale = true;

    // the tables, a piece at a time through the kernel's arguments, into the array
    hipStream_t st = (hipStream_t)stream;
    for (uint32_t off = 0; off < std::max(need_src, need_dst); off += kArgTableEntries) {
        TableChunk c{};
        const uint32_t ns = off < need_src ? std::min(kArgTableEntries, need_src - off) : 0u;
        const uint32_t nt = off < need_dst ? std::min(kArgTableEntries, need_dst - off) : 0u;
        if (ns) memcpy(c.src, src_tbl + off, (size_t)ns * sizeof(int32_t));
        if (nt) memcpy(c.dst, dst_tbl + off, (size_t)nt * sizeof(int32_t));
        hipLaunchKernelGGL(kvd_stage_tables_kernel, dim3(1), dim3(kArgTableEntries), 0, st, c, p->tables_src_dev + off, ns,
                           p->tables_dst_dev + off, nt);
        KVD_HIP(hipGetLastError());
    }
    BuildArgs a = build_args(p, g, layer_begin, n_layers, n_txn, items);
    a.first = ReqDev{0, 0, len, 0};
    p->sorted_by_build = build_sorts(p, true, n_txn, items);
    a.sort_inline = p->sorted_by_build ? 1u : 0u;
    p->order_stale = !p->sorted_by_build;
    hipLaunchKernelGGL(kvd_build_kernel, dim3(1), dim3(kBuildThreads), 0, st, g, a);
    KVD_HIP(hipGetLastError());
    if (!a.expand_inline) {
        hipLaunchKernelGGL(kvd_expand_kernel, dim3(items / 256 + 1), dim3(256), 0, st, g, p->desc_dev, p->desc_hi_dev,
                           p->items_dev, p->hdr_dev, a.layers);
        KVD_HIP(hipGetLastError());
    }
    return launch_pull(p, stream, true, 0, 0);
}

int kvd_complete(uint64_t *flag, uint64_t value, void *stream)
{
    if (!flag) return fail(KVD_ERR_INVALID, "null flag");
    if ((uintptr_t)flag % 8) return fail(KVD_ERR_INVALID, "flag must be 8-byte aligned");
    // the kernel must be able to reach the word: device memory, or pinned host memory that is mapped
    hipPointerAttribute_t at;
    if (hipPointerGetAttributes(&at, flag) != hipSuccess) {
        (void)hipGetLastError();
        return fail(KVD_ERR_INVALID, "flag is not memory the GPU can reach (device memory or pinned host memory)");
    }
    if (!at.devicePointer) return fail(KVD_ERR_INVALID, "flag is host memory that is not mapped into the device");
    hipLaunchKernelGGL(kvd_complete_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, (uint64_t *)at.devicePointer, 1u, value);
    KVD_HIP(hipGetLastError());
    return KVD_OK;
}

int kvd_pull_staged(kvd_plan_t *p, void *send_buffer, void *recv_buffer, uint64_t buffer_bytes, void *stream)
{
    if (!as_plan(p)) return fail(KVD_ERR_INVALID, "not a plan handle");
    if (!send_buffer || !recv_buffer) return fail(KVD_ERR_INVALID, "null buffer");
    if (buffer_bytes < 4096 || ((uintptr_t)send_buffer % 16) || ((uintptr_t)recv_buffer % 16))
        return fail(KVD_ERR_INVALID, "buffers must hold at least 4096 bytes and be 16-byte aligned");
    if (p->reqs.empty()) return KVD_OK;
    hipStream_t st = (hipStream_t)stream;
    KVD_HIP(hipStreamSynchronize(st));
    Header h;
    KVD_HIP(hipMemcpy(&h, p->hdr_dev, sizeof(h), hipMemcpyDeviceToHost));
    PullArgs a{};
    a.src_base = (const unsigned char *)p->src.base;
    a.dst_base = (unsigned char *)p->dst.base;
    a.items = p->items_dev;
    a.hdr = p->hdr_dev;
    a.slabs = p->max_layers << p->geo.kv_shift;
    a.absolute_layers = 0;
    a.layer0 = 0;
    a.req_item = nullptr;
    a.req = a.req_end = a.n_req = 0;
    a.announce = nullptr;
    a.announce_value = 0;
    a.announce_n = 0;
    a.flat_deal = 0;
    const uint32_t cap = (uint32_t)std::min<uint64_t>(buffer_bytes / 4096, 1u << 20);
    for (uint32_t y = 0; y < a.slabs; ++y)
        for (uint32_t c0 = 0; c0 < h.n_items; c0 += cap) {
            const uint32_t n = std::min(cap, h.n_items - c0);
            // prefill side: gather into the send buffer; "send" it; the CPU waits for the GPU
            hipLaunchKernelGGL(kvd_stage_kernel<true>, dim3(n * 4), dim3(64), 0, st, p->geo, a,
                               (unsigned char *)send_buffer, c0, n, y);
            KVD_HIP(hipGetLastError());
            KVD_HIP(hipMemcpyAsync(recv_buffer, send_buffer, (size_t)n * 4096, hipMemcpyDeviceToDevice, st));
            KVD_HIP(hipStreamSynchronize(st));
            // decode side: scatter out of the receive buffer, then notify (another wait)
            hipLaunchKernelGGL(kvd_stage_kernel<false>, dim3(n * 4), dim3(64), 0, st, p->geo, a,
                               (unsigned char *)recv_buffer, c0, n, y);
            KVD_HIP(hipGetLastError());
            KVD_HIP(hipStreamSynchronize(st));
        }
    return KVD_OK;
}

int kvd_pull_blockwise_memcpy(kvd_plan_t *p, void *stream)
{
    if (!as_plan(p)) return fail(KVD_ERR_INVALID, "not a plan handle");
    const Geo &g = p->geo;
    if (g.mode >= kRelayoutHT2TH || g.tb_src != g.tb_dst)
        return fail(KVD_ERR_MISMATCH, "blockwise memcpy baseline needs equal layout and block size");
    const uint64_t e = p->src.elem_bytes;
    const uint64_t row = (uint64_t)g.du * kUnitBytes;  // bytes of one (token, head) row
    const char *sb = (const char *)p->src.base;
    char *db = (char *)p->dst.base;
    for (const ReqHost &r : p->reqs) {
        const uint32_t whole = r.seq_len / g.tb_src, tail = r.seq_len % g.tb_src;
        // layers folded into the block: one copy covers the request's layers of a block
        const uint32_t hk = p->fold_layers ? p->planes_per_layer * (r.layer_end - r.layer_begin) : g.hk;
        const uint32_t layer_stop = p->fold_layers ? r.layer_begin + 1 : r.layer_end;
        const uint64_t tile = (uint64_t)g.tb_src * hk * row;
        for (uint32_t layer = r.layer_begin; layer < layer_stop; ++layer)
            for (uint32_t kv = 0; kv < (1u << g.kv_shift); ++kv) {
                const uint64_t so = layer * g.src_layer_bytes + kv * g.src_kv_bytes;
                const uint64_t dof = layer * g.dst_layer_bytes + kv * g.dst_kv_bytes;
                for (uint32_t b = 0; b < whole; ++b) {
                    const uint64_t s = so + (uint64_t)p->tables_src[r.table_off_src + b] * p->src.stride_block * e;
                    const uint64_t d = dof + (uint64_t)p->tables_dst[r.table_off_dst + b] * p->dst.stride_block * e;
                    KVD_HIP(hipMemcpyAsync(db + d, sb + s, tile, hipMemcpyDeviceToDevice, (hipStream_t)stream));
                }
                if (tail) {
                    const uint64_t s = so + (uint64_t)p->tables_src[r.table_off_src + whole] * p->src.stride_block * e;
                    const uint64_t d = dof + (uint64_t)p->tables_dst[r.table_off_dst + whole] * p->dst.stride_block * e;
                    if (g.mode == kSpanTokenMajor) {
                        KVD_HIP(hipMemcpyAsync(db + d, sb + s, tail * g.hk * row, hipMemcpyDeviceToDevice, (hipStream_t)stream));
                    } else {
                        for (uint32_t h = 0; h < hk; ++h)
                            KVD_HIP(hipMemcpyAsync(db + d + h * g.tb_dst * row, sb + s + h * g.tb_src * row,
                                                   tail * row, hipMemcpyDeviceToDevice, (hipStream_t)stream));
                    }
                }
            }
    }
    return KVD_OK;
}

int kvd_plan_stats(kvd_plan_t *p, void *stream, kvd_stats_t *out)
{
    if (!as_plan(p) || !out) return fail(KVD_ERR_INVALID, "null or wrong handle");
    memset(out, 0, sizeof(*out));
    out->num_requests = (uint32_t)p->reqs.size();
    out->relayout = p->geo.mode >= kRelayoutHT2TH ? 1u : 0u;
    out->num_src_blocks = p->used_src;
    out->num_dst_blocks = p->used_dst;
    out->num_transactions = p->txns_total;
    out->payload_bytes = p->payload_bytes;
    if (!p->reqs.empty()) {
        KVD_HIP(hipStreamSynchronize((hipStream_t)stream));
        Header h;
        KVD_HIP(hipMemcpy(&h, p->hdr_dev, sizeof(h), hipMemcpyDeviceToHost));
        out->num_descriptors = h.n_desc;
        out->num_work_items = h.n_items;
        // the device keeps the queue order when merging made the descriptors longer than the host expected
        out->work_order = (p->hint.rough && (uint64_t)h.n_items > (uint64_t)kSortItemsPerDesc * h.n_desc) ? (uint32_t)KVD_ORDER_QUEUE
                                                                                                           : work_order(p);
    }
    return KVD_OK;
}

int kvd_plan_get_descriptors(kvd_plan_t *p, void *stream, kvd_span_t *spans, kvd_piece_t *pieces,
                             uint64_t cap, uint64_t *n_out)
{
    if (!as_plan(p) || !n_out) return fail(KVD_ERR_INVALID, "null or wrong handle");
    *n_out = 0;
    if (p->reqs.empty()) return KVD_OK;
    const bool relayout = p->geo.mode >= kRelayoutHT2TH;
    if ((relayout && !pieces) || (!relayout && !spans))
        return fail(KVD_ERR_INVALID, "output array for this plan's descriptor kind is null");
    KVD_HIP(hipStreamSynchronize((hipStream_t)stream));
    Header h;
    KVD_HIP(hipMemcpy(&h, p->hdr_dev, sizeof(h), hipMemcpyDeviceToHost));
    if (h.n_desc > p->max_txns) return fail(KVD_ERR_HIP, "corrupt plan header");
    std::vector<Desc> d;
    std::vector<uint32_t> hi;
    try {
        d.resize(h.n_desc);
        hi.resize(h.n_desc);
    } catch (const std::exception &) {
        return fail(KVD_ERR_CAPACITY, "out of host memory for %u descriptors", h.n_desc);
    }
    KVD_HIP(hipMemcpy(d.data(), p->desc_dev, (size_t)h.n_desc * sizeof(Desc), hipMemcpyDeviceToHost));
    if (p->geo.wide)  // written only for plans with 48-bit offsets
        KVD_HIP(hipMemcpy(hi.data(), p->desc_hi_dev, (size_t)h.n_desc * sizeof(uint32_t), hipMemcpyDeviceToHost));
    for (uint32_t i = 0; i < h.n_desc && i < cap; ++i) {
        if (relayout) {
            pieces[i].src_block = (int32_t)(d[i].src16 / p->geo.src_block16);
            pieces[i].dst_block = (int32_t)(d[i].dst16 / p->geo.dst_block16);
            pieces[i].src_token = d[i].a & 1023u;
            pieces[i].dst_token = (d[i].a >> 10) & 1023u;
            pieces[i].num_tokens = d[i].a >> 20;
        } else {
            spans[i].src_offset = (((uint64_t)(hi[i] & 0xFFFFu) << 32) | d[i].src16) * kUnitBytes;
            spans[i].dst_offset = (((uint64_t)(hi[i] >> 16) << 32) | d[i].dst16) * kUnitBytes;
            spans[i].bytes = (uint64_t)(d[i].a - d[i].src16) * kUnitBytes;
        }
    }
    *n_out = h.n_desc;
    return KVD_OK;
}

int kvd_copy_plain(void *dst, const void *src, uint64_t bytes, void *stream)
{
    if (!dst || !src) return fail(KVD_ERR_INVALID, "null pointer");
    if ((bytes % 16) || ((uintptr_t)dst % 16) || ((uintptr_t)src % 16))
        return fail(KVD_ERR_INVALID, "pointers and size must be multiples of 16 bytes");
    if (bytes == 0) return KVD_OK;
    const uint64_t units = bytes / 16;
    const uint64_t grid = (units + 255) / 256;
    if (grid >= (1ull << 31)) return fail(KVD_ERR_CAPACITY, "copy too large for one launch");
    hipLaunchKernelGGL(kvd_copy_kernel, dim3((uint32_t)grid), dim3(256), 0, (hipStream_t)stream, (u32x4 *)dst,
                       (const u32x4 *)src, units);
    KVD_HIP(hipGetLastError());
    return KVD_OK;
}

int kvd_stream_probe(void *dst, const void *src, uint64_t bytes, uint32_t mode, void *stream)
{
    if (!dst || !src) return fail(KVD_ERR_INVALID, "null pointer");
    if ((bytes % 4096) || bytes == 0 || ((uintptr_t)dst % 16) || ((uintptr_t)src % 16))
        return fail(KVD_ERR_INVALID, "size must be a positive multiple of 4096 bytes and the pointers multiples of 16");
    if (mode > 5) return fail(KVD_ERR_INVALID, "mode %u: 0..5", mode);
    const uint64_t units = bytes / 16, grid = units / 256;
    if (grid >= (1ull << 31)) return fail(KVD_ERR_CAPACITY, "buffer too large for one launch");
    int dev = 0;
    hipDeviceProp_t prop;
    KVD_HIP(hipGetDevice(&dev));
    KVD_HIP(hipGetDeviceProperties(&prop, dev));
    const uint32_t resident = (uint32_t)std::min<uint64_t>(grid, (uint64_t)prop.multiProcessorCount * 8);  // 8 workgroups of 4 waves per CU
    const u32x4 fill = {0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
    u32x4 *d = (u32x4 *)dst;
    const u32x4 *s = (const u32x4 *)src;
    hipStream_t st = (hipStream_t)stream;
    switch (mode) {
    case KVD_PROBE_COPY: hipLaunchKernelGGL((kvd_probe_kernel<true, true, true>), dim3((uint32_t)grid), dim3(256), 0, st, d, s, units, fill); break;
    case KVD_PROBE_READ: hipLaunchKernelGGL((kvd_probe_kernel<true, false, true>), dim3((uint32_t)grid), dim3(256), 0, st, d, s, units, fill); break;
    case KVD_PROBE_WRITE: hipLaunchKernelGGL((kvd_probe_kernel<false, true, true>), dim3((uint32_t)grid), dim3(256), 0, st, d, s, units, fill); break;
    case KVD_PROBE_COPY_PERSISTENT: hipLaunchKernelGGL((kvd_probe_kernel<true, true, false>), dim3(resident), dim3(256), 0, st, d, s, units, fill); break;
    case KVD_PROBE_READ_PERSISTENT: hipLaunchKernelGGL((kvd_probe_kernel<true, false, false>), dim3(resident), dim3(256), 0, st, d, s, units, fill); break;
    default: hipLaunchKernelGGL((kvd_probe_kernel<false, true, false>), dim3(resident), dim3(256), 0, st, d, s, units, fill); break;
    }
    KVD_HIP(hipGetLastError());
    return KVD_OK;
}

void kvd_free(void *handle)
{
    // only a handle that is still on the list of live ones is touched: a second release of the
    // same handle, or a pointer that never was one, is ignored without being read
    if (!handle || !retire_handle(handle)) return;
    const uint32_t tag = *(const uint32_t *)handle;
    if (tag == kPoolTag) {
        kvd_pool *p = (kvd_pool *)handle;
        p->tag = 0;
        delete p;
    } else if (tag == kPlanTag) {
        release_plan((kvd_plan *)handle);
    }
}

}  // extern "C"
