// kvd - paged KV-cache pull for MI355X (gfx950): kernels and C ABI.
//
// Data path of KVDirect (arXiv 2501.14743), sections 4.1-4.3, with both pools in one GPU's
// HBM.  Kernels:
//   kvd_build_kernel   one workgroup per appended request or batch: block ids -> byte ranges (section
//                      4.1), coalescing of queued ranges with a wave64 ballot + prefix scan
//                      (section 4.2), then expansion of the coalesced ranges into a table of
//                      fixed 4 KiB work items.
//   kvd_expand_kernel  that expansion as a wide launch of its own, for builds with many items.
//   kvd_pull_kernel    moves the bytes: one small workgroup per (work item, layer, K/V), one
//                      16-byte load and one 16-byte store per lane, non-temporal.  The
//                      hardware dispatcher hands the work items out in table order, which
//                      keeps the traffic an orderly sweep; measured on MI355X this beats a
//                      persistent grid that walks LDS-staged descriptors.
//   kvd_pull_by_descriptor_kernel  the same move for re-layout plans between block-major pools,
//                      walking block by block instead of slab by slab.
//   kvd_order_kernel   for plans of short scattered descriptors: groups the work items by
//                      destination region before the first pull.
//   kvd_pull_persistent_kernel  persistent grid with the descriptors staged in LDS (kept for
//                      comparison).
//   kvd_stage_kernel   gather into / scatter out of a staging buffer (message-style baseline).
//   kvd_copy_kernel    plain streaming copy (counter calibration / practical ceiling).
//
// Descriptors and work items are relative to the (layer 0, K) slab; the pull kernel adds the
// slab offset of each side, so one list serves every layer and both K and V (the receiver
// computes locations from the tensor metadata, section 4.1).

#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <thread>
#include <vector>

#include "kvd.h"

namespace {

constexpr uint32_t kUnitBytes = 16;    // one lane moves 16 bytes per access
constexpr uint32_t kChunkUnits = 256;  // work item: at most 256 units = 4 KiB
constexpr uint32_t kBuildThreads = 1024;
constexpr uint32_t kWave = 64;

enum Mode : uint32_t {
    kSpanTokenMajor = 0,  // same layout, any token sub-range of a block is one byte range
    kSpanHeadMajor = 1,   // both [head][token][dim] with several heads: one range per head
    kRelayoutHT2TH = 2,   // source [head][token][dim] -> destination [token][head][dim]
    kRelayoutTH2HT = 3    // source [token][head][dim] -> destination [head][token][dim]
};

// Coalesced read transaction, 16 bytes.  Offsets and lengths count 16-byte units.  src16 / dst16
// are the low 32 bits of the offsets; bits 32..47 (pools above 64 GiB) sit in a parallel array.
//   byte-copy path: a = low 32 bits of the first unit past the end on the source side
//                   (length = a - src16, modulo 2^32)
//   re-layout path: a = src_token | dst_token << 10 | num_tokens << 20; src16/dst16 = block base
struct Desc {
    uint32_t src16;
    uint32_t dst16;
    uint32_t a;
    uint32_t prefix;  // work items needed by all earlier descriptors
};

// Work item, 16 bytes: what the pull kernel moves per (layer, K/V) for one table entry.
//   byte-copy path: n = units (1..256) starting at src16 / dst16
//   re-layout path: n = first_row | (rows - 1) << 20, rows of one (token, head) each, numbered
//                   token-major inside the piece; src16 / dst16 = the piece's first token
//   layers = layer_begin | num_layers << 16; with 48-bit offsets (Geo::wide, one slab only):
//            bits 32..47 of the source offset | those of the destination offset << 16
struct Item {
    uint32_t src16;
    uint32_t dst16;
    uint32_t n;
    uint32_t layers;
};

struct Header {
    uint32_t n_desc;
    uint32_t n_items;
    // what the last build left for kvd_expand_kernel: descriptors [exp_desc, n_desc) cover work
    // items [exp_item, n_items), which are not written yet
    uint32_t exp_desc;
    uint32_t exp_item;
};

// Exact unsigned division by a run-time constant through multiply-high and shifts
// (Granlund & Montgomery, "Division by invariant integers using multiplication", 1994).
struct FastDiv {
    uint32_t m, s1, s2;
};

FastDiv make_fastdiv(uint32_t d)
{
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;
    FastDiv f;
    f.m = (uint32_t)(((1ull << 32) * ((1ull << l) - d)) / d + 1);
    f.s1 = l < 1 ? l : 1;
    f.s2 = l > 0 ? l - 1 : 0;
    return f;
}

__device__ __forceinline__ uint32_t fdiv(uint32_t n, FastDiv f)
{
    uint32_t t = __umulhi(f.m, n);
    return (t + ((n - t) >> f.s1)) >> f.s2;
}

struct Geo {
    uint64_t src_layer_bytes, src_kv_bytes, dst_layer_bytes, dst_kv_bytes;
    uint32_t src_block16, dst_block16;  // block stride in 16-byte units
    uint32_t tb_src, tb_dst;            // tokens per block
    uint32_t hk, du;                    // KV heads; 16-byte units per (token, head) row
    uint32_t piece_tokens;              // min(tb_src, tb_dst): tokens that share a block on both sides
    uint32_t rows_per_item;             // re-layout: (token, head) rows per work item = 256 / du
    uint32_t kv_shift;                  // 1: K and V are separate slabs; 0: K/V folded into the head axis
    uint32_t wide;                      // 1: offsets have 48 bits (layers folded too, so there is one slab)
    uint32_t mode;
    FastDiv div_du, div_hk, div_tb_src, div_tb_dst;
};

// ------------------------------------------------------------------ build: translate + coalesce + expand

constexpr uint32_t kMaxBatch = 512;  // requests one launch of the build kernel can take
// Builds that add at most this many work items write them from the build kernel itself; larger
// ones leave that to a second, wide launch (one workgroup would take about 1 us per thousand items).
constexpr uint32_t kInlineItems = 8192;

// One request of a batch, as the build kernel sees it.
struct ReqDev {
    uint32_t table_off_src, table_off_dst;  // where its block tables start in the plan's tables
    uint32_t seq_len;
    uint32_t txn_begin;                     // its first read transaction within the batch
};

struct BuildArgs {
    const int32_t *tables_src;  // the plan's block tables (device-visible pinned host memory)
    const int32_t *tables_dst;
    const ReqDev *reqs;         // the batch (device-visible pinned host memory)
    ReqDev first;               // copy of reqs[0]: a single request needs no extra host read
    Desc *desc;
    uint32_t *desc_hi;          // per descriptor: bits 32..47 of src offset | those of dst offset << 16
    Item *items;
    Header *hdr;
    uint32_t n_req;
    uint32_t base_src16;       // added to every offset: the first layer's place inside a block when
    uint32_t base_dst16;       // the layers are folded into the block (0 otherwise)
    uint32_t n_txn;            // read transactions of the whole batch per (layer, K/V)
    uint32_t layers;           // layer_begin | num_layers << 16
    uint32_t fresh;            // 1: the plan is empty (header contents are stale)
    uint32_t may_merge_prev;   // 1: the previous request moves the same layers
    uint32_t no_coalesce;
    uint32_t expand_inline;    // 1: this workgroup also writes the work items (few of them)
    uint32_t *done;            // pinned host word that receives `seq` once the tables have been read
    uint32_t seq;
};

struct Txn {
    uint64_t s16, d16;
    uint32_t len16, meta;
};

// Section 4.1: block id -> offset through the strides.  Transaction j of request rq, in the
// order Transfer() is called for its blocks.
__device__ __forceinline__ Txn make_txn(const Geo &g, const BuildArgs &a, const ReqDev rq, uint32_t j)
{
    uint32_t piece, head = 0;
    bool per_head = false;
    if (g.mode == kSpanHeadMajor) {
        if (g.tb_src == g.tb_dst) {
            const uint32_t n_single = fdiv(rq.seq_len, g.div_tb_src);  // leading whole blocks
            if (j < n_single) {
                piece = j;
            } else {
                piece = n_single;
                head = j - n_single;
                per_head = true;
            }
        } else {
            piece = fdiv(j, g.div_hk);
            head = j - piece * g.hk;
            per_head = true;
        }
    } else {
        piece = j;
    }
    const uint32_t t0 = piece * g.piece_tokens;
    const uint32_t ntok = min(g.piece_tokens, rq.seq_len - t0);
    const uint32_t sb_i = fdiv(t0, g.div_tb_src), db_i = fdiv(t0, g.div_tb_dst);
    const uint32_t st0 = t0 - sb_i * g.tb_src, dt0 = t0 - db_i * g.tb_dst;
    const uint64_t sbase = (uint64_t)(uint32_t)a.tables_src[rq.table_off_src + sb_i] * g.src_block16 + a.base_src16;
    const uint64_t dbase = (uint64_t)(uint32_t)a.tables_dst[rq.table_off_dst + db_i] * g.dst_block16 + a.base_dst16;
    Txn t;
    t.meta = 0;
    if (g.mode == kSpanTokenMajor) {
        t.s16 = sbase + st0 * g.hk * g.du;
        t.d16 = dbase + dt0 * g.hk * g.du;
        t.len16 = ntok * g.hk * g.du;
    } else if (g.mode == kSpanHeadMajor) {
        if (per_head) {
            t.s16 = sbase + (head * g.tb_src + st0) * g.du;
            t.d16 = dbase + (head * g.tb_dst + dt0) * g.du;
            t.len16 = ntok * g.du;
        } else {
            t.s16 = sbase;
            t.d16 = dbase;
            t.len16 = g.tb_src * g.hk * g.du;
        }
    } else {
        t.s16 = sbase;
        t.d16 = dbase;
        t.len16 = ntok * g.hk * g.du;
        t.meta = st0 | (dt0 << 10) | (ntok << 20);
    }
    return t;
}

// Work item number cl of descriptor d (hi = the upper halves of its offsets).
__device__ __forceinline__ Item make_item(const Geo &g, const Desc d, uint32_t hi, uint32_t cl, uint32_t layers)
{
    Item it;
    it.layers = layers;
    if (g.mode < kRelayoutHT2TH) {
        const uint64_t s = (((uint64_t)(hi & 0xFFFFu) << 32) | d.src16) + (uint64_t)cl * kChunkUnits;
        const uint64_t t = (((uint64_t)(hi >> 16) << 32) | d.dst16) + (uint64_t)cl * kChunkUnits;
        it.src16 = (uint32_t)s;
        it.dst16 = (uint32_t)t;
        it.n = min(kChunkUnits, d.a - d.src16 - cl * kChunkUnits);
        if (g.wide) it.layers = (uint32_t)(s >> 32) | ((uint32_t)(t >> 32) << 16);
    } else {
        const uint32_t st0 = d.a & 1023u, dt0 = (d.a >> 10) & 1023u, ntok = d.a >> 20;
        const uint32_t row0 = cl * g.rows_per_item;
        const uint32_t rows = min(g.rows_per_item, ntok * g.hk - row0);
        // fold the first token's slot into the bases (both layouts are linear in the slot)
        const uint32_t s_tok = (g.mode == kRelayoutHT2TH) ? g.du : g.hk * g.du;
        const uint32_t d_tok = (g.mode == kRelayoutHT2TH) ? g.hk * g.du : g.du;
        it.src16 = d.src16 + st0 * s_tok;
        it.dst16 = d.dst16 + dt0 * d_tok;
        it.n = row0 | ((rows - 1) << 20);
    }
    return it;
}

__device__ __forceinline__ uint32_t desc_items(const Geo &g, const Desc &d)
{
    if (g.mode >= kRelayoutHT2TH) return ((d.a >> 20) * g.hk + g.rows_per_item - 1) / g.rows_per_item;
    return (d.a - d.src16 + kChunkUnits - 1) / kChunkUnits;
}

__global__ __launch_bounds__(kBuildThreads) void kvd_build_kernel(Geo g, BuildArgs a)
{
    __shared__ uint64_t s_end[2 * kBuildThreads];  // where every transaction of the tile ends, per side
    uint64_t *const s_end_s = s_end, *const s_end_d = s_end + kBuildThreads;
    uint32_t *const s_buf = (uint32_t *)s_end;     // the same memory as 4096 words, for the expansion
    __shared__ uint64_t s_win[kBuildThreads];      // 2^31-unit windows the transactions start in
    __shared__ uint8_t s_brk[kBuildThreads];
    __shared__ uint32_t s_wave[kBuildThreads / kWave];
    __shared__ ReqDev s_req[kMaxBatch];

    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    if (a.n_req > 1) {
        for (uint32_t i = tid; i < a.n_req; i += kBuildThreads) s_req[i] = a.reqs[i];
        __syncthreads();
    }
    const bool relayout = g.mode >= kRelayoutHT2TH;
    const bool never_merge = relayout || a.no_coalesce;
    const uint32_t n0 = a.fresh ? 0u : a.hdr->n_desc;

    // The queue's last transaction so far: a new transaction that continues it on both sides
    // is merged into it, also when it belongs to another request (section 4.2).
    bool have_prev = false;
    uint64_t prev_s = 0, prev_d = 0, prev_w = 0;
    if (n0 > 0 && !never_merge && a.may_merge_prev) {
        const Desc p = a.desc[n0 - 1];
        const uint32_t hi = g.wide ? a.desc_hi[n0 - 1] : 0u;
        const uint64_t s0 = ((uint64_t)(hi & 0xFFFFu) << 32) | p.src16, d0 = ((uint64_t)(hi >> 16) << 32) | p.dst16;
        have_prev = true;
        prev_s = s0 + (p.a - p.src16);
        prev_d = d0 + (p.a - p.src16);
        prev_w = g.wide ? (((s0 >> 31) << 32) | (d0 >> 31)) : 0ull;
    }
    const bool had_open = have_prev;
    uint32_t runs = n0;

    for (uint32_t tile = 0; tile < a.n_txn; tile += kBuildThreads) {
        const uint32_t j = tile + tid;
        const bool valid = j < a.n_txn;
        Txn t = {0, 0, 0, 0};
        if (valid) {
            ReqDev rq = a.first;
            if (a.n_req > 1) {
                uint32_t lo = 0, hi = a.n_req;  // the request transaction j belongs to
                while (hi - lo > 1) {
                    const uint32_t mid = (lo + hi) >> 1;
                    if (s_req[mid].txn_begin <= j) lo = mid; else hi = mid;
                }
                rq = s_req[lo];
            }
            t = make_txn(g, a, rq, j - rq.txn_begin);
        }
        // With 48-bit offsets a descriptor's length must still fit 32 bits: its transactions all
        // start in one 2^31-unit window (32 GiB) per side, so a run breaks where it enters the next one.
        const uint64_t my_w = g.wide ? (((t.s16 >> 31) << 32) | (t.d16 >> 31)) : 0ull;
        s_end_s[tid] = t.s16 + t.len16;
        s_end_d[tid] = t.d16 + t.len16;
        s_win[tid] = my_w;
        __syncthreads();
        uint64_t ps = prev_s, pd = prev_d, pw = prev_w;
        bool hp = have_prev;
        if (tid > 0) {
            ps = s_end_s[tid - 1];
            pd = s_end_d[tid - 1];
            pw = s_win[tid - 1];
            hp = true;
        }
        const uint32_t tile_last = min(kBuildThreads, a.n_txn - tile) - 1;
        const uint64_t next_prev_s = s_end_s[tile_last], next_prev_d = s_end_d[tile_last], next_prev_w = s_win[tile_last];

        // break flag: this transaction starts a new descriptor
        const bool brk = valid && (never_merge || !hp || ps != t.s16 || pd != t.d16 || pw != my_w);
        const uint64_t ballot = __ballot(brk);
        const uint32_t before = __popcll(ballot & ((1ull << lane) - 1ull));
        if (lane == 0) s_wave[wave] = __popcll(ballot);
        s_brk[tid] = brk ? 1 : 0;
        __syncthreads();
        uint32_t wave_prefix = 0, total = 0;
#pragma unroll
        for (uint32_t w = 0; w < kBuildThreads / kWave; ++w) {
            const uint32_t c = s_wave[w];
            wave_prefix += (w < wave) ? c : 0u;
            total += c;
        }
        if (valid) {
            // descriptor this transaction belongs to = (breaks up to and including it) - 1
            const uint32_t run = runs + wave_prefix + before + (brk ? 1u : 0u) - 1u;
            if (brk) {
                a.desc[run].src16 = (uint32_t)t.s16;
                a.desc[run].dst16 = (uint32_t)t.d16;
                if (g.wide) a.desc_hi[run] = (uint32_t)(t.s16 >> 32) | ((uint32_t)(t.d16 >> 32) << 16);
                if (relayout) a.desc[run].a = t.meta;
            }
            // the last member of a descriptor (so far) records where it ends; a later tile or
            // a later request that continues it overwrites this
            const bool closes = (tid == tile_last) || s_brk[tid + 1];
            if (!relayout && closes) a.desc[run].a = (uint32_t)(t.s16 + t.len16);
        }
        runs += total;
        prev_s = next_prev_s;
        prev_d = next_prev_d;
        prev_w = next_prev_w;
        have_prev = true;
        __syncthreads();
    }

    // The host's block tables and request list are not read again: tell the host, which may then
    // overwrite them for the next build while this one is still running.  Every lane has used what
    // it loaded from them before the barrier that ends the loop above, so the loads are complete;
    // nothing is published to the host with this word, hence no release (which would write the
    // L2 back first).
    if (tid == 0) __hip_atomic_store(a.done, a.seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);

    // work-item prefix over the descriptors that are new or were extended
    const uint32_t n1 = runs;
    const uint32_t from = had_open ? n0 - 1 : n0;
    uint32_t first_item = 0;
    if (from > 0) {
        Desc p = a.desc[from - 1];
        first_item = p.prefix + desc_items(g, p);
    }
    uint32_t carry = first_item;
    for (uint32_t base = from; base < n1; base += kBuildThreads) {
        const uint32_t i = base + tid;
        const bool v = i < n1;
        Desc d = {0, 0, 0, 0};
        if (v) d = a.desc[i];
        const uint32_t c = v ? desc_items(g, d) : 0u;
        uint32_t incl = c;  // inclusive scan inside the wave
#pragma unroll
        for (uint32_t o = 1; o < kWave; o <<= 1) {
            uint32_t up = __shfl_up(incl, o);
            if (lane >= o) incl += up;
        }
        if (lane == kWave - 1) s_wave[wave] = incl;
        __syncthreads();
        uint32_t wave_prefix = 0, total = 0;
#pragma unroll
        for (uint32_t w = 0; w < kBuildThreads / kWave; ++w) {
            const uint32_t x = s_wave[w];
            wave_prefix += (w < wave) ? x : 0u;
            total += x;
        }
        if (v) a.desc[i].prefix = carry + wave_prefix + incl - c;
        carry += total;
        __syncthreads();
    }
    const uint32_t n_items = carry;

    // expand descriptors [from, n1) into work items [first_item, n_items), a window of
    // descriptors at a time with their prefixes staged in LDS for the item -> descriptor search
    constexpr uint32_t kWin = 2 * kBuildThreads;
    for (uint32_t w0 = from; a.expand_inline && w0 < n1; w0 += kWin) {
        const uint32_t nw = min(kWin, n1 - w0);
        for (uint32_t i = tid; i < nw; i += kBuildThreads) s_buf[i] = a.desc[w0 + i].prefix;
        __syncthreads();
        const uint32_t item_lo = s_buf[0];
        const uint32_t item_hi = (w0 + nw == n1) ? n_items : a.desc[w0 + nw].prefix;
        for (uint32_t c = item_lo + tid; c < item_hi; c += kBuildThreads) {
            uint32_t lo = 0, hi = nw;  // largest i with prefix[i] <= c
            while (hi - lo > 1) {
                const uint32_t mid = (lo + hi) >> 1;
                if (s_buf[mid] <= c) lo = mid; else hi = mid;
            }
            const Desc d = a.desc[w0 + lo];
            const uint32_t cl = c - d.prefix;
            const Item it = make_item(g, d, g.wide ? a.desc_hi[w0 + lo] : 0u, cl, a.layers);
            a.items[c] = it;
        }
        __syncthreads();
    }
    if (tid == 0) {
        // Left to kvd_expand_kernel when there are many items.  An extended descriptor keeps the
        // items it had; only its last one, which may have been short, is written again.
        uint32_t exp_item = first_item;
        if (had_open) exp_item = a.hdr->n_items - 1;
        a.hdr->n_desc = n1;
        a.hdr->n_items = n_items;
        a.hdr->exp_desc = from;
        a.hdr->exp_item = a.expand_inline ? n_items : exp_item;
    }
}

// The expansion of descriptors into work items for builds with many items: one lane per item,
// the item's descriptor found by a search over the descriptors' item prefixes.
// grid * 256 >= the number of items the build added + 1.
__global__ __launch_bounds__(256) void kvd_expand_kernel(Geo g, const Desc *desc, const uint32_t *desc_hi, Item *items,
                                                         const Header *hdr, uint32_t layers)
{
    const Header h = *hdr;
    const uint32_t c = h.exp_item + blockIdx.x * 256 + threadIdx.x;
    if (c >= h.n_items) return;
    uint32_t lo = h.exp_desc, hi = h.n_desc;  // largest i with prefix[i] <= c
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (desc[mid].prefix <= c) lo = mid; else hi = mid;
    }
    const Desc d = desc[lo];
    items[c] = make_item(g, d, g.wide ? desc_hi[lo] : 0u, c - d.prefix, layers);
}

// ------------------------------------------------------------------ pull

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct PullArgs {
    const unsigned char *src_base;
    unsigned char *dst_base;
    const Item *items;
    const Header *hdr;  // descriptor and work-item counts, written by the build kernel
    uint32_t slabs;     // (K, V slabs) * the largest layer count of any request
    // 0: slab y of the grid is the y-th of each work item's own layers (the whole plan is moved);
    // 1: slab y is layer `layer0 + y / (K, V slabs)` of the pools, and items without it sit out
    uint32_t absolute_layers;
    uint32_t layer0;
};

// Streaming 16-byte store: non-temporal at device scope.  Measured on MI355X, this cache policy
// moves the scattered 32 KiB-block transfer from 75 % to 80 % of HBM peak compared with the
// plain non-temporal store the compiler emits for __builtin_nontemporal_store.
__device__ __forceinline__ void stream_store(u32x4 v, u32x4 *p)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt" : : "v"(p), "v"(v) : "memory");
}

// Where lane unit u of work item `it` sits on both sides, in 16-byte units from the slab base.
// False if the item has no such unit or does not take part in slab y.
__device__ __forceinline__ bool unit_offsets(const Geo &g, const Item it, uint32_t y, uint32_t u,
                                             uint64_t *s16, uint64_t *d16)
{
    if (g.wide) {  // one slab; the item's last word holds the upper halves of the offsets
        if (y > 0 || u >= it.n) return false;
        *s16 = (((uint64_t)(it.layers & 0xFFFFu) << 32) | it.src16) + u;
        *d16 = (((uint64_t)(it.layers >> 16) << 32) | it.dst16) + u;
        return true;
    }
    if (y >= (it.layers >> 16) << g.kv_shift) return false;
    if (g.mode < kRelayoutHT2TH) {
        if (u >= it.n) return false;
        *s16 = (uint64_t)it.src16 + u;
        *d16 = (uint64_t)it.dst16 + u;
    } else {
        const uint32_t r = fdiv(u, g.div_du), x = u - r * g.du;
        if (r > (it.n >> 20)) return false;
        const uint32_t row = (it.n & 0xFFFFFu) + r;
        const uint32_t tok = fdiv(row, g.div_hk), head = row - tok * g.hk;
        const uint32_t in_ht_src = head * g.tb_src + tok, in_ht_dst = head * g.tb_dst + tok;
        *s16 = (uint64_t)it.src16 + ((g.mode == kRelayoutHT2TH) ? in_ht_src : row) * g.du + x;
        *d16 = (uint64_t)it.dst16 + ((g.mode == kRelayoutHT2TH) ? row : in_ht_dst) * g.du + x;
    }
    return true;
}

__device__ __forceinline__ const unsigned char *src_slab(const Geo &g, const PullArgs &a, const Item it, uint32_t y)
{
    if (g.wide) return a.src_base;
    const uint32_t layer = (it.layers & 0xFFFFu) + (y >> g.kv_shift), kv = y & g.kv_shift;
    return a.src_base + layer * g.src_layer_bytes + kv * g.src_kv_bytes;
}

__device__ __forceinline__ unsigned char *dst_slab(const Geo &g, const PullArgs &a, const Item it, uint32_t y)
{
    if (g.wide) return a.dst_base;
    const uint32_t layer = (it.layers & 0xFFFFu) + (y >> g.kv_shift), kv = y & g.kv_shift;
    return a.dst_base + layer * g.dst_layer_bytes + kv * g.dst_kv_bytes;
}

// One 16-byte unit of work item `it` for slab `y` (= layer offset, K/V): lane unit u.
__device__ __forceinline__ void move_unit(const Geo &g, const PullArgs &a, const Item it, uint32_t y,
                                          uint32_t u)
{
    uint64_t s16, d16;
    if (!unit_offsets(g, it, y, u, &s16, &d16)) return;
    const unsigned char *sp = src_slab(g, a, it, y);
    unsigned char *dp = dst_slab(g, a, it, y);
    const u32x4 v = __builtin_nontemporal_load((const u32x4 *)(sp + (size_t)s16 * kUnitBytes));
    stream_store(v, (u32x4 *)(dp + (size_t)d16 * kUnitBytes));
}

// Message-style baseline (section 4.1, the buffer-based transfer the paper compares against): work
// items [first_item, first_item + n) of slab y are packed into a contiguous buffer (GATHER) or
// unpacked from one (scatter), 4 KiB per item.
template <bool GATHER>
__global__ __launch_bounds__(64) void kvd_stage_kernel(Geo g, PullArgs a, unsigned char *buffer,
                                                       uint32_t first_item, uint32_t n, uint32_t y)
{
    const uint32_t c = blockIdx.x >> 2, u = (blockIdx.x & 3u) * 64 + threadIdx.x;
    if (c >= n) return;
    const Item it = a.items[first_item + c];
    uint64_t s16, d16;
    if (!unit_offsets(g, it, y, u, &s16, &d16)) return;
    u32x4 *packed = (u32x4 *)(buffer + ((size_t)c * kChunkUnits + u) * kUnitBytes);
    if (GATHER)
        *packed = *(const u32x4 *)(src_slab(g, a, it, y) + (size_t)s16 * kUnitBytes);
    else
        *(u32x4 *)(dst_slab(g, a, it, y) + (size_t)d16 * kUnitBytes) = *packed;
}

// Which piece (T consecutive units of a work item) workgroup `b` of a slab's row of the grid moves.
// Workgroups are dealt round-robin to the 8 XCDs.  When descriptors are long on average (at least
// four work items each) every XCD is given one contiguous eighth of the item list, so that one
// XCD's L2 sees whole runs (+3..5 % of HBM peak measured on 32 KiB-block transfers); with short,
// scattered descriptors the plain order is kept (the contiguous deal measured 2 % slower there).
// Returns false if there is nothing to do for this workgroup.
template <int T>
__device__ __forceinline__ bool pick_piece(const Header h, uint32_t b, uint32_t *piece)
{
    constexpr uint32_t kParts = kChunkUnits / T;
    const uint32_t pieces = h.n_items * kParts;
    if (h.n_items >= 4 * h.n_desc) {
        const uint32_t per = (pieces + 7) >> 3;
        if ((b >> 3) >= per) return false;
        b = (b & 7) * per + (b >> 3);
    }
    *piece = b;
    return b < pieces;
}

// grid = (ceil8(item bound * 256 / T), slabs): one workgroup per T units of a work item and slab.
template <int T>
__global__ __launch_bounds__(T) void kvd_pull_kernel(Geo g, PullArgs a)
{
    constexpr uint32_t kParts = kChunkUnits / T;
    uint32_t piece;
    if (!pick_piece<T>(*a.hdr, blockIdx.x, &piece)) return;
    const Item it = a.items[piece / kParts];
    uint32_t y = blockIdx.y;
    if (a.absolute_layers) {
        const uint32_t rel = a.layer0 + (y >> g.kv_shift) - (it.layers & 0xFFFFu);  // wraps below the item's first layer
        if (rel >= (it.layers >> 16)) return;
        y = (rel << g.kv_shift) | (y & g.kv_shift);
    }
    move_unit(g, a, it, y, (piece % kParts) * T + threadIdx.x);
}

// Re-layout between pools that keep a block's layers together: the grid walks descriptor by
// descriptor (a descriptor = the tokens that share one block on both sides) and, inside one, slab
// by slab, so that everything a block holds is touched in one go instead of once per slab sweep
// (measured on MI355X with lone blocks: 78 % of HBM peak against 72 %; walking the descriptors
// that share a block of the side with the larger blocks together gained nothing more).
// grid = (items of a whole descriptor * 256 / T * slabs, descriptors up to 65535, the rest of them).
template <int T>
__global__ __launch_bounds__(T) void kvd_pull_by_descriptor_kernel(Geo g, PullArgs a, const Desc *desc, uint32_t items_per_desc)
{
    constexpr uint32_t kParts = kChunkUnits / T;
    const Header h = *a.hdr;
    const uint32_t d = blockIdx.y + blockIdx.z * 65535u;
    if (d >= h.n_desc) return;
    // gridDim.x is a multiple of 8 (K and V slabs times four pieces per item): XCD k, which gets the
    // workgroups with blockIdx.x = k mod 8, takes the k-th contiguous eighth of the descriptor
    const uint32_t x = (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const uint32_t per_slab = items_per_desc * kParts;
    uint32_t y = x / per_slab;
    const uint32_t piece = x - y * per_slab;
    const Desc dd = desc[d];
    if (piece / kParts >= desc_items(g, dd)) return;
    const Item it = a.items[dd.prefix + piece / kParts];
    if (a.absolute_layers) {
        const uint32_t rel = a.layer0 + (y >> g.kv_shift) - (it.layers & 0xFFFFu);
        if (rel >= (it.layers >> 16)) return;
        y = (rel << g.kv_shift) | (y & g.kv_shift);
    }
    move_unit(g, a, it, y, (piece % kParts) * T + threadIdx.x);
}

// Order of the work items for plans made of short, scattered descriptors (fewer than four work
// items each): items are grouped by the region of the destination slab they write to (buckets of
// 2^shift units, at least 2 MiB), regions in address order.  Measured on MI355X: 80 layers of
// 2048 lone 4 KiB blocks go from 69 % to 74 % of HBM peak; buckets as coarse as 2 MiB give the
// whole gain, the order inside a bucket does not matter.  Plans with long descriptors keep the
// queue order (grouping measured slower there).  One workgroup; a counting sort with the bucket
// counters in LDS.
constexpr uint32_t kOrderBuckets = 4096;

__global__ __launch_bounds__(kBuildThreads) void kvd_order_kernel(const Item *items, Item *ordered, const Header *hdr,
                                                                   uint32_t shift, uint32_t wide)
{
    __shared__ uint32_t s_count[kOrderBuckets];
    __shared__ uint32_t s_wave[kBuildThreads / kWave];
    const Header h = *hdr;
    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    if (h.n_items >= 4 * h.n_desc) {  // long descriptors: keep the queue order
        for (uint32_t i = tid; i < h.n_items; i += kBuildThreads) ordered[i] = items[i];
        return;
    }
    for (uint32_t b = tid; b < kOrderBuckets; b += kBuildThreads) s_count[b] = 0;
    __syncthreads();
    auto region = [&](const Item &it) {
        const uint64_t d = wide ? (((uint64_t)(it.layers >> 16) << 32) | it.dst16) : (uint64_t)it.dst16;
        return (uint32_t)min(d >> shift, (uint64_t)(kOrderBuckets - 1));
    };
    for (uint32_t i = tid; i < h.n_items; i += kBuildThreads) atomicAdd(&s_count[region(items[i])], 1u);
    __syncthreads();
    // exclusive scan of the bucket counts: four consecutive buckets per lane
    constexpr uint32_t kPer = kOrderBuckets / kBuildThreads;
    uint32_t c[kPer], sum = 0;
#pragma unroll
    for (uint32_t k = 0; k < kPer; ++k) {
        c[k] = s_count[tid * kPer + k];
        sum += c[k];
    }
    uint32_t incl = sum;
#pragma unroll
    for (uint32_t o = 1; o < kWave; o <<= 1) {
        const uint32_t up = __shfl_up(incl, o);
        if (lane >= o) incl += up;
    }
    if (lane == kWave - 1) s_wave[wave] = incl;
    __syncthreads();
    uint32_t base = incl - sum;
    for (uint32_t w = 0; w < wave; ++w) base += s_wave[w];
#pragma unroll
    for (uint32_t k = 0; k < kPer; ++k) {
        s_count[tid * kPer + k] = base;
        base += c[k];
    }
    __syncthreads();
    for (uint32_t i = tid; i < h.n_items; i += kBuildThreads) {
        const Item it = items[i];
        ordered[atomicAdd(&s_count[region(it)], 1u)] = it;
    }
}

// Persistent form, kept for comparison: a fixed grid of 1024-lane workgroups stages the coalesced
// descriptors in LDS (a window of kLdsDescs at a time), every wave finds the descriptor of its
// 4 KiB work item by a search over the staged prefixes and moves it with four loads and four
// stores per lane, for one slab after the other.  On MI355X this is 15-20 % of HBM peak slower
// than kvd_pull_kernel: waves of a persistent grid drift apart and the store stream loses its order.
constexpr uint32_t kLdsDescs = 2048;

__global__ __launch_bounds__(1024) void kvd_pull_persistent_kernel(Geo g, PullArgs a, const Desc *desc,
                                                                  uint32_t layers)
{
    __shared__ Desc s_desc[kLdsDescs];
    const Header h = *a.hdr;
    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1);
    const uint32_t W = blockIdx.x * (blockDim.x / kWave) + tid / kWave, NW = gridDim.x * (blockDim.x / kWave);
    for (uint32_t w0 = 0; w0 < h.n_desc; w0 += kLdsDescs) {
        const uint32_t nw = min(kLdsDescs, h.n_desc - w0);
        __syncthreads();
        for (uint32_t i = tid; i < nw; i += blockDim.x) s_desc[i] = desc[w0 + i];
        __syncthreads();
        const uint32_t item_lo = s_desc[0].prefix;
        const uint32_t nc = ((w0 + nw == h.n_desc) ? h.n_items : desc[w0 + nw].prefix) - item_lo;
        // rounds 0..full-1: wave W takes item r*NW + W through every slab; last round: the
        // remaining items are spread over all waves by also splitting the slabs
        const uint32_t full = nc / NW, rem = nc - full * NW;
        for (uint32_t r = 0; r <= full; ++r) {
            uint32_t c, y0 = 0, ystep = 1;
            if (r < full) {
                c = r * NW + W;
            } else {
                if (rem == 0) break;
                const uint32_t phases = min(NW / rem, a.slabs);
                if (W >= rem * phases) break;
                y0 = W / rem;
                c = full * NW + (W - y0 * rem);
                ystep = phases;
            }
            c += item_lo;
            uint32_t lo = 0, hi = nw;  // largest i with prefix[i] <= c
            while (hi - lo > 1) {
                const uint32_t mid = (lo + hi) >> 1;
                if (s_desc[mid].prefix <= c) lo = mid; else hi = mid;
            }
            const Desc d = s_desc[lo];
            const Item it = make_item(g, d, 0u, c - d.prefix, layers);  // 32-bit offsets only (checked by the host)
            uint64_t s16[4], d16[4];
            bool ok[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) ok[k] = unit_offsets(g, it, 0, k * kWave + lane, &s16[k], &d16[k]);
            for (uint32_t y = y0; y < a.slabs; y += ystep) {
                const unsigned char *sp = src_slab(g, a, it, y);
                unsigned char *dp = dst_slab(g, a, it, y);
                u32x4 v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (ok[k]) v[k] = __builtin_nontemporal_load((const u32x4 *)(sp + (size_t)s16[k] * kUnitBytes));
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (ok[k]) stream_store(v[k], (u32x4 *)(dp + (size_t)d16[k] * kUnitBytes));
            }
        }
    }
}

// Complete() of section 4.1 as a message in memory: one word that says which request is done.
// Stream order puts it behind the pulls; the release at system scope makes their writes visible
// to whoever reads the word (another GPU, the host) before the word itself.
__global__ void kvd_complete_kernel(uint64_t *flag, uint64_t value)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) __hip_atomic_store(flag, value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__global__ __launch_bounds__(256) void kvd_copy_kernel(u32x4 *__restrict__ dst,
                                                       const u32x4 *__restrict__ src, uint64_t units)
{
    const uint64_t u = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (u < units) stream_store(__builtin_nontemporal_load(src + u), dst + u);
}

// ------------------------------------------------------------------ host side

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

struct ReqHost {
    uint32_t table_off_src, table_off_dst;  // into the plan's table mirrors
    uint32_t n_src, n_dst;                  // entries used
    uint32_t seq_len, layer_begin, layer_end;
};

}  // namespace

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
    Item *ordered_dev;     // items grouped by destination region (plans of short descriptors)
    bool order_stale;      // requests were appended since ordered_dev was last written
    uint32_t order_shift;  // log2 of the region size in 16-byte units
    Header *hdr_dev;
    // Completion of the build kernels, as far as the host's tables are concerned: every launch
    // carries a sequence number and stores it into a pinned host word when it has read them.
    // (An event recorded between the build and the pull would cost a few microseconds of every
    // step on the GPU's queue.)
    uint32_t *done_host, *done_dev;
    uint32_t build_seq;
    hipStream_t build_stream;
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
    const uint64_t block_axis = ((uint64_t)(d.num_blocks - 1) * d.stride_block + tile) * e;
    if (block_axis >= (1ull << 50))
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

// Frees whatever of the plan's scratch exists (pointers are null until allocated).
void free_scratch(kvd_plan *p)
{
    if (p->done_host) (void)hipHostFree(p->done_host);
    if (p->tables_src) (void)hipHostFree(p->tables_src);
    if (p->tables_dst) (void)hipHostFree(p->tables_dst);
    if (p->reqs_pinned) (void)hipHostFree(p->reqs_pinned);
    if (p->desc_dev) (void)hipFree(p->desc_dev);
    if (p->desc_hi_dev) (void)hipFree(p->desc_hi_dev);
    if (p->items_dev) (void)hipFree(p->items_dev);
    if (p->ordered_dev) (void)hipFree(p->ordered_dev);
    if (p->hdr_dev) (void)hipFree(p->hdr_dev);
    p->done_host = nullptr;
    p->tables_src = p->tables_dst = nullptr;
    p->reqs_pinned = nullptr;
    p->desc_dev = nullptr;
    p->desc_hi_dev = nullptr;
    p->items_dev = p->ordered_dev = nullptr;
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
    KVD_HIP(hipMalloc((void **)&p->hdr_dev, sizeof(Header)));
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
    kvd_plan *p = (kvd_plan *)h;
    return (p && p->tag == kPlanTag) ? p : nullptr;
}

// The launch(es) of a pull: the whole plan (whole = true), or layers [l0, l1) of the pools.
int launch_pull(kvd_plan *p, void *stream, bool whole, uint32_t l0, uint32_t l1)
{
    PullArgs a;
    a.src_base = (const unsigned char *)p->src.base;
    a.dst_base = (unsigned char *)p->dst.base;
    a.items = p->items_dev;
    a.hdr = p->hdr_dev;
    a.slabs = (whole ? p->max_layers : l1 - l0) << p->geo.kv_shift;
    a.absolute_layers = whole ? 0u : 1u;
    a.layer0 = l0;
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
        // transactions shorter than four work items on average (known on the host before merging):
        // the items may be scattered 4-16 KiB pieces, which move faster grouped by destination
        // region; the extra launch (about 8 us) pays from roughly half a GiB of payload on
        if (!(p->flags & KVD_PLAN_QUEUE_ORDER) && p->item_bound < 4 * p->txns_total &&
            p->item_bound * ((uint64_t)p->max_layers << p->geo.kv_shift) >= (1u << 17)) {
            // recorded into a graph, the ordering runs at every replay and the plan still counts
            // as unordered for pulls outside the graph
            const bool capturing = is_capturing(stream);
            if (p->order_stale || capturing) {
                hipLaunchKernelGGL(kvd_order_kernel, dim3(1), dim3(kBuildThreads), 0, (hipStream_t)stream,
                                   p->items_dev, p->ordered_dev, p->hdr_dev, p->order_shift, p->geo.wide);
                KVD_HIP(hipGetLastError());
                if (!capturing) p->order_stale = false;
            }
            a.items = p->ordered_dev;
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
    *out = p;
    return KVD_OK;
}

int kvd_plan_create(const kvd_pool_t *src, const kvd_pool_t *dst, uint32_t max_requests,
                    uint32_t max_total_blocks, uint32_t flags, kvd_plan_t **out)
{
    if (!src || !dst || !out) return fail(KVD_ERR_INVALID, "null argument");
    *out = nullptr;
    if (src->tag != kPoolTag || dst->tag != kPoolTag) return fail(KVD_ERR_INVALID, "not a pool handle");
    if (!max_requests || !max_total_blocks) return fail(KVD_ERR_INVALID, "zero capacity");
    const kvd_pool_desc_t &s = src->d, &d = dst->d;
    if (s.num_kv_heads != d.num_kv_heads || s.head_dim != d.head_dim || s.elem_bytes != d.elem_bytes)
        return fail(KVD_ERR_MISMATCH, "pools differ in num_kv_heads, head_dim or elem_bytes");
    const uint32_t tmin = std::min(s.block_tokens, d.block_tokens);
    const uint32_t tmax = std::max(s.block_tokens, d.block_tokens);
    if (tmax % tmin)
        return fail(KVD_ERR_MISMATCH, "block sizes %u and %u: neither divides the other",
                    s.block_tokens, d.block_tokens);
    const uintptr_t sb = (uintptr_t)s.base, db = (uintptr_t)d.base;
    if (sb < db + dst->extent_bytes && db < sb + src->extent_bytes)
        return fail(KVD_ERR_ALIAS, "source and destination pools overlap");

    kvd_plan *p = new (std::nothrow) kvd_plan();
    if (!p) return fail(KVD_ERR_INVALID, "out of host memory");
    p->tag = kPlanTag;
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
    if (!p->fold_layers && (block_axis_bytes(s) >= (1ull << 36) || block_axis_bytes(d) >= (1ull << 36))) {
        delete p;
        return fail(KVD_ERR_RANGE, "a block axis that spans more than 64 GiB needs block-major pools with the same inner "
                                   "order on both sides");
    }
    if ((flags & KVD_PLAN_WIDE_OFFSETS) && !p->fold_layers) {
        delete p;
        return fail(KVD_ERR_MISMATCH, "48-bit offsets are for block-major pools with the same inner order on both sides");
    }
    if ((flags & KVD_PLAN_PERSISTENT) && g.wide) {
        delete p;
        return fail(KVD_ERR_MISMATCH, "the persistent form has 32-bit offsets only");
    }
    const uint32_t hk_max = p->fold_layers ? g.hk * std::min(s.num_layers, d.num_layers) : g.hk;
    g.rows_per_item = g.du <= kChunkUnits ? kChunkUnits / g.du : 0;
    p->by_descriptor = g.mode >= kRelayoutHT2TH && !(flags & (KVD_PLAN_PERSISTENT | KVD_PLAN_QUEUE_ORDER)) &&
                       s.stride_block > s.stride_layer && s.stride_block > s.stride_kv &&
                       d.stride_block > d.stride_layer && d.stride_block > d.stride_kv;
    p->items_per_desc = g.rows_per_item ? ceil_div(tmin * g.hk, g.rows_per_item) : 0;
    if ((flags & KVD_PLAN_WHOLE_BLOCKS) && s.block_tokens != d.block_tokens) {
        delete p;
        return fail(KVD_ERR_MISMATCH, "whole-block transfers need equal block sizes");
    }
    g.div_du = make_fastdiv(g.du);
    g.div_hk = make_fastdiv(g.hk);
    g.div_tb_src = make_fastdiv(g.tb_src);
    g.div_tb_dst = make_fastdiv(g.tb_dst);

    // upper bounds of what the plan can hold: read transactions and work items
    const uint64_t pieces_max = (uint64_t)max_total_blocks * (tmax / tmin);
    if (g.mode == kSpanHeadMajor)
        p->max_txns = (g.tb_src == g.tb_dst) ? pieces_max + (uint64_t)max_requests * hk_max
                                             : pieces_max * hk_max;
    else
        p->max_txns = pieces_max;
    const uint64_t units_max = pieces_max * tmin * hk_max * g.du;
    if (g.mode >= kRelayoutHT2TH)
        p->max_items = pieces_max * tmin * g.hk / g.rows_per_item + p->max_txns + 1;
    else
        p->max_items = units_max / kChunkUnits + p->max_txns + 1;
    if (p->max_items >= (1ull << 31) || p->max_txns >= (1ull << 31)) {
        delete p;
        return fail(KVD_ERR_CAPACITY, "plan capacity too large");
    }
    // destination regions for kvd_order_kernel: 2 MiB, or wider if the slab's block axis would
    // need more buckets than the kernel keeps
    const uint64_t dst_span16 = ((uint64_t)(d.num_blocks - 1) * d.stride_block +
                                 (uint64_t)d.block_tokens * d.num_kv_heads * d.head_dim) * e / kUnitBytes;
    p->order_shift = 17;
    while ((dst_span16 >> p->order_shift) >= kOrderBuckets) ++p->order_shift;
    p->order_stale = true;
    p->dst_used.assign(d.num_blocks, 0);
    p->reqs.reserve(max_requests);
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
    p->max_layers = 0;
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
    if (rc != KVD_OK) {
        unmark_call(n_requests, 0);
        return rc;
    }

    // 3. commit on the host, then one launch per kMaxBatch requests
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
        memcpy(p->tables_src + r.table_off_src, src_tbls[k], (size_t)r.n_src * sizeof(int32_t));
        memcpy(p->tables_dst + r.table_off_dst, dst_tbls[k], (size_t)r.n_dst * sizeof(int32_t));
        for (uint32_t i = 0; i < r.n_dst; ++i) p->dst_used[(uint32_t)dst_tbls[k][i]] = 1;
        p->used_src += r.n_src;
        p->used_dst += r.n_dst;
        p->payload_bytes += ((uint64_t)seq_len * slab_layers * g.hk * g.du * kUnitBytes) << g.kv_shift;
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
            p->reqs_pinned[b0 + i] = ReqDev{r.table_off_src, r.table_off_dst, r.seq_len, batch_txn};
            batch_txn += n_txn;
            batch_items += items;
        }
        BuildArgs a;
        a.tables_src = p->tables_src_dev;
        a.tables_dst = p->tables_dst_dev;
        a.reqs = p->reqs_pinned_dev + b0;
        a.first = p->reqs_pinned[b0];
        a.desc = p->desc_dev;
        a.desc_hi = p->desc_hi_dev;
        a.items = p->items_dev;
        a.hdr = p->hdr_dev;
        a.n_req = nb;
        a.base_src16 = p->fold_layers ? (uint32_t)(layer_begin * g.src_layer_bytes / kUnitBytes) : 0u;
        a.base_dst16 = p->fold_layers ? (uint32_t)(layer_begin * g.dst_layer_bytes / kUnitBytes) : 0u;
        a.n_txn = batch_txn;
        a.layers = p->fold_layers ? (1u << 16) : (layer_begin | (n_layers << 16));
        a.fresh = (b0 == 0) ? 1u : 0u;
        a.may_merge_prev = (b0 > first_new || same_layers) ? 1u : 0u;
        a.no_coalesce = (p->flags & KVD_PLAN_NO_COALESCE) ? 1u : 0u;
        a.expand_inline = batch_items <= kInlineItems ? 1u : 0u;
        a.done = p->done_dev;
        a.seq = ++p->build_seq;
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
        p->order_stale = true;
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
    hipLaunchKernelGGL(kvd_complete_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, (uint64_t *)at.devicePointer, value);
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
    PullArgs a;
    a.src_base = (const unsigned char *)p->src.base;
    a.dst_base = (unsigned char *)p->dst.base;
    a.items = p->items_dev;
    a.hdr = p->hdr_dev;
    a.slabs = p->max_layers << p->geo.kv_shift;
    a.absolute_layers = 0;
    a.layer0 = 0;
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
    std::vector<Desc> d(h.n_desc);
    std::vector<uint32_t> hi(h.n_desc);
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

void kvd_free(void *handle)
{
    if (!handle) return;
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
