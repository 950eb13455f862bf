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
//   kvd_order_kernel, kvd_order_copy_kernel  for plans of short scattered descriptors: put the
//                      work items in the order of their destination before the first pull.
//   kvd_pull_persistent_kernel  persistent grid with the descriptors staged in LDS (kept for
//                      comparison).
//   kvd_stage_kernel   gather into / scatter out of a staging buffer (message-style baseline).
//   kvd_copy_kernel    plain streaming copy (counter calibration / practical ceiling).
//   kvd_probe_kernel   read-only / write-only / copy streams, dispatched or persistent (calibration).
//
// Descriptors and work items are relative to the (layer 0, K) slab; the pull kernel adds the
// slab offset of each side, so one list serves every layer and both K and V (the receiver
// computes locations from the tensor metadata, section 4.1).

#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

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
// A build that adds at most this many descriptors keeps them in LDS from the translation to the
// expansion, so that the prefix scan and the work items do not wait for global memory again.
constexpr uint32_t kBuildLdsDescs = 1024;

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
    // Plans that complete request by request (section 4.2: a completion transaction sits behind the
    // reads of its own request, and reads are merged only up to the first completion): a request's
    // first transaction always starts a descriptor, and the descriptor / work item each request of
    // the batch starts at are recorded for the per-request pulls.  Null otherwise.
    uint32_t *req_desc;        // [requests of the plan] first descriptor
    uint32_t *req_item;        // [requests of the plan] first work item
    uint32_t req_base;         // index of the batch's first request within the plan
    // 1: a fresh plan's first launch, which adds at most kBuildLdsDescs descriptors and writes its work
    // items itself, also writes them a second time into `ordered`, the descriptors sorted by destination
    // address (what kvd_order_kernel and kvd_order_copy_kernel do for larger plans, without their launches)
    uint32_t sort_inline;
    Item *ordered;
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

// Sorts np2 keys (a power of two, at least one wave's 64) with their 16-bit companions in LDS, ascending:
// a bitonic network, every lane of the kBuildThreads-lane workgroup takes part, the arrays are final
// after the call (it ends with a workgroup barrier; one must precede it, after the arrays were filled).
__device__ __forceinline__ void bitonic_sort_lds(uint32_t *s_key, uint16_t *s_idx, uint32_t np2, uint32_t tid)
{
    // One compare-exchange stage: pair t is (lo, lo | j), lo with bit j clear.
    auto stage = [&](uint32_t k, uint32_t j) {
        for (uint32_t t = tid; t < np2 / 2; t += kBuildThreads) {
            const uint32_t lo = ((t & ~(j - 1)) << 1) | (t & (j - 1)), hi = lo | j;
            const uint32_t x = s_key[lo], y = s_key[hi];
            if ((x > y) == ((lo & k) == 0)) {
                s_key[lo] = y;
                s_key[hi] = x;
                const uint16_t ix = s_idx[lo];
                s_idx[lo] = s_idx[hi];
                s_idx[hi] = ix;
            }
        }
    };
    for (uint32_t k = 2; k <= np2; k <<= 1) {
        uint32_t j = k >> 1;
        for (; j >= 2 * kWave; j >>= 1) {
            stage(k, j);
            __syncthreads();
        }
        // Pairs at most 64 apart lie inside one 128-element block, and pairs 64 t .. 64 t + 63 - one wave's -
        // are exactly the pairs of block t: these stages touch nothing another wave touches, so they need
        // no workgroup barrier, only the wave's own LDS accesses kept in program order.
        for (; j > 0; j >>= 1) {
            stage(k, j);
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
        if (k >= 2 * kWave) __syncthreads();  // the next k starts with pairs that cross waves
    }
    __syncthreads();
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
    __shared__ Desc s_desc[kBuildLdsDescs];             // descriptors [from, from + kBuildLdsDescs) as they are written

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
        if (tid == 0) s_desc[0] = p;  // it is descriptor `from` below; the loop's first barrier publishes it
        const uint32_t hi = g.wide ? a.desc_hi[n0 - 1] : 0u;
        const uint64_t s0 = ((uint64_t)(hi & 0xFFFFu) << 32) | p.src16, d0 = ((uint64_t)(hi >> 16) << 32) | p.dst16;
        have_prev = true;
        prev_s = s0 + (p.a - p.src16);
        prev_d = d0 + (p.a - p.src16);
        prev_w = g.wide ? (((s0 >> 31) << 32) | (d0 >> 31)) : 0ull;
    }
    const bool had_open = have_prev;
    const uint32_t from = had_open ? n0 - 1 : n0;  // first descriptor this launch writes or extends
    uint32_t runs = n0;

    for (uint32_t tile = 0; tile < a.n_txn; tile += kBuildThreads) {
        const uint32_t j = tile + tid;
        const bool valid = j < a.n_txn;
        Txn t = {0, 0, 0, 0};
        uint32_t req = 0;                // the request transaction j belongs to (index within the batch)
        bool first_of_request = false;   // ... and whether it opens that request's own descriptors
        if (valid) {
            ReqDev rq = a.first;
            if (a.n_req > 1) {
                uint32_t lo = 0, hi = a.n_req;
                while (hi - lo > 1) {
                    const uint32_t mid = (lo + hi) >> 1;
                    if (s_req[mid].txn_begin <= j) lo = mid; else hi = mid;
                }
                rq = s_req[lo];
                req = lo;
            }
            t = make_txn(g, a, rq, j - rq.txn_begin);
            first_of_request = a.req_desc && j == rq.txn_begin;
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
        const bool brk = valid && (never_merge || !hp || ps != t.s16 || pd != t.d16 || pw != my_w || first_of_request);
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
            if (first_of_request) a.req_desc[a.req_base + req] = run;
            const bool in_lds = run - from < kBuildLdsDescs;
            if (brk) {
                a.desc[run].src16 = (uint32_t)t.s16;
                a.desc[run].dst16 = (uint32_t)t.d16;
                if (g.wide) a.desc_hi[run] = (uint32_t)(t.s16 >> 32) | ((uint32_t)(t.d16 >> 32) << 16);
                if (relayout) a.desc[run].a = t.meta;
                if (in_lds) {
                    s_desc[run - from].src16 = (uint32_t)t.s16;
                    s_desc[run - from].dst16 = (uint32_t)t.d16;
                    if (relayout) s_desc[run - from].a = t.meta;
                }
            }
            // the last member of a descriptor (so far) records where it ends; a later tile or
            // a later request that continues it overwrites this
            const bool closes = (tid == tile_last) || s_brk[tid + 1];
            if (!relayout && closes) {
                a.desc[run].a = (uint32_t)(t.s16 + t.len16);
                if (in_lds) s_desc[run - from].a = (uint32_t)(t.s16 + t.len16);
            }
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
    const bool in_lds = n1 - from <= kBuildLdsDescs;  // s_desc holds every descriptor of this launch
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
        if (v) d = in_lds ? s_desc[i - from] : a.desc[i];
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
        if (v) {
            a.desc[i].prefix = carry + wave_prefix + incl - c;
            if (in_lds) s_desc[i - from].prefix = carry + wave_prefix + incl - c;
        }
        carry += total;
        __syncthreads();
    }
    const uint32_t n_items = carry;
    // where each request of the batch starts in the work-item table (the prefixes above were written
    // by this workgroup and the loop's last barrier has passed)
    if (a.req_item)
        for (uint32_t i = tid; i < a.n_req; i += kBuildThreads) a.req_item[a.req_base + i] = a.desc[a.req_desc[a.req_base + i]].prefix;

    // expand descriptors [from, n1) into work items [first_item, n_items), a window of
    // descriptors at a time with their prefixes staged in LDS for the item -> descriptor search
    if (a.expand_inline && in_lds) {
        // Every lane writes `per` consecutive work items: one search over the prefixes in LDS for
        // its first item, then it walks on from descriptor to descriptor (each has at least one item).
        const uint32_t nd = n1 - from;
        const uint32_t per = (n_items - first_item + kBuildThreads - 1) / kBuildThreads;
        const uint32_t c0 = first_item + tid * per, c1 = min(n_items, c0 + per);
        if (c0 < c1) {
            uint32_t lo = 0, hi = nd;  // largest i with prefix[i] <= c0
            while (hi - lo > 1) {
                const uint32_t mid = (lo + hi) >> 1;
                if (s_desc[mid].prefix <= c0) lo = mid; else hi = mid;
            }
            Desc d = s_desc[lo];
            uint32_t next = (lo + 1 < nd) ? s_desc[lo + 1].prefix : n_items;
            uint32_t dhi = g.wide ? a.desc_hi[from + lo] : 0u;
            for (uint32_t c = c0; c < c1; ++c) {
                while (c >= next) {
                    ++lo;
                    d = s_desc[lo];
                    next = (lo + 1 < nd) ? s_desc[lo + 1].prefix : n_items;
                    if (g.wide) dhi = a.desc_hi[from + lo];
                }
                a.items[c] = make_item(g, d, dhi, c - d.prefix, a.layers);
            }
        }
    }
    if (a.sort_inline && a.expand_inline && in_lds && from == 0) {
        // the same work items once more, in the order of their descriptors' destination addresses
        uint32_t *const s_key = (uint32_t *)s_end;  // the translation's memory is free by now
        uint32_t *const s_off = s_key + kBuildLdsDescs;
        uint16_t *const s_idx = (uint16_t *)(s_off + kBuildLdsDescs);
        const uint32_t nd = n1;
        uint32_t np2 = kWave;
        while (np2 < nd) np2 <<= 1;
        __syncthreads();
        if (tid < np2) {
            s_key[tid] = tid < nd ? s_desc[tid].dst16 : 0xFFFFFFFFu;  // padding sorts to the end
            s_idx[tid] = (uint16_t)tid;
        }
        __syncthreads();
        bitonic_sort_lds(s_key, s_idx, np2, tid);
        // items of the descriptor at sorted position tid, then where each position's items start
        uint32_t cnt = 0;
        if (tid < nd) {
            const uint32_t i = s_idx[tid];
            cnt = ((i + 1 < nd) ? s_desc[i + 1].prefix : n_items) - s_desc[i].prefix;
        }
        uint32_t incl = cnt;
#pragma unroll
        for (uint32_t o = 1; o < kWave; o <<= 1) {
            const uint32_t up = __shfl_up(incl, o);
            if (lane >= o) incl += up;
        }
        if (lane == kWave - 1) s_wave[wave] = incl;
        __syncthreads();
        uint32_t start = incl - cnt;
        for (uint32_t w = 0; w < wave; ++w) start += s_wave[w];
        s_off[tid] = start;
        __syncthreads();
        const uint32_t per = (n_items + kBuildThreads - 1) / kBuildThreads;
        const uint32_t o0 = tid * per, o1 = min(n_items, o0 + per);
        if (o0 < o1) {
            uint32_t pos = 0, top = nd;  // largest position whose items start at or before o0
            while (top - pos > 1) {
                const uint32_t mid = (pos + top) >> 1;
                if (s_off[mid] <= o0) pos = mid; else top = mid;
            }
            Desc d = s_desc[s_idx[pos]];
            uint32_t next = (pos + 1 < nd) ? s_off[pos + 1] : n_items;
            for (uint32_t o = o0; o < o1; ++o) {
                while (o >= next) {
                    ++pos;
                    d = s_desc[s_idx[pos]];
                    next = (pos + 1 < nd) ? s_off[pos + 1] : n_items;
                }
                a.ordered[o] = make_item(g, d, 0u, o - s_off[pos], a.layers);
            }
        }
    }
    constexpr uint32_t kWin = 2 * kBuildThreads;
    for (uint32_t w0 = from; a.expand_inline && !in_lds && w0 < n1; w0 += kWin) {
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

// A piece of the host's two block tables carried in the kernel's argument buffer and written to
// device memory: the way the tables reach the GPU for a caller that has no pinned memory to put
// them in.  2 * 448 ids fill 3584 of the 4096 bytes a kernel's arguments may take.
constexpr uint32_t kArgTableEntries = 448;

struct TableChunk {
    int32_t src[kArgTableEntries];
    int32_t dst[kArgTableEntries];
};

__global__ __launch_bounds__(kArgTableEntries) void kvd_stage_tables_kernel(TableChunk c, int32_t *tables_src, uint32_t n_src,
                                                                            int32_t *tables_dst, uint32_t n_dst)
{
    const uint32_t i = threadIdx.x;
    if (i < n_src) tables_src[i] = c.src[i];
    if (i < n_dst) tables_dst[i] = c.dst[i];
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
    // requests [req, req_end) of the plan only (per-request completion): work items
    // [req_item[req], req_item[req_end]) of the table, up to the table's end if req_end = n_req.
    // Null: the whole table.
    const uint32_t *req_item;
    uint32_t req, req_end, n_req;
    // Completion words to store (null: none): those of the announce_n consecutive requests whose pull
    // ran before this launch on the same stream, so that they cost no launch of their own.
    uint64_t *announce;
    uint64_t announce_value;
    uint32_t announce_n;
    // 1: workgroups are dealt to the XCDs item by item whatever the descriptors look like (lone blocks
    // sorted by destination that fill an eighth of the pool or more lie close enough to move like one
    // contiguous range, for which this deal is the faster one)
    uint32_t flat_deal;
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
// scattered descriptors the plain order is kept (the contiguous deal measured 2 % slower there),
// and so it is when the host asks for it (PullArgs::flat_deal).
// Returns false if there is nothing to do for this workgroup.
template <int T>
__device__ __forceinline__ bool pick_piece(const Header h, const PullArgs &a, uint32_t b, uint32_t *piece)
{
    constexpr uint32_t kParts = kChunkUnits / T;
    uint32_t lo = 0, hi = h.n_items;  // the part of the item table this launch moves
    if (a.req_item) {
        lo = a.req_item[a.req];
        if (a.req_end < a.n_req) hi = a.req_item[a.req_end];
    }
    const uint32_t pieces = (hi - lo) * kParts;
    if (h.n_items >= 4 * h.n_desc && !a.flat_deal) {
        const uint32_t per = (pieces + 7) >> 3;
        if ((b >> 3) >= per) return false;
        b = (b & 7) * per + (b >> 3);
    }
    *piece = lo * kParts + b;
    return b < pieces;
}

// grid = (ceil8(item bound * 256 / T), slabs): one workgroup per T units of a work item and slab.
template <int T>
__global__ __launch_bounds__(T) void kvd_pull_kernel(Geo g, PullArgs a)
{
    constexpr uint32_t kParts = kChunkUnits / T;
    uint32_t piece;
    if (pick_piece<T>(*a.hdr, a, blockIdx.x, &piece)) {
        const Item it = a.items[piece / kParts];
        uint32_t y = blockIdx.y;
        bool mine = true;
        if (a.absolute_layers) {
            const uint32_t rel = a.layer0 + (y >> g.kv_shift) - (it.layers & 0xFFFFu);  // wraps below the item's first layer
            mine = rel < (it.layers >> 16);
            y = (rel << g.kv_shift) | (y & g.kv_shift);
        }
        if (mine) move_unit(g, a, it, y, (piece % kParts) * T + threadIdx.x);
    }
    // Stream order has put the previous launch's writes behind this one's start; the release at
    // system scope makes them visible to whoever reads the word, before the word.  Kept at the very
    // end: the loads above stay scalar loads only while no atomic precedes them in program order
    // (with this store first, the header and item loads become vector loads and the whole kernel
    // runs a quarter slower, measured).
    if (a.announce && blockIdx.x == 0 && blockIdx.y == 0)
        for (uint32_t i = threadIdx.x; i < a.announce_n; i += T)
            __hip_atomic_store(a.announce + i, a.announce_value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
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

// Order of the work items for plans made of short, scattered descriptors; the host chooses the form
// from the tables; where its picture of them is a rough one (`guard`), the device keeps the queue order
// if merging made the descriptors long after all.
//  - group_items (most of the work in descriptors below four work items): items are grouped by the region of the
//    destination slab they write to (buckets of 2^shift units, at least 2 MiB), regions in address
//    order; a counting sort with the bucket counters in LDS.  Measured on MI355X: 80 layers of 2048
//    lone 4 KiB blocks go from 69 % to 74 % of HBM peak; buckets as coarse as 2 MiB give the whole
//    gain, the order inside a bucket does not matter.
//  - otherwise (most of it in descriptors of four to eight work items: lone 16 and 32 KiB blocks): whole
//    descriptors are sorted by destination address, kSortMax of them at a time (a bitonic sort of
//    their keys in LDS), and each keeps its items together and in order.  This kernel writes, per
//    sorted position, where its items go and where they come from; kvd_order_copy_kernel, a wide
//    launch right behind it, moves the items.  Measured: 2048 lone 32 KiB blocks out of 16384 go
//    from 65 % to 72 %, 4096 to 74 %, 512 to 68 %.
//  - Plans with a quarter or more of the work in longer descriptors keep the queue order and never get
//    here (sorting runs of two blocks gains 1.5 points, about
//    what the sort costs; runs of four gain nothing; the 1-8 block runs of the 8192-token
//    configuration lose a point).
// One workgroup.
constexpr uint32_t kOrderBuckets = 4096;
constexpr uint32_t kSortMax = 8192;  // descriptors sorted together
constexpr uint32_t kSortItemsPerDesc = 8;

// Sorted position -> (first work item in the ordered table, first work item in the queue-ordered one).
struct OrderEntry {
    uint32_t to, from;
};

// With `guard` the device has the last word: the host's picture of the descriptors was a rough one
// (block sizes differ between the pools), and if merging made them long after all the queue order stays.
__device__ __forceinline__ bool sorts_descriptors(const Header h, uint32_t guard)
{
    return !guard || h.n_items <= kSortItemsPerDesc * h.n_desc;
}

__global__ __launch_bounds__(kBuildThreads) void kvd_order_kernel(const Item *items, Item *ordered, const Header *hdr,
                                                                   const Desc *desc, const uint32_t *desc_hi, OrderEntry *order,
                                                                   uint32_t group_items, uint32_t guard, uint32_t shift, uint32_t wide)
{
    __shared__ uint32_t s_mem[kSortMax + kSortMax / 2];  // bucket counters; or sort keys, then 16-bit indices
    __shared__ uint32_t s_wave[kBuildThreads / kWave];
    uint32_t *const s_count = s_mem;
    const Header h = *hdr;
    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    if (!sorts_descriptors(h, guard)) {  // long descriptors: keep the queue order
        for (uint32_t i = tid; i < h.n_items; i += kBuildThreads) ordered[i] = items[i];
        return;
    }
    if (!group_items) {
        uint32_t *const s_key = s_mem;                           // keys while sorting, item offsets afterwards
        uint16_t *const s_idx = (uint16_t *)(s_mem + kSortMax);  // descriptor (within the chunk) at each sorted position
        constexpr uint32_t kPer = kSortMax / kBuildThreads;
        for (uint32_t c0 = 0; c0 < h.n_desc; c0 += kSortMax) {
            const uint32_t n = min(kSortMax, h.n_desc - c0);
            uint32_t np2 = kWave;
            while (np2 < n) np2 <<= 1;
            for (uint32_t i = tid; i < np2; i += kBuildThreads) {
                uint32_t key = 0xFFFFFFFFu;  // padding sorts to the end
                if (i < n) key = wide ? (uint32_t)(((((uint64_t)(desc_hi[c0 + i] >> 16)) << 32) | desc[c0 + i].dst16) >> 16)
                                      : desc[c0 + i].dst16;
                s_key[i] = key;
                s_idx[i] = (uint16_t)i;
            }
            __syncthreads();
            bitonic_sort_lds(s_key, s_idx, np2, tid);
            // how many items each sorted position brings, then where its items start within the chunk
            uint32_t c[kPer], sum = 0;
#pragma unroll
            for (uint32_t k = 0; k < kPer; ++k) {
                const uint32_t pos = tid * kPer + k;
                c[k] = 0;
                if (pos < n) {
                    const uint32_t gi = c0 + s_idx[pos];
                    c[k] = ((gi + 1 < h.n_desc) ? desc[gi + 1].prefix : h.n_items) - desc[gi].prefix;
                }
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
                s_key[tid * kPer + k] = base;
                base += c[k];
            }
            __syncthreads();
            // the chunk's items keep their range of the table
            const uint32_t item0 = desc[c0].prefix;
#pragma unroll
            for (uint32_t k = 0; k < kPer; ++k) {
                const uint32_t pos = tid * kPer + k;
                if (pos < n) order[c0 + pos] = OrderEntry{item0 + s_key[pos], desc[c0 + s_idx[pos]].prefix};
            }
            __syncthreads();
        }
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

// Second half of the descriptor sort: one lane per work item of the ordered table; its sorted
// position is found by a search over the entries kvd_order_kernel wrote.  grid * 256 >= work items.
// Does nothing when that kernel kept the queue order (it has then copied the items itself).
__global__ __launch_bounds__(256) void kvd_order_copy_kernel(const Item *items, Item *ordered, const Header *hdr,
                                                              const OrderEntry *order, uint32_t guard)
{
    const Header h = *hdr;
    const uint32_t o = blockIdx.x * 256 + threadIdx.x;
    if (!sorts_descriptors(h, guard) || o >= h.n_items) return;
    uint32_t lo = 0, hi = h.n_desc;  // largest position whose items start at or before o
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (order[mid].to <= o) lo = mid; else hi = mid;
    }
    const OrderEntry e = order[lo];
    ordered[o] = items[e.from + (o - e.to)];
}

// Persistent form, kept for comparison: a fixed grid of 1024-lane workgroups stages the coalesced
// descriptors in LDS (a window of kBuildLdsDescs at a time), every wave finds the descriptor of its
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
__global__ void kvd_complete_kernel(uint64_t *flags, uint32_t n, uint64_t value)
{
    if (blockIdx.x == 0)
        for (uint32_t i = threadIdx.x; i < n; i += blockDim.x)
            __hip_atomic_store(flags + i, value, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

__global__ __launch_bounds__(256) void kvd_copy_kernel(u32x4 *__restrict__ dst,
                                                       const u32x4 *__restrict__ src, uint64_t units)
{
    const uint64_t u = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    if (u < units) stream_store(__builtin_nontemporal_load(src + u), dst + u);
}

// Probes of the memory system on plain buffers, with the pull kernel's access width and cache
// policies: what a stream of reads, a stream of writes and a copy reach when every workgroup does
// one access per lane and the hardware dispatcher hands the workgroups out in address order
// (DISPATCHED), and when a fixed grid of resident workgroups strides over the buffer instead
// (the persistent form).  READ / WRITE select the streams.
template <bool READ, bool WRITE, bool DISPATCHED>
__global__ __launch_bounds__(256) void kvd_probe_kernel(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src,
                                                        uint64_t units, u32x4 fill)
{
    const uint64_t stride = DISPATCHED ? units : (uint64_t)gridDim.x * 256;
    u32x4 seen = fill;
    for (uint64_t u = (uint64_t)blockIdx.x * 256 + threadIdx.x; u < units; u += stride) {
        u32x4 v = fill;
        if (READ) v = __builtin_nontemporal_load(src + u);
        if (WRITE) stream_store(v, dst + u);
        seen ^= v;
    }
    // keeps the loads of the read-only form alive: no buffer of N(0,1) values xors to this pattern
    if (READ && !WRITE && seen.x == 0x7FA57FA5u && seen.y == 0x7FA57FA5u && seen.z == 0x12345678u) stream_store(seen, dst);
}

}  // namespace
