// kvd - paged KV-cache pull for MI355X (gfx950): kernels and C ABI.
//
// Data path of KVDirect (arXiv 2501.14743), sections 4.1-4.3, with both pools in one GPU's
// HBM.  Three kernels:
//   kvd_build_kernel   block ids -> byte ranges (section 4.1) and coalescing of queued ranges
//                      (section 4.2) with a wave64 ballot + prefix scan; one workgroup.
//   kvd_pull_kernel    persistent grid; stages the coalesced descriptors in LDS and moves
//                      16 bytes per lane per access for every (layer, K/V) slab.
//   kvd_copy_kernel    plain streaming copy (counter calibration / practical ceiling).
//
// A descriptor is relative to the (layer 0, K) slab; the pull kernel adds the slab offset of
// each side, so one descriptor list serves every layer and both K and V (the receiver
// computes locations from the tensor metadata, section 4.1).

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "kvd.h"

namespace {

constexpr uint32_t kUnitBytes = 16;     // one lane moves 16 bytes per access
constexpr uint32_t kChunkUnits = 256;   // one wave step: 64 lanes x 4 accesses = 4 KiB
constexpr uint32_t kSegCap = 4096;      // descriptors per segment (LDS: 16 B each = 64 KiB)
constexpr uint32_t kBuildThreads = 1024;
constexpr uint32_t kPullThreads = 1024;
constexpr uint32_t kWave = 64;

enum Mode : uint32_t {
    kSpanTokenMajor = 0,  // same layout, any token sub-range of a block is one byte range
    kSpanHeadMajor = 1,   // both [head][token][dim] with several heads: one range per head
    kRelayoutHT2TH = 2,   // source [head][token][dim] -> destination [token][head][dim]
    kRelayoutTH2HT = 3    // source [token][head][dim] -> destination [head][token][dim]
};

// 16 bytes.  Offsets and lengths count 16-byte units.
//   byte-copy path: a = first unit past the end on the source side (length = a - src16)
//   re-layout path: a = src_token | dst_token << 10 | num_tokens << 20; src16/dst16 = block base
struct Desc {
    uint32_t src16;
    uint32_t dst16;
    uint32_t a;
    uint32_t prefix;  // 4 KiB wave steps needed by all earlier descriptors of the segment
};

struct SegHeader {
    uint32_t n_desc;
    uint32_t n_chunks;
    uint32_t layer_begin;
    uint32_t layer_end;
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
    uint32_t mode;
    FastDiv div_du, div_hkdu, div_piecedu, div_tb_src, div_tb_dst;
};

// ------------------------------------------------------------------ build: translate + coalesce

struct BuildArgs {
    const int32_t *src_table;  // this request's tables (device-visible pinned host memory)
    const int32_t *dst_table;
    Desc *desc;                // the segment's descriptor array
    SegHeader *seg;
    uint32_t seq_len;
    uint32_t j_begin, j_end;   // transactions of this request that go into this segment
    uint32_t n_single;         // head-major, equal block size: leading whole-block transactions
    uint32_t layer_begin, layer_end;
    uint32_t fresh;            // 1: the segment is empty (header contents are stale)
    uint32_t no_coalesce;
};

struct Txn {
    uint32_t s16, d16, len16, meta;
};

// Section 4.1: block id -> offset through the strides.  Transaction j of a request, in the
// order Transfer() is called for its blocks.
__device__ __forceinline__ Txn make_txn(const Geo &g, const BuildArgs &a, uint32_t j)
{
    uint32_t piece, head = 0;
    bool per_head = false;
    if (g.mode == kSpanHeadMajor) {
        if (g.tb_src == g.tb_dst) {
            if (j < a.n_single) {
                piece = j;
            } else {
                piece = a.n_single;
                head = j - a.n_single;
                per_head = true;
            }
        } else {
            piece = j / g.hk;
            head = j - piece * g.hk;
            per_head = true;
        }
    } else {
        piece = j;
    }
    const uint32_t t0 = piece * g.piece_tokens;
    const uint32_t ntok = min(g.piece_tokens, a.seq_len - t0);
    const uint32_t sb_i = fdiv(t0, g.div_tb_src), db_i = fdiv(t0, g.div_tb_dst);
    const uint32_t st0 = t0 - sb_i * g.tb_src, dt0 = t0 - db_i * g.tb_dst;
    const uint32_t sbase = (uint32_t)a.src_table[sb_i] * g.src_block16;
    const uint32_t dbase = (uint32_t)a.dst_table[db_i] * g.dst_block16;
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

__device__ __forceinline__ uint32_t desc_chunks(const Geo &g, const Desc &d)
{
    uint32_t units = (g.mode >= kRelayoutHT2TH) ? (d.a >> 20) * g.hk * g.du : d.a - d.src16;
    return (units + kChunkUnits - 1) / kChunkUnits;
}

__global__ __launch_bounds__(kBuildThreads) void kvd_build_kernel(Geo g, BuildArgs a)
{
    __shared__ uint32_t s_end_s[kBuildThreads];
    __shared__ uint32_t s_end_d[kBuildThreads];
    __shared__ uint8_t s_brk[kBuildThreads];
    __shared__ uint32_t s_wave[kBuildThreads / kWave];

    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const bool relayout = g.mode >= kRelayoutHT2TH;
    const bool never_merge = relayout || a.no_coalesce;
    const uint32_t n0 = a.fresh ? 0u : a.seg->n_desc;

    // The queue's last transaction so far: a new transaction that continues it on both sides
    // is merged into it, also when it belongs to another request (section 4.2).
    bool have_prev = false;
    uint32_t prev_s = 0, prev_d = 0;
    if (n0 > 0 && !never_merge) {
        Desc p = a.desc[n0 - 1];
        have_prev = true;
        prev_s = p.a;
        prev_d = p.dst16 + (p.a - p.src16);
    }
    const bool had_open = have_prev;
    uint32_t runs = n0;

    for (uint32_t tile = a.j_begin; tile < a.j_end; tile += kBuildThreads) {
        const uint32_t j = tile + tid;
        const bool valid = j < a.j_end;
        Txn t = {0, 0, 0, 0};
        if (valid) t = make_txn(g, a, j);
        s_end_s[tid] = t.s16 + t.len16;
        s_end_d[tid] = t.d16 + t.len16;
        __syncthreads();
        uint32_t ps = prev_s, pd = prev_d;
        bool hp = have_prev;
        if (tid > 0) {
            ps = s_end_s[tid - 1];
            pd = s_end_d[tid - 1];
            hp = true;
        }
        const uint32_t tile_last = min(kBuildThreads, a.j_end - tile) - 1;
        const uint32_t next_prev_s = s_end_s[tile_last], next_prev_d = s_end_d[tile_last];

        // break flag: this transaction starts a new descriptor
        const bool brk = valid && (never_merge || !hp || ps != t.s16 || pd != t.d16);
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
                a.desc[run].src16 = t.s16;
                a.desc[run].dst16 = t.d16;
                if (relayout) a.desc[run].a = t.meta;
            }
            // the last member of a descriptor (so far) records where it ends; a later tile or
            // a later request that continues it overwrites this
            const bool closes = (tid == tile_last) || s_brk[tid + 1];
            if (!relayout && closes) a.desc[run].a = t.s16 + t.len16;
        }
        runs += total;
        prev_s = next_prev_s;
        prev_d = next_prev_d;
        have_prev = true;
        __syncthreads();
    }

    // chunk prefix over the descriptors that are new or were extended
    const uint32_t n1 = runs;
    const uint32_t from = had_open ? n0 - 1 : n0;
    uint32_t carry = 0;
    if (from > 0) {
        Desc p = a.desc[from - 1];
        carry = p.prefix + desc_chunks(g, p);
    }
    for (uint32_t base = from; base < n1; base += kBuildThreads) {
        const uint32_t i = base + tid;
        const bool v = i < n1;
        Desc d = {0, 0, 0, 0};
        if (v) d = a.desc[i];
        const uint32_t c = v ? desc_chunks(g, d) : 0u;
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
    if (tid == 0) {
        a.seg->n_desc = n1;
        a.seg->n_chunks = carry;
        a.seg->layer_begin = a.layer_begin;
        a.seg->layer_end = a.layer_end;
    }
}

// ------------------------------------------------------------------ pull

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct PullArgs {
    const unsigned char *src_base;
    unsigned char *dst_base;
    const Desc *desc;       // n_segments arrays of kSegCap descriptors
    const SegHeader *segs;
    uint32_t n_segments;
    uint32_t lds_cap;       // descriptors the dynamic LDS can hold
};

__device__ __forceinline__ uint32_t find_desc(const uint32_t *l_prefix, uint32_t n, uint32_t c)
{
    // largest i with prefix[i] <= c
    uint32_t lo = 0, hi = n;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (l_prefix[mid] <= c) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ __launch_bounds__(kPullThreads) void kvd_pull_kernel(Geo g, PullArgs a)
{
    extern __shared__ uint32_t lds[];
    uint32_t *l_prefix = lds;
    uint32_t *l_src = lds + a.lds_cap;
    uint32_t *l_dst = lds + 2 * a.lds_cap;
    uint32_t *l_a = lds + 3 * a.lds_cap;

    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1);
    const uint32_t waves_per_block = blockDim.x / kWave;
    const uint32_t W = blockIdx.x * waves_per_block + tid / kWave;
    const uint32_t NW = gridDim.x * waves_per_block;
    const bool relayout = g.mode >= kRelayoutHT2TH;

    for (uint32_t s = 0; s < a.n_segments; ++s) {
        const SegHeader h = a.segs[s];
        const Desc *d = a.desc + (size_t)s * kSegCap;
        __syncthreads();
        for (uint32_t i = tid; i < h.n_desc; i += blockDim.x) {
            const Desc x = d[i];
            l_prefix[i] = x.prefix;
            l_src[i] = x.src16;
            l_dst[i] = x.dst16;
            l_a[i] = relayout ? x.a : x.a - x.src16;
        }
        __syncthreads();

        const uint32_t slabs = (h.layer_end - h.layer_begin) * 2;
        const uint32_t nc = h.n_chunks;
        if (nc == 0 || slabs == 0) continue;
        const uint32_t full_rounds = nc / NW;
        const uint32_t rem = nc - full_rounds * NW;
        // Rounds 0..full_rounds-1: wave W takes chunk r*NW + W through every slab.  Last round:
        // the remaining chunks are spread over all waves by also splitting the slabs.
        for (uint32_t r = 0; r <= full_rounds; ++r) {
            uint32_t c, slab0, slab_step;
            if (r < full_rounds) {
                c = r * NW + W;
                slab0 = 0;
                slab_step = 1;
            } else {
                if (rem == 0) break;
                const uint32_t phases = min(NW / rem, slabs);
                if (W >= rem * phases) break;
                slab0 = W / rem;
                c = full_rounds * NW + (W - slab0 * rem);
                slab_step = phases;
            }
            const uint32_t i = find_desc(l_prefix, h.n_desc, c);
            const uint32_t cl = c - l_prefix[i];
            uint32_t s_off[4], d_off[4];
            bool ok[4];
            if (!relayout) {
                const uint32_t left = l_a[i] - cl * kChunkUnits;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t u = k * kWave + lane;
                    ok[k] = u < left;
                    s_off[k] = l_src[i] + cl * kChunkUnits + u;
                    d_off[k] = l_dst[i] + cl * kChunkUnits + u;
                }
            } else {
                const uint32_t meta = l_a[i];
                const uint32_t st0 = meta & 1023u, dt0 = (meta >> 10) & 1023u, ntok = meta >> 20;
                const uint32_t units = ntok * g.hk * g.du;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t u = cl * kChunkUnits + k * kWave + lane;
                    ok[k] = u < units;
                    uint32_t tok, head, x;
                    if (g.mode == kRelayoutHT2TH) {
                        // destination order: token, head, dim
                        tok = fdiv(u, g.div_hkdu);
                        const uint32_t r2 = u - tok * g.hk * g.du;
                        head = fdiv(r2, g.div_du);
                        x = r2 - head * g.du;
                        s_off[k] = l_src[i] + (head * g.tb_src + st0 + tok) * g.du + x;
                        d_off[k] = l_dst[i] + ((dt0 + tok) * g.hk + head) * g.du + x;
                    } else {
                        // destination order: head, token, dim
                        head = (ntok == g.piece_tokens) ? fdiv(u, g.div_piecedu) : u / (ntok * g.du);
                        const uint32_t r2 = u - head * ntok * g.du;
                        tok = fdiv(r2, g.div_du);
                        x = r2 - tok * g.du;
                        s_off[k] = l_src[i] + ((st0 + tok) * g.hk + head) * g.du + x;
                        d_off[k] = l_dst[i] + (head * g.tb_dst + dt0 + tok) * g.du + x;
                    }
                }
            }
            for (uint32_t slab = slab0; slab < slabs; slab += slab_step) {
                const uint32_t layer = h.layer_begin + (slab >> 1), kv = slab & 1u;
                const unsigned char *sp = a.src_base + layer * g.src_layer_bytes + kv * g.src_kv_bytes;
                unsigned char *dp = a.dst_base + layer * g.dst_layer_bytes + kv * g.dst_kv_bytes;
                u32x4 v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (ok[k]) v[k] = *(const u32x4 *)(sp + (size_t)s_off[k] * kUnitBytes);
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (ok[k]) *(u32x4 *)(dp + (size_t)d_off[k] * kUnitBytes) = v[k];
            }
        }
    }
}

__global__ __launch_bounds__(256) void kvd_copy_kernel(u32x4 *__restrict__ dst,
                                                       const u32x4 *__restrict__ src, uint64_t units)
{
    // every workgroup step moves 256 lanes x 4 x 16 B = 16 KiB, grid-stride
    const uint64_t step = (uint64_t)gridDim.x * 1024;
    for (uint64_t base = (uint64_t)blockIdx.x * 1024; base < units; base += step) {
        u32x4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint64_t u = base + k * 256 + threadIdx.x;
            if (u < units) v[k] = src[u];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint64_t u = base + k * 256 + threadIdx.x;
            if (u < units) dst[u] = v[k];
        }
    }
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

struct SegHost {
    uint32_t txns;
    uint32_t layer_begin, layer_end;
};

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

struct kvd_plan {
    uint32_t tag;
    kvd_pool_desc_t src, dst;
    uint32_t max_requests, max_total_blocks, flags;
    Geo geo;
    uint64_t max_txns;
    uint32_t max_segments;
    // host bookkeeping
    std::vector<ReqHost> reqs;
    std::vector<SegHost> segs;
    std::vector<uint8_t> dst_used;  // one byte per destination block
    uint64_t used_src, used_dst, txns_total, payload_bytes;
    // device / pinned scratch (allocated on first use)
    bool allocated;
    int device;
    int num_cus;
    int32_t *tables_src, *tables_dst;  // pinned host, device-visible
    int32_t *tables_src_dev, *tables_dst_dev;
    Desc *desc_dev;
    SegHeader *segs_dev;
    hipEvent_t build_done;
    bool build_pending;
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
    if (d.stride_layer < 0 || d.stride_kv < 0 || d.stride_block < 0)
        return fail(KVD_ERR_INVALID, "negative stride");
    const uint64_t e = d.elem_bytes;
    const uint64_t tile = (uint64_t)d.block_tokens * d.num_kv_heads * d.head_dim;
    if ((uint64_t)d.stride_block < tile)
        return fail(KVD_ERR_INVALID, "stride_block smaller than one block");
    if (((uintptr_t)d.base % 16) || ((uint64_t)d.stride_layer * e % 16) ||
        ((uint64_t)d.stride_kv * e % 16) || ((uint64_t)d.stride_block * e % 16) ||
        ((uint64_t)d.head_dim * e % 16))
        return fail(KVD_ERR_INVALID, "base, strides and head_dim*elem_bytes must be multiples of 16 bytes");
    const uint64_t block_axis = ((uint64_t)(d.num_blocks - 1) * d.stride_block + tile) * e;
    if (block_axis >= (1ull << 36))
        return fail(KVD_ERR_RANGE, "block axis of one slab spans more than 64 GiB");
    *extent_out = ((uint64_t)(d.num_layers - 1) * d.stride_layer + (uint64_t)d.stride_kv) * e + block_axis;
    return KVD_OK;
}

uint32_t ceil_div(uint32_t a, uint32_t b) { return (a + b - 1) / b; }

// number of read transactions of one request per (layer, kv), and the leading whole-block ones
uint32_t request_txns(const Geo &g, uint32_t seq_len, uint32_t *n_single)
{
    const uint32_t pieces = ceil_div(seq_len, g.piece_tokens);
    *n_single = 0;
    if (g.mode != kSpanHeadMajor) return pieces;
    if (g.tb_src != g.tb_dst) return pieces * g.hk;
    const uint32_t whole = seq_len / g.tb_src;
    *n_single = whole;
    return whole + ((seq_len % g.tb_src) ? g.hk : 0);
}

int ensure_allocated(kvd_plan *p)
{
    if (p->allocated) return KVD_OK;
    KVD_HIP(hipGetDevice(&p->device));
    hipDeviceProp_t prop;
    KVD_HIP(hipGetDeviceProperties(&prop, p->device));
    p->num_cus = prop.multiProcessorCount;
    const size_t tb = (size_t)p->max_total_blocks * sizeof(int32_t);
    KVD_HIP(hipHostMalloc((void **)&p->tables_src, tb, hipHostMallocMapped));
    KVD_HIP(hipHostMalloc((void **)&p->tables_dst, tb, hipHostMallocMapped));
    KVD_HIP(hipHostGetDevicePointer((void **)&p->tables_src_dev, p->tables_src, 0));
    KVD_HIP(hipHostGetDevicePointer((void **)&p->tables_dst_dev, p->tables_dst, 0));
    KVD_HIP(hipMalloc((void **)&p->desc_dev, (size_t)p->max_segments * kSegCap * sizeof(Desc)));
    KVD_HIP(hipMalloc((void **)&p->segs_dev, (size_t)p->max_segments * sizeof(SegHeader)));
    KVD_HIP(hipMemset(p->segs_dev, 0, (size_t)p->max_segments * sizeof(SegHeader)));
    KVD_HIP(hipEventCreateWithFlags(&p->build_done, hipEventDisableTiming));
    p->allocated = true;
    return KVD_OK;
}

void release_plan(kvd_plan *p)
{
    if (p->allocated) {
        if (p->build_pending) (void)hipEventSynchronize(p->build_done);
        (void)hipHostFree(p->tables_src);
        (void)hipHostFree(p->tables_dst);
        (void)hipFree(p->desc_dev);
        (void)hipFree(p->segs_dev);
        (void)hipEventDestroy(p->build_done);
    }
    p->tag = 0;
    delete p;
}

kvd_plan *as_plan(void *h)
{
    kvd_plan *p = (kvd_plan *)h;
    return (p && p->tag == kPlanTag) ? p : nullptr;
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
    if (s.layout == d.layout || g.hk == 1)
        g.mode = (s.layout == KVD_LAYOUT_BTHD || g.hk == 1) ? kSpanTokenMajor : kSpanHeadMajor;
    else
        g.mode = (s.layout == KVD_LAYOUT_BHTD) ? kRelayoutHT2TH : kRelayoutTH2HT;
    g.div_du = make_fastdiv(g.du);
    g.div_hkdu = make_fastdiv(g.hk * g.du);
    g.div_piecedu = make_fastdiv(g.piece_tokens * g.du);
    g.div_tb_src = make_fastdiv(g.tb_src);
    g.div_tb_dst = make_fastdiv(g.tb_dst);

    // upper bound of transactions the plan can hold -> number of descriptor segments
    const uint64_t pieces_max = (uint64_t)max_total_blocks * (tmax / tmin);
    if (g.mode == kSpanHeadMajor)
        p->max_txns = (g.tb_src == g.tb_dst) ? pieces_max + (uint64_t)max_requests * g.hk
                                             : pieces_max * g.hk;
    else
        p->max_txns = pieces_max;
    p->max_segments = (uint32_t)((p->max_txns + kSegCap - 1) / kSegCap) + max_requests;
    p->dst_used.assign(d.num_blocks, 0);
    p->reqs.reserve(max_requests);
    p->allocated = false;
    p->build_pending = false;
    *out = p;
    return KVD_OK;
}

int kvd_plan_reset(kvd_plan_t *p)
{
    if (!as_plan(p)) return fail(KVD_ERR_INVALID, "not a plan handle");
    if (p->build_pending) {
        KVD_HIP(hipEventSynchronize(p->build_done));
        p->build_pending = false;
    }
    for (const ReqHost &r : p->reqs)
        for (uint32_t i = 0; i < r.n_dst; ++i)
            p->dst_used[(uint32_t)p->tables_dst[r.table_off_dst + i]] = 0;
    p->reqs.clear();
    p->segs.clear();
    p->used_src = p->used_dst = p->txns_total = p->payload_bytes = 0;
    return KVD_OK;
}

int kvd_build_descriptors(kvd_plan_t *p, const int32_t *src_tbl, uint32_t n_src,
                          const int32_t *dst_tbl, uint32_t n_dst, uint32_t seq_len,
                          uint32_t layer_begin, uint32_t layer_end, void *stream)
{
    if (!as_plan(p)) return fail(KVD_ERR_INVALID, "not a plan handle");
    if (layer_begin >= layer_end) return fail(KVD_ERR_INVALID, "empty layer range [%u, %u)", layer_begin, layer_end);
    if (layer_end > p->src.num_layers || layer_end > p->dst.num_layers)
        return fail(KVD_ERR_RANGE, "layer range [%u, %u) outside a pool", layer_begin, layer_end);
    if (seq_len == 0) return KVD_OK;
    if (!src_tbl || !dst_tbl) return fail(KVD_ERR_INVALID, "null block table");
    const Geo &g = p->geo;
    const uint32_t need_src = ceil_div(seq_len, g.tb_src), need_dst = ceil_div(seq_len, g.tb_dst);
    if (n_src < need_src || n_dst < need_dst)
        return fail(KVD_ERR_RANGE, "block table too short for %u tokens (source %u of %u, destination %u of %u)",
                    seq_len, n_src, need_src, n_dst, need_dst);
    for (uint32_t i = 0; i < need_src; ++i)
        if (src_tbl[i] < 0 || (uint32_t)src_tbl[i] >= p->src.num_blocks)
            return fail(KVD_ERR_RANGE, "source block id %d at entry %u outside [0, %u)", src_tbl[i], i, p->src.num_blocks);
    for (uint32_t i = 0; i < need_dst; ++i)
        if (dst_tbl[i] < 0 || (uint32_t)dst_tbl[i] >= p->dst.num_blocks)
            return fail(KVD_ERR_RANGE, "destination block id %d at entry %u outside [0, %u)", dst_tbl[i], i, p->dst.num_blocks);
    // every destination byte is written at most once per plan
    for (uint32_t i = 0; i < need_dst; ++i) {
        uint8_t &u = p->dst_used[(uint32_t)dst_tbl[i]];
        if (u) {
            for (uint32_t k = 0; k < i; ++k)  // undo this request's marks; earlier requests keep theirs
                if (p->dst_used[(uint32_t)dst_tbl[k]] == 2) p->dst_used[(uint32_t)dst_tbl[k]] = 0;
            return fail(KVD_ERR_ALIAS, "destination block %d (entry %u) is already a target in this plan", dst_tbl[i], i);
        }
        u = 2;
    }
    auto unmark = [&]() { for (uint32_t i = 0; i < need_dst; ++i) p->dst_used[(uint32_t)dst_tbl[i]] = 0; };
    if (p->reqs.size() >= p->max_requests) { unmark(); return fail(KVD_ERR_CAPACITY, "plan already holds %u requests", p->max_requests); }
    if (p->used_src + need_src > p->max_total_blocks || p->used_dst + need_dst > p->max_total_blocks) {
        unmark();
        return fail(KVD_ERR_CAPACITY, "plan holds at most %u block-table entries per side", p->max_total_blocks);
    }
    int rc = ensure_allocated(p);
    if (rc != KVD_OK) { unmark(); return rc; }
    for (uint32_t i = 0; i < need_dst; ++i) p->dst_used[(uint32_t)dst_tbl[i]] = 1;

    ReqHost r;
    r.table_off_src = (uint32_t)p->used_src;
    r.table_off_dst = (uint32_t)p->used_dst;
    r.n_src = need_src;
    r.n_dst = need_dst;
    r.seq_len = seq_len;
    r.layer_begin = layer_begin;
    r.layer_end = layer_end;
    memcpy(p->tables_src + r.table_off_src, src_tbl, (size_t)need_src * sizeof(int32_t));
    memcpy(p->tables_dst + r.table_off_dst, dst_tbl, (size_t)need_dst * sizeof(int32_t));
    p->used_src += need_src;
    p->used_dst += need_dst;
    p->reqs.push_back(r);
    p->payload_bytes += (uint64_t)seq_len * (layer_end - layer_begin) * 2 * g.hk * g.du * kUnitBytes;

    uint32_t n_single = 0;
    const uint32_t m = request_txns(g, seq_len, &n_single);
    p->txns_total += m;
    uint32_t j = 0;
    while (j < m) {
        bool fresh = false;
        if (p->segs.empty() || p->segs.back().txns == kSegCap ||
            p->segs.back().layer_begin != layer_begin || p->segs.back().layer_end != layer_end) {
            if (p->segs.size() >= p->max_segments) return fail(KVD_ERR_CAPACITY, "plan is out of descriptor segments");
            p->segs.push_back(SegHost{0, layer_begin, layer_end});
            fresh = true;
        }
        SegHost &sh = p->segs.back();
        const uint32_t take = std::min(m - j, kSegCap - sh.txns);
        const size_t si = p->segs.size() - 1;
        BuildArgs a;
        a.src_table = p->tables_src_dev + r.table_off_src;
        a.dst_table = p->tables_dst_dev + r.table_off_dst;
        a.desc = p->desc_dev + si * kSegCap;
        a.seg = p->segs_dev + si;
        a.seq_len = seq_len;
        a.j_begin = j;
        a.j_end = j + take;
        a.n_single = n_single;
        a.layer_begin = layer_begin;
        a.layer_end = layer_end;
        a.fresh = fresh ? 1u : 0u;
        a.no_coalesce = (p->flags & KVD_PLAN_NO_COALESCE) ? 1u : 0u;
        hipLaunchKernelGGL(kvd_build_kernel, dim3(1), dim3(kBuildThreads), 0, (hipStream_t)stream, g, a);
        KVD_HIP(hipGetLastError());
        sh.txns += take;
        j += take;
    }
    KVD_HIP(hipEventRecord(p->build_done, (hipStream_t)stream));
    p->build_pending = true;
    return KVD_OK;
}

int kvd_pull(kvd_plan_t *p, void *stream)
{
    if (!as_plan(p)) return fail(KVD_ERR_INVALID, "not a plan handle");
    if (p->segs.empty()) return KVD_OK;
    uint32_t lds_cap = 0;
    for (const SegHost &s : p->segs) lds_cap = std::max(lds_cap, s.txns);
    lds_cap = (lds_cap + 63u) & ~63u;
    PullArgs a;
    a.src_base = (const unsigned char *)p->src.base;
    a.dst_base = (unsigned char *)p->dst.base;
    a.desc = p->desc_dev;
    a.segs = p->segs_dev;
    a.n_segments = (uint32_t)p->segs.size();
    a.lds_cap = lds_cap;
    const uint32_t grid = (uint32_t)p->num_cus * 2;  // persistent: two 1024-thread workgroups per CU
    hipLaunchKernelGGL(kvd_pull_kernel, dim3(grid), dim3(kPullThreads), (size_t)lds_cap * 16,
                       (hipStream_t)stream, p->geo, a);
    KVD_HIP(hipGetLastError());
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
    const uint64_t tile = (uint64_t)g.tb_src * g.hk * row;
    const char *sb = (const char *)p->src.base;
    char *db = (char *)p->dst.base;
    for (const ReqHost &r : p->reqs) {
        const uint32_t whole = r.seq_len / g.tb_src, tail = r.seq_len % g.tb_src;
        for (uint32_t layer = r.layer_begin; layer < r.layer_end; ++layer)
            for (uint32_t kv = 0; kv < 2; ++kv) {
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
                        for (uint32_t h = 0; h < g.hk; ++h)
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
    out->num_segments = (uint32_t)p->segs.size();
    out->relayout = p->geo.mode >= kRelayoutHT2TH ? 1u : 0u;
    out->num_src_blocks = p->used_src;
    out->num_dst_blocks = p->used_dst;
    out->num_transactions = p->txns_total;
    out->payload_bytes = p->payload_bytes;
    if (!p->segs.empty()) {
        KVD_HIP(hipStreamSynchronize((hipStream_t)stream));
        std::vector<SegHeader> h(p->segs.size());
        KVD_HIP(hipMemcpy(h.data(), p->segs_dev, h.size() * sizeof(SegHeader), hipMemcpyDeviceToHost));
        for (const SegHeader &x : h) out->num_descriptors += x.n_desc;
    }
    return KVD_OK;
}

int kvd_plan_get_descriptors(kvd_plan_t *p, void *stream, kvd_span_t *spans, kvd_piece_t *pieces,
                             uint64_t cap, uint64_t *n_out)
{
    if (!as_plan(p) || !n_out) return fail(KVD_ERR_INVALID, "null or wrong handle");
    *n_out = 0;
    if (p->segs.empty()) return KVD_OK;
    const bool relayout = p->geo.mode >= kRelayoutHT2TH;
    if ((relayout && !pieces) || (!relayout && !spans))
        return fail(KVD_ERR_INVALID, "output array for this plan's descriptor kind is null");
    KVD_HIP(hipStreamSynchronize((hipStream_t)stream));
    std::vector<SegHeader> h(p->segs.size());
    KVD_HIP(hipMemcpy(h.data(), p->segs_dev, h.size() * sizeof(SegHeader), hipMemcpyDeviceToHost));
    std::vector<Desc> d(kSegCap);
    uint64_t n = 0;
    for (size_t s = 0; s < h.size(); ++s) {
        if (h[s].n_desc > kSegCap) return fail(KVD_ERR_HIP, "corrupt segment header");
        KVD_HIP(hipMemcpy(d.data(), p->desc_dev + s * kSegCap, h[s].n_desc * sizeof(Desc), hipMemcpyDeviceToHost));
        for (uint32_t i = 0; i < h[s].n_desc; ++i, ++n) {
            if (n >= cap) continue;
            if (relayout) {
                pieces[n].src_block = (int32_t)(d[i].src16 / p->geo.src_block16);
                pieces[n].dst_block = (int32_t)(d[i].dst16 / p->geo.dst_block16);
                pieces[n].src_token = d[i].a & 1023u;
                pieces[n].dst_token = (d[i].a >> 10) & 1023u;
                pieces[n].num_tokens = d[i].a >> 20;
            } else {
                spans[n].src_offset = (uint64_t)d[i].src16 * kUnitBytes;
                spans[n].dst_offset = (uint64_t)d[i].dst16 * kUnitBytes;
                spans[n].bytes = (uint64_t)(d[i].a - d[i].src16) * kUnitBytes;
            }
        }
    }
    *n_out = n;
    return KVD_OK;
}

int kvd_copy_plain(void *dst, const void *src, uint64_t bytes, void *stream)
{
    if (!dst || !src) return fail(KVD_ERR_INVALID, "null pointer");
    if ((bytes % 16) || ((uintptr_t)dst % 16) || ((uintptr_t)src % 16))
        return fail(KVD_ERR_INVALID, "pointers and size must be multiples of 16 bytes");
    if (bytes == 0) return KVD_OK;
    int dev = 0;
    KVD_HIP(hipGetDevice(&dev));
    int cus = 0;
    KVD_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    const uint64_t units = bytes / 16;
    const uint64_t want = (units + 1023) / 1024;
    const uint32_t grid = (uint32_t)std::min<uint64_t>(want, (uint64_t)cus * 32);
    hipLaunchKernelGGL(kvd_copy_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (u32x4 *)dst,
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
