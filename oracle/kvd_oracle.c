/*
 * CPU oracle for the paged KV-cache transfer of KVDirect (arXiv 2501.14743).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the GPU library and must never be called from a product path.
 *
 * Everything is integer / raw-byte work, so every result is exact.
 *
 * Notation follows the paper, section 4.1: a KV cache tensor has five axes
 * whose roles are B (blocks), KV (K or V), L (tokens inside a block), H (heads)
 * and D (head dimension).  The order of the axes is free; Shape and Stride are
 * listed in the same order as Dims, strides count elements.  There is one such
 * tensor per model layer.
 *
 * Pins (tests/test_oracle_pins.py): the worked example of section 4.1
 * (offsets of block 8, span size, blocks 0 and 1 merging), the queue example
 * of section 4.2 (R1 0->5 merges with R2 1->6), closed-form sizes from
 * sections 3 and 5.1, an element-by-element brute force with write counts,
 * unique-id closed form, sentinel preservation, round trip, and the special
 * case that reduces to one memcpy.  Nothing here is "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { KVDO_B = 0, KVDO_KV = 1, KVDO_L = 2, KVDO_H = 3, KVDO_D = 4 };

typedef struct {
    unsigned char *address; /* base address of the tensor (section 4.1, item i)   */
    int32_t dims[5];        /* role of every axis, in axis order (item ii)        */
    int64_t shape[5];       /* extent of every axis, same order as dims (item iii) */
    int64_t stride[5];      /* elements between neighbours on every axis (item iv) */
    int64_t elem_bytes;     /* bytes per element (2 for bfloat16 in the example)   */
} kvdo_tensor;

static int axis_of(const kvdo_tensor *t, int role)
{
    for (int a = 0; a < 5; ++a)
        if (t->dims[a] == role)
            return a;
    return -1;
}

/* Section 4.1, address translation: the starting offset of an element is the
 * dot product of its index with the stride vector, times the element size.
 * `index` is given in the tensor's own axis order. */
int64_t kvdo_offset_bytes(const kvdo_tensor *t, const int64_t index[5])
{
    int64_t dot = 0;
    for (int a = 0; a < 5; ++a)
        dot += index[a] * t->stride[a];
    return dot * t->elem_bytes;
}

/* Same dot product with the index given by role (block, kv, token, head, dim);
 * role_axis[r] is the axis that plays role r (see roles_to_axes). */
static void roles_to_axes(const kvdo_tensor *t, int role_axis[5])
{
    for (int r = 0; r < 5; ++r)
        role_axis[r] = axis_of(t, r);
}

static int64_t offset_by_role(const kvdo_tensor *t, const int role_axis[5], int64_t b, int64_t kv,
                              int64_t l, int64_t h, int64_t d)
{
    int64_t index[5];
    index[role_axis[KVDO_B]] = b;
    index[role_axis[KVDO_KV]] = kv;
    index[role_axis[KVDO_L]] = l;
    index[role_axis[KVDO_H]] = h;
    index[role_axis[KVDO_D]] = d;
    return kvdo_offset_bytes(t, index);
}

/* Section 4.1, transaction size: the contiguous space that covers the L, H
 * and D axes of one block is found from the one of these three axes that has
 * the largest stride: its extent times its stride, in bytes. */
int64_t kvdo_block_span_bytes(const kvdo_tensor *t)
{
    const int roles[3] = { KVDO_L, KVDO_H, KVDO_D };
    int best = axis_of(t, roles[0]);
    for (int i = 1; i < 3; ++i) {
        int a = axis_of(t, roles[i]);
        if (t->stride[a] > t->stride[best])
            best = a;
    }
    return t->shape[best] * t->stride[best] * t->elem_bytes;
}

/* Bytes of KV cache that belong to `tokens` tokens: K and V, every layer,
 * every KV head, every dimension (section 5.1 quotes this per token). */
int64_t kvdo_transfer_bytes(int64_t tokens, int64_t layers, int64_t kv_heads,
                            int64_t head_dim, int64_t elem_bytes)
{
    return tokens * layers * 2 * kv_heads * head_dim * elem_bytes;
}

/*
 * The transfer itself, written as its definition (sections 2.1 and 4.1):
 * token t of the request lives in the source pool at block src_table[t / Ls],
 * slot t % Ls, and must arrive in the destination pool at block
 * dst_table[t / Ld], slot t % Ld, for every layer of the range, for K and V,
 * for every head and every dimension.  Elements are copied as raw bytes.
 * Nothing else in either pool is touched.
 *
 * src[i] / dst[i] describe layer i.  Returns 0, or -1 when the two sides do
 * not describe the same kind of element.
 */
int kvdo_pull(const kvdo_tensor *src, const kvdo_tensor *dst,
              int64_t layer_begin, int64_t layer_end,
              const int32_t *src_table, const int32_t *dst_table,
              int64_t seq_len)
{
    for (int64_t layer = layer_begin; layer < layer_end; ++layer) {
        const kvdo_tensor *s = &src[layer];
        const kvdo_tensor *d = &dst[layer];
        int sa[5], da[5];
        roles_to_axes(s, sa);
        roles_to_axes(d, da);
        const int64_t Ls = s->shape[axis_of(s, KVDO_L)];
        const int64_t Ld = d->shape[axis_of(d, KVDO_L)];
        const int64_t H = s->shape[axis_of(s, KVDO_H)];
        const int64_t D = s->shape[axis_of(s, KVDO_D)];
        const int64_t e = s->elem_bytes;
        if (H != d->shape[axis_of(d, KVDO_H)] || D != d->shape[axis_of(d, KVDO_D)] ||
            e != d->elem_bytes)
            return -1;
        for (int64_t kv = 0; kv < 2; ++kv)
            for (int64_t t = 0; t < seq_len; ++t)
                for (int64_t h = 0; h < H; ++h)
                    for (int64_t x = 0; x < D; ++x) {
                        int64_t so = offset_by_role(s, sa, src_table[t / Ls], kv, t % Ls, h, x);
                        int64_t dofs = offset_by_role(d, da, dst_table[t / Ld], kv, t % Ld, h, x);
                        memcpy(d->address + dofs, s->address + so, (size_t)e);
                    }
    }
    return 0;
}

/* ---- read transactions and their coalescing (sections 4.1 and 4.2) ---- */

typedef struct {
    int64_t remote; /* byte offset in the source (remote, prefill) tensor   */
    int64_t local;  /* byte offset in the destination (local, decode) tensor */
    int64_t size;   /* bytes                                                 */
} kvdo_txn;

static int cmp_txn_remote(const void *a, const void *b)
{
    const kvdo_txn *x = (const kvdo_txn *)a, *y = (const kvdo_txn *)b;
    return (x->remote > y->remote) - (x->remote < y->remote);
}

/*
 * Read transactions of one request for one tensor, in the order the blocks
 * are handed to Transfer(): for kv = 0 or 1 only the K or only the V half, for
 * kv < 0 both, K then V of every block (a block "consists of the K and V" and
 * gives one transaction for each, section 4.1).  A transaction is a maximal byte
 * range that is contiguous on both sides and holds only tokens of the request
 * (only tokens below seq_len move).  They are found the slow way: list every
 * element of a (source block, destination block) pair with both its offsets,
 * order by source offset, and join neighbours that touch on both sides.  With
 * full blocks of equal size this gives the paper's one span per block.
 *
 * Returns the number of transactions, or -1 if `cap` is too small.
 */
int64_t kvdo_request_transactions(const kvdo_tensor *s, const kvdo_tensor *d, int64_t kv,
                                  const int32_t *src_table, const int32_t *dst_table,
                                  int64_t seq_len, kvdo_txn *out, int64_t cap)
{
    const int64_t Ls = s->shape[axis_of(s, KVDO_L)];
    const int64_t Ld = d->shape[axis_of(d, KVDO_L)];
    const int64_t H = s->shape[axis_of(s, KVDO_H)];
    const int64_t D = s->shape[axis_of(s, KVDO_D)];
    const int64_t e = s->elem_bytes;
    const int64_t max_tokens = Ls < Ld ? Ls : Ld;
    int sa[5], da[5];
    roles_to_axes(s, sa);
    roles_to_axes(d, da);
    kvdo_txn *elems = (kvdo_txn *)malloc((size_t)(max_tokens * H * D) * sizeof(kvdo_txn));
    int64_t n_out = 0;
    int64_t t0 = 0;
    while (t0 < seq_len) {
        /* tokens [t0, t1) share one source block and one destination block */
        int64_t t1 = t0 + 1;
        while (t1 < seq_len && t1 / Ls == t0 / Ls && t1 / Ld == t0 / Ld)
            ++t1;
        for (int64_t part = (kv < 0 ? 0 : kv); part <= (kv < 0 ? 1 : kv); ++part) {
            int64_t n = 0;
            for (int64_t t = t0; t < t1; ++t)
                for (int64_t h = 0; h < H; ++h)
                    for (int64_t x = 0; x < D; ++x) {
                        elems[n].remote = offset_by_role(s, sa, src_table[t / Ls], part, t % Ls, h, x);
                        elems[n].local = offset_by_role(d, da, dst_table[t / Ld], part, t % Ld, h, x);
                        elems[n].size = e;
                        ++n;
                    }
            qsort(elems, (size_t)n, sizeof(kvdo_txn), cmp_txn_remote);
            for (int64_t i = 0; i < n; ++i) {
                if (i > 0 && out[n_out - 1].remote + out[n_out - 1].size == elems[i].remote &&
                    out[n_out - 1].local + out[n_out - 1].size == elems[i].local) {
                    out[n_out - 1].size += elems[i].size;
                } else {
                    if (n_out == cap) {
                        free(elems);
                        return -1;
                    }
                    out[n_out++] = elems[i];
                }
            }
        }
        t0 = t1;
    }
    free(elems);
    return n_out;
}

/*
 * Section 4.2, coalescing: walk the queued read transactions in order and
 * merge a transaction into the one before it only when it continues that one
 * on BOTH the remote and the local side.  `out` may alias `in`.
 * Returns the number of merged transactions.
 */
int64_t kvdo_coalesce(const kvdo_txn *in, int64_t n, kvdo_txn *out)
{
    int64_t m = 0;
    for (int64_t i = 0; i < n; ++i) {
        kvdo_txn cur = in[i];
        if (m > 0 && out[m - 1].remote + out[m - 1].size == cur.remote &&
            out[m - 1].local + out[m - 1].size == cur.local)
            out[m - 1].size += cur.size;
        else
            out[m++] = cur;
    }
    return m;
}
