// Hybrid cache assigner: host-side bookkeeping of the unified block pool (Section 4.3).
// Every block of the pool holds the K, V or hidden vectors of block_size consecutive token
// positions of one request; a request's cache map lists its blocks in position order.  A block
// is picked on demand by scanning for unused blocks, lowest block id first.
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <new>
#include <vector>
#include "apt_internal.h"

struct apt_pool {
    int64_t n_blocks;
    int32_t block_size, max_blocks, max_requests;
    int64_t n_free;
    int64_t scan_from;                    // every block below this id is in use
    std::vector<uint8_t> used;            // [n_blocks]
    std::vector<int32_t> map;             // [max_requests][2][max_blocks], -1 = no block
    std::vector<int32_t> len;             // tokens of the slot, 0 = slot empty
    std::vector<uint8_t> kind;
};

namespace {
inline int64_t blocks_for(const apt_pool* p, int64_t n_tokens) { return (n_tokens + p->block_size - 1) / p->block_size; }
inline int rows_of(uint8_t kind) { return kind == APT_KIND_KV ? 2 : 1; }

int64_t take_lowest_unused(apt_pool* p) {
    int64_t b = p->scan_from;
    while (p->used[b]) ++b;               // the caller has checked that an unused block exists
    p->used[b] = 1;
    p->scan_from = b + 1;
    --p->n_free;
    return b;
}
void give_back(apt_pool* p, int64_t b) {
    p->used[b] = 0;
    if (b < p->scan_from) p->scan_from = b;
    ++p->n_free;
}
// grows the map of `slot` (kind already set) from `have` to `want` logical blocks
void grow(apt_pool* p, int32_t slot, int64_t have, int64_t want) {
    int32_t* m = p->map.data() + (int64_t)slot * 2 * p->max_blocks;
    for (int64_t i = have; i < want; ++i)
        for (int row = 0; row < rows_of(p->kind[slot]); ++row) m[row * p->max_blocks + i] = (int32_t)take_lowest_unused(p);
}
}  // namespace

extern "C" int apt_pool_create(int64_t n_blocks, int32_t block_size, int32_t max_blocks_per_req, int32_t max_requests,
                               apt_pool** out) {
    if (!out || n_blocks < 1 || n_blocks > 0x7fffffff || block_size < 1 || max_blocks_per_req < 1 || max_requests < 1)
        return APT_EINVAL;
    apt_pool* p = new (std::nothrow) apt_pool;
    if (!p) return APT_EINVAL;
    p->n_blocks = n_blocks;
    p->block_size = block_size;
    p->max_blocks = max_blocks_per_req;
    p->max_requests = max_requests;
    p->n_free = n_blocks;
    p->scan_from = 0;
    p->used.assign((size_t)n_blocks, 0);
    p->map.assign((size_t)max_requests * 2 * max_blocks_per_req, -1);
    p->len.assign((size_t)max_requests, 0);
    p->kind.assign((size_t)max_requests, 0);
    *out = p;
    return APT_OK;
}

extern "C" void apt_pool_destroy(apt_pool* p) { delete p; }

extern "C" int apt_pool_free_blocks(const apt_pool* p, int64_t* n_free) {
    if (!p || !n_free) return APT_EINVAL;
    *n_free = p->n_free;
    return APT_OK;
}

extern "C" int apt_pool_blocks_needed(const apt_pool* p, uint8_t kind, int32_t n_tokens, int64_t* n) {
    if (!p || !n || n_tokens < 0 || kind > APT_KIND_HIDDEN) return APT_EINVAL;
    *n = blocks_for(p, n_tokens) * rows_of(kind);
    return APT_OK;
}

extern "C" int apt_pool_assign(apt_pool* p, int32_t slot, uint8_t kind, int32_t n_tokens) {
    if (!p || slot < 0 || slot >= p->max_requests || kind > APT_KIND_HIDDEN || n_tokens < 1) return APT_EINVAL;
    if (p->len[slot] != 0) return APT_EINVAL;                 // slot in use
    const int64_t nb = blocks_for(p, n_tokens);
    if (nb > p->max_blocks) return APT_ERANGE;
    if (nb * rows_of(kind) > p->n_free) return APT_EFULL;
    p->kind[slot] = kind;
    p->len[slot] = n_tokens;
    grow(p, slot, 0, nb);
    return APT_OK;
}

extern "C" int apt_pool_extend(apt_pool* p, int32_t slot, int32_t n_tokens) {
    if (!p || slot < 0 || slot >= p->max_requests) return APT_EINVAL;
    if (p->len[slot] == 0 || n_tokens < p->len[slot]) return APT_EINVAL;
    const int64_t have = blocks_for(p, p->len[slot]), want = blocks_for(p, n_tokens);
    if (want > p->max_blocks) return APT_ERANGE;
    if ((want - have) * rows_of(p->kind[slot]) > p->n_free) return APT_EFULL;
    grow(p, slot, have, want);
    p->len[slot] = n_tokens;
    return APT_OK;
}

extern "C" int apt_pool_release(apt_pool* p, int32_t slot) {
    if (!p || slot < 0 || slot >= p->max_requests || p->len[slot] == 0) return APT_EINVAL;
    int32_t* m = p->map.data() + (int64_t)slot * 2 * p->max_blocks;
    const int64_t nb = blocks_for(p, p->len[slot]);
    for (int row = 0; row < rows_of(p->kind[slot]); ++row)
        for (int64_t i = 0; i < nb; ++i) {
            give_back(p, m[row * p->max_blocks + i]);
            m[row * p->max_blocks + i] = -1;
        }
    p->len[slot] = 0;
    return APT_OK;
}

extern "C" int apt_pool_switch_kind(apt_pool* p, int32_t slot, uint8_t new_kind) {
    if (!p || slot < 0 || slot >= p->max_requests || p->len[slot] == 0 || new_kind > APT_KIND_HIDDEN) return APT_EINVAL;
    if (new_kind == p->kind[slot]) return APT_OK;
    const int32_t n = p->len[slot];
    const int64_t nb = blocks_for(p, n);
    // the old blocks are discarded first, so they count as free for the new cache
    if (nb * rows_of(new_kind) > p->n_free + nb * rows_of(p->kind[slot])) return APT_EFULL;
    apt_pool_release(p, slot);
    return apt_pool_assign(p, slot, new_kind, n);
}

extern "C" int apt_pool_export(const apt_pool* p, const int32_t* slots, int B, int32_t* block_tables, int32_t* ctx_lens,
                               uint8_t* cache_kind) {
    if (!p || !slots || B < 1 || !block_tables || !ctx_lens || !cache_kind) return APT_EINVAL;
    for (int r = 0; r < B; ++r) {
        const int32_t s = slots[r];
        if (s < 0 || s >= p->max_requests || p->len[s] == 0) return APT_EINVAL;
        memcpy(block_tables + (int64_t)r * 2 * p->max_blocks, p->map.data() + (int64_t)s * 2 * p->max_blocks,
               sizeof(int32_t) * 2 * p->max_blocks);
        ctx_lens[r] = p->len[s];
        cache_kind[r] = p->kind[s];
    }
    return APT_OK;
}
