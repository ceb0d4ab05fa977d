// Host side of the library: status strings, shape checks, the ragged work
// partitioner and the cache-map range check.  No device code here.
#include <string.h>
#include <algorithm>
#include <vector>
#include "apt_internal.h"

extern "C" const char* apt_strerror(int status) {
    switch (status) {
    case APT_OK: return "ok";
    case APT_EINVAL: return "invalid argument";
    case APT_ESHAPE: return "unsupported or inconsistent shape";
    case APT_EDTYPE: return "unsupported dtype";
    case APT_EWORKSPACE: return "buffer too small";
    case APT_EHIP: return "HIP runtime error";
    case APT_ERANGE: return "value out of range";
    case APT_EFULL: return "not enough unused cache blocks";
    default: return "unknown status";
    }
}

extern "C" int apt_version(void) { return 100; }

static bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }

int apt_resolve(const apt_shape* in, apt_resolved* out) {
    if (!in || !out) return APT_EINVAL;
    apt_shape s = *in;
    if (s.dtype != APT_F32 && s.dtype != APT_F16 && s.dtype != APT_BF16) return APT_EDTYPE;
    if (s.out_dtype != APT_F32 && s.out_dtype != s.dtype) return APT_EDTYPE;
    const int e = s.dtype == APT_F32 ? 4 : 2;
    if (s.d_model < 1 || s.n_heads < 1 || s.max_blocks_per_req < 1 || s.reserved != 0) return APT_ESHAPE;
    if (s.head_dim != 64 && s.head_dim != 128) return APT_ESHAPE;
    if ((int64_t)s.n_heads * s.head_dim != s.d_model) return APT_ESHAPE;
    if (!is_pow2(s.block_size) || s.block_size > 64) return APT_ESHAPE;
    // a (block, head) run of the K/V layout is read in 1 KB wave loads
    const int lanes_per_row = s.head_dim * e / 16;
    if ((s.block_size * lanes_per_row) % 64 != 0) return APT_ESHAPE;
    if (!(s.softmax_scale == s.softmax_scale)) return APT_EINVAL;

    const bool mfma_ok = (s.dtype != APT_F32) && s.head_dim == 128 && (s.d_model % 128 == 0);
    if (s.hidden_impl == APT_HIDDEN_AUTO) s.hidden_impl = mfma_ok ? APT_HIDDEN_MFMA : APT_HIDDEN_VALU;
    if (s.hidden_impl == APT_HIDDEN_MFMA) {
        if (!mfma_ok) return APT_ESHAPE;
        // the larger tile moves fewer bytes per flop but costs more per item: it pays when an item's k loop is long
        if (s.hidden_chunk == 0)
            s.hidden_chunk = s.d_model >= APT_MFMA_LARGE_TILE_D_MODEL ? APT_MFMA_HIDDEN_CHUNK : APT_MFMA_HIDDEN_CHUNK_SMALL;
        if (s.hidden_chunk != APT_MFMA_HIDDEN_CHUNK && s.hidden_chunk != APT_MFMA_HIDDEN_CHUNK_SMALL) return APT_ESHAPE;
    } else if (s.hidden_impl == APT_HIDDEN_ABSORBED) {
        // heads: groups of 64 rows per operand part on the matrix cores (16-bit inputs), 4 x 10 register tiles otherwise
        const int max_heads = s.dtype == APT_F32 ? APT_ABSORBED_HEAD_GROUPS * APT_ABSORBED_HEADS_PER_THREAD : 128;
        if (s.d_model % 32 != 0 || s.n_heads > max_heads) return APT_ESHAPE;
        if (s.hidden_chunk == 0) s.hidden_chunk = APT_ABSORBED_CHUNK;
        if (s.hidden_chunk != APT_ABSORBED_CHUNK) return APT_ESHAPE;
    } else if (s.hidden_impl == APT_HIDDEN_VALU) {
        if (s.hidden_chunk == 0) s.hidden_chunk = APT_DEFAULT_VALU_HIDDEN_CHUNK;
        if (s.hidden_chunk < 1 || s.hidden_chunk > APT_MAX_VALU_HIDDEN_CHUNK) return APT_ESHAPE;
    } else {
        return APT_ESHAPE;
    }
    out->kv_auto = s.kv_chunk == 0;
    if (out->kv_auto) s.kv_chunk = APT_DEFAULT_KV_CHUNK;
    if (!apt_kv_chunk_ok(s.kv_chunk, s.block_size)) return APT_ESHAPE;
    out->s = s;
    out->elem_bytes = e;
    return APT_OK;
}

static int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

static size_t plan_words(int B, int64_t n_items) {
    size_t w = APT_PW_HEADER + APT_PA_COUNT * (size_t)B;
    w = (w + 3) & ~(size_t)3;
    return w + 4 * (size_t)n_items;
}

extern "C" int apt_plan_max_bytes(const apt_shape* s, int B, int max_ctx, size_t* bytes) {
    apt_resolved rs;
    int rc = apt_resolve(s, &rs);
    if (rc) return rc;
    if (B < 1 || max_ctx < 1 || !bytes) return APT_EINVAL;
    const int cmin = rs.s.hidden_chunk < rs.s.kv_chunk ? rs.s.hidden_chunk : rs.s.kv_chunk;
    const int64_t n_items = (int64_t)B * rs.s.n_heads * ceil_div64(max_ctx, cmin);
    *bytes = plan_words(B, n_items) * 4;
    return APT_OK;
}

extern "C" int apt_workspace_bytes(const apt_shape* s, int max_batch, int max_ctx, size_t* dev_bytes, size_t* host_bytes) {
    apt_resolved rs;
    int rc = apt_resolve(s, &rs);
    if (rc) return rc;
    if (max_batch < 1 || max_ctx < 1 || (!dev_bytes && !host_bytes)) return APT_EINVAL;
    if ((int64_t)max_ctx > (int64_t)rs.s.max_blocks_per_req * rs.s.block_size) return APT_ERANGE;
    // every workspace section grows with each of these counts, so the layout of their separate maxima bounds
    // the layout of any batch: ranges are most numerous when every request is of the kind with the shorter
    // chunk; the sections of the absorbed-weight path are largest when every request is hidden-kind
    const int cmin = rs.s.hidden_chunk < rs.s.kv_chunk ? rs.s.hidden_chunk : rs.s.kv_chunk;
    const int64_t n_partials = (int64_t)max_batch * ceil_div64(max_ctx, cmin);
    const int64_t hid_chunks = (int64_t)max_batch * ceil_div64(max_ctx, rs.s.hidden_chunk);
    if (n_partials * (int64_t)rs.s.n_heads > 0x7fffffff || (int64_t)max_batch * max_ctx > 0x7fffffff) return APT_ERANGE;
    if (dev_bytes)
        *dev_bytes = (size_t)apt_ws_sections(n_partials, rs.s.n_heads, rs.s.head_dim, rs.s.hidden_impl, max_batch,
                                             (int64_t)max_batch * max_ctx, hid_chunks, rs.s.d_model, rs.s.dtype).total;
    if (host_bytes) return apt_plan_max_bytes(s, max_batch, max_ctx, host_bytes);
    return APT_OK;
}

extern "C" int apt_plan(const apt_shape* s, const int32_t* ctx_lens, const uint8_t* cache_kind, int B,
                        void* plan_host, size_t plan_bytes, apt_plan_info* info) {
    apt_resolved rs;
    int rc = apt_resolve(s, &rs);
    if (rc) return rc;
    if (!ctx_lens || !cache_kind || !plan_host || B < 1) return APT_EINVAL;
    const int H = rs.s.n_heads;
    const int64_t max_len = (int64_t)rs.s.max_blocks_per_req * rs.s.block_size;

    // KV-kind range length left to the library: a short range costs an item's start-up and wind-down more often
    // per byte, a long one leaves too few items to fill the device; take the longest that still yields enough items
    if (rs.kv_auto) {
        for (int c = APT_MAX_AUTO_KV_CHUNK; c > rs.s.kv_chunk; c /= 2) {
            if (!apt_kv_chunk_ok(c, rs.s.block_size)) continue;
            int64_t kv_items = 0;
            for (int r = 0; r < B; ++r)
                if (cache_kind[r] == APT_KIND_KV && ctx_lens[r] > 0) kv_items += ceil_div64(ctx_lens[r], c) * H;
            if (kv_items >= APT_KV_ITEMS_TARGET) { rs.s.kv_chunk = c; break; }
        }
    }

    // pass 1: validate and count
    const bool absorbed = rs.s.hidden_impl == APT_HIDDEN_ABSORBED;
    int64_t n_partials = 0, n_hidden_items = 0, n_items = 0, tok = 0, htok = 0, n_hid_req = 0;
    for (int r = 0; r < B; ++r) {
        const int n = ctx_lens[r];
        if (n < 1) return APT_EINVAL;
        if (n > max_len) return APT_ERANGE;
        if (cache_kind[r] != APT_KIND_KV && cache_kind[r] != APT_KIND_HIDDEN) return APT_EINVAL;
        const bool hid = cache_kind[r] == APT_KIND_HIDDEN;
        const int64_t sp = ceil_div64(n, hid ? rs.s.hidden_chunk : rs.s.kv_chunk);
        const int64_t per_range = (hid && absorbed) ? 1 : H;      // absorbed: one item serves all heads
        n_partials += sp;
        n_items += sp * per_range;
        if (hid) { n_hidden_items += sp * per_range; htok += n; ++n_hid_req; }
        tok += n;
    }
    if (n_items > 0x7fffffff || n_partials * (int64_t)H > 0x7fffffff || htok > 0x7fffffff) return APT_ERANGE;
    const size_t words = plan_words(B, n_items);
    if (plan_bytes < words * 4) return APT_EWORKSPACE;

    int32_t* w = (int32_t*)plan_host;
    const size_t items_off = words - 4 * (size_t)n_items;
    memset(w, 0, items_off * 4);
    w[APT_PW_MAGIC] = APT_PLAN_MAGIC;
    w[APT_PW_BATCH] = B;
    w[APT_PW_HEADS] = H;
    w[APT_PW_NITEMS] = (int32_t)n_items;
    w[APT_PW_NHIDDEN] = (int32_t)n_hidden_items;
    w[APT_PW_NPARTIALS] = (int32_t)n_partials;
    w[APT_PW_HCHUNK] = rs.s.hidden_chunk;
    w[APT_PW_KCHUNK] = rs.s.kv_chunk;
    w[APT_PW_HIMPL] = rs.s.hidden_impl;
    w[APT_PW_ITEMS_OFF] = (int32_t)items_off;
    w[APT_PW_TOK_LO] = (int32_t)(tok & 0xffffffff);
    w[APT_PW_TOK_HI] = (int32_t)(tok >> 32);
    w[APT_PW_HTOK_LO] = (int32_t)(htok & 0xffffffff);
    w[APT_PW_HTOK_HI] = (int32_t)(htok >> 32);
    w[APT_PW_HEAD_DIM] = rs.s.head_dim;
    w[APT_PW_WORDS] = (int32_t)words;
    w[APT_PW_D_MODEL] = rs.s.d_model;
    w[APT_PW_BLOCK_SIZE] = rs.s.block_size;
    w[APT_PW_MAX_BLOCKS] = rs.s.max_blocks_per_req;
    w[APT_PW_DTYPE] = rs.s.dtype;
    w[APT_PW_NHIDREQ] = (int32_t)n_hid_req;

    int32_t* split_count = w + APT_PW_HEADER + APT_PA_SPLIT_COUNT * B;
    int32_t* ws_offset = w + APT_PW_HEADER + APT_PA_WS_OFFSET * B;
    int32_t* kind = w + APT_PW_HEADER + APT_PA_KIND * B;
    int32_t* hid_index = w + APT_PW_HEADER + APT_PA_HID_INDEX * B;
    int32_t* hid_tok_off = w + APT_PW_HEADER + APT_PA_HID_TOK_OFF * B;
    int32_t* hid_chunk_off = w + APT_PW_HEADER + APT_PA_HID_CHUNK_OFF * B;
    int32_t* hid_req = w + APT_PW_HEADER + APT_PA_HID_REQ * B;
    int32_t* ctx_len = w + APT_PW_HEADER + APT_PA_CTX_LEN * B;
    for (int r = 0; r < B; ++r) hid_req[r] = -1;
    int32_t run = 0, hi = 0, ht = 0, hc = 0;
    for (int r = 0; r < B; ++r) {
        const bool hid = cache_kind[r] == APT_KIND_HIDDEN;
        split_count[r] = (int32_t)ceil_div64(ctx_lens[r], hid ? rs.s.hidden_chunk : rs.s.kv_chunk);
        ws_offset[r] = run;
        run += split_count[r];
        kind[r] = cache_kind[r];
        ctx_len[r] = ctx_lens[r];
        if (hid) hid_req[hi] = r;
        hid_index[r] = hid ? hi : -1;
        hid_tok_off[r] = hid ? ht : -1;
        hid_chunk_off[r] = hid ? hc : -1;
        if (hid) { ++hi; ht += ctx_lens[r]; hc += split_count[r]; }
    }
    // pass 2: items.  Hidden kind first, in APT_N_QUEUES queues by head % 8; in a queue the
    // full ranges come first (request, range, head order), then the last, shorter ranges by
    // decreasing length.  Then the KV kind by decreasing range length.
    int32_t* it = w + items_off;
    int32_t* const it0 = it;
    std::vector<int32_t> tails;     // requests with a shorter last range, to be ordered by its length
    auto emit_kind = [&](uint8_t want, int c, int h_first, int h_step) {
        for (int r = 0; r < B; ++r) {       // full ranges
            if (cache_kind[r] != want) continue;
            const int nfull = ctx_lens[r] / c;
            for (int sp = 0; sp < nfull; ++sp)
                for (int h = h_first; h < H; h += h_step) {
                    it[0] = r; it[1] = h; it[2] = sp * c; it[3] = sp * c + c;
                    it += 4;
                }
        }
        tails.clear();
        for (int r = 0; r < B; ++r)
            if (cache_kind[r] == want && ctx_lens[r] % c != 0) tails.push_back(r);
        std::stable_sort(tails.begin(), tails.end(),
                         [&](int32_t a, int32_t b) { return ctx_lens[a] % c > ctx_lens[b] % c; });
        for (int32_t r : tails) {
            const int t0 = (ctx_lens[r] / c) * c;
            for (int h = h_first; h < H; h += h_step) {
                it[0] = r; it[1] = h; it[2] = t0; it[3] = ctx_lens[r];
                it += 4;
            }
        }
    };
    for (int x = 0; x < APT_N_QUEUES; ++x) {
        w[APT_PW_QUEUE0 + x] = (int32_t)((it - it0) / 4);
        if (!absorbed) {
            emit_kind(APT_KIND_HIDDEN, rs.s.hidden_chunk, x, APT_N_QUEUES);
        } else if (x == 0) {           // one item per range, by request and range, all in queue 0
            for (int r = 0; r < B; ++r) {
                if (cache_kind[r] != APT_KIND_HIDDEN) continue;
                for (int sp = 0; sp < split_count[r]; ++sp) {
                    const int t0 = sp * rs.s.hidden_chunk;
                    it[0] = r; it[1] = 0; it[2] = t0;
                    it[3] = t0 + rs.s.hidden_chunk < ctx_lens[r] ? t0 + rs.s.hidden_chunk : ctx_lens[r];
                    it += 4;
                }
            }
        }
    }
    w[APT_PW_QUEUE0 + APT_N_QUEUES] = (int32_t)((it - it0) / 4);
    emit_kind(APT_KIND_KV, rs.s.kv_chunk, 0, 1);
    if (info) return apt_plan_get_info(plan_host, info);
    return APT_OK;
}

extern "C" int apt_plan_get_info(const void* plan_host, apt_plan_info* info) {
    if (!plan_host || !info) return APT_EINVAL;
    const int32_t* w = (const int32_t*)plan_host;
    if (w[APT_PW_MAGIC] != APT_PLAN_MAGIC) return APT_EINVAL;
    memset(info, 0, sizeof(*info));
    info->batch = w[APT_PW_BATCH];
    info->n_items = w[APT_PW_NITEMS];
    info->n_hidden_items = w[APT_PW_NHIDDEN];
    info->n_partials = w[APT_PW_NPARTIALS];
    info->hidden_chunk = w[APT_PW_HCHUNK];
    info->kv_chunk = w[APT_PW_KCHUNK];
    info->hidden_impl = w[APT_PW_HIMPL];
    info->total_tokens = ((int64_t)w[APT_PW_TOK_HI] << 32) | (uint32_t)w[APT_PW_TOK_LO];
    info->hidden_tokens = ((int64_t)w[APT_PW_HTOK_HI] << 32) | (uint32_t)w[APT_PW_HTOK_LO];
    info->plan_bytes = (uint64_t)(uint32_t)w[APT_PW_WORDS] * 4u;
    info->workspace_bytes = apt_ws_sections(w[APT_PW_NPARTIALS], w[APT_PW_HEADS], w[APT_PW_HEAD_DIM], w[APT_PW_HIMPL],
                                            w[APT_PW_NHIDREQ], info->hidden_tokens, w[APT_PW_NHIDDEN], w[APT_PW_D_MODEL],
                                            w[APT_PW_DTYPE]).total;
    return APT_OK;
}

extern "C" int apt_validate_host(const apt_shape* s, const int32_t* ctx_lens, const uint8_t* cache_kind,
                                 const int32_t* block_tables, int B, int64_t n_pool_blocks) {
    apt_resolved rs;
    int rc = apt_resolve(s, &rs);
    if (rc) return rc;
    if (!ctx_lens || !cache_kind || !block_tables || B < 1 || n_pool_blocks < 1) return APT_EINVAL;
    const int mb = rs.s.max_blocks_per_req, bs = rs.s.block_size;
    // the MFMA kernel addresses hidden rows by 32-bit offsets in 16-byte units
    if (rs.s.hidden_impl == APT_HIDDEN_MFMA &&
        (uint64_t)n_pool_blocks * (uint64_t)bs * (uint64_t)rs.s.d_model * (uint64_t)rs.elem_bytes > ((uint64_t)1 << 36))
        return APT_ERANGE;
    for (int r = 0; r < B; ++r) {
        const int n = ctx_lens[r];
        if (n < 1) return APT_EINVAL;
        if (cache_kind[r] != APT_KIND_KV && cache_kind[r] != APT_KIND_HIDDEN) return APT_EINVAL;
        const int nb = (n + bs - 1) / bs;
        if (nb > mb) return APT_ERANGE;
        const int rows = cache_kind[r] == APT_KIND_KV ? 2 : 1;
        for (int row = 0; row < rows; ++row)
            for (int i = 0; i < nb; ++i) {
                const int32_t b = block_tables[((int64_t)r * 2 + row) * mb + i];
                if (b < 0 || b >= n_pool_blocks) return APT_ERANGE;
            }
    }
    return APT_OK;
}
