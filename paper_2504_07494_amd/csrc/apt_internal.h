// Internal definitions shared by the host planner and the kernel launchers.
#pragma once
#include <stdint.h>
#include "apt_hybrid.h"

// Plan blob: int32 words.
enum {
    APT_PW_MAGIC = 0,
    APT_PW_BATCH = 1,
    APT_PW_HEADS = 2,
    APT_PW_NITEMS = 3,
    APT_PW_NHIDDEN = 4,
    APT_PW_NPARTIALS = 5,
    APT_PW_HCHUNK = 6,
    APT_PW_KCHUNK = 7,
    APT_PW_HIMPL = 8,
    APT_PW_ITEMS_OFF = 9,   // word offset of items[]
    APT_PW_TOK_LO = 10,
    APT_PW_TOK_HI = 11,
    APT_PW_HTOK_LO = 12,
    APT_PW_HTOK_HI = 13,
    APT_PW_HEAD_DIM = 14,
    APT_PW_WORDS = 15,      // total words of the blob
    APT_PW_QUEUE0 = 16,     // 9 words: start of each hidden-kind queue (in items), then the end
    APT_PW_KV_TICKET = 25,  // device copy only: next KV-kind item to hand out (0 between launches)
    APT_PW_D_MODEL = 26,    // the shape the plan was made for
    APT_PW_BLOCK_SIZE = 27,
    APT_PW_MAX_BLOCKS = 28,
    APT_PW_DTYPE = 29,
    APT_PW_NHIDREQ = 30,    // number of hidden-kind requests
    APT_PW_HEADER = 32
};
#define APT_N_QUEUES 8
#define APT_PLAN_MAGIC 0x41505431

// Tokens per work item.
#define APT_DEFAULT_KV_CHUNK 512         // shortest range the planner chooses by itself; it doubles it (to at most
#define APT_MAX_AUTO_KV_CHUNK 2048       // this) while the batch still yields APT_KV_ITEMS_TARGET KV-kind items:
#define APT_KV_ITEMS_TARGET 2048         // two per workgroup slot of a 256-CU device at four workgroups per CU
#define APT_MFMA_HIDDEN_CHUNK 320       // token rows of the MFMA kernel's tile: 320 ...
#define APT_MFMA_HIDDEN_CHUNK_SMALL 256 // ... or 256 (default for d_model < APT_MFMA_LARGE_TILE_D_MODEL)
#define APT_MFMA_LARGE_TILE_D_MODEL 8192
#define APT_DEFAULT_VALU_HIDDEN_CHUNK 32
#define APT_MAX_VALU_HIDDEN_CHUNK 64
#define APT_KV_MAX_PAGES_PER_WAVE 64
#define APT_ABSORBED_HEAD_GROUPS 4       // absorbed-weight kernels: threads of a workgroup = 64 x 4 (token or column
#define APT_ABSORBED_HEADS_PER_THREAD 10 // group, head group), 8 tokens/columns x 10 heads per thread
#define APT_ABSORBED_CHUNK 512           // = 64 groups x 8 tokens
#define APT_ABSORBED_OUT_ROWS 256        // d_model rows per partial of the output projection

// per-request arrays of the plan blob, each B words, starting at APT_PW_HEADER
enum {
    APT_PA_SPLIT_COUNT = 0,    // ranges of the request
    APT_PA_WS_OFFSET = 1,      // its first partial
    APT_PA_KIND = 2,           // APT_KIND_*
    APT_PA_CTX_LEN = 3,        // cached tokens
    APT_PA_HID_INDEX = 4,      // hidden-kind requests only (-1 otherwise): index among them,
    APT_PA_HID_TOK_OFF = 5,    //   tokens of the hidden-kind requests before it,
    APT_PA_HID_CHUNK_OFF = 6,  //   ranges of the hidden-kind requests before it
    APT_PA_HID_REQ = 7,        // entry i: the request that is hidden-kind request i (-1 past their number)
    APT_PA_COUNT = 8
};

struct apt_resolved {
    apt_shape s;        // chunks and hidden_impl filled in
    int elem_bytes;
    bool kv_auto;       // kv_chunk was 0: s.kv_chunk holds the shortest range, the planner may choose a longer one
};

// Whether c tokens can be a KV-kind range of this shape (whole blocks, within the item kernel's page loop).
static inline bool apt_kv_chunk_ok(int c, int block_size) {
    return c >= block_size && c % block_size == 0 && c / block_size <= 4 * APT_KV_MAX_PAGES_PER_WAVE;
}

// Validates a shape and fills the defaults.  Returns an apt_status.
int apt_resolve(const apt_shape* in, apt_resolved* out);

static inline uint64_t apt_align256(uint64_t v) { return (v + 255u) & ~(uint64_t)255u; }

// Workspace sections.  Always: the partials (per slot head_dim floats of un-normalised output, then (m, l)).
// Absorbed-weight hidden path in addition (fp32), with KS = ceil(d / 512) slices of d_model: absorbed queries
// QT [n_hid_req][H][d] (16-bit inputs: [n_hid_req][d / 32][parts * 64][32] 16-bit parts), score offsets CB [n_hid_req][H], score partials S [KS][H][hidden_tokens] (slice 0 then
// holds the scores), statistics ML [n_hid_req][H] (m, l), the partial weighted sums YP [n_hidden_chunks][H][d]
// the output partials OP [ceil(d / 256)][n_hid_req][H][hd], and (16-bit inputs) the softmax weights PP as 16-bit parts.
struct apt_ws_layout {
    uint64_t acc, ml, qt, cb, s, stat, yp, op, pp, total;
};
static inline apt_ws_layout apt_ws_sections(int64_t n_partials, int H, int hd, int himpl, int64_t n_hid_req,
                                            int64_t hidden_tokens, int64_t n_hid_chunks, int d, int dtype) {
    apt_ws_layout L;
    const uint64_t slots = (uint64_t)n_partials * (uint64_t)H;
    L.acc = 0;
    L.ml = slots * (uint64_t)hd * 4u;
    uint64_t end = L.ml + slots * 8u;
    L.qt = L.cb = L.s = L.stat = L.yp = L.op = L.pp = 0;
    if (himpl == APT_HIDDEN_ABSORBED) {
        const uint64_t ks = (uint64_t)(d + APT_ABSORBED_CHUNK - 1) / APT_ABSORBED_CHUNK;
        L.qt = apt_align256(end);
        // 16-bit inputs: QT is kept as 16-bit parts (2 for fp16, 3 for bf16) of the heads padded to a multiple of 64 instead
        const uint64_t head_groups = (uint64_t)(H + 63) / 64;
        const uint64_t qt_per_elem = dtype == APT_F32 ? (uint64_t)H * 4u : head_groups * (dtype == APT_F16 ? 256u : 384u);
        L.cb = apt_align256(L.qt + (uint64_t)n_hid_req * d * qt_per_elem);
        L.s = apt_align256(L.cb + (uint64_t)n_hid_req * H * 4u);
        L.stat = apt_align256(L.s + ks * (uint64_t)hidden_tokens * H * 4u);
        L.yp = apt_align256(L.stat + (uint64_t)n_hid_req * H * 8u);
        L.op = apt_align256(L.yp + (uint64_t)n_hid_chunks * H * d * 4u);
        const uint64_t os = (uint64_t)(d + APT_ABSORBED_OUT_ROWS - 1) / APT_ABSORBED_OUT_ROWS;
        L.pp = apt_align256(L.op + os * (uint64_t)n_hid_req * H * hd * 4u);
        // 16-bit inputs: the softmax weights as 16-bit parts, 16 tiles of 32 tokens per range, 64 padded heads
        end = L.pp + (dtype == APT_F32 ? 0u : (uint64_t)n_hid_chunks * 16u * 32u * qt_per_elem);
    }
    L.total = end;
    return L;
}
