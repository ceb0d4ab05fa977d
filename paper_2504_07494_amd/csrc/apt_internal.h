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
    APT_PW_HEADER = 32
};
#define APT_N_QUEUES 8
#define APT_PLAN_MAGIC 0x41505431

// Tokens per work item.
#define APT_DEFAULT_KV_CHUNK 512
#define APT_MFMA_HIDDEN_CHUNK 256   // token rows of the MFMA kernel's tile
#define APT_DEFAULT_VALU_HIDDEN_CHUNK 32
#define APT_MAX_VALU_HIDDEN_CHUNK 64
#define APT_KV_MAX_PAGES_PER_WAVE 64

struct apt_resolved {
    apt_shape s;        // chunks and hidden_impl filled in
    int elem_bytes;
};

// Validates a shape and fills the defaults.  Returns an apt_status.
int apt_resolve(const apt_shape* in, apt_resolved* out);

static inline uint64_t apt_ws_bytes(int64_t n_partials, int H, int hd) {
    // per slot: head_dim floats of un-normalised output + (m, l)
    return (uint64_t)n_partials * (uint64_t)H * (uint64_t)(hd + 2) * 4u;
}
