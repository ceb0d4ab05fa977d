/*
 * apt_hybrid.h - C ABI of the MI355X (gfx950) hybrid-cache decode attention library.
 *
 * One decode step of one Transformer layer's attention over a ragged batch in
 * which every request keeps its context either in a paged KV cache or in a
 * hidden cache: the layer's input hidden vectors, from which K and V are
 * projected again on the fly (Section 3.1, "Opportunity I: Utilizing Hybrid
 * Cache"; Section 2.1, Eq. 1-3 for the attention itself; Section 2.2 for the KV
 * cache and block-wise storage; Section 4.3 for the unified block pool and the
 * per-request cache map).
 *
 * For request r (n = ctx_lens[r] attended positions, the current token
 * included and already present in the cache) and head h:
 *     KV kind:      k_j, v_j read from the request's K and V blocks
 *     hidden kind:  k_j = x_j W_K[:, h] + b_K[h],  v_j = x_j W_V[:, h] + b_V[h]    (Eq. 1)
 *     out[r][h] = sum_j softmax_j(softmax_scale * <q[r][h], k_j>) v_j              (Eq. 2-3)
 * The output projection W_o of Eq. 3 is NOT applied.
 *
 * Conventions
 *   - Plain C, no exceptions cross the boundary.  Every function returns 0
 *     (APT_OK) or a negative apt_status; apt_strerror() names it.
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HIP device
 *     memory of the current device.  The caller owns every buffer.  The library
 *     allocates no device memory.  The only state it keeps between calls is a small
 *     per-device record made by apt_init() (compute-unit count, "kernel attributes are
 *     set", address of the static workspace), written once per device under a mutex and
 *     read-only afterwards, so calls from several host threads are safe.  apt_pool_* keep
 *     their state in the host handle the caller holds; apt_schedule is a pure function.
 *   - Launching functions take a HIP stream as void* (NULL = default stream) and
 *     return after enqueueing; inputs are read-only, only `out`, `workspace`,
 *     `packed` (apt_pack_weights), the cache pools (apt_cache_append, apt_cache_write) and one
 *     counter word of `plan_dev` are written.
 *   - Arguments are validated on the host before anything is launched.  Block
 *     ids inside block_tables are NOT range-checked on the device; use
 *     apt_validate_host() on a host copy.
 *
 * Memory layout (T = element type of apt_shape.dtype)
 *   pool block       block_size * d_model elements of T.  The three pool base
 *                    pointers may alias one unified pool: a block holds K, V or
 *                    hidden vectors of block_size consecutive token positions
 *                    (Section 4.3).
 *   hidden block     T [slot][d_model]
 *   K block, V block T [head][slot][head_dim]
 *   block_tables     int32 [B][2][max_blocks_per_req] (device): row 0 = K blocks
 *                    (KV kind) or hidden blocks (hidden kind), row 1 = V blocks
 *                    (KV kind).  Token j is in entry j / block_size at slot
 *                    j % block_size.  Entries past the request's last block and
 *                    the unused slots of the last block are never read.
 *   q                T [B][n_heads][head_dim]
 *   W_K, W_V         T [d_in = d_model][d_out = n_heads*head_dim] row-major, so
 *                    that k = x W + b; this is the transpose of an [out][in]
 *                    linear-layer weight (the paper writes W x for column vectors).
 *   b_K, b_V         T [d_model]
 *   out              [B][n_heads][head_dim] of apt_shape.out_dtype
 */
#ifndef APT_HYBRID_H
#define APT_HYBRID_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum apt_status {
    APT_OK = 0,
    APT_EINVAL = -1,     /* null pointer, non-positive count, bad length or kind */
    APT_ESHAPE = -2,     /* unsupported or inconsistent shape                     */
    APT_EDTYPE = -3,     /* unknown dtype / unsupported out_dtype                 */
    APT_EWORKSPACE = -4, /* workspace or plan buffer too small                    */
    APT_EHIP = -5,       /* a HIP runtime call failed                             */
    APT_ERANGE = -6,     /* a block id or length is out of range                  */
    APT_EFULL = -7       /* not enough unused blocks in the pool (nothing changed) */
} apt_status;

enum { APT_F32 = 0, APT_F16 = 1, APT_BF16 = 2 };
enum { APT_KIND_KV = 0, APT_KIND_HIDDEN = 1 };
enum { APT_HIDDEN_AUTO = 0, APT_HIDDEN_VALU = 1, APT_HIDDEN_MFMA = 2, APT_HIDDEN_ABSORBED = 3 };

typedef struct apt_shape {
    int32_t d_model;            /* = n_heads * head_dim                                   */
    int32_t n_heads;
    int32_t head_dim;           /* 64 or 128                                               */
    int32_t block_size;         /* tokens per cache block; 16 (or 4, 8, 32)               */
    int32_t dtype;              /* APT_F32 / APT_F16 / APT_BF16: q, pools, W, b           */
    int32_t out_dtype;          /* APT_F32 or the same as dtype                           */
    int32_t max_blocks_per_req; /* row length of block_tables                             */
    int32_t hidden_chunk;       /* tokens per hidden-kind work item; 0 = library default
                                   (MFMA kernel: 256 or 320, default 320 for d_model >= 8192)  */
    int32_t kv_chunk;           /* tokens per KV-kind work item, whole blocks, at most 256
                                   of them; 0 = chosen by apt_plan for each batch: the
                                   longest of 2048 / 1024 / 512 that still gives 2048
                                   KV-kind items (apt_plan_info.kv_chunk reports it)      */
    int32_t hidden_impl;        /* APT_HIDDEN_AUTO: MFMA kernel for 16-bit dtypes with
                                   head_dim 128, plain-ALU kernel otherwise.
                                   APT_HIDDEN_ABSORBED (never chosen by AUTO): the same
                                   output without projecting K and V, see below           */
    float softmax_scale;        /* multiplies <q, k>; 1/sqrt(head_dim) in Eq. 2's
                                   multi-head reading                                     */
    int32_t reserved;           /* must be 0                                              */
} apt_shape;

typedef struct apt_plan_info {
    int32_t batch;
    int32_t n_items;            /* work items = workgroups of the attention launch        */
    int32_t n_hidden_items;     /* the first n_hidden_items items are hidden-kind         */
    int32_t n_partials;         /* sum over requests of their token ranges                */
    int32_t hidden_chunk;       /* resolved values                                        */
    int32_t kv_chunk;
    int32_t hidden_impl;        /* resolved: APT_HIDDEN_VALU, _MFMA or _ABSORBED          */
    int32_t reserved;
    int64_t total_tokens;
    int64_t hidden_tokens;
    uint64_t plan_bytes;        /* bytes of the plan blob actually used                   */
    uint64_t workspace_bytes;   /* device workspace apt_hybrid_decode_attn needs          */
} apt_plan_info;

/* Utilities of the boundary (no counterpart in the paper): name of a status code; library
 * version (major*10000 + minor*100 + patch). */
const char* apt_strerror(int status);
int apt_version(void);

/*
 * One-off set-up for the CURRENT device: reads the compute-unit count (the hidden-kind MFMA kernel
 * runs one persistent workgroup per compute unit), raises the dynamic-LDS limit of the kernels that
 * need more than 64 KB, and looks up the device address of the static workspace used by
 * apt_hybrid_decode_attn_static.  Idempotent and thread-safe.  Every launching entry point calls it
 * by itself on its first use on a device, so calling it is optional, EXCEPT before capturing calls
 * into a HIP graph: call apt_init() (or run one eager call) on that device first, because setting
 * kernel attributes is not a stream operation and does not belong into a capture.
 * (Utility of the boundary; the operation it prepares is the attention step of Eq. 1-3.)
 * Errors: APT_EHIP.
 */
int apt_init(void);

/*
 * Sizes a caller needs BEFORE any batch is known (Section 4.3: the cache pool and everything
 * around it are set up once for the serving process; Section 4.2: batches of at most max_batch
 * requests whose cache kinds change from iteration to iteration):
 *   *dev_bytes   upper bound of apt_plan_info.workspace_bytes over every batch of 1..max_batch
 *                requests with contexts of 1..max_ctx tokens and ANY mix of the two cache kinds.
 *                For hidden_impl = APT_HIDDEN_AUTO, _VALU or _MFMA this is the partial-result
 *                workspace (ranges of the shorter of the two chunk lengths); for
 *                APT_HIDDEN_ABSORBED the sections of that path are added.  A workspace of this
 *                size serves every such batch, so it can be allocated once.
 *   *host_bytes  the same bound for the plan blob (= apt_plan_max_bytes), needed once on the host
 *                and once on the device.
 * Either pointer may be NULL.  Host only.  Errors: APT_EINVAL (max_batch < 1, max_ctx < 1, both
 * pointers NULL), APT_ERANGE (max_ctx beyond max_blocks_per_req*block_size), APT_ESHAPE, APT_EDTYPE.
 */
int apt_workspace_bytes(const apt_shape* s, int max_batch, int max_ctx, size_t* dev_bytes, size_t* host_bytes);

/*
 * Size in bytes of the largest plan blob a batch of B requests with contexts of at
 * most max_ctx tokens can need (host and device copy have the same size).  Helper of apt_plan
 * (Section 4.2: one batch per iteration).
 */
int apt_plan_max_bytes(const apt_shape* s, int B, int max_ctx, size_t* bytes);

/*
 * Ragged work partitioner (host).  Cuts the batch into work items
 * (request, head, token range) of the two cache kinds, hidden-kind items first,
 * so that one launch serves both (the cache type is a per-request decision,
 * Section 4.2; requests of both types share a batch, Section 4.3).
 *   ctx_lens_host   int32 [B], every entry >= 1 and <= max_blocks_per_req*block_size
 *   cache_kind_host uint8 [B], APT_KIND_KV or APT_KIND_HIDDEN
 *   plan_host       caller's buffer of plan_bytes bytes (see apt_plan_max_bytes); filled
 *                   with a self-contained blob of int32 words:
 *                     [0..15] header, [16..24] queue_offset, [32..32+B) split_count,
 *                     then ws_offset[B] and six more per-request arrays of B words (cache
 *                     kind, length; index, first token and first range among the hidden-kind
 *                     requests; the list of hidden-kind requests), then (padded to a multiple of 4 words)
 *                     items[n_items][4] = (request, head, t0, t1)
 *   info            optional, receives the counts and the workspace size
 * The rule: a request of n tokens is cut into ceil(n/C) ranges [s*C, min(n,(s+1)*C)),
 * C = hidden_chunk or kv_chunk by kind; ws_offset is the exclusive prefix sum of
 * split_count in request order; the partial result of (r, range s, head h) lives in
 * slot (ws_offset[r]+s)*n_heads + h.  Items are ordered hidden kind first: 8 queues, queue x
 * holding the heads with h % 8 == x (queue_offset[x] = its first item, queue_offset[8] = the
 * number of hidden-kind items), in a queue first the full ranges by request, range, head, then
 * the shorter last ranges by decreasing length (ties by request, head); then the KV kind by
 * decreasing range length (ties by request, range, head).  With APT_HIDDEN_ABSORBED a hidden-kind
 * item covers all heads of its range: one item (request, 0, t0, t1) per range, all in queue 0, by
 * request and range.  The order only steers which workgroup takes which item (cache locality,
 * balance); every item is independent.
 * Integer-only; the same inputs always give the same bytes.
 * Errors: APT_EINVAL (null, B < 1, length < 1, unknown kind), APT_ERANGE (length
 * beyond max_blocks_per_req*block_size), APT_EWORKSPACE (plan_bytes too small),
 * APT_ESHAPE / APT_EDTYPE (bad shape).
 */
int apt_plan(const apt_shape* s, const int32_t* ctx_lens_host, const uint8_t* cache_kind_host, int B,
             void* plan_host, size_t plan_bytes, apt_plan_info* info);

/* Read the counts back from a plan blob made by apt_plan (host; helper of apt_plan). */
int apt_plan_get_info(const void* plan_host, apt_plan_info* info);

/* Asynchronous copy of a plan blob to device memory (plan_dev: at least
 * info.plan_bytes bytes; helper of apt_plan: the device half of the work partition).  plan_host
 * must stay unchanged until the copy is done (re-planning into the same host buffer before that
 * tears the copy: use one host buffer per step in flight, or wait for an event recorded after
 * this call); use page-locked host memory for a truly asynchronous copy. */
int apt_plan_upload(const void* plan_host, void* plan_dev, void* stream);

/*
 * Debug helper (host): range-check a host copy of the cache maps (Section 4.3, "Cache Block
 * Allocation": a cache map associates each token position of a request with a block of the
 * unified pool; K and V lists for the KV kind, one list for the hidden kind).  Every entry of
 * the first ceil(n/block_size) positions of the rows a request uses must lie in
 * [0, n_pool_blocks).  Returns APT_ERANGE on the first violation, APT_EINVAL for a length < 1 or
 * an unknown kind.  Also APT_ERANGE when the resolved hidden_impl is APT_HIDDEN_MFMA and the pool
 * (n_pool_blocks blocks) is larger than 64 GiB: that kernel addresses hidden rows by 32-bit offsets
 * in 16-byte units from hidden_pages (a larger pool gives wrong results, not a fault).
 */
int apt_validate_host(const apt_shape* s, const int32_t* ctx_lens_host, const uint8_t* cache_kind_host,
                      const int32_t* block_tables_host, int B, int64_t n_pool_blocks);

/*
 * One-off re-layout of a layer's projection weights for the MFMA kernel (Eq. 1's
 * W_k, W_v restricted to one head at a time).  Needed only when the resolved
 * hidden_impl is APT_HIDDEN_MFMA.  `packed` (device) needs apt_packed_weight_bytes()
 * bytes = 2 * d_model^2 elements.  Layout of `packed`, in 16-byte units of 8 elements:
 *   [head][k-tile of 32 inputs][row 0..255][unit 0..3], row < 128: W_K output channel
 *   head*128+row, row >= 128: W_V output channel head*128+row-128; the unit holding
 *   inputs k-tile*32 + 8*c .. +7 sits at position c ^ ((row >> 1) & 3).
 */
int apt_packed_weight_bytes(const apt_shape* s, size_t* bytes);
int apt_pack_weights(const apt_shape* s, const void* W_K, const void* W_V, void* packed, void* stream);

/*
 * The decode attention step for one layer (Eq. 1-3 over both cache kinds).
 *   plan_host / plan_dev   the blob from apt_plan and its device copy.  One word of the device
 *               copy (a ticket counter that hands out KV-kind items inside the launch) is
 *               written by the item kernel and reset by the merge kernel, so two calls that
 *               share one plan_dev must be ordered on one stream (calls for successive layers
 *               are); everything else in it is read-only
 *   q, k_pages, v_pages, hidden_pages, b_K, b_V, block_tables, out   device, see layout
 *   W_K, W_V    device, raw [d_in][d_out]; read only by the plain-ALU hidden kernel
 *               (may be NULL when the resolved hidden_impl is MFMA or no request is
 *               hidden-kind)
 *   W_packed    device, from apt_pack_weights; read only by the MFMA hidden kernel
 *               (may be NULL otherwise)
 *   workspace   device, at least info.workspace_bytes bytes; holds the per-range
 *               partial results (running maximum, sum, un-normalised output) that the
 *               merge kernel combines; contents are undefined afterwards
 * Two kernels are enqueued on `stream`: the item kernel (one workgroup per work item,
 * hidden-kind and KV-kind items in the same launch) and the merge kernel.
 * Errors: APT_EINVAL (null pointer that is needed), APT_EWORKSPACE, APT_ESHAPE,
 * APT_EDTYPE, APT_EHIP (launch failure; nothing is written in the other cases).
 */
int apt_hybrid_decode_attn(const apt_shape* s, const void* plan_host, void* plan_dev,
                           const void* q, const void* k_pages, const void* v_pages, const void* hidden_pages,
                           const void* W_K, const void* W_V, const void* W_packed,
                           const void* b_K, const void* b_V, const int32_t* block_tables,
                           void* out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * APT_HIDDEN_ABSORBED.  Not in the paper: an exact re-association of Eq. 1-3 for hidden-kind
 * requests.  With qt = W_K[:, h] q (a d_model vector per request and head) the score of token j is
 * scale * (<x_j, qt> + <q, b_K[h]>), and because the softmax weights a_j sum to one,
 * out = (sum_j a_j x_j) W_V[:, h] + b_V[h].  The cached hidden rows are then read twice (scores,
 * weighted sum) like the K and V rows of a KV-kind request, and the two projections shrink to one
 * matrix-vector product per request and head.  Work per hidden token: 4 * d_model * n_heads flops
 * instead of 4 * d_model^2.  Results agree with the other implementations to fp32 rounding.  Needs
 * the raw W_K, W_V (not W_packed), d_model a multiple of 32, n_heads <= 128 (fp32 inputs: <= 40), and a larger workspace
 * (apt_plan_info.workspace_bytes says how much); hidden_chunk must be 0 or 512.
 */

/*
 * For callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same step as apt_hybrid_decode_attn with the
 * partial-result workspace taken from a static device array inside the library instead of a
 * caller buffer.  Arguments as for apt_hybrid_decode_attn, without workspace / workspace_bytes.
 * The array has APT_STATIC_WORKSPACE_BYTES bytes per device (each GPU the library runs on holds it
 * until the process ends); a plan that needs more (apt_plan_info.workspace_bytes) is rejected with
 * APT_EWORKSPACE, and so is APT_HIDDEN_ABSORBED (its workspace is far larger: APT_ESHAPE).  The call
 * allocates nothing and frees nothing.  Every partial the merge reads is written earlier in the same
 * call, so nothing needs clearing between calls; the array keeps the last call's partials.  All calls
 * on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two host
 * threads) race and give wrong results; order them on one stream.  Call apt_init() before
 * capturing this call into a graph.
 */
#define APT_STATIC_WORKSPACE_BYTES ((size_t)64 << 20)
int apt_hybrid_decode_attn_static(const apt_shape* s, const void* plan_host, void* plan_dev,
                                  const void* q, const void* k_pages, const void* v_pages, const void* hidden_pages,
                                  const void* W_K, const void* W_V, const void* W_packed,
                                  const void* b_K, const void* b_V, const int32_t* block_tables,
                                  void* out, void* stream);

/*
 * Hybrid cache assigner: host-side bookkeeping of the unified block pool (Section 4.3,
 * "Tailored Global Memory Pool" and "Cache Block Allocation").  The pool has n_blocks blocks;
 * each holds the K, V or hidden vectors of block_size consecutive token positions of one
 * request, so a KV-kind request of n tokens occupies 2*ceil(n/block_size) blocks and a
 * hidden-kind request half of that (the (1 - beta/2) m of Definition 1).  Requests live in
 * numbered slots (0 .. max_requests-1).  A request's cache map lists its blocks in position
 * order; blocks are picked on demand by scanning for unused blocks, lowest block id first (for a
 * KV-kind request the K block of a position range is taken before its V block).  All memory is
 * host memory owned by the handle; nothing here touches the device.
 *   apt_pool_assign       new request in an empty slot: blocks for n_tokens positions
 *   apt_pool_extend       grow a request to n_tokens (>= its current length); takes blocks
 *                         only when a block boundary is crossed
 *   apt_pool_release      return all blocks of the slot, empty the slot
 *   apt_pool_switch_kind  discard the cache and take blocks for the same length in the other
 *                         kind (Section 5: the caller then recomputes the contents by a prefill)
 *   apt_pool_export       block_tables int32 [B][2][max_blocks_per_req] (-1 = no block),
 *                         ctx_lens int32 [B], cache_kind uint8 [B] of the listed slots, in the
 *                         layout the attention and cache-write calls take (host arrays)
 *   apt_pool_blocks_needed  blocks a request of n_tokens occupies in the given kind
 * Errors: APT_EINVAL (null, bad slot, slot empty / in use, shrinking), APT_ERANGE (more than
 * max_blocks_per_req blocks), APT_EFULL (not enough unused blocks; the pool is unchanged).
 */
typedef struct apt_pool apt_pool;
int apt_pool_create(int64_t n_blocks, int32_t block_size, int32_t max_blocks_per_req, int32_t max_requests,
                    apt_pool** out);
void apt_pool_destroy(apt_pool* pool);
int apt_pool_free_blocks(const apt_pool* pool, int64_t* n_free);
int apt_pool_blocks_needed(const apt_pool* pool, uint8_t kind, int32_t n_tokens, int64_t* n_blocks);
int apt_pool_assign(apt_pool* pool, int32_t slot, uint8_t kind, int32_t n_tokens);
int apt_pool_extend(apt_pool* pool, int32_t slot, int32_t n_tokens);
int apt_pool_release(apt_pool* pool, int32_t slot);
int apt_pool_switch_kind(apt_pool* pool, int32_t slot, uint8_t new_kind);
int apt_pool_export(const apt_pool* pool, const int32_t* slots, int B, int32_t* block_tables, int32_t* ctx_lens,
                    uint8_t* cache_kind);

/*
 * Greedy solution of the hybrid-cache scheduling problem (Section 5, Definition 1): choose for
 * every candidate request i whether it is scheduled (alpha_i) and whether it gets hidden cache
 * (beta_i), maximising sum alpha_i g_i with g_i = p_i - beta_i * n_unfinished * rho * m_i under
 * sum (1 - beta_i/2) m_i alpha_i <= mem_limit.  pending[i] = p_i >= 0 (pending time), mem[i] = m_i
 * (memory of the request's KV cache, any unit, even and >= 2 so that the hidden cache takes
 * exactly m_i/2), n_unfinished = |W| + |R|, rho = the extra time per unit of memory of a
 * hidden-cache request (Eq. 6; the slope bench.py --sweep fits).  Candidate schedules and their
 * marginal gains theta are the two case tables after Definition 1; they are taken by decreasing
 * theta (ties: lower request index, first increment first) while they fit, a second increment
 * only after its first, and the result is compared with the best single request.  The value
 * reached is at least half of the optimum.  alpha, beta: uint8 [n] outputs; value (may be NULL)
 * receives the objective.  Host only, O(n log n).  Errors: APT_EINVAL.
 */
int apt_schedule(const double* pending, const int64_t* mem, int n, int64_t mem_limit, int32_t n_unfinished,
                 double rho, uint8_t* alpha, uint8_t* beta, double* value);

/*
 * Cache append: writes the vectors of the token just processed into the request's cache
 * blocks, with the layout change fused into the write (the paper's block-wise cache I/O
 * kernel, Section 5.1; block placement per Section 4.3).  For request r with
 * n = ctx_lens[r] tokens AFTER the append, position n-1 (block entry (n-1)/block_size, slot
 * (n-1)%block_size) receives
 *     hidden kind: x_new[r][0..d_model)                      -> hidden block [slot][d_model]
 *     KV kind:     k_new[r][head][0..head_dim), v_new[...]   -> K / V block [head][slot][head_dim]
 * All pointers are device memory; ctx_lens_dev int32 [B], cache_kind_dev uint8 [B];
 * x_new may be NULL if no request is hidden-kind, k_new/v_new if none is KV-kind (the kernel
 * does not check the kinds against NULL: pass what the batch needs).  Elements are copied
 * bit for bit.  One launch on `stream`.  Run it before apt_hybrid_decode_attn of the same
 * step (ctx_lens counts the current token).
 * Errors: APT_EINVAL (B < 1, missing tables or all three sources NULL), APT_ESHAPE, APT_EDTYPE, APT_EHIP.
 */
int apt_cache_append(const apt_shape* s, int B, const void* x_new, const void* k_new, const void* v_new,
                     void* k_pages, void* v_pages, void* hidden_pages, const int32_t* block_tables,
                     const int32_t* ctx_lens_dev, const uint8_t* cache_kind_dev, void* stream);

/*
 * Cache write of a run of new tokens per request: the prefill's cache write (all prompt
 * positions at once, both cache kinds; Section 2.2 and Section 5.1) and the general form of
 * apt_cache_append.  Request r has n_r = new_offsets[r+1] - new_offsets[r] new tokens; their
 * vectors are rows new_offsets[r] .. new_offsets[r+1]-1 of x_new [rows][d_model] (hidden kind)
 * or k_new, v_new [rows][n_heads][head_dim] (KV kind) and go to positions
 * ctx_lens[r] - n_r .. ctx_lens[r] - 1 of the request's cache map (ctx_lens counts the tokens
 * AFTER the write), with the same layout change as apt_cache_append.  n_r may be 0.
 * new_offsets_dev int32 [B+1] (device, non-decreasing, first entry 0); max_new_tokens >= every
 * n_r sizes the launch (host value).  Pointer rules, aliasing rules and errors as for
 * apt_cache_append; APT_ERANGE if max_new_tokens exceeds 524280.  One launch.
 */
int apt_cache_write(const apt_shape* s, int B, const int32_t* new_offsets_dev, int32_t max_new_tokens,
                    const void* x_new, const void* k_new, const void* v_new, void* k_pages, void* v_pages,
                    void* hidden_pages, const int32_t* block_tables, const int32_t* ctx_lens_dev,
                    const uint8_t* cache_kind_dev, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* APT_HYBRID_H */
