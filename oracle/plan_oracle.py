"""Plain reference of the ragged work partition.  TEST INFRASTRUCTURE ONLY.

The decode attention step over a batch of requests with two cache kinds
(Section 4.2: the cache type is chosen per request; Section 4.3: one cache map
per request) is cut into independent work items, one per (request, head, token
range).  The paper does not prescribe an intra-kernel partition; the rule below
is this build's, stated in full so that the library's planner can be checked
against it bit for bit:

* a request of n tokens is cut into ceil(n / C) ranges [s*C, min(n, (s+1)*C)),
  with C = hidden_chunk for hidden-kind and C = kv_chunk for KV-kind requests;
* split_count[r] = number of ranges of request r; ws_offset[r] = sum of
  split_count over requests before r (request order);
* the partial result of (request r, range s, head h) is stored in slot
  (ws_offset[r] + s) * H + h;
* an item is (r, h, t0, t1).  Items are listed hidden-kind first, then KV-kind.
* hidden-kind items are grouped into N_QUEUES = 8 queues, queue x holding the items
  whose head h has h % 8 == x; the queues are concatenated in order x = 0..7 and
  queue_offset[x] (9 entries) is the position of queue x's first item.  Inside a
  queue: first the items whose range is a full hidden_chunk, ordered by request,
  range, head; then the shorter (last) ranges, ordered by decreasing length, ties by
  request, then head.
* KV-kind items are ordered by decreasing length of their range, ties by request,
  range, head.
* when the caller leaves kv_chunk open, it is the longest of 2048, 1024 and 512 tokens
  that consists of whole blocks, at most 256 of them, and with which the KV-kind
  requests of the batch still make at least 2048 items (ranges x heads); 512 if neither
  of the longer ones does (auto_kv_chunk below).

Block arithmetic of the cache map (Section 4.3): token j of a request lives in
its (j // block_size)-th block at slot j % block_size; a request of n tokens owns
ceil(n / block_size) blocks per cached vector type (K and V for the KV kind, the
input hidden vector for the hidden kind).
"""
KIND_KV = 0
KIND_HIDDEN = 1
N_QUEUES = 8


def ceil_div(a, b):
    return -(-a // b)


def auto_kv_chunk(ctx_lens, cache_kind, n_heads, block_size):
    """The range length of KV-kind requests when the caller does not fix it."""
    kv_lens = [int(n) for n, k in zip(ctx_lens, cache_kind) if int(k) == KIND_KV]
    for c in (2048, 1024):
        if c % block_size or c // block_size > 256:
            continue
        if sum(ceil_div(n, c) for n in kv_lens) * n_heads >= 2048:
            return c
    return 512


def plan(ctx_lens, cache_kind, n_heads, hidden_chunk, kv_chunk, hidden_item_per_head=True):
    """hidden_item_per_head=False: the absorbed-weight hidden path, whose items serve all heads of a
    range at once: one item (r, 0, t0, t1) per range of a hidden-kind request, by request and range,
    all in queue 0."""
    B = len(ctx_lens)
    split_count, ws_offset = [], []
    run = 0
    for r in range(B):
        n = int(ctx_lens[r])
        if n < 1:
            raise ValueError("ctx_len must be >= 1")
        if int(cache_kind[r]) not in (KIND_KV, KIND_HIDDEN):
            raise ValueError("unknown cache kind")
        c = hidden_chunk if int(cache_kind[r]) == KIND_HIDDEN else kv_chunk
        split_count.append(ceil_div(n, c))
        ws_offset.append(run)
        run += split_count[-1]
    def all_items(kind, c):
        out = []
        for r in range(B):
            if int(cache_kind[r]) != kind:
                continue
            n = int(ctx_lens[r])
            for s in range(split_count[r]):
                for h in range(n_heads):
                    out.append((r, h, s * c, min(n, (s + 1) * c)))
        return out

    items = []
    queue_offset = []
    hidden = all_items(KIND_HIDDEN, hidden_chunk)
    if not hidden_item_per_head:
        hidden = [it for it in hidden if it[1] == 0]
    for x in range(N_QUEUES):
        queue_offset.append(len(items))
        if not hidden_item_per_head:
            if x == 0:
                items += sorted(hidden, key=lambda it: (it[0], it[2]))
            continue
        mine = [it for it in hidden if it[1] % N_QUEUES == x]
        full = [it for it in mine if it[3] - it[2] == hidden_chunk]
        tails = [it for it in mine if it[3] - it[2] != hidden_chunk]
        full.sort(key=lambda it: (it[0], it[2], it[1]))
        tails.sort(key=lambda it: (-(it[3] - it[2]), it[0], it[1]))
        items += full + tails
    queue_offset.append(len(items))
    n_hidden_items = len(items)
    kv = all_items(KIND_KV, kv_chunk)
    kv.sort(key=lambda it: (-(it[3] - it[2]), it[0], it[2], it[1]))
    items += kv
    return {
        "split_count": split_count,
        "ws_offset": ws_offset,
        "items": items,
        "n_hidden_items": n_hidden_items,
        "n_partials": run,
        "queue_offset": queue_offset,
    }


def partial_slot(ws_offset, n_heads, r, s, h):
    return (ws_offset[r] + s) * n_heads + h


def token_location(block_list, block_size, j):
    """(block id, slot) of token j given the request's list of blocks."""
    return block_list[j // block_size], j % block_size


def blocks_for(n_tokens, block_size):
    return ceil_div(n_tokens, block_size)


def cache_bytes(n_tokens, d_model, elem_bytes, kind):
    """Bytes of cached vectors for n tokens of one layer (un-padded)."""
    per_token = d_model * elem_bytes
    return n_tokens * per_token * (1 if kind == KIND_HIDDEN else 2)
