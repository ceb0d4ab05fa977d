"""Test infrastructure: the unified block pool's bookkeeping by its plain definition
(Section 4.3, "Tailored Global Memory Pool" and "Cache Block Allocation").

A pool of n_blocks blocks; a block holds the K, V or hidden vectors of block_size consecutive
token positions of one request.  A request's cache map lists its blocks in position order (two
lists, K and V, for the KV kind; one for the hidden kind).  Blocks are chosen on demand by
scanning for unused blocks: always the unused block with the smallest id, the K block of a
position range before its V block.  Only tests may import this module."""

KIND_KV, KIND_HIDDEN = 0, 1


class Full(Exception):
    pass


class Pool:
    def __init__(self, n_blocks, block_size):
        self.block_size = block_size
        self.unused = set(range(n_blocks))
        self.requests = {}                     # slot -> dict(kind, len, maps=[list, ...])

    def _blocks(self, n_tokens):
        return -(-n_tokens // self.block_size)

    def needed(self, kind, n_tokens):
        return self._blocks(n_tokens) * (2 if kind == KIND_KV else 1)

    def _grow(self, req, want):
        have = len(req["maps"][0])
        if (want - have) * len(req["maps"]) > len(self.unused):
            raise Full()
        for _ in range(have, want):
            for m in req["maps"]:
                b = min(self.unused)
                self.unused.remove(b)
                m.append(b)

    def assign(self, slot, kind, n_tokens):
        assert slot not in self.requests and n_tokens >= 1
        req = {"kind": kind, "len": n_tokens, "maps": [[], []] if kind == KIND_KV else [[]]}
        self._grow(req, self._blocks(n_tokens))
        self.requests[slot] = req

    def extend(self, slot, n_tokens):
        req = self.requests[slot]
        assert n_tokens >= req["len"]
        self._grow(req, self._blocks(n_tokens))
        req["len"] = n_tokens

    def release(self, slot):
        for m in self.requests.pop(slot)["maps"]:
            self.unused.update(m)

    def switch_kind(self, slot, new_kind):
        req = self.requests[slot]
        if req["kind"] == new_kind:
            return
        nb = self._blocks(req["len"])
        if self.needed(new_kind, req["len"]) > len(self.unused) + nb * len(req["maps"]):
            raise Full()
        n = req["len"]
        self.release(slot)
        self.assign(slot, new_kind, n)

    def export(self, slots, max_blocks):
        """(block_tables [B][2][max_blocks] with -1 padding, ctx_lens, cache_kind) as nested lists."""
        bt, lens, kinds = [], [], []
        for s in slots:
            req = self.requests[s]
            rows = [m + [-1] * (max_blocks - len(m)) for m in req["maps"]]
            if len(rows) == 1:
                rows.append([-1] * max_blocks)
            bt.append(rows)
            lens.append(req["len"])
            kinds.append(req["kind"])
        return bt, lens, kinds
