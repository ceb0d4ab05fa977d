"""Pins of oracle/pool_oracle.Pool itself (not through the product): the worked example of the
unified block pool (Section 4.3: 16 blocks of 4 positions, request A with KV cache of 11 tokens,
request B with hidden cache of 14 tokens), block counts and placements computed by hand for the
"lowest unused id, K before V" scan, the storage law hidden = half of KV (Section 3.1), and the
invariants every sequence of operations must keep."""
import os

import numpy as np
import pytest

from oracle import pool_oracle as po

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "pool_example.txt")


def _golden():
    g = {}
    for line in open(GOLDEN):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] in ("pool_blocks", "block_size"):
            g[t[0]] = int(t[1])
            continue
        req = {"kind": t[2], "tokens": int(t[4]), "lists": []}      # "<name> kind <kv|hidden> tokens <n> <x>_blocks ids..."
        for w in t[5:]:
            if w.endswith("_blocks"):
                req["lists"].append([])
            else:
                req["lists"][-1].append(int(w))
        g[t[0]] = req
    return g


def test_worked_example_of_the_paper_sizes_and_positions():
    g = _golden()
    pool = po.Pool(g["pool_blocks"], g["block_size"])
    a, b = g["A"], g["B"]
    assert (a["kind"], b["kind"]) == ("kv", "hidden")
    pool.assign(0, po.KIND_KV, a["tokens"])
    pool.assign(1, po.KIND_HIDDEN, b["tokens"])
    # the paper's block counts: A has 3 K blocks and 3 V blocks, B has 4 hidden blocks, 6 of 16 stay unused
    ra, rb = pool.requests[0], pool.requests[1]
    assert [len(m) for m in ra["maps"]] == [len(l) for l in a["lists"]] == [3, 3]
    assert [len(m) for m in rb["maps"]] == [len(l) for l in b["lists"]] == [4]
    assert len(pool.unused) == g["pool_blocks"] - sum(len(l) for l in a["lists"] + b["lists"]) == 6
    assert pool.needed(po.KIND_KV, a["tokens"]) == 6 and pool.needed(po.KIND_HIDDEN, b["tokens"]) == 4
    # position -> (entry of the cache map, slot): A's 11th token sits in its 3rd block at slot 2, B's 14th in its
    # 4th block at slot 1 (Section 4.3: a block holds contiguous positions, the map lists blocks in position order)
    bt, lens, kinds = pool.export([0, 1], max_blocks=5)
    assert lens == [11, 14] and kinds == [po.KIND_KV, po.KIND_HIDDEN]
    assert (10 // pool.block_size, 10 % pool.block_size) == (2, 2) and bt[0][0][2] == ra["maps"][0][2]
    assert (13 // pool.block_size, 13 % pool.block_size) == (3, 1) and bt[1][0][3] == rb["maps"][0][3]
    # a hidden-kind request has no V list; unused entries are -1
    assert bt[1][1] == [-1] * 5 and bt[0][0][3:] == [-1, -1] and bt[1][0][4:] == [-1]


def test_hand_computed_placements_extend_release_switch():
    pool = po.Pool(16, 4)
    pool.assign(0, po.KIND_KV, 11)           # K, V alternate over the lowest unused ids
    assert pool.requests[0]["maps"] == [[0, 2, 4], [1, 3, 5]]
    pool.assign(1, po.KIND_HIDDEN, 14)
    assert pool.requests[1]["maps"] == [[6, 7, 8, 9]]
    pool.extend(0, 12)                       # still 3 blocks per list
    assert pool.requests[0]["maps"] == [[0, 2, 4], [1, 3, 5]] and len(pool.unused) == 6
    pool.extend(0, 13)                       # crosses a block boundary: one K and one V block
    assert pool.requests[0]["maps"] == [[0, 2, 4, 10], [1, 3, 5, 11]] and pool.requests[0]["len"] == 13
    pool.extend(1, 16)                       # 16 positions still fit 4 blocks
    assert pool.requests[1]["maps"] == [[6, 7, 8, 9]]
    pool.release(0)
    assert sorted(pool.unused) == [0, 1, 2, 3, 4, 5, 10, 11, 12, 13, 14, 15] and 0 not in pool.requests
    pool.switch_kind(1, po.KIND_KV)          # B's cache is discarded, then 4 K + 4 V blocks from the lowest ids
    assert pool.requests[1]["maps"] == [[0, 2, 4, 6], [1, 3, 5, 7]] and pool.requests[1]["len"] == 16
    assert sorted(pool.unused) == [8, 9, 10, 11, 12, 13, 14, 15]
    pool.switch_kind(1, po.KIND_HIDDEN)
    assert pool.requests[1]["maps"] == [[0, 1, 2, 3]] and len(pool.unused) == 12
    pool.switch_kind(1, po.KIND_HIDDEN)      # same kind: nothing happens
    assert pool.requests[1]["maps"] == [[0, 1, 2, 3]]


def test_full_pool_raises_and_changes_nothing():
    pool = po.Pool(8, 4)
    pool.assign(0, po.KIND_KV, 9)            # 3 + 3 blocks, 2 unused
    with pytest.raises(po.Full):
        pool.assign(1, po.KIND_KV, 5)        # needs 4
    assert 1 not in pool.requests and sorted(pool.unused) == [6, 7]
    with pytest.raises(po.Full):
        pool.extend(0, 17)                   # 5 blocks per list: 4 more
    assert pool.requests[0]["maps"] == [[0, 2, 4], [1, 3, 5]] and pool.requests[0]["len"] == 9
    pool.extend(0, 16)                       # 4 blocks per list: exactly the 2 unused ones
    assert pool.requests[0]["maps"] == [[0, 2, 4, 6], [1, 3, 5, 7]] and not pool.unused
    pool2 = po.Pool(8, 4)
    pool2.assign(0, po.KIND_HIDDEN, 20)      # 5 blocks
    with pytest.raises(po.Full):
        pool2.switch_kind(0, po.KIND_KV)     # 10 > 8 even after giving its own 5 back
    assert pool2.requests[0]["maps"] == [[0, 1, 2, 3, 4]] and len(pool2.unused) == 3


@pytest.mark.parametrize("bs", [1, 4, 16])
def test_storage_law_hidden_is_half_of_kv(bs):
    pool = po.Pool(10, bs)
    for n in range(1, 200):
        assert 2 * pool.needed(po.KIND_HIDDEN, n) == pool.needed(po.KIND_KV, n) == 2 * -(-n // bs)


@pytest.mark.parametrize("seed", range(5))
def test_invariants_over_random_operation_sequences(seed):
    g = np.random.default_rng(seed)
    n_blocks, bs = 64, 4
    pool = po.Pool(n_blocks, bs)
    for _ in range(400):
        op = g.integers(0, 4)
        slot = int(g.integers(0, 8))
        try:
            if op == 0 and slot not in pool.requests:
                pool.assign(slot, int(g.integers(0, 2)), int(g.integers(1, 40)))
            elif op == 1 and slot in pool.requests:
                pool.extend(slot, pool.requests[slot]["len"] + int(g.integers(0, 9)))
            elif op == 2 and slot in pool.requests:
                pool.release(slot)
            elif op == 3 and slot in pool.requests:
                pool.switch_kind(slot, 1 - pool.requests[slot]["kind"])
        except po.Full:
            pass
        held = [b for r in pool.requests.values() for m in r["maps"] for b in m]
        assert len(held) == len(set(held))                             # no block serves two positions ranges
        assert set(held).isdisjoint(pool.unused) and set(held) | pool.unused == set(range(n_blocks))
        for r in pool.requests.values():
            rows = 2 if r["kind"] == po.KIND_KV else 1
            assert len(r["maps"]) == rows and all(len(m) == -(-r["len"] // bs) for m in r["maps"])
