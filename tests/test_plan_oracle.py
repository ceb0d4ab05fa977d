"""Pins of the plain work-partition rule: coverage and slot invariants by brute force."""
import numpy as np
import pytest

from oracle import plan_oracle as po


def _random_batch(seed, B, hi):
    g = np.random.default_rng(seed)
    return g.integers(1, hi + 1, size=B), g.integers(0, 2, size=B)


@pytest.mark.parametrize("seed,B,hi,H,ch,ck", [(0, 1, 1, 1, 4, 4), (1, 7, 40, 3, 8, 16), (2, 16, 300, 5, 64, 128),
                                               (3, 9, 64, 2, 64, 64), (4, 12, 50, 4, 256, 512)])
def test_every_token_is_covered_exactly_once(seed, B, hi, H, ch, ck):
    lens, kinds = _random_batch(seed, B, hi)
    p = po.plan(lens, kinds, H, ch, ck)
    cover = [np.zeros((H, int(n)), dtype=np.int32) for n in lens]
    slots = set()
    for i, (r, h, t0, t1) in enumerate(p["items"]):
        assert 0 <= t0 < t1 <= lens[r]
        c = ch if kinds[r] == po.KIND_HIDDEN else ck
        assert t1 - t0 <= c and t0 % c == 0
        assert (i < p["n_hidden_items"]) == (kinds[r] == po.KIND_HIDDEN)
        if i < p["n_hidden_items"]:
            x = h % po.N_QUEUES
            assert p["queue_offset"][x] <= i < p["queue_offset"][x + 1]
        cover[r][h, t0:t1] += 1
        slot = po.partial_slot(p["ws_offset"], H, r, t0 // c, h)
        assert slot not in slots
        slots.add(slot)
    for c in cover:
        assert np.all(c == 1)
    # slots are dense: 0 .. n_partials*H - 1
    assert slots == set(range(p["n_partials"] * H))
    assert p["n_partials"] == sum(p["split_count"])
    assert p["ws_offset"] == [int(x) for x in np.concatenate([[0], np.cumsum(p["split_count"])[:-1]])]
    for r in range(B):
        c = ch if kinds[r] == po.KIND_HIDDEN else ck
        assert p["split_count"][r] == (int(lens[r]) + c - 1) // c
    assert len(p["items"]) == sum(H * s for s in p["split_count"])
    assert p["queue_offset"][0] == 0 and p["queue_offset"][-1] == p["n_hidden_items"]
    assert all(a <= b for a, b in zip(p["queue_offset"][:-1], p["queue_offset"][1:]))
    # inside a queue and inside the KV part the cost (range length) never increases
    for lo, hi in list(zip(p["queue_offset"][:-1], p["queue_offset"][1:])) + [(p["n_hidden_items"], len(p["items"]))]:
        lens_ = [t1 - t0 for (_, _, t0, t1) in p["items"][lo:hi]]
        assert lens_ == sorted(lens_, reverse=True)


def test_item_order_hand_example():
    # 3 requests: KV(5), hidden(9), KV(3); H=2, hidden chunk 4, KV chunk 4
    p = po.plan([5, 9, 3], [0, 1, 0], 2, 4, 4)
    assert p["split_count"] == [2, 3, 1]
    assert p["ws_offset"] == [0, 2, 5]
    assert p["n_hidden_items"] == 6
    # queue 0 = head 0 (full ranges, then the 1-token tail), queue 1 = head 1, queues 2..7 empty;
    # KV items by decreasing length: 4, 4, 3, 3, 1, 1
    assert p["items"] == [
        (1, 0, 0, 4), (1, 0, 4, 8), (1, 0, 8, 9),
        (1, 1, 0, 4), (1, 1, 4, 8), (1, 1, 8, 9),
        (0, 0, 0, 4), (0, 1, 0, 4), (2, 0, 0, 3), (2, 1, 0, 3), (0, 0, 4, 5), (0, 1, 4, 5),
    ]
    assert p["queue_offset"] == [0, 3, 6, 6, 6, 6, 6, 6, 6]


def test_plan_rejects_bad_input():
    with pytest.raises(ValueError):
        po.plan([0], [0], 1, 4, 4)
    with pytest.raises(ValueError):
        po.plan([3], [2], 1, 4, 4)
