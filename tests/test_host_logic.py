"""CPU-only checks of two index rules that the kernels rely on, written out again in Python from
their descriptions (the device code is not run here): the XCD-aware numbering of the wide FFN
kernels' workgroups must be a one-to-one map onto the (item, part) pairs, and the cut of a long
expert into equal work items must give positive, tile-sized items that add up to the expert's rows."""
import random


def xcd_virtual_id(wg: int, total: int, xcds: int = 8) -> int:
    """Workgroups go to the XCDs round-robin by linear id; XCD x gets the contiguous range of
    virtual ids that starts after the ranges of the XCDs before it."""
    x, q, r = wg % xcds, total // xcds, total % xcds
    return x * q + min(x, r) + wg // xcds


def test_xcd_numbering_is_a_bijection_and_keeps_an_item_on_one_xcd():
    rng = random.Random(7)
    for _ in range(300):
        items, parts = rng.randint(1, 700), rng.choice([1, 2, 3, 6, 8, 11, 12, 16, 24])
        total = items * parts
        seen = [xcd_virtual_id(w, total) for w in range(total)]
        assert sorted(seen) == list(range(total))
        # consecutive virtual ids of one XCD are consecutive: an item's parts meet on one XCD
        # except where an XCD's range ends inside an item (at most 7 items in all)
        owner = {}
        for w, v in enumerate(seen):
            owner.setdefault(v // parts, set()).add(w % 8)
        split = sum(1 for xs in owner.values() if len(xs) > 1)
        assert split <= 7, (items, parts, split)


def cut_expert(rows: int, item_rows: int):
    """Items of one expert: as many as rows / item_rows rounded up; from 128-row items on, two to
    four items share the rows equally, rounded up to 16-row tiles."""
    n = -(-rows // item_rows)
    per = item_rows
    if item_rows >= 128 and 2 <= n <= 4:
        per = (-(-rows // n) + 15) // 16 * 16
    return [min(per, rows - j * per) for j in range(n)]


def test_long_experts_are_cut_into_positive_tile_sized_items():
    for item_rows in (32, 64, 128, 256):
        for rows in range(1, 4 * item_rows + 40):
            items = cut_expert(rows, item_rows)
            assert sum(items) == rows
            assert all(0 < c <= item_rows for c in items), (rows, item_rows, items)
            assert all(c % 16 == 0 for c in items[:-1]) or item_rows < 128 or len(items) > 4
