"""The helpers that choose where x, G and z lie in device memory (allocation plumbing only)."""
import pytest
import torch

from paper_2208_05631_amd import placement


def test_choose_rows_takes_the_fastest_ordered_choice():
    rows = ["a", "b", "c", "d"]
    cost = {"a": 1.0, "b": 5.0, "c": 0.5, "d": 3.0}
    seen = []

    def probe(r0, r1):                       # order matters: the first row weighs double
        seen.append((r0, r1))
        return 2 * cost[r0] + cost[r1]

    best, table = placement.choose_rows(rows, 2, probe, ordered=True)
    assert best == (2, 0)                    # c then a: 2 * 0.5 + 1.0
    assert len(table) == 12 and len(seen) == 12 and table[(2, 0)] == 2.0
    assert table[(0, 2)] == 2.5              # the reverse order is a different choice
    # combinations in index order, stopping at the first that is good enough
    del seen[:]
    best, table = placement.choose_rows(rows, 2, probe, good_enough_ms=2.6)
    assert best == (0, 2) and list(table) == [(0, 1), (0, 2)] and len(seen) == 2
    best, table = placement.choose_rows(rows, 2, probe, good_enough_ms=0.1)      # never met: all tried
    assert len(table) == 6 and best == (0, 2)


@pytest.mark.gpu
def test_spread_rows_are_zero_and_distinct_and_the_spacers_are_returned():
    dev = torch.device("cuda:0")
    before = torch.cuda.memory_reserved(dev)
    rows, spacer = placement.spread_rows(3, 1 << 24, dev, spacer_bytes=256 << 20, reserve_bytes=1 << 30)
    assert spacer == 256 << 20 and len(rows) == 3
    ptrs = sorted(r.data_ptr() for r in rows)
    assert all(b - a >= 64 << 20 for a, b in zip(ptrs, ptrs[1:]))            # no overlap
    print("distances between the rows' addresses, MiB:", [(b - a) >> 20 for a, b in zip(ptrs, ptrs[1:])])
    assert all(r.dtype == torch.float32 and r.numel() == 1 << 24 and not r.any() for r in rows)
    # the spacers went back to the driver: only the rows (and what torch rounds them to) stay
    assert torch.cuda.memory_reserved(dev) - before < 256 << 20
