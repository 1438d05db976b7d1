"""Pins for oracle/pagetable.py: hand cases and churn invariants.  CPU only."""
import pytest

from oracle.pagetable import PageTable
from workloads import churn_script


def test_hand_case():
    pt = PageTable(10)
    assert pt.alloc(1, 33) == [0, 1, 2]          # ceil(33/16) = 3 lowest pages
    assert pt.alloc(2, 16) == [3]
    assert pt.alloc(3, 1) == [4]
    pt.release(2)
    pt.release(1)
    assert pt.alloc(4, 70) == [0, 1, 2, 3, 5]    # lowest free first, skipping page 4
    assert pt.slot(4, 0) == 0 and pt.slot(4, 69) == 5 * 16 + 5 and pt.slot(4, 63) == 3 * 16 + 15
    assert pt.alloc(5, 0) == []
    with pytest.raises(MemoryError):
        pt.alloc(6, 16 * 5)
    assert pt.n_free() == 4


def test_churn_keeps_pages_exclusive_and_lowest_first():
    for seed in range(5):
        pt = PageTable(64)
        for op in churn_script(seed, 64):
            if op[0] == "alloc":
                free_before = [p for p in range(64) if pt.free[p]]
                got = pt.alloc(op[1], op[2])
                assert got == free_before[:len(got)]
            else:
                pt.release(op[1])
            owned = [p for t in pt.tables.values() for p in t]
            assert len(owned) == len(set(owned))
            assert all(not pt.free[p] for p in owned)
            assert pt.n_free() == 64 - len(owned)
