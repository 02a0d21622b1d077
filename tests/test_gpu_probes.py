"""The machine probes do what the header says (they only serve the benchmark's denominators,
so the checks are about bounds and bookkeeping, not about the paper's method)."""
import pytest
import torch

from paper_2201_05989_amd import probe_atomic_add, probe_copy, probe_gather, probe_gather_lines

pytestmark = pytest.mark.gpu


def test_copy_copies_every_byte_including_a_ragged_grid():
    for n in (4, 4 * 1000 + 4, 1 << 22):
        src = torch.arange(n, dtype=torch.int32, device="cuda")
        dst = torch.zeros_like(src)
        probe_copy(src, dst)
        assert torch.equal(src, dst)


def test_gather_reads_only_inside_the_table_and_sums_what_it_read():
    table = torch.full((1 << 12,), 3, dtype=torch.int32, device="cuda")
    n = 4096 * 5
    sink = torch.zeros(n // 16, dtype=torch.int32, device="cuda")
    probe_gather(table, n, sink)
    assert bool((sink == 48).all())  # 16 loads of the value 3 per thread, wherever they fall


def test_atomic_add_adds_exactly_n_ones_spread_over_the_table():
    table = torch.zeros(1 << 10, dtype=torch.float32, device="cuda")
    guard = torch.zeros(1 << 10, dtype=torch.float32, device="cuda")
    n = 4096 * 8
    probe_atomic_add(table, n, seed=5)
    assert float(table.sum()) == float(n)
    assert int((table > 0).sum()) > 900  # pseudo-random addresses reach nearly every word
    assert float(guard.sum()) == 0.0


def test_gather_lines_reads_only_inside_its_slices_and_sums_what_it_read():
    # 3 slices of 2^10 words holding 1, 2, 3; a guard slice after them must never be read (its value would show)
    words, levels, n = 1 << 10, 7, 1024 * 3
    table = torch.cat([torch.full((words,), v, dtype=torch.int32, device="cuda") for v in (1, 2, 3, 1000000)])
    sink = torch.zeros(n, dtype=torch.int32, device="cuda")
    probe_gather_lines(table, words, 3, n, levels, sink)
    expect = 8 * sum((1, 2, 3)[l % 3] for l in range(levels))  # 8 words per point and level
    assert bool((sink == expect).all())
