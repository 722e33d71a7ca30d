"""Host logic of partial-range updates, checked on the CPU: which chunks of the
gradient row a call launches.  A chunk that holds a column of some tensor
must be launched (else parameters would silently stay un-updated); chunks in
wide gaps must not be; gaps of up to 64 chunks stay inside a run."""
import numpy as np
import pytest

import paper_1604_00981_amd as bs

A = 0x1000                                              # a fake, aligned device address: never dereferenced
MERGE = 64


def _runs(layout, chunk_cols):
    tz = bs.make_tensors([(A, None, None, o, n) for o, n in layout])
    return bs.bsgd_debug_chunk_runs(tz, chunk_cols)


def _needed_chunks(layout, chunk_cols):
    live = [(o, n) for o, n in layout if n > 0]
    base = min(o for o, _ in live) // 4 * 4
    need = set()
    for o, n in live:
        need.update(range((o - base) // chunk_cols, (o + n - 1 - base) // chunk_cols + 1))
    return need


def _random_layout(r, tensors, max_size, gap_p, max_gap):
    layout, o = [], int(r.integers(0, 9))
    for _ in range(tensors):
        n = int(r.integers(0, max_size))
        layout.append((o, n))
        o += n
        if r.random() < gap_p:
            o += int(r.integers(1, max_gap))
    order = r.permutation(len(layout))
    return [layout[i] for i in order]                   # tensors may be listed in any order


@pytest.mark.parametrize("chunk_cols", [1024, 4096, 8192])
@pytest.mark.parametrize("seed", range(40))
def test_runs_cover_every_chunk_that_holds_a_tensor_column_and_skip_wide_gaps(seed, chunk_cols):
    r = np.random.default_rng(seed)
    layout = _random_layout(r, tensors=int(r.integers(2, 60)), max_size=int(r.choice([50, 5000, 300_000])),
                            gap_p=float(r.choice([0.05, 0.3, 0.9])), max_gap=int(r.choice([40, 20_000, 3_000_000])))
    if not any(n > 0 for _, n in layout):
        layout.append((0, 5))
    runs = _runs(layout, chunk_cols)
    need = _needed_chunks(layout, chunk_cols)
    launched = set()
    for first, count in runs:
        assert count >= 1
        assert first in need and first + count - 1 in need          # a run starts and ends on a chunk with work
        launched.update(range(first, first + count))
    assert need <= launched                                          # nothing that needs updating is skipped
    for (f0, c0), (f1, _) in zip(runs, runs[1:]):
        assert f1 - (f0 + c0) > MERGE                                # runs are apart by more than the tolerated gap
    # inside a run no stretch of more than MERGE chunks is idle
    idle = sorted(launched - need)
    streak = 0
    for a, b in zip(idle, idle[1:]):
        streak = streak + 1 if b == a + 1 else 0
        assert streak < MERGE
    assert len(launched) - len(need) <= MERGE * max(0, len([1 for _ in layout]) - 1)


def test_hand_cases():
    # one tensor: one run over all of its chunks, counted from its own first column
    assert _runs([(5000, 10_000)], 1024) == [(0, 10)]                # base 5000: columns 5000..14999 in chunks of 1024
    # two tensors 1000 chunks apart: two runs; 10 chunks apart: one
    assert _runs([(0, 2048), (2048 + 1000 * 1024, 1024)], 1024) == [(0, 2), (1002, 1)]
    assert _runs([(0, 2048), (2048 + 10 * 1024, 1024)], 1024) == [(0, 13)]
    # exactly at the tolerance: 64 idle chunks are kept, 65 are not
    assert _runs([(0, 1024), (1024 + 64 * 1024, 1024)], 1024) == [(0, 66)]
    assert _runs([(0, 1024), (1024 + 65 * 1024, 1024)], 1024) == [(0, 1), (66, 1)]
    # empty tensors take no part; order of the list does not matter
    assert _runs([(9_000_000, 0), (4096, 100), (0, 100)], 4096) == [(0, 2)]
    # overlap is refused
    with pytest.raises(bs.BsgdError):
        _runs([(0, 100), (50, 100)], 1024)
