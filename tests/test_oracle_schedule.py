"""Pins for the oracle's round-robin schedule (paper Section 3, Eq. (3), Figure 1)."""
import os

import numpy as np
import pytest

from oracle import givens_oracle as O


def _read_golden(golden_dir):
    seqs, blocks = [], []
    with open(os.path.join(golden_dir, "rr_schedule_n6.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            left, right = line.split("|")
            seqs.append([int(t) for t in left.replace("seq:", "").split()])
            blocks.append([tuple(int(v) for v in tok.split("-"))
                           for tok in right.replace("pairs:", "").split()])
    return seqs, blocks


def test_worked_example_n6_is_reproduced_exactly(golden_dir):
    seqs, blocks = _read_golden(golden_dir)
    assert len(seqs) == 5 and len(blocks) == 5
    got_seqs = O.circle_method_sequences(6)
    got = O.circle_method_schedule(6)
    assert got_seqs.tolist() == seqs
    assert got.shape == (5, 3, 2)
    for k in range(5):
        assert [tuple(int(v) for v in p) for p in got[k]] == blocks[k]


@pytest.mark.parametrize("n", [2, 4, 6, 8, 10, 12, 16, 30, 64, 126, 256])
def test_blocks_are_perfect_matchings_and_cover_each_pair_once(n):
    sched = O.circle_method_schedule(n)
    assert sched.shape == (n - 1, n // 2, 2)
    assert sched.dtype == np.int32
    seen = set()
    for k in range(n - 1):
        coords = sched[k].reshape(-1)
        assert sorted(coords.tolist()) == list(range(n)), "block is not a perfect matching"
        for i, j in sched[k]:
            assert 0 <= i < j < n
            assert (int(i), int(j)) not in seen
            seen.add((int(i), int(j)))
    assert len(seen) == n * (n - 1) // 2


def test_angle_counts_of_the_five_workloads():
    for n, count in [(8, 28), (256, 32640), (1024, 523776), (4096, 8386560), (2048, 2096128)]:
        assert n * (n - 1) // 2 == count
        assert (n - 1) * (n // 2) == count


@pytest.mark.parametrize("n", [4, 6, 8, 34, 128])
def test_closed_form_of_the_dimension_sequences(n):
    """seq_k[0] = 0 and seq_k[p] = 1 + ((p - 1 - k) mod (n - 1)): a restatement of
    'hold the first element, shift the rest by one per step'."""
    seqs = O.circle_method_sequences(n)
    for k in range(n - 1):
        assert seqs[k, 0] == 0
        for p in range(1, n):
            assert seqs[k, p] == 1 + ((p - 1 - k) % (n - 1))
    sched = O.circle_method_schedule(n)
    for k in range(n - 1):
        # arc 0 always joins the held element with the element at the far end
        assert tuple(sched[k, 0]) == (0, n - 1 - k)


def test_n4_sequence_from_the_circle_method():
    # Section 2's E-tilde for n = 4 is only an illustration of an ordering; the circle
    # method itself, started from (0,1,2,3), gives these three blocks.
    got = O.circle_method_schedule(4).tolist()
    assert got == [[[0, 3], [1, 2]], [[0, 2], [1, 3]], [[0, 1], [2, 3]]]


def test_odd_or_tiny_n_is_rejected():
    for n in (0, 1, 3, 7):
        with pytest.raises(ValueError):
            O.circle_method_schedule(n)
