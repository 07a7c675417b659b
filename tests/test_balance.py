"""Token-balanced dispatch: the library's host entry point (C++, no GPU involved) against the oracle, part by
part.  The oracle's own pins are in test_balance_oracle_pins.py."""
import numpy as np
import pytest

import paper_2507_01663_amd as ra
from oracle.balance import partition


def sums(w, part, k):
    s = [0] * k
    for x, p in zip(w, part):
        s[p] += int(x)
    return s


@pytest.mark.parametrize("eq", [False, True])
def test_library_matches_the_oracle_part_by_part(eq):
    rng = np.random.default_rng(5)
    cases = [([8, 7, 6, 5, 4], 2), ([8, 7, 6, 5, 4], 3), ([0, 0, 0, 0], 3), ([5], 4), ([], 2), ([3, 3, 3, 3, 3, 3], 4)]
    for _ in range(40):
        n = int(rng.integers(1, 300))
        hi = int(rng.choice([3, 50, 100000]))              # many ties, some ties, hardly any
        cases.append((rng.integers(0, hi, size=n).tolist(), int(rng.integers(1, 20))))
    for w, k in cases:
        part, s = ra.rollout_attn_balance(w, k, eq)
        assert part.tolist() == partition(w, k, eq), (w, k, eq)
        assert s.tolist() == sums(w, part.tolist(), k)


def test_library_at_the_size_of_a_real_dispatch_and_bad_arguments():
    rng = np.random.default_rng(6)
    w = rng.integers(16, 40000, size=20000)
    part, s = ra.rollout_attn_balance(w, 64, True)
    cnt = np.bincount(part, minlength=64)
    assert cnt.max() - cnt.min() <= 1 and s.sum() == w.sum()
    assert (s.max() - s.min()) / s.mean() < 1e-3
    assert part.tolist() == partition(w.tolist(), 64, True)
    with pytest.raises(ra.RolloutAttnError):
        ra.rollout_attn_balance([1, -2, 3], 2)
    with pytest.raises(ra.RolloutAttnError):
        ra.rollout_attn_balance([1, 2, 3], 0)
