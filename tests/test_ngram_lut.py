"""The library's host-side n-gram drafter against the oracle's (no GPU): same tables, same
drafts, on the hand-worked example and on random streams."""
import os

import numpy as np
import pytest

from oracle import exspec as X
from paper_2605_10380_amd import binding as B
from paper_2605_10380_amd import inputs as I

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_example():
    stream = [7, 8, 9, 7, 8, 5, 7, 8, 9, 3, 3, 3, 4, 3, 3, 4, 3, 3, 6]
    lut = B.ax_lut_build(stream, 3, 100)
    assert B.ax_lut_size(lut) == 9
    assert B.ax_lut_draft(lut, [1, 7, 8], 4) == ([9, 7, 8, 9], 4)
    assert B.ax_lut_draft(lut, [8, 9], 1) == ([7], 1)            # tie 7 / 3: first recorded wins
    assert B.ax_lut_draft(lut, [3, 3], 1) == ([4], 1)
    assert B.ax_lut_draft(lut, [2, 2], 4, selective=True) == ([], 0)
    d, hits = B.ax_lut_draft(lut, [2, 2], 4, selective=False, seed=5)
    assert len(d) == 4 and d[0] == X.splitmix64(5) % 100
    assert B.ax_lut_draft(lut, [7], 2) == ([], 0)                 # not enough context
    B.ax_lut_free(lut)
    assert B.ax_lut_size(lut) == -1


@pytest.mark.parametrize("n", [1, 2, 3, 4])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_random_streams_match_oracle(n, seed):
    vocab = 23                                                   # small: many repeated keys and ties
    stream = I.zipf_tokens(vocab, seed, "lut", 400)
    ref = X.build_lut(stream, n)
    lut = B.ax_lut_build(stream, n, vocab)
    assert B.ax_lut_size(lut) == len(ref)
    rng = np.random.default_rng(seed)
    for trial in range(60):
        ctx = rng.integers(0, vocab, size=int(rng.integers(0, 6))).tolist()
        sel = bool(trial % 2)
        k = int(rng.integers(0, 7))
        want = X.draft(ref, n, ctx, k, sel, vocab, seed * 7, trial)
        got = B.ax_lut_draft(lut, ctx, k, sel, seed * 7, trial)
        assert got == (want[0], want[1]), (n, ctx, k, sel)
    B.ax_lut_free(lut)


def test_bad_arguments():
    with pytest.raises(B.AxError):
        B.ax_lut_build([1, 2, 3], 0, 10)
    with pytest.raises(B.AxError):
        B.ax_lut_build([1, 2, 30], 3, 10)
    lut = B.ax_lut_build([], 3, 10)                               # empty stream: empty table
    assert B.ax_lut_size(lut) == 0 and B.ax_lut_draft(lut, [1, 2], 3) == ([], 0)
    B.ax_lut_free(lut)
