"""Pins for the oracle's retrieval drafter (no GPU)."""
import os

import numpy as np
from hypothesis import given, settings, strategies as st

from oracle.drafter import suffix_match_draft

HERE = os.path.dirname(os.path.abspath(__file__))


def test_hand_worked_cases():
    n = 0
    for line in open(os.path.join(HERE, "golden", "drafter_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        hist, k, mx, mn, want = [[int(t) for t in f.split()] for f in line.split("|")]
        assert suffix_match_draft(hist, k[0], mx[0], mn[0]) == want, line
        n += 1
    assert n == 8


@settings(max_examples=300, deadline=None)
@given(st.lists(st.integers(0, 2), min_size=0, max_size=40), st.integers(1, 6), st.integers(1, 5), st.integers(1, 3))
def test_against_a_string_search(history, k, max_suffix, min_suffix):
    """Another route: the history as a byte string; bytes.rfind looks for the suffix ending before the
    last token; the longest suffix with a hit decides."""
    got = suffix_match_draft(history, k, max_suffix, min_suffix)
    data = bytes(history)
    n = len(history)
    want = []
    for length in range(min(max_suffix, n - 1), min_suffix - 1, -1):
        pos = data.rfind(data[n - length:], 0, n - 1)     # the occurrence must end at or before n - 1
        if pos >= 0:
            want = history[pos + length:pos + length + k]
            break
    assert got == want
    if got:   # the draft follows an occurrence of the matched suffix and is not longer than k
        assert len(got) <= k
