"""The library's host-side reuse pool against the oracle's, and the argument checks of the reuse
entry points (no GPU: these functions run on the host or fail before anything is launched)."""
import ctypes as C

import numpy as np
from hypothesis import given, settings, strategies as st

from oracle.reuse import ReusePool
import paper_2510_15312_amd as vf

_step = st.tuples(st.lists(st.integers(0, 99), min_size=0, max_size=32),   # drafts of a step
                  st.integers(0, 31), st.integers(0, 32),                  # raw segment start / length
                  st.integers(0, 34))                                      # fresh drafts of the next step


@settings(max_examples=200, deadline=None)
@given(st.integers(0, 4), st.integers(1, 32), st.lists(_step, min_size=1, max_size=12))
def test_pool_follows_the_oracle_through_random_steps(max_age, cap, steps):
    pool = vf.vf_reuse_pool_init(max_age, cap)
    ref = ReusePool(max_age, cap)
    for drafts, s0, ln, n_fresh in steps:
        n = len(drafts)
        ln = min(ln, n)
        start = 0 if ln == 0 else 1 + s0 % (n - ln + 1)
        vf.vf_reuse_pool_update(pool, drafts, start, ln)
        ref.update(drafts, start, ln)
        assert list(pool.tokens[:pool.len]) == ref.tokens and pool.age == ref.age
        fresh = list(range(1000, 1000 + min(n_fresh, cap)))
        assert vf.vf_reuse_pool_extend(pool, fresh) == ref.extend(fresh)
        assert list(pool.tokens[:pool.len]) == ref.tokens and pool.age == ref.age


def test_reuse_argument_errors():
    L = vf.lib
    pool = vf.binding.vf_reuse_pool()
    assert L.vf_reuse_pool_init(None, 1, 8) == vf.VF_ERR_ARG
    assert L.vf_reuse_pool_init(C.byref(pool), -1, 8) == vf.VF_ERR_ARG
    assert L.vf_reuse_pool_init(C.byref(pool), 1, 0) == vf.VF_ERR_ARG
    assert L.vf_reuse_pool_init(C.byref(pool), 1, vf.VF_MAX_DRAFTS + 1) == vf.VF_ERR_ARG
    assert L.vf_reuse_pool_init(C.byref(pool), 1, 8) == vf.VF_OK
    d = (C.c_int32 * 4)(1, 2, 3, 4)
    assert L.vf_reuse_pool_update(C.byref(pool), d, 4, 3, 3) == vf.VF_ERR_ARG      # runs past the drafts
    assert L.vf_reuse_pool_update(C.byref(pool), d, 4, 0, 2) == vf.VF_ERR_ARG      # positions are 1-based
    assert L.vf_reuse_pool_update(C.byref(pool), None, 4, 1, 2) == vf.VF_ERR_ARG
    assert pool.len == 0
    assert L.vf_reuse_pool_extend(C.byref(pool), d, 9) == vf.VF_ERR_ARG           # more fresh drafts than cap
    assert L.vf_reuse_pool_extend(None, d, 1) == vf.VF_ERR_ARG
    ro = (C.c_int32 * 2)(0, 3)
    assert L.vf_reuse_select(1, None, ro, None, None, None, None) == vf.VF_ERR_ARG
    assert L.vf_reuse_select(0, None, ro, None, None, None, None) == vf.VF_ERR_ARG
    assert L.vf_reuse_select(vf.VF_MAX_BATCH + 1, None, ro, None, None, None, None) == vf.VF_ERR_ARG
    assert vf.lib.vf_last_error()


@settings(max_examples=300, deadline=None)
@given(st.lists(st.integers(0, 2), min_size=0, max_size=60), st.integers(0, 8), st.integers(1, 6), st.integers(1, 3))
def test_retrieval_drafter_follows_the_oracle(history, k, max_suffix, min_suffix):
    from oracle.drafter import suffix_match_draft
    if min_suffix > max_suffix:
        min_suffix = max_suffix
    assert vf.vf_draft_suffix_match(history, k, max_suffix, min_suffix) == suffix_match_draft(history, k, max_suffix,
                                                                                             min_suffix)


def test_retrieval_drafter_hand_worked_cases_and_errors():
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    n = 0
    for line in open(os.path.join(here, "golden", "drafter_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        hist, k, mx, mn, want = [[int(t) for t in f.split()] for f in line.split("|")]
        assert vf.vf_draft_suffix_match(hist, k[0], mx[0], mn[0]) == want, line
        n += 1
    assert n == 8
    L = vf.lib
    h = (C.c_int32 * 4)(1, 2, 1, 2)
    out = (C.c_int32 * 32)()
    assert L.vf_draft_suffix_match(None, 4, 2, 1, 2, out) == vf.VF_ERR_ARG
    assert L.vf_draft_suffix_match(h, 4, 0, 1, 2, out) == vf.VF_ERR_ARG
    assert L.vf_draft_suffix_match(h, 4, 2, 3, 2, out) == vf.VF_ERR_ARG
    assert L.vf_draft_suffix_match(h, 4, 2, 1, 33, out) == vf.VF_ERR_ARG
    assert L.vf_draft_suffix_match(h, 4, 2, 1, 2, None) == vf.VF_ERR_ARG
    assert L.vf_draft_suffix_match(h, 4, 2, 1, 0, None) == 0
