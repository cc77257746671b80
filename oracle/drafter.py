"""Retrieval drafter over the token history (test infrastructure only).

Sec. 3 ("retrieval-based SD ... drafts candidate tokens directly from context")
and Sec. 5.1 (the suffix-automaton retrieval of the compared systems): the
draft is what followed, earlier in the text, the longest suffix of the text so
far.  `suffix_match_draft` is that definition written out as a search: suffix
lengths from the longest allowed down to the shortest, earlier occurrences
from the most recent back; the first hit gives the continuation.

Readings where the text is silent: an occurrence must end before the last token
(it is an *earlier* occurrence and has at least one token after it); among
occurrences of the longest matching suffix the most recent one is used; the
continuation may run into the suffix itself and stops at the end of the
history or after k tokens.
"""


def suffix_match_draft(history, k, max_suffix, min_suffix=1):
    """history: token ids so far (prompt and generated); returns up to k draft tokens ([] if no
    suffix of length min_suffix..max_suffix occurs earlier)."""
    history = [int(t) for t in history]
    n = len(history)
    if k <= 0:
        return []
    for length in range(min(max_suffix, n - 1), min_suffix - 1, -1):
        suffix = history[n - length:]
        for start in range(n - length - 1, -1, -1):
            if history[start:start + length] == suffix:
                return history[start + length:start + length + k]
    return []
