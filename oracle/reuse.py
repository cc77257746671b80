"""Draft extension by reuse of rejected draft tokens (test infrastructure only).

Sec. 4.3 ("Reuse strategy", Eq. (reuse)): with drafts x = [T, x_1..x_n], the
model's predictions y = [y_1..y_{n+1}] (y_i follows x_{i-1}) and a rejection at
position e, the segment of x kept for later steps is the longest run of
positions after e on which draft and prediction agree,

    gamma, epsilon = argmax (epsilon - gamma)  s.t.  y_i = x_i  for all i in [e+gamma, e+epsilon].

The paper calls the search over all (gamma, epsilon) cubic; `reuse_segment` is
exactly that enumeration.  The kept segment "is retained across at least one
decoding step and discarded once its accumulated lifetime or total draft length
exceeds a predefined threshold"; the total length cap is 32 (Sec. 5.1).

Readings where the text is silent:
  * the run starts after e (gamma >= 1): position e itself now holds the
    corrected token y_e, so x_e is never part of the segment, also when a
    stochastic rejection happened at a position whose arg-max equals x_e;
  * among runs of equal length the earliest one is kept;
  * no rejection (all n drafts accepted) keeps nothing;
  * one segment is held at a time; a newly found segment replaces the held one
    only if it is longer ("length-first"), and then starts a new lifetime;
  * the lifetime counts verify steps since the segment was found; a segment is
    dropped when its age exceeds the limit, or when appending it to the fresh
    drafts of a step would exceed the cap (it is not truncated).
"""


def reuse_segment(x, y, n_accept):
    """x: drafts x_1..x_n; y: predictions y_1..y_{n+1}; n_accept = e - 1 accepted drafts.

    Returns (start, length): the kept segment is x_start..x_{start+length-1}
    (1-based draft indices), (0, 0) if there is none.  Every pair of end points
    is tried, in increasing order of start then end, and a strictly longer
    all-equal range replaces the best so far.
    """
    n = len(x)
    assert len(y) == n + 1 and 0 <= n_accept <= n
    if n_accept == n:
        return 0, 0
    e = n_accept + 1
    best = (0, 0)
    for first in range(e + 1, n + 1):
        for last in range(first, n + 1):
            if all(x[i - 1] == y[i - 1] for i in range(first, last + 1)):
                if last - first + 1 > best[1]:
                    best = (first, last - first + 1)
    return best


class ReusePool:
    """The one segment held between steps, with its age in verify steps."""

    def __init__(self, max_age, cap=32):
        self.max_age = max_age
        self.cap = cap
        self.tokens = []
        self.age = 0

    def update(self, x, start, length):
        """After a verify step with drafts x and the segment found in it."""
        if self.tokens:
            self.age += 1
            if self.age > self.max_age:
                self.tokens, self.age = [], 0
        if length > len(self.tokens):
            self.tokens, self.age = [int(t) for t in x[start - 1:start - 1 + length]], 0

    def extend(self, fresh):
        """Drafts of the next step: the fresh ones, then the held segment if the total fits the cap
        (a segment that does not fit is dropped)."""
        fresh = [int(t) for t in fresh]
        if not self.tokens:
            return fresh
        if len(fresh) + len(self.tokens) > self.cap:
            self.tokens, self.age = [], 0
            return fresh
        return fresh + self.tokens
