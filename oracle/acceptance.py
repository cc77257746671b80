"""Acceptance rules of the draft-verify step (test infrastructure only).

Greedy ("strict verify", lossless): Sec. 3 and Sec. 4.3 -- with drafts
x = [T, x_1..x_k] and predictions y = [y_1..y_{k+1}], the first e with
x_e != y_e ends the accepted prefix; the step emits x_1..x_{e-1}, y_e.  If no
draft mismatches, all k are kept and y_{k+1} is emitted as a bonus.

Stochastic: the paper relies on speculative sampling, from the work it cites
in Sec. 3 for keeping the target's output distribution, without printing the rule; the
rule below is the standard one from that literature: accept x_i with
probability min(1, p_i(x_i)/q_i(x_i)); at the first rejection draw the
replacement from the normalised positive part of p_i - q_i; if nothing is
rejected draw a bonus token from p_{k+1}.  All random numbers are inputs.

Decisions on floating point follow one convention on both sides of the parity
tests: logits are float32 values; the arg-max is taken on those values with the
lowest id winning ties; probabilities are float64.
"""
import numpy as np


def _argmax_rows(z):
    return np.argmax(np.asarray(z, dtype=np.float32), axis=-1).astype(np.int32)


def first_token(z_last, temperature=0.0, u=None):
    """First generated token after prefill, from the last prompt row's logits.

    temperature == 0: arg-max; otherwise inverse-CDF sample of
    softmax(z / temperature) with the supplied uniform u in [0, 1).
    """
    z = np.asarray(z_last, dtype=np.float32)
    if temperature == 0.0:
        return int(np.argmax(z))
    p = softmax_t(z, temperature)
    return inverse_cdf(p, u)


def softmax_t(z_row, temperature):
    """softmax(z / T) in float64 from float32 logits; T is a float32 value."""
    z = np.asarray(z_row, dtype=np.float32).astype(np.float64)
    t = np.float64(np.float32(temperature))
    e = np.exp((z - z.max()) / t)
    return e / e.sum()


def inverse_cdf(weights, u):
    """Smallest id w with sum_{j<=w} weights[j] > u * sum_j weights[j].

    `weights` need not be normalised.  u in [0, 1) always yields an id of
    positive weight.
    """
    c = np.cumsum(np.asarray(weights, dtype=np.float64))
    w = int(np.searchsorted(c, np.float64(u) * c[-1], side="right"))
    return min(w, len(c) - 1)


def greedy_accept(z, drafts):
    """Greedy rule.  z: logits [k+1, V]; drafts: ids [k].

    Returns (n_accept, out_tokens[n_accept+1], y[k+1]) where y is the per-row
    arg-max, n_accept = number of leading drafts with x_i == y_i, and
    out_tokens = x_1..x_a followed by y_{a+1}.
    """
    drafts = np.asarray(drafts, dtype=np.int32)
    y = _argmax_rows(z)
    a = 0
    while a < len(drafts) and drafts[a] == y[a]:
        a += 1
    out = np.concatenate([drafts[:a], y[a:a + 1]]).astype(np.int32)
    return a, out, y


def stochastic_accept(z, drafts, q, u, temperature):
    """Speculative-sampling rule.

    z: logits [k+1, V] (float32 values); drafts: ids [k];
    q: draft distributions [k, V] (each row sums to 1) or None for a
       deterministic drafter (one-hot at the draft token);
    u: 2*(k+1) uniforms in [0,1): u[i] decides acceptance of draft i+1 (u[k] is
       unused), u[k+1+i] drives the replacement / bonus draw made at row i;
    temperature: applied to the target logits only.

    Returns (n_accept, out_tokens[n_accept+1], y[k+1]); y is the per-row
    arg-max of z (what a greedy target would have said at every row).
    """
    drafts = np.asarray(drafts, dtype=np.int32)
    k = len(drafts)
    m = k + 1
    u = np.asarray(u, dtype=np.float32).astype(np.float64)
    y = _argmax_rows(z)
    out = []
    for i in range(k):
        p = softmax_t(z[i], temperature)
        x = int(drafts[i])
        if q is None:
            qi = np.zeros_like(p)
            qi[x] = 1.0
        else:
            qi = np.asarray(q[i], dtype=np.float32).astype(np.float64)
        if u[i] * qi[x] < p[x]:
            out.append(x)
            continue
        r = np.maximum(p - qi, 0.0)
        if r.sum() == 0.0:
            r = p
        out.append(inverse_cdf(r, u[m + i]))
        return i, np.asarray(out, dtype=np.int32), y
    p = softmax_t(z[k], temperature)
    out.append(inverse_cdf(p, u[m + k]))
    return k, np.asarray(out, dtype=np.int32), y
