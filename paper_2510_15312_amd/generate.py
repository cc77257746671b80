"""Greedy generation by repeated draft-verify steps: the host loop around the library's calls.

Every piece of work is a call of the C ABI: chunked prefill (`vf_prefill_chunk`), the retrieval
drafter over the text so far (`vf_draft_suffix_match`), the pool of reusable rejected drafts
(`vf_reuse_pool_*`), the verify forward (`vf_verify`), acceptance (`vf_accept`) and the reuse
segment (`vf_reuse_select`).  This module only strings them together and moves the few integers a
step decides (accepted count, emitted tokens, reuse segment) to the host, once per step.
"""
import torch

from . import binding as vf


def generate(model, seq, prompt, n_new, k=16, max_suffix=8, min_suffix=1, chunk=256, reuse_max_age=2, drafter=None, reuse=True):
    """prompt: host ints; returns (the n_new generated tokens, statistics).  Greedy acceptance: the
    result is what plain greedy decoding would produce.  drafter(text, k) -> list of at most k draft
    ids replaces the library's suffix-match drafter (any drafter gives the same text); reuse=False
    leaves the pool of rejected drafts out."""
    dev = model.buf.device
    k = min(int(k), vf.VF_MAX_DRAFTS)
    toks = torch.as_tensor(list(prompt), dtype=torch.int32, device=dev)
    for c0 in range(0, len(prompt), chunk):
        vf.vf_prefill_chunk(model, seq, toks[c0:c0 + chunk], sample_first=c0 + chunk >= len(prompt))
    length, pending = vf.vf_seq_get_state(seq)
    text = [int(t) for t in prompt] + [pending]        # the pending token is the first generated one
    pool = vf.vf_reuse_pool_init(reuse_max_age, max(k, 1))
    n_acc = torch.zeros(1, dtype=torch.int32, device=dev)
    out = torch.zeros(vf.VF_MAX_DRAFTS + 1, dtype=torch.int32, device=dev)
    y = torch.zeros_like(out)
    seg = torch.zeros(2, dtype=torch.int32, device=dev)
    greedy = [(vf.VF_GREEDY, 0.0, None, None)]
    steps, accepted, drafted = 0, 0, 0
    while len(text) - len(prompt) < n_new:
        if not k:
            fresh = []
        elif drafter is not None:
            fresh = [int(t) for t in drafter(text, k)][:k]
        else:
            fresh = vf.vf_draft_suffix_match(text, k, max_suffix, min_suffix)
        drafts = vf.vf_reuse_pool_extend(pool, fresh) if k and reuse else fresh
        m = len(drafts) + 1
        tokens = torch.as_tensor([vf.VF_PENDING] + drafts, dtype=torch.int32, device=dev)
        vf.vf_verify(model, [seq], tokens, [0, m])
        vf.vf_accept(model, [seq], tokens, [0, m], greedy, n_acc, out[:m], y[:m])
        if drafts and reuse:
            vf.vf_reuse_select(tokens, [0, m], y[:m], n_acc, seg)
        host = torch.cat([n_acc, seg, out[:m]]).cpu().tolist()          # the step's one synchronisation
        a, seg_start, seg_len, emitted = host[0], host[1], host[2], host[3:4 + host[0]]
        if drafts and reuse:
            vf.vf_reuse_pool_update(pool, drafts, seg_start, seg_len)
        text += emitted
        length += 1 + a
        vf.vf_seq_note_len(seq, length)                 # vf_accept counted all m rows; 1 + a were kept
        steps += 1
        accepted += a
        drafted += len(drafts)
    new = text[len(prompt):len(prompt) + n_new]
    return new, {"steps": steps, "accepted_drafts": accepted, "drafted": drafted,
                 "tokens_per_step": (len(text) - len(prompt) - 1) / max(steps, 1)}
