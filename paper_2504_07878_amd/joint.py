"""Token-level routing loop over two models on one GPU (the paper's `joint` mode, Section 3.1 and Figure 2).

The small model decodes; whenever its router flags a position, the large model produces that token instead, and the small
model continues from it. Both models keep KV caches: the large model is brought up to date only when it is needed, with a
prefill the first time and a catch-up step (`tr_extend`) afterwards, so the several rounds of prefill and decode inside one
request (Figure 2) never recompute a prefix (the prototype of Section 4.1 has no cache and re-runs it).

This module is host control flow only: every tensor operation runs in the library's kernels, called through the C ABI
binding. One device-to-host copy of the flags and tokens per step decides which sequences call the large model.
"""
from __future__ import annotations

import numpy as np

NEEDED = ("token", "flag")     # all the host loop reads back per step: 8 bytes per sequence


def generate(slm, llm, prompts, max_new: int):
    """Greedy joint decoding of len(prompts) sequences (slot b of both models serves sequence b).

    slm: tokroute.Model with a router; llm: tokroute.Model of the large model (its own outputs are used, its router
    fields ignored). Returns (tokens int32 [B][max_new], routed bool [B][max_new]): routed[b][t] says the large model
    produced tokens[b][t].
    """
    B = len(prompts)
    slots = list(range(B))
    seq = [list(map(int, p)) for p in prompts]
    llm_len = [0] * B                      # tokens of seq[b] the large model's cache holds
    tokens = np.zeros((B, max_new), np.int32)
    routed = np.zeros((B, max_new), bool)
    out = slm.prefill(slots, prompts).cpu(NEEDED)
    for t in range(max_new):
        tok = out.token.astype(np.int32).copy()
        flagged = [b for b in slots if out.flag[b]]
        first = [b for b in flagged if llm_len[b] == 0]
        later = [b for b in flagged if llm_len[b] > 0]
        if first:
            lo = llm.prefill(first, [seq[b] for b in first]).cpu(("token",))
            for i, b in enumerate(first):
                tok[b] = lo.token[i]
        if later:
            lo = llm.extend(later, [seq[b][llm_len[b]:] for b in later]).cpu(("token",))
            for i, b in enumerate(later):
                tok[b] = lo.token[i]
        for b in flagged:
            llm_len[b] = len(seq[b])
            routed[b, t] = True
        for b in slots:
            seq[b].append(int(tok[b]))
        tokens[:, t] = tok
        if t + 1 < max_new:
            out = slm.decode_step(slots, tok).cpu(NEEDED)
    return tokens, routed
