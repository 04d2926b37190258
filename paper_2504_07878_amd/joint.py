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


def generate_overlapped(slm, llm, prompts, max_new: int):
    """The same decoding as `generate`, sequence by sequence, scheduled for throughput: a flagged sequence waits for the
    large model while the others keep decoding.

    The large model runs on a stream of its own, one call at a time, on every sequence that is waiting when the previous call
    has finished (prefill for a sequence's first call, catch-up segments afterwards); the small model steps the sequences that
    are not waiting. What a sequence emits does not depend on the schedule (each of its positions is still the small model's
    token unless the router flags it, and the large model's otherwise), only the order in which the sequences advance does.
    Returns (tokens, routed) like `generate`.
    """
    import torch
    B = len(prompts)
    seq = [list(map(int, p)) for p in prompts]
    llm_len = [0] * B
    done = [0] * B                         # tokens emitted per sequence
    next_tok = np.zeros(B, np.int32)       # input of a running sequence's next small-model step
    running = [False] * B
    tokens = np.zeros((B, max_new), np.int32)
    routed = np.zeros((B, max_new), bool)
    pending = []                           # flagged, not yet handed to the large model
    s_small, s_large = torch.cuda.Stream(), torch.cuda.Stream()
    host_tok = torch.empty(2 * B, dtype=torch.int32, pin_memory=True)
    inflight = None                        # (sequences, output objects kept alive, event)

    def emit(b, tok, by_large):
        tokens[b, done[b]] = tok
        routed[b, done[b]] = by_large
        seq[b].append(int(tok))
        done[b] += 1
        running[b] = done[b] < max_new
        next_tok[b] = tok

    def take(bs, out):
        for i, b in enumerate(bs):
            running[b] = False
            if out.flag[i]:
                pending.append(b)
            else:
                emit(b, out.token[i], False)

    start = torch.cuda.current_stream()
    s_small.wait_stream(start); s_large.wait_stream(start)
    with torch.cuda.stream(s_small):
        take(list(range(B)), slm.prefill(list(range(B)), prompts).cpu(NEEDED, stream_only=True))
    while inflight or pending or any(running):
        if inflight and (inflight[2].query() or not any(running)):
            bs, _, ev = inflight
            ev.synchronize()
            for i, b in enumerate(bs):
                llm_len[b] = len(seq[b])
                emit(b, int(host_tok[i]), True)
            inflight = None
        if not inflight and pending:
            first = [b for b in pending if llm_len[b] == 0]
            later = [b for b in pending if llm_len[b] > 0]
            keep = []
            with torch.cuda.stream(s_large):
                if first:
                    keep.append(llm.prefill(first, [seq[b] for b in first]))
                    host_tok[:len(first)].copy_(keep[-1].token[:len(first)], non_blocking=True)
                if later:
                    keep.append(llm.extend(later, [seq[b][llm_len[b]:] for b in later]))
                    host_tok[len(first):len(first) + len(later)].copy_(keep[-1].token[:len(later)], non_blocking=True)
                ev = torch.cuda.Event()
                ev.record(s_large)
            inflight = (first + later, keep, ev)
            pending = []
        run = [b for b in range(B) if running[b]]
        if run:
            with torch.cuda.stream(s_small):
                take(run, slm.decode_step(run, next_tok[run]).cpu(NEEDED, stream_only=True))
    start.wait_stream(s_small); start.wait_stream(s_large)
    return tokens, routed
