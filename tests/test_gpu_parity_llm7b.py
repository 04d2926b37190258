"""GPU parity for the large model's decode step on routed tokens (7B-class shapes, bf16): 32 sequences with a
synthetic cache at context 2048; per step a Bernoulli(0.07) subset of the slots is stepped. The oracle follows
two slots. Run with -s to see progress lines (drawing 7.6e9 weights takes about a minute)."""
import time

import numpy as np
import pytest
import torch

from paper_2504_07878_amd import synth
from parity import compare_outputs

pytestmark = pytest.mark.gpu
SEED = 7878
S = synth.LLM_7B


def say(*a):
    print(*a, flush=True)


def test_routed_subset_decode_on_7b_shapes(tro):
    from paper_2504_07878_amd import tokroute as tr
    tr.load_library()
    B, CTX, STEPS = 32, 2048, 48
    t = time.time()
    w = synth.make_weights(S, SEED, qkv_bias=True, workers=16)
    say(f"[7b weights drawn in {time.time() - t:.0f}s]")
    t = time.time()
    g = tr.Model(S.asdict(), w, B, CTX + STEPS + 1)
    say(f"[7b weights on the GPU in {time.time() - t:.0f}s]")
    flags = synth.bernoulli_flags(SEED, "cfg5.flags", (STEPS, B), 0.07)
    hits = flags.sum(0)
    watch = [int(i) for i in np.argsort(-hits)[:2]]          # the two slots routed most often in this window
    say(f"[routed per step: {flags.sum(1).tolist()}; oracle follows slots {watch} ({hits[watch].tolist()} activations)]")
    o = tro.Model(S.asdict(), w, len(watch), CTX + STEPS + 1)
    gen = torch.Generator(device="cuda").manual_seed(SEED)
    for b in range(B):
        if b in watch:
            k, v = synth.kv_fill(SEED, f"cfg5.kv{b}", S, CTX)
            o.load_kv(watch.index(b), synth.bf16_bits_to_f32(k), synth.bf16_bits_to_f32(v))
            g.load_kv(b, tr.to_device(k, synth.BF16), tr.to_device(v, synth.BF16))
        else:   # the other slots only have to hold plausible values
            shape = (S.n_layers, S.n_kv_heads, CTX, S.head_dim)
            g.load_kv(b, torch.randn(shape, device="cuda", generator=gen).to(torch.bfloat16),
                      torch.randn(shape, device="cuda", generator=gen).to(torch.bfloat16))
    toks = synth.prompt_tokens(SEED, "cfg5.toks", STEPS * B, S.vocab).reshape(STEPS, B)
    compared, exempt, gpu_s, gpu_tokens = 0, 0, 0.0, 0
    for step in range(STEPS):
        active = [b for b in range(B) if flags[step, b]]
        if not active:
            continue
        torch.cuda.synchronize(); t0 = time.perf_counter()
        go = g.decode_step(active, toks[step, active], want_logits=True).cpu()
        gpu_s += time.perf_counter() - t0; gpu_tokens += len(active)
        for b in active:
            if b in watch:                     # every activation of the followed slots, so that both sides hold the same caches
                oo = o.decode_step([watch.index(b)], [toks[step, b]], want_logits=True)
                i = active.index(b)
                sub = type("O", (), dict(token=go.token[i:i + 1], conf=go.conf[i:i + 1], score=go.score[i:i + 1], flag=go.flag[i:i + 1],
                                         hidden=go.hidden[i:i + 1], logits=go.logits[i:i + 1]))()
                exempt += compare_outputs(sub, oo, S.dtype, 0.5, f"7b step {step} slot {b}")
                compared += 1
                say(f"[7b step {step} slot {b} ok ({len(active)} active)]")
    assert compared >= 4 and exempt <= 1
    assert (go.flag == 0).all() and (go.score == 1.0).all()          # the large model has no router
    for b in range(B):
        assert g.seq_len(b) == CTX + int(flags[:, b].sum())
    say(f"[7b: {gpu_tokens} routed tokens in {gpu_s * 1e3:.1f} ms of GPU steps (incl. logits copy) = {gpu_tokens / gpu_s:.0f} routed tok/s]")
    # catch-up of 12 tokens on the two followed slots: more than 4 rows, i.e. the split-K matrix-core path of wide models
    # (all linear layers through partials, rotary/cache append, SwiGLU and the head's softmax statistics finished separately)
    segs = [synth.prompt_tokens(SEED, f"cfg5.seg{b}", 12, S.vocab) for b in watch]
    t = time.time()
    go = g.extend(watch, segs, want_logits=True).cpu()
    oo = o.extend([0, 1], segs, want_logits=True)
    say(f"[7b catch-up of 2 x 12 tokens: oracle {time.time() - t:.0f}s]")
    assert compare_outputs(go, oo, S.dtype, 0.5, "7b extend") <= 1
    for i, b in enumerate(watch):
        assert g.seq_len(b) == o.seq_len(i)
