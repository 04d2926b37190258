"""GPU parity with the paged KV cache (kv_page > 0): the same function as with contiguous slots, so the oracle (which knows
nothing of pages) is the reference for every call; page sharing after a fork, copies before writes into shared pages,
pages given back by rollbacks and restarts, and an exhausted pool are exercised through the C ABI."""
import numpy as np
import pytest

from paper_2504_07878_amd import synth
from parity import compare_outputs

pytestmark = pytest.mark.gpu
SEED = 7878


@pytest.fixture(scope="module")
def tr():
    from paper_2504_07878_amd import tokroute
    tokroute.load_library()
    return tokroute


def small(dtype=synth.BF16):
    s = synth.TINY.with_(dtype=dtype, kv_dtype=synth.BF16)
    return s, synth.make_weights(s, SEED + 21, std=0.05, bias_std=0.05, gain_std=0.1)


@pytest.mark.parametrize("page,B", [(32, 3), (64, 3), (64, 21), (128, 70), (32, 70)])
def test_paged_prefill_decode_and_catch_up(tr, tro, page, B):
    """Ragged prompts, decode steps and a catch-up step on every kernel family (3 rows: streaming kernels and the chunked
    attention; 21: matrix-core GEMMs; 70: the row attention kernel), pages of 32 to 128 positions."""
    s, w = small()
    max_seq = 260
    g = tr.Model(s.asdict(), w, B, max_seq, kv_page=page); o = tro.Model(s.asdict(), w, B, max_seq)
    lens = synth.prompt_lengths(SEED, f"pg.lens{page}.{B}", B, 1, 200)
    lens[0], lens[1] = 1, page            # a single token; exactly one full page
    prompts = [synth.prompt_tokens(SEED, f"pg{page}.{B}.{i}", int(n), s.vocab) for i, n in enumerate(lens)]
    slots = list(np.random.default_rng(B + page).permutation(B))
    go = g.prefill(slots, prompts, want_logits=True).cpu(); oo = o.prefill(slots, prompts, want_logits=True)
    ex = compare_outputs(go, oo, s.dtype, s.threshold, f"paged {page} B={B} prefill")
    for step in range(3):
        toks = oo.token.copy()
        go = g.decode_step(slots, toks, want_logits=True).cpu(); oo = o.decode_step(slots, toks, want_logits=True)
        ex += compare_outputs(go, oo, s.dtype, s.threshold, f"paged {page} B={B} step {step}")
    segs = [synth.prompt_tokens(SEED, f"pg{page}.{B}.seg{i}", 1 + 7 * (i % 6), s.vocab) for i in range(B)]
    go = g.extend(slots, segs, want_logits=True).cpu(); oo = o.extend(slots, segs, want_logits=True)
    ex += compare_outputs(go, oo, s.dtype, s.threshold, f"paged {page} B={B} catch-up")
    assert ex <= 2
    for i, slot in enumerate(slots):
        assert g.seq_len(slot) == o.seq_len(slot) == lens[i] + 3 + len(segs[i])


@pytest.mark.parametrize("B,ctx", [(3, 1200), (12, 2300)])
def test_paged_long_contexts(tr, tro, B, ctx):
    """Contexts of many pages: the chunked attention with its merges, and rows split into parts."""
    s, w = small()
    max_seq = ctx + 8
    g = tr.Model(s.asdict(), w, B, max_seq, kv_page=64); o = tro.Model(s.asdict(), w, B, max_seq)
    lens = [ctx - 37 * i for i in range(B)]
    prompts = [synth.prompt_tokens(SEED, f"pgl{ctx}.{i}", n, s.vocab) for i, n in enumerate(lens)]
    slots = list(range(B))
    go = g.prefill(slots, prompts, want_logits=True).cpu(); oo = o.prefill(slots, prompts, want_logits=True)
    ex = compare_outputs(go, oo, s.dtype, s.threshold, "paged long prefill")
    for step in range(3):
        toks = oo.token.copy()
        go = g.decode_step(slots, toks, want_logits=True).cpu(); oo = o.decode_step(slots, toks, want_logits=True)
        ex += compare_outputs(go, oo, s.dtype, s.threshold, f"paged long step {step}")
    assert ex <= 1


def test_paged_fork_shares_pages_and_copies_before_writing(tr, tro):
    """A fork must leave both sequences independent although they start on the same pages: both continue with different
    tokens (each write into the shared last page needs a private copy first), one is rolled back INTO a shared page and
    continues from there, one is restarted; all against the oracle, whose forks are plain copies."""
    s, w = small()
    B, max_seq, page = 4, 300, 32
    g = tr.Model(s.asdict(), w, B, max_seq, kv_page=page); o = tro.Model(s.asdict(), w, B, max_seq)
    p0 = synth.prompt_tokens(SEED, "pgf.p0", 77, s.vocab)          # 2 full pages + 13 positions
    for m in (g, o):
        m.prefill([0], [p0])
        m.seq_fork(0, 1); m.seq_fork(0, 2)
    ex = 0
    rng = np.random.default_rng(5)
    for step in range(40):                                           # crosses a page boundary on the way
        toks = rng.integers(0, s.vocab, 3).astype(np.int32)
        go = g.decode_step([0, 1, 2], toks, want_logits=True).cpu(); oo = o.decode_step([0, 1, 2], toks, want_logits=True)
        ex += compare_outputs(go, oo, s.dtype, s.threshold, f"fork step {step}")
    for m in (g, o):
        m.seq_truncate(1, 40)                                        # back into page 1, which slots 0 and 2 still share
        m.seq_fork(1, 3)
    seg = [synth.prompt_tokens(SEED, f"pgf.seg{i}", n, s.vocab) for i, n in enumerate((50, 9))]
    go = g.extend([1, 3], seg, want_logits=True).cpu(); oo = o.extend([1, 3], seg, want_logits=True)
    ex += compare_outputs(go, oo, s.dtype, s.threshold, "extend after rollback into a shared page")
    toks = rng.integers(0, s.vocab, 4).astype(np.int32)
    go = g.decode_step([0, 1, 2, 3], toks, want_logits=True).cpu(); oo = o.decode_step([0, 1, 2, 3], toks, want_logits=True)
    ex += compare_outputs(go, oo, s.dtype, s.threshold, "everyone after the rollback")
    p2 = synth.prompt_tokens(SEED, "pgf.p2", 33, s.vocab)
    go = g.prefill([2], [p2], want_logits=True).cpu(); oo = o.prefill([2], [p2], want_logits=True)      # restart a sharer
    ex += compare_outputs(go, oo, s.dtype, s.threshold, "restart of a sharer")
    toks = rng.integers(0, s.vocab, 4).astype(np.int32)
    go = g.decode_step([3, 2, 1, 0], toks, want_logits=True).cpu(); oo = o.decode_step([3, 2, 1, 0], toks, want_logits=True)
    ex += compare_outputs(go, oo, s.dtype, s.threshold, "everyone after the restart")
    assert ex <= 2
    cnt = g.counters()
    for b in range(B):
        assert g.seq_len(b) == o.seq_len(b) and tuple(cnt[b]) == o.counters(b)


def test_paged_pool_runs_out_and_recovers(tr, tro):
    """With fewer pages than the slots could ask for, a call that does not fit is refused as a whole and changes nothing;
    once another sequence has given pages back, the same call goes through, and results still equal the oracle's."""
    s, w = small()
    B, max_seq, page = 3, 256, 32
    g = tr.Model(s.asdict(), w, B, max_seq, kv_page=page, kv_pool_pages=10); o = tro.Model(s.asdict(), w, B, max_seq)
    pa, pb = synth.prompt_tokens(SEED, "pgx.a", 150, s.vocab), synth.prompt_tokens(SEED, "pgx.b", 100, s.vocab)   # 5 + 4 pages
    go = g.prefill([0, 1], [pa, pb], want_logits=True).cpu(); oo = o.prefill([0, 1], [pa, pb], want_logits=True)
    ex = compare_outputs(go, oo, s.dtype, s.threshold, "small pool prefill")
    pc = synth.prompt_tokens(SEED, "pgx.c", 70, s.vocab)                                                      # 3 pages, 1 free
    with pytest.raises(tr.TokrouteError):
        g.prefill([2], [pc])
    with pytest.raises(tr.TokrouteError):
        g.extend([1, 0], [pc[:30], pc[:20]])                                                                  # 1 + 1 pages, 1 free
    assert g.seq_len(0) == 150 and g.seq_len(1) == 100
    toks = oo.token.copy()
    go = g.decode_step([0, 1], toks, want_logits=True).cpu(); oo = o.decode_step([0, 1], toks, want_logits=True)   # no new page needed
    ex += compare_outputs(go, oo, s.dtype, s.threshold, "step after the refused calls")
    for m in (g, o):
        m.seq_truncate(0, 60)                                                                                  # gives 3 pages back
    go = g.prefill([2], [pc], want_logits=True).cpu(); oo = o.prefill([2], [pc], want_logits=True)
    ex += compare_outputs(go, oo, s.dtype, s.threshold, "prefill after a rollback freed pages")
    toks = np.array([5, 6, 7], np.int32)
    go = g.decode_step([0, 1, 2], toks, want_logits=True).cpu(); oo = o.decode_step([0, 1, 2], toks, want_logits=True)
    ex += compare_outputs(go, oo, s.dtype, s.threshold, "everyone after the recovery")
    assert ex <= 1


def test_paged_other_paths(tr, tro):
    """fp32 weights over a paged bf16 cache (streaming kernels), an imported cache, and a wide model on the split-K path
    (its finishing kernel appends to the cache)."""
    s, w = small(dtype=synth.F32)
    g = tr.Model(s.asdict(), w, 2, 200, kv_page=64); o = tro.Model(s.asdict(), w, 2, 200)
    k, v = synth.kv_fill(SEED, "pgo.kv", s, 130)
    g.load_kv(1, tr.to_device(k, s.kv_dtype), tr.to_device(v, s.kv_dtype)); o.load_kv(1, synth.bf16_bits_to_f32(k), synth.bf16_bits_to_f32(v))
    p = synth.prompt_tokens(SEED, "pgo.p", 70, s.vocab)
    go = g.prefill([0], [p], want_logits=True).cpu(); oo = o.prefill([0], [p], want_logits=True)
    ex = compare_outputs(go, oo, s.dtype, s.threshold, "fp32 weights, paged cache: prefill")
    toks = np.array([3, 4], np.int32)
    go = g.decode_step([0, 1], toks, want_logits=True).cpu(); oo = o.decode_step([0, 1], toks, want_logits=True)
    ex += compare_outputs(go, oo, s.dtype, s.threshold, "fp32 weights, paged cache: step over a prefilled and an imported cache")

    sw = synth.TINY.with_(name="wide", d_model=1024, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ffn=2048, dtype=synth.BF16, kv_dtype=synth.BF16)
    ww = synth.make_weights(sw, SEED + 22, std=0.03)
    for B in (12, 40):                                   # 40 sequences x 2 kv heads: the row attention kernel at head_dim 128
        g = tr.Model(sw.asdict(), ww, B, 160, kv_page=32); o = tro.Model(sw.asdict(), ww, B, 160)
        prompts = [synth.prompt_tokens(SEED, f"pgw.{i}", 5 + (9 * i) % 120, sw.vocab) for i in range(B)]
        slots = list(range(B))
        go = g.prefill(slots, prompts, want_logits=True).cpu(); oo = o.prefill(slots, prompts, want_logits=True)
        ex += compare_outputs(go, oo, sw.dtype, sw.threshold, f"wide model, paged cache, B={B}: prefill")
        for step in range(2):
            toks = oo.token.copy()
            go = g.decode_step(slots, toks, want_logits=True).cpu(); oo = o.decode_step(slots, toks, want_logits=True)
            ex += compare_outputs(go, oo, sw.dtype, sw.threshold, f"wide model, paged cache, B={B}: step {step}")
    assert ex <= 3


@pytest.mark.parametrize("B", [2, 33])
def test_paged_and_contiguous_caches_give_identical_bits(tr, B):
    """Paging changes where keys and values are stored, not one arithmetic operation: logits, scores and confidences of a
    paged and a contiguous context must agree bit for bit through prefill, decode steps, a catch-up step and a fork."""
    s, w = small()
    max_seq = 500
    a = tr.Model(s.asdict(), w, B + 1, max_seq); b = tr.Model(s.asdict(), w, B + 1, max_seq, kv_page=32)
    lens = synth.prompt_lengths(SEED, f"pgb.{B}", B, 1, 300)
    prompts = [synth.prompt_tokens(SEED, f"pgb.{B}.{i}", int(n), s.vocab) for i, n in enumerate(lens)]
    slots = list(range(B))

    def same(x, y, what):
        for f in ("logits", "score", "conf", "token", "flag", "hidden"):
            assert np.array_equal(getattr(x, f), getattr(y, f)), f"{what}: {f}"

    x = a.prefill(slots, prompts, want_logits=True).cpu(); y = b.prefill(slots, prompts, want_logits=True).cpu()
    same(x, y, "prefill")
    for step in range(5):
        toks = x.token.copy()
        x = a.decode_step(slots, toks, want_logits=True).cpu(); y = b.decode_step(slots, toks, want_logits=True).cpu()
        same(x, y, f"step {step}")
    for m in (a, b):
        m.seq_fork(0, B)
    segs = [synth.prompt_tokens(SEED, f"pgb.{B}.seg{i}", 1 + 5 * (i % 7), s.vocab) for i in range(B + 1)]
    x = a.extend(slots + [B], segs, want_logits=True).cpu(); y = b.extend(slots + [B], segs, want_logits=True).cpu()
    same(x, y, "catch-up after a fork")


def test_paged_config_is_validated(tr):
    s, w = small()
    for bad in (dict(kv_page=48), dict(kv_page=16), dict(kv_page=0, kv_pool_pages=4)):
        with pytest.raises(tr.TokrouteError):
            tr.Model(s.asdict(), w, 2, 64, **bad)
    s32 = synth.TINY                                     # fp32 cache: pages are refused
    with pytest.raises(tr.TokrouteError):
        tr.Model(s32.asdict(), synth.make_weights(s32, SEED), 2, 64, kv_page=32)
