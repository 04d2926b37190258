"""GPU parity on the tiny fp32 model: the HIP path, called through the C ABI, against the CPU oracle."""
import numpy as np
import pytest
import torch

from paper_2504_07878_amd import synth
from parity import compare_outputs, assert_rows_close

pytestmark = pytest.mark.gpu
SEED = 7878


@pytest.fixture(scope="module")
def tr():
    from paper_2504_07878_amd import tokroute
    tokroute.load_library()
    return tokroute


@pytest.fixture(scope="module")
def tiny_weights():
    return synth.make_weights(synth.TINY, SEED)


def test_tiny_prefill_and_free_running_greedy_decode(tr, tro, tiny_weights):
    """Workload 1: batch 1, 32-token uniform prompt, 16 greedy steps, free-running: tokens must equal the oracle's."""
    s = synth.TINY
    g = tr.Model(s.asdict(), tiny_weights, 1, 64)
    o = tro.Model(s.asdict(), tiny_weights, 1, 64)
    prompt = synth.prompt_tokens(SEED, "cfg1.prompt", 32, s.vocab)
    go = g.prefill([0], [prompt], want_logits=True).cpu()
    oo = o.prefill([0], [prompt], want_logits=True)
    assert compare_outputs(go, oo, s.dtype, s.threshold, "prefill") == 0
    gt, ot = int(go.token[0]), int(oo.token[0])
    for step in range(16):
        assert gt == ot, f"free-running tokens diverged at step {step}"
        go = g.decode_step([0], [gt], want_logits=True).cpu()
        oo = o.decode_step([0], [ot], want_logits=True)
        assert compare_outputs(go, oo, s.dtype, s.threshold, f"step {step}") == 0
        gt, ot = int(go.token[0]), int(oo.token[0])
    assert g.seq_len(0) == o.seq_len(0) == 48
    assert tuple(g.counters()[0]) == o.counters(0)


def test_tiny_ragged_batch_with_biases_and_gains(tr, tro):
    """Several slots, prompts of different lengths (1 .. several attention tiles), non-zero biases and non-unit gains."""
    s = synth.TINY
    w = synth.make_weights(s, SEED + 1, std=0.05, bias_std=0.05, gain_std=0.1)
    B, max_seq = 7, 700
    g = tr.Model(s.asdict(), w, B, max_seq)
    o = tro.Model(s.asdict(), w, B, max_seq)
    lens = [1, 2, 63, 64, 65, 300, 640]
    prompts = [synth.prompt_tokens(SEED, f"rag{i}", n, s.vocab) for i, n in enumerate(lens)]
    slots = [3, 0, 6, 1, 5, 2, 4]
    go = g.prefill(slots, prompts, want_logits=True).cpu()
    oo = o.prefill(slots, prompts, want_logits=True)
    compare_outputs(go, oo, s.dtype, s.threshold, "ragged prefill")
    for step in range(5):
        toks = oo.token.copy()                      # teacher-forced with the oracle's tokens
        order = np.roll(np.arange(B), step)         # the order of slots in a call is free
        go = g.decode_step([slots[i] for i in order], toks[order], want_logits=True).cpu()
        o2 = o.decode_step([slots[i] for i in order], toks[order], want_logits=True)
        compare_outputs(go, o2, s.dtype, s.threshold, f"ragged step {step}")
        inv = np.argsort(order)
        oo = type("O", (), dict(token=o2.token[inv]))()
    for i, slot in enumerate(slots):
        assert g.seq_len(slot) == o.seq_len(slot) == lens[i] + 5
    cnt = g.counters()
    for slot in slots:
        assert tuple(cnt[slot]) == o.counters(slot)


def test_tiny_subset_of_slots_and_cache_contents(tr, tro, tiny_weights):
    s = synth.TINY
    g = tr.Model(s.asdict(), tiny_weights, 4, 128)
    o = tro.Model(s.asdict(), tiny_weights, 4, 128)
    prompts = [synth.prompt_tokens(SEED, f"sub{i}", 20 + 7 * i, s.vocab) for i in range(4)]
    g.prefill([0, 1, 2, 3], prompts); o.prefill([0, 1, 2, 3], prompts)
    # step only two of the four
    go = g.decode_step([2, 0], [5, 9], want_logits=True).cpu(); oo = o.decode_step([2, 0], [5, 9], want_logits=True)
    compare_outputs(go, oo, s.dtype, s.threshold, "subset step")
    assert [g.seq_len(i) for i in range(4)] == [o.seq_len(i) for i in range(4)] == [21, 27, 35, 41]
    # the other slots are untouched: stepping them now gives what the oracle gives
    go = g.decode_step([1, 3], [7, 8], want_logits=True).cpu(); oo = o.decode_step([1, 3], [7, 8], want_logits=True)
    compare_outputs(go, oo, s.dtype, s.threshold, "other slots")


def test_tiny_error_paths_leave_state_unchanged(tr, tiny_weights):
    s = synth.TINY
    g = tr.Model(s.asdict(), tiny_weights, 2, 16)
    g.prefill([0], [[1, 2, 3]])
    before = (g.seq_len(0), g.seq_len(1), g.counters().copy())
    cases = [(lambda: g.decode_step([1], [0]), tr.ERR_STATE),
             (lambda: g.decode_step([0, 0], [1, 1]), tr.ERR_INVALID_ARG),
             (lambda: g.decode_step([0], [s.vocab]), tr.ERR_INVALID_ARG),
             (lambda: g.decode_step([0], [-1]), tr.ERR_INVALID_ARG),
             (lambda: g.decode_step([2], [0]), tr.ERR_INVALID_ARG),
             (lambda: g.prefill([1], [list(range(17))]), tr.ERR_CAPACITY),
             (lambda: g.prefill([1], [[]]), tr.ERR_INVALID_ARG),
             (lambda: g.seq_truncate(0, 4), tr.ERR_INVALID_ARG),
             (lambda: g.seq_truncate(1, 0), tr.ERR_STATE),
             (lambda: g.set_mode(7), tr.ERR_INVALID_ARG)]
    for fn, code in cases:
        with pytest.raises(tr.TokrouteError) as e:
            fn()
        assert e.value.code == code, (code, e.value)
        assert (g.seq_len(0), g.seq_len(1)) == before[:2] and np.array_equal(g.counters(), before[2])
    while g.seq_len(0) < 16:
        g.decode_step([0], [1])
    with pytest.raises(tr.TokrouteError) as e:
        g.decode_step([0], [1])
    assert e.value.code == tr.ERR_CAPACITY and g.seq_len(0) == 16


def test_tiny_modes_threshold_and_options(tr, tro, tiny_weights):
    s = synth.TINY
    prompt = synth.prompt_tokens(SEED, "modes", 12, s.vocab)
    g = tr.Model(s.asdict(), tiny_weights, 1, 64); o = tro.Model(s.asdict(), tiny_weights, 1, 64)
    g.prefill([0], [prompt]); o.prefill([0], [prompt])
    for thr, mode in ((0.0, tr.JOINT), (1.0, tr.JOINT), (1.0, tr.SMALL_ONLY), (0.5, tr.JOINT)):
        g.set_threshold(thr); o.set_threshold(thr); g.set_mode(mode); o.set_mode(mode)
        go = g.decode_step([0], [3], want_logits=True).cpu(); oo = o.decode_step([0], [3], want_logits=True)
        compare_outputs(go, oo, s.dtype, thr, f"thr {thr} mode {mode}", joint=mode == tr.JOINT)
        assert int(go.flag[0]) == (1 if (thr == 1.0 and mode == tr.JOINT) else 0 if thr != 0.5 else int(go.flag[0]))
    assert tuple(g.counters()[0]) == o.counters(0)
    # pre-norm hidden tap and the opposite routing direction
    g2 = tr.Model(s.asdict(), tiny_weights, 1, 64, route_dir=tr.ROUTE_IF_ABOVE, hidden_tap=tr.PRE_FINAL_NORM)
    o2 = tro.Model(s.asdict(), tiny_weights, 1, 64, route_dir=tro.ROUTE_IF_ABOVE, hidden_tap=tro.PRE_FINAL_NORM)
    go = g2.prefill([0], [prompt], want_logits=True).cpu(); oo = o2.prefill([0], [prompt], want_logits=True)
    compare_outputs(go, oo, s.dtype, s.threshold, "options", route_dir_below=False)


def test_tiny_truncate_and_replace_token(tr, tro, tiny_weights):
    """A token from the large model replaces the small model's next input; rolling back needs no recompute."""
    s = synth.TINY
    g = tr.Model(s.asdict(), tiny_weights, 1, 64); o = tro.Model(s.asdict(), tiny_weights, 1, 64)
    prompt = synth.prompt_tokens(SEED, "trunc", 30, s.vocab)
    g.prefill([0], [prompt]); o.prefill([0], [prompt])
    a = g.decode_step([0], [11], want_logits=True).cpu()
    g.decode_step([0], [12]); g.seq_truncate(0, 30)
    b = g.decode_step([0], [11], want_logits=True).cpu()
    assert np.array_equal(a.logits, b.logits) and a.token[0] == b.token[0]   # deterministic, bit for bit
    o.decode_step([0], [11])
    compare_outputs(g.decode_step([0], [99], want_logits=True).cpu(), o.decode_step([0], [99], want_logits=True), s.dtype, s.threshold, "after replace")


def test_tiny_load_kv_and_no_router_untied_head(tr, tro):
    s = synth.TINY.with_(router_hidden=0, tie_lm_head=0, kv_dtype=synth.BF16)
    w = synth.make_weights(s, SEED + 2)
    g = tr.Model(s.asdict(), w, 2, 300); o = tro.Model(s.asdict(), w, 2, 300)
    k, v = synth.kv_fill(SEED, "kvfill", s, 257)
    o.load_kv(1, synth.bf16_bits_to_f32(k), synth.bf16_bits_to_f32(v))
    g.load_kv(1, tr.to_device(k, synth.BF16), tr.to_device(v, synth.BF16))
    go = g.decode_step([1], [17], want_logits=True).cpu(); oo = o.decode_step([1], [17], want_logits=True)
    assert_rows_close(go.logits, oo.logits, 1e-4, "loaded-cache logits")
    assert go.token[0] == oo.token[0] and go.flag[0] == 0 and go.score[0] == 1.0 and g.seq_len(1) == 258


def test_tiny_isolated_tail(tr, tro, tiny_weights):
    s = synth.TINY
    g = tr.Model(s.asdict(), tiny_weights, 9, 8)
    x = synth.hidden_rows(SEED, "tailx", 9, s.d_model, False)
    go = g.tail(torch.from_numpy(x).cuda(), want_logits=True).cpu()
    w = tiny_weights
    for i in range(9):
        hn = tro.rmsnorm(x[i], w["final_norm"], s.dtype, s.rms_eps)
        z = tro.linear(w["tok_emb"], None, s.dtype, hn)
        tok, conf = tro.softmax_stats(z)
        sc = tro.router_score(hn, w["r_w1"], w["r_b1"], w["r_w2"], w["r_b2"], s.dtype)
        assert_rows_close(go.logits[i], z, 1e-4, "tail logits"); assert_rows_close(go.hidden[i], hn, 1e-4, "tail hidden")
        assert go.token[i] == tok and go.conf[i] == pytest.approx(conf, rel=1e-4) and go.score[i] == pytest.approx(sc, abs=1e-5)
        assert go.flag[i] == tro.route_flag(go.score[i], s.threshold)
    assert not g.counters().any()


def test_tiny_run_twice_is_bit_identical(tr, tiny_weights):
    s = synth.TINY
    prompts = [synth.prompt_tokens(SEED, f"det{i}", 40 + 100 * i, s.vocab) for i in range(3)]
    res = []
    for _ in range(2):
        g = tr.Model(s.asdict(), tiny_weights, 3, 400)
        a = g.prefill([0, 1, 2], prompts, want_logits=True).cpu()
        b = g.decode_step([0, 1, 2], a.token, want_logits=True).cpu()
        res.append((a, b))
    for x, y in zip(res[0], res[1]):
        assert np.array_equal(x.logits, y.logits) and np.array_equal(x.score, y.score) and np.array_equal(x.conf, y.conf)


@pytest.mark.parametrize("B", [9, 33, 70, 256])
def test_small_bf16_model_on_the_matrix_core_path(tr, tro, B):
    """bf16 weights and 3 or more rows take the MFMA kernels: batches of 9 (one column block), 33 (two) and 70 (two row
    groups) and 256 (four row groups, the LM head's XCD-aware placement), ragged prompts up to several 64-row groups,
    non-zero biases, non-unit gains."""
    s = synth.TINY.with_(dtype=synth.BF16, kv_dtype=synth.BF16)
    w = synth.make_weights(s, SEED + 3, std=0.05, bias_std=0.05, gain_std=0.1)
    max_seq = 200
    g = tr.Model(s.asdict(), w, B, max_seq); o = tro.Model(s.asdict(), w, B, max_seq)
    lens = synth.prompt_lengths(SEED, f"mfma.lens{B}", B, 1, 150)
    lens[0], lens[1], lens[2] = 1, 9, 150
    prompts = [synth.prompt_tokens(SEED, f"mfma{B}.{i}", int(n), s.vocab) for i, n in enumerate(lens)]
    slots = list(np.random.default_rng(B).permutation(B))
    go = g.prefill(slots, prompts, want_logits=True).cpu(); oo = o.prefill(slots, prompts, want_logits=True)
    ex = compare_outputs(go, oo, s.dtype, s.threshold, f"mfma B={B} prefill")
    for step in range(4):
        toks = oo.token.copy()
        go = g.decode_step(slots, toks, want_logits=True).cpu(); oo = o.decode_step(slots, toks, want_logits=True)
        ex += compare_outputs(go, oo, s.dtype, s.threshold, f"mfma B={B} step {step}")
    assert ex <= 2
    cnt = g.counters()
    for i, slot in enumerate(slots):
        assert g.seq_len(slot) == lens[i] + 4 and cnt[slot][0] == 5


@pytest.mark.parametrize("B,ctx", [(3, 1200), (1, 4500), (12, 2300), (40, 900)])
def test_small_bf16_model_long_contexts(tr, tro, B, ctx):
    """Long loaded caches with a bf16 KV cache: many attention chunks per row (merged by a separate kernel for a few rows,
    by the consumer or the batched merge otherwise), chunks longer than 64 keys past 4096 positions, contexts of very
    different lengths in one call, and decoding right up to the last position of the cache (max_seq not a multiple of 32)."""
    s = synth.TINY.with_(dtype=synth.BF16, kv_dtype=synth.BF16)
    w = synth.make_weights(s, SEED + 4, std=0.05, bias_std=0.05, gain_std=0.1)
    max_seq = ctx + 3
    g = tr.Model(s.asdict(), w, B, max_seq); o = tro.Model(s.asdict(), w, B, max_seq)
    lens = [ctx] + [int(n) for n in synth.prompt_lengths(SEED, f"long.lens{B}", B - 1, 1, ctx)]
    for b, n in enumerate(lens):
        k, v = synth.kv_fill(SEED, f"long{B}.{b}", s, n)
        o.load_kv(b, synth.bf16_bits_to_f32(k), synth.bf16_bits_to_f32(v))
        g.load_kv(b, tr.to_device(k, synth.BF16), tr.to_device(v, synth.BF16))
    slots = list(range(B))
    toks = synth.prompt_tokens(SEED, f"long.tok{B}", B, s.vocab)
    ex = 0
    for step in range(3):
        go = g.decode_step(slots, toks, want_logits=True).cpu(); oo = o.decode_step(slots, toks, want_logits=True)
        ex += compare_outputs(go, oo, s.dtype, s.threshold, f"long B={B} step {step}")
        toks = oo.token.copy()
    assert ex <= 1
    assert g.seq_len(0) == max_seq
    with pytest.raises(tr.TokrouteError):
        g.decode_step([0], [1])            # the cache of slot 0 is full


@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
def test_catch_up_step_over_an_existing_cache(tr, tro, dtype):
    """tr_extend against the oracle's definition (cached decode steps, only the last one visible): segments of 1, 5, 14
    (the paper's ~7 % routing means about 14 small-model tokens between two routed ones), 40 and 130 tokens — one or two rows
    run the GEMV kernels, more run the matrix-core ones (bf16) — over caches of very different lengths, several slots per call,
    alternating with ordinary decode steps; counters, lengths and error paths included."""
    s = synth.TINY.with_(dtype=dtype, kv_dtype=dtype)
    w = synth.make_weights(s, SEED + 5, std=0.05, bias_std=0.05, gain_std=0.1)
    B, max_seq = 5, 700
    g = tr.Model(s.asdict(), w, B, max_seq); o = tro.Model(s.asdict(), w, B, max_seq)
    lens = [3, 64, 200, 511, 33]
    prompts = [synth.prompt_tokens(SEED, f"cu.p{i}", n, s.vocab) for i, n in enumerate(lens)]
    slots = list(range(B))
    g.prefill(slots, prompts); o.prefill(slots, prompts)
    ex = 0
    for rnd, seg_lens in enumerate(([1, 5, 14, 40, 130], [14, 130, 1, 5, 40])):
        segs = [synth.prompt_tokens(SEED, f"cu.s{rnd}.{i}", n, s.vocab) for i, n in enumerate(seg_lens)]
        order = [4, 2, 0, 3, 1] if rnd else slots
        go = g.extend(order, [segs[i] for i in order], want_logits=True).cpu()
        oo = o.extend(order, [segs[i] for i in order], want_logits=True)
        ex += compare_outputs(go, oo, s.dtype, s.threshold, f"extend round {rnd}")
        go = g.decode_step(slots, oo.token[np.argsort(order)], want_logits=True).cpu()
        oo = o.decode_step(slots, oo.token[np.argsort(order)], want_logits=True)
        ex += compare_outputs(go, oo, s.dtype, s.threshold, f"decode after extend round {rnd}")
    assert ex <= 1
    cnt = g.counters()
    total = [1 + 14, 5 + 130, 14 + 1, 40 + 5, 130 + 40]
    for b in range(B):
        assert g.seq_len(b) == o.seq_len(b) == lens[b] + total[b] + 2 and tuple(cnt[b]) == o.counters(b)
        assert cnt[b][0] == 5                     # prefill + 2 x (extend + decode step)
    room = max_seq - g.seq_len(3)
    with pytest.raises(tr.TokrouteError):
        g.extend([3], [synth.prompt_tokens(SEED, "cu.big", room + 1, s.vocab)])
    with pytest.raises(tr.TokrouteError):
        g.extend([0], [[]])
    fresh = tr.Model(s.asdict(), w, 2, 16)
    with pytest.raises(tr.TokrouteError):
        fresh.extend([0], [[1, 2]])               # no cache yet
    assert g.seq_len(3) == max_seq - room and g.seq_len(0) == lens[0] + total[0] + 2
    go = g.extend([3], [synth.prompt_tokens(SEED, "cu.fill", room, s.vocab)], want_logits=True).cpu()      # exactly up to the last position
    oo = o.extend([3], [synth.prompt_tokens(SEED, "cu.fill", room, s.vocab)], want_logits=True)
    assert compare_outputs(go, oo, s.dtype, s.threshold, "extend to the end of the cache") == 0 and g.seq_len(3) == max_seq


@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
def test_one_call_mixes_new_prompts_decode_steps_and_catch_up(tr, tro, dtype):
    """One tr_extend call whose segments are a new prompt for an emptied slot (a prefill), single tokens (decode steps) and
    catch-up segments, in the same passes over the weights, against the oracle; then an ordinary decode step of everyone."""
    s = synth.TINY.with_(dtype=dtype, kv_dtype=dtype)
    w = synth.make_weights(s, SEED + 9, std=0.05, bias_std=0.05, gain_std=0.1)
    B, max_seq = 6, 400
    g = tr.Model(s.asdict(), w, B, max_seq); o = tro.Model(s.asdict(), w, B, max_seq)
    lens = [40, 7, 130, 64, 9, 250]
    slots = list(range(B))
    prompts = [synth.prompt_tokens(SEED, f"mx.p{i}", n, s.vocab) for i, n in enumerate(lens)]
    g.prefill(slots, prompts); o.prefill(slots, prompts)
    for m in (g, o):
        m.seq_truncate(0, 0); m.seq_truncate(3, 0)            # two requests ended; their slots take new prompts
    seg_lens = [90, 1, 14, 33, 1, 6]
    segs = [synth.prompt_tokens(SEED, f"mx.s{i}", n, s.vocab) for i, n in enumerate(seg_lens)]
    go = g.extend(slots, segs, want_logits=True).cpu()
    oo = o.extend(slots, segs, want_logits=True)
    ex = compare_outputs(go, oo, s.dtype, s.threshold, "mixed call")
    go = g.decode_step(slots, oo.token, want_logits=True).cpu()
    oo = o.decode_step(slots, oo.token, want_logits=True)
    ex += compare_outputs(go, oo, s.dtype, s.threshold, "decode after the mixed call")
    assert ex <= 1
    want = [90, 8, 144, 33, 10, 256]
    cnt = g.counters()
    for b in range(B):
        assert g.seq_len(b) == o.seq_len(b) == want[b] + 1 and tuple(cnt[b]) == o.counters(b)


@pytest.mark.parametrize("dtype,B", [(synth.F32, 3), (synth.BF16, 20)])
def test_other_routing_scores(tr, tro, dtype, B):
    """The softmax-confidence score (Figure 1) and the linear deferral head compared with '>' (Section 2.2) in the fused tail,
    on the GEMV path (3 rows, fp32) and on the matrix-core path (20 rows, bf16), against the oracle."""
    s = synth.TINY.with_(dtype=dtype, kv_dtype=dtype, router_hidden=0)
    w = synth.make_weights(s, SEED + 6, std=0.05, bias_std=0.05, gain_std=0.1)
    w["r_w2"] = synth.normal(SEED, "lin.w", (s.d_model,), 0.1, dtype)
    w["r_b2"] = synth.normal(SEED, "lin.b", (1,), 0.1, dtype)
    prompts = [synth.prompt_tokens(SEED, f"pol{b}", 3 + 5 * b, s.vocab) for b in range(B)]
    slots = list(range(B))
    # a threshold inside the range of the confidences the model actually produces, so that both outcomes occur
    probe = tro.Model(s.asdict(), w, B, 128, route_policy=tro.POLICY_CONFIDENCE).prefill(slots, prompts)
    conf_thr = float(np.median(probe.conf))
    for policy, thr, below in ((tr.POLICY_CONFIDENCE, conf_thr, True), (tr.POLICY_LINEAR, 0.5, False)):
        sh = s.with_(threshold=thr).asdict()
        rd = tr.ROUTE_IF_BELOW if below else tr.ROUTE_IF_ABOVE
        g = tr.Model(sh, w, B, 128, route_dir=rd, route_policy=policy)
        o = tro.Model(sh, w, B, 128, route_dir=rd, route_policy=policy)
        go = g.prefill(slots, prompts, want_logits=True).cpu(); oo = o.prefill(slots, prompts, want_logits=True)
        ex = compare_outputs(go, oo, s.dtype, thr, f"policy {policy} prefill", route_dir_below=below)
        flags = list(oo.flag)
        for step in range(3):
            go = g.decode_step(slots, oo.token, want_logits=True).cpu(); oo = o.decode_step(slots, oo.token, want_logits=True)
            ex += compare_outputs(go, oo, s.dtype, thr, f"policy {policy} step {step}", route_dir_below=below)
            flags += list(oo.flag)
        assert ex <= 2 and 0 < sum(flags) < len(flags)
        if policy == tr.POLICY_CONFIDENCE:
            assert np.array_equal(go.score, go.conf)
        cnt = g.counters()
        for b in range(B):
            assert tuple(cnt[b]) == o.counters(b)


@pytest.mark.parametrize("B", [12, 70])
def test_wide_bf16_model_on_the_split_k_path(tr, tro, B):
    """A model wider than one workgroup's share of K (d_model 1024 > 896, head dim 128): with more than 2 rows every linear
    layer goes through split-K partials and the rotary/cache-append and SwiGLU steps are finished by their own kernels; the
    tail stays on the streaming kernels. Ragged prefill, decode steps, a catch-up step, and the row counts in between."""
    s = synth.TINY.with_(name="wide", d_model=1024, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ffn=2048, dtype=synth.BF16, kv_dtype=synth.BF16)
    w = synth.make_weights(s, SEED + 7, std=0.03, bias_std=0.05, gain_std=0.1)
    max_seq = 260
    g = tr.Model(s.asdict(), w, B, max_seq); o = tro.Model(s.asdict(), w, B, max_seq)
    lens = synth.prompt_lengths(SEED, f"wide.lens{B}", B, 1, 150)
    lens[0], lens[1], lens[2] = 1, 9, 150
    prompts = [synth.prompt_tokens(SEED, f"wide{B}.{i}", int(n), s.vocab) for i, n in enumerate(lens)]
    slots = list(np.random.default_rng(B).permutation(B))
    go = g.prefill(slots, prompts, want_logits=True).cpu(); oo = o.prefill(slots, prompts, want_logits=True)
    ex = compare_outputs(go, oo, s.dtype, s.threshold, f"wide B={B} prefill")
    for step in range(3):
        toks = oo.token.copy()
        go = g.decode_step(slots, toks, want_logits=True).cpu(); oo = o.decode_step(slots, toks, want_logits=True)
        ex += compare_outputs(go, oo, s.dtype, s.threshold, f"wide B={B} step {step}")
    segs = [synth.prompt_tokens(SEED, f"wide{B}.seg{i}", 1 + (7 * i) % 40, s.vocab) for i in range(B)]
    go = g.extend(slots, segs, want_logits=True).cpu(); oo = o.extend(slots, segs, want_logits=True)
    ex += compare_outputs(go, oo, s.dtype, s.threshold, f"wide B={B} extend")
    assert ex <= 2
    cnt = g.counters()
    for i, slot in enumerate(slots):
        assert g.seq_len(slot) == lens[i] + 3 + len(segs[i]) and tuple(cnt[slot]) == o.counters(slot)


ROWS_SHAPES = {
    # gate/up and q|k|v with a ragged last 512-column chunk, down projection over two chunks per wavefront, fp32 cache
    "d2560": dict(d_model=2560, n_q_heads=10, n_kv_heads=2, head_dim=128, d_ffn=6152, vocab=3001, router_hidden=0, tie_lm_head=0, kv_dtype=synth.F32),
    # three and four chunks per wavefront in the down projection, q width different from d, 64-wide heads
    "d1536": dict(d_model=1536, n_q_heads=20, n_kv_heads=4, head_dim=64, d_ffn=12296, vocab=3001, router_hidden=40),
    # the widest rows the kernels take: every register array full
    "d4096": dict(d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, d_ffn=20480, vocab=2003, router_hidden=0, tie_lm_head=0),
}


@pytest.mark.parametrize("name,kv_page", [("d2560", 0), ("d1536", 32), ("d4096", 0)])
def test_wide_models_with_the_rows_in_registers(tr, tro, name, kv_page):
    """bf16 models of 1025 to 4096 columns at 1 to 4 rows: the q|k|v projection, the output projection and the FFN run on the
    kernels that keep the rows' columns in registers (every chunk count the kernels are built for, ragged last chunks, fp32 and
    paged caches); 5 rows take the matrix-core path. Decode steps at each row count and a short catch-up step against the oracle."""
    s = synth.TINY.with_(name=name, n_layers=2, dtype=synth.BF16, **{"kv_dtype": synth.BF16, **ROWS_SHAPES[name]})
    w = synth.make_weights(s, SEED + 17, std=0.02, bias_std=0.05, gain_std=0.1)
    B, max_seq = 5, 96
    kw = dict(kv_page=kv_page) if kv_page else {}
    g = tr.Model(s.asdict(), w, B, max_seq, **kw); o = tro.Model(s.asdict(), w, B, max_seq)
    prompts = [synth.prompt_tokens(SEED, f"rows.{name}.{i}", 3 + 9 * i, s.vocab) for i in range(B)]
    slots = list(range(B))
    go = g.prefill(slots, prompts, want_logits=True).cpu(); oo = o.prefill(slots, prompts, want_logits=True)
    ex = compare_outputs(go, oo, s.dtype, s.threshold, f"{name} prefill", joint=s.router_hidden > 0)
    toks = oo.token.copy()
    for n in (1, 2, 3, 4, 5, 4, 2):                                   # rows of each step: the first n sequences
        go = g.decode_step(slots[:n], toks[:n], want_logits=True).cpu(); oo = o.decode_step(slots[:n], toks[:n], want_logits=True)
        ex += compare_outputs(go, oo, s.dtype, s.threshold, f"{name} step of {n} rows", joint=s.router_hidden > 0)
        toks[:n] = oo.token
    segs = [synth.prompt_tokens(SEED, f"rows.{name}.seg{i}", 1 + i, s.vocab) for i in range(2)]      # 3 rows: one and two tokens
    go = g.extend(slots[:2], segs, want_logits=True).cpu(); oo = o.extend(slots[:2], segs, want_logits=True)
    ex += compare_outputs(go, oo, s.dtype, s.threshold, f"{name} catch-up", joint=s.router_hidden > 0)
    assert ex <= 2
    cnt = g.counters()
    for b in range(B):
        assert g.seq_len(b) == o.seq_len(b) and tuple(cnt[b]) == o.counters(b)
    # fixed reduction shapes: a second context gives the same bits at every row count
    g2 = tr.Model(s.asdict(), w, B, max_seq, **kw)
    g2.prefill(slots, prompts)
    g3 = tr.Model(s.asdict(), w, B, max_seq, **kw)
    g3.prefill(slots, prompts)
    for n in (1, 2, 3, 4):
        a = g2.decode_step(slots[:n], toks[:n], want_logits=True).cpu(); b = g3.decode_step(slots[:n], toks[:n], want_logits=True).cpu()
        assert np.array_equal(a.logits, b.logits) and np.array_equal(a.hidden, b.hidden) and np.array_equal(a.score, b.score), f"{name}: {n} rows differ between two runs"


@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
def test_fork_of_a_sequence(tr, tro, dtype):
    """tr_seq_fork against the oracle: the copy and the original continue independently and each matches the oracle's
    corresponding slot, for the row-major fp32 cache and for the block-transposed bf16 V cache."""
    s = synth.TINY.with_(dtype=dtype, kv_dtype=dtype)
    w = synth.make_weights(s, SEED + 8, std=0.05, bias_std=0.05, gain_std=0.1)
    g = tr.Model(s.asdict(), w, 3, 200); o = tro.Model(s.asdict(), w, 3, 200)
    toks = synth.prompt_tokens(SEED, "fork", 140, s.vocab)
    for m in (g, o):
        m.prefill([0, 2], [toks[:77], toks[:5]])
        m.seq_fork(0, 2)                              # replaces slot 2
        m.seq_fork(0, 1)                              # fills an empty slot
    assert [g.seq_len(b) for b in range(3)] == [77, 77, 77]
    ex = 0
    for step in range(3):
        t3 = [toks[100 + step], toks[110 + step], toks[120 + step]]      # the three copies diverge
        go = g.decode_step([0, 1, 2], t3, want_logits=True).cpu(); oo = o.decode_step([0, 1, 2], t3, want_logits=True)
        ex += compare_outputs(go, oo, s.dtype, s.threshold, f"fork step {step}")
    assert ex == 0
    cnt = g.counters()
    for b in range(3):
        assert tuple(cnt[b]) == o.counters(b)
    fresh = tr.Model(s.asdict(), w, 2, 16)
    with pytest.raises(tr.TokrouteError):
        fresh.seq_fork(0, 1)


ODD_SHAPES = {
    # fp32 everywhere, GEMV + FMA attention kernels: nothing a multiple of 16 or 32, one query head per kv head
    "f32_g1": dict(d_model=72, n_q_heads=3, n_kv_heads=3, head_dim=64, d_ffn=200, vocab=1003, router_hidden=40, dtype=synth.F32, kv_dtype=synth.F32),
    # bf16 on the fused matrix-core path: ragged last tiles of the FFN, the residual stream and the vocabulary, 8 query heads on one kv head
    "bf16_g8": dict(d_model=272, n_q_heads=8, n_kv_heads=1, head_dim=64, d_ffn=1040, vocab=5003, router_hidden=72, dtype=synth.BF16, kv_dtype=synth.BF16),
    # bf16 weights over an fp32 cache
    "bf16_f32kv": dict(d_model=272, n_q_heads=6, n_kv_heads=2, head_dim=64, d_ffn=1040, vocab=5003, router_hidden=72, dtype=synth.BF16, kv_dtype=synth.F32),
    # wide model on the split-K path: 65 k-steps, 5 query heads per kv head, ragged vocabulary, no router, untied head
    "wide_g5": dict(d_model=1040, n_q_heads=10, n_kv_heads=2, head_dim=128, d_ffn=2080, vocab=4099, router_hidden=0, tie_lm_head=0,
                    dtype=synth.BF16, kv_dtype=synth.BF16),
    # a single sequence with FFN widths of 1025 to 8192: the output projection splits each weight row over the four wavefronts
    # of a workgroup, 1, 2 or 4 steps of 512 columns each (the 0.5B-class model's 4864 gives 3)
    "ffn_1544": dict(d_ffn=1544, dtype=synth.F32, kv_dtype=synth.F32),
    "ffn_3000": dict(d_ffn=3000, dtype=synth.BF16, kv_dtype=synth.BF16),
    "ffn_6152": dict(d_ffn=6152, dtype=synth.BF16, kv_dtype=synth.F32),
}


@pytest.mark.parametrize("name,B", [("f32_g1", 5), ("bf16_g8", 3), ("bf16_g8", 21), ("bf16_f32kv", 21), ("wide_g5", 3), ("wide_g5", 12),
                                    ("wide_g5", 1), ("ffn_1544", 1), ("ffn_3000", 1), ("ffn_6152", 1),
                                    # one and two rows: the LDS-free short path, the split rows of the output projections and, with bf16
                                    # weights and cache, the fused projection + attention kernel (272 columns: one partly used step; 8 heads per group)
                                    ("bf16_g8", 1), ("bf16_g8", 2), ("ffn_3000", 2), ("ffn_6152", 2), ("bf16_f32kv", 2), ("f32_g1", 2), ("wide_g5", 2)])
def test_shapes_that_fill_no_tile_exactly(tr, tro, name, B):
    """Model shapes whose widths are not multiples of the kernels' tiles (reduction length, FFN width, vocabulary, router
    width, heads per group), on every kernel family: prefill, decode steps and a catch-up step against the oracle."""
    s = synth.TINY.with_(name=name, **ODD_SHAPES[name])
    w = synth.make_weights(s, SEED + 11, std=0.05, bias_std=0.05, gain_std=0.1)
    max_seq = 160
    g = tr.Model(s.asdict(), w, B, max_seq); o = tro.Model(s.asdict(), w, B, max_seq)
    lens = synth.prompt_lengths(SEED, f"odd.{name}.{B}", B, 1, 120)
    lens[0] = 1 if B > 1 else 37
    prompts = [synth.prompt_tokens(SEED, f"odd.{name}.{i}", int(n), s.vocab) for i, n in enumerate(lens)]
    slots = list(range(B))
    go = g.prefill(slots, prompts, want_logits=True).cpu(); oo = o.prefill(slots, prompts, want_logits=True)
    ex = compare_outputs(go, oo, s.dtype, s.threshold, f"{name} B={B} prefill")
    for step in range(3):
        toks = oo.token.copy()
        go = g.decode_step(slots, toks, want_logits=True).cpu(); oo = o.decode_step(slots, toks, want_logits=True)
        ex += compare_outputs(go, oo, s.dtype, s.threshold, f"{name} B={B} step {step}")
    segs = [synth.prompt_tokens(SEED, f"odd.{name}.seg{i}", 1 + 3 * (i % 5), s.vocab) for i in range(B)]
    go = g.extend(slots, segs, want_logits=True).cpu(); oo = o.extend(slots, segs, want_logits=True)
    ex += compare_outputs(go, oo, s.dtype, s.threshold, f"{name} B={B} catch-up")
    assert ex <= 2
    cnt = g.counters()
    for b in range(B):
        assert g.seq_len(b) == o.seq_len(b) and tuple(cnt[b]) == o.counters(b)


@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
def test_decode_steps_fed_from_device_memory(tr, tro, tiny_weights, dtype):
    """tr_decode_step_dev: a chain of greedy steps that feeds each step's token output straight into the next step without
    the host seeing it must produce the token stream of the same chain fed through the host (bit-identical logits at every
    step), and for the fp32 model the oracle's own free-running stream; out-of-vocabulary device tokens are clamped."""
    s = synth.TINY.with_(dtype=dtype, kv_dtype=dtype)
    w = tiny_weights if dtype == synth.F32 else synth.make_weights(s, SEED + 31, std=0.05)
    B, steps = 3, 12
    a = tr.Model(s.asdict(), w, B, 128); b = tr.Model(s.asdict(), w, B, 128); o = tro.Model(s.asdict(), w, B, 128)
    prompts = [synth.prompt_tokens(SEED, f"dev.p{i}", 5 + 11 * i, s.vocab) for i in range(B)]
    slots = list(range(B))
    xa = a.prefill(slots, prompts, want_logits=True); xb = b.prefill(slots, prompts, want_logits=True); oo = o.prefill(slots, prompts, want_logits=True)
    dev_stream = []
    for t in range(steps):
        host_tok = xa.cpu().token.copy()
        xa = a.decode_step(slots, host_tok, want_logits=True)              # through the host
        xb = b.decode_step_dev(slots, xb.token, xb, want_logits=True)      # device to device: the outputs object feeds itself
        oo = o.decode_step(slots, oo.token, want_logits=True)
        ca, cb = xa.cpu(), xb.cpu()
        assert np.array_equal(ca.logits, cb.logits) and np.array_equal(ca.token, cb.token) and np.array_equal(ca.flag, cb.flag), f"step {t}"
        dev_stream.append(cb.token.copy())
        if dtype == synth.F32:
            assert np.array_equal(cb.token, oo.token), f"free-running token stream differs from the oracle at step {t}"
    assert b.seq_len(0) == len(prompts[0]) + steps and tuple(b.counters()[1]) == tuple(a.counters()[1])
    bad = torch.tensor([-5, s.vocab + 7, 3], dtype=torch.int32, device="cuda")
    good = np.array([0, s.vocab - 1, 3], np.int32)
    ya = a.decode_step(slots, good, want_logits=True).cpu(); yb = b.decode_step_dev(slots, bad, want_logits=True).cpu()
    assert np.array_equal(ya.logits, yb.logits)


@pytest.mark.parametrize("B", [2, 8])
def test_decode_step_replayed_from_a_captured_graph(tr, B):
    """A device-fed decode step enqueues kernels only (no allocation, no host copy, no memset), so it can be captured into a
    HIP graph. Every replay, with eager work of the same model and synchronisations in between, must give the bits of the
    eager step it was captured from (2 rows: the streaming kernels; 8 rows: the matrix-core path with its exchange counters)."""
    s = synth.TINY.with_(name="graph", dtype=synth.BF16, kv_dtype=synth.BF16, vocab=5003)
    w = synth.make_weights(s, SEED + 41, std=0.05, bias_std=0.05, gain_std=0.1)
    g = tr.Model(s.asdict(), w, B, 1200)
    prompts = [synth.prompt_tokens(SEED, f"graph.p{i}", 900 + 37 * i if i == 0 else 5 + 23 * i, s.vocab) for i in range(B)]   # one row long enough for several attention parts
    slots = list(range(B))
    base = [len(p) for p in prompts]
    g.prefill(slots, prompts)
    toks = torch.from_numpy(synth.prompt_tokens(SEED, "graph.t", B, s.vocab)).cuda()
    other = torch.from_numpy(synth.prompt_tokens(SEED, "graph.o", B, s.vocab)).cuda()
    eager = g.decode_step_dev(slots, toks, want_logits=True).cpu()
    for sl, n in zip(slots, base):
        g.seq_truncate(sl, n)
    out = g.outputs(B, want_logits=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        g.decode_step_dev(slots, toks, out)
    torch.cuda.synchronize()
    for rep in range(4):
        for f in (out.token, out.flag, out.conf, out.score, out.logits, out.hidden):
            f.fill_(0)
        graph.replay()
        torch.cuda.synchronize()
        got = out.cpu()
        for name in ("token", "flag", "conf", "score", "logits", "hidden"):
            assert np.array_equal(getattr(got, name), getattr(eager, name)), f"replay {rep}: {name}"
        # eager work of the same model between the replays: a step on the next position with other tokens, rolled back again
        g.decode_step_dev(slots, other, want_logits=True)
        torch.cuda.synchronize()
        for sl, n in zip(slots, base):
            g.seq_truncate(sl, n + 1)


@pytest.mark.parametrize("kv_page", [0, 32])
def test_one_and_two_row_decode_steps_at_chunk_boundaries(tr, tro, kv_page):
    """Decode steps of one or two sequences with bf16 weights and cache run the projection and the attention over the cached
    keys as one kernel, whose partials (chunks of 128 cached keys) the output projection merges with the row's own new key.
    Cases: a sequence rolled back to nothing and decoded from position 0 (no cached key at all), one whose cache crosses
    positions 127, 128 and 129 (first chunk filling up, second chunk starting), both in one call (very different contexts)
    and each alone; the same on the paged cache (pages of 32)."""
    s = synth.TINY.with_(dtype=synth.BF16, kv_dtype=synth.BF16)
    w = synth.make_weights(s, SEED + 41, std=0.05, bias_std=0.05, gain_std=0.1)
    g = tr.Model(s.asdict(), w, 2, 300, kv_page=kv_page); o = tro.Model(s.asdict(), w, 2, 300)
    p0 = synth.prompt_tokens(SEED, "qa.p0", 3, s.vocab)
    g.prefill([0], [p0]); o.prefill([0], [p0])
    g.seq_truncate(0, 0); o.seq_truncate(0, 0)
    k, v = synth.kv_fill(SEED, "qa.kv", s, 126)
    o.load_kv(1, synth.bf16_bits_to_f32(k), synth.bf16_bits_to_f32(v)); g.load_kv(1, tr.to_device(k, synth.BF16), tr.to_device(v, synth.BF16))
    toks = synth.prompt_tokens(SEED, "qa.tok", 2, s.vocab)
    ex = 0
    for step in range(5):     # slot 0 at positions 0..4, slot 1 at 126..130
        go = g.decode_step([0, 1], toks, want_logits=True).cpu(); oo = o.decode_step([0, 1], toks, want_logits=True)
        ex += compare_outputs(go, oo, s.dtype, s.threshold, f"two rows, step {step}")
        toks = oo.token.copy()
    for slot in (1, 0):
        t1 = toks[slot:slot + 1]
        for step in range(2):
            go = g.decode_step([slot], t1, want_logits=True).cpu(); oo = o.decode_step([slot], t1, want_logits=True)
            ex += compare_outputs(go, oo, s.dtype, s.threshold, f"slot {slot} alone, step {step}")
            t1 = oo.token.copy()
    # a catch-up call whose segments are one token each is a decode step and takes the same kernels
    segs = [synth.prompt_tokens(SEED, f"qa.seg{i}", 1, s.vocab) for i in range(2)]
    go = g.extend([1, 0], segs, want_logits=True).cpu(); oo = o.extend([1, 0], segs, want_logits=True)
    ex += compare_outputs(go, oo, s.dtype, s.threshold, "one-token segments")
    assert ex <= 1
    assert g.seq_len(0) == 8 and g.seq_len(1) == 134


def test_exchanges_between_workgroups_give_the_same_bits_every_time(tr):
    """The two places where workgroups hand partial results to whichever of them arrives last (attention rows split over
    several workgroups; the router's hidden units split over the workgroups of a row), each repeated a few hundred times:
    every repetition must reproduce the first result bit for bit. Stops at the first difference."""
    REPS = 300
    # (1) attention: 64 rows of a bf16 model with contexts of up to ~2000 keys, i.e. up to three parts per (row, kv head)
    s = synth.TINY.with_(dtype=synth.BF16, kv_dtype=synth.BF16)
    w = synth.make_weights(s, SEED + 9, std=0.05)
    B, ctx = 64, 2000
    g = tr.Model(s.asdict(), w, B, ctx + 4)
    lens = [ctx] + [int(n) for n in synth.prompt_lengths(SEED, "soak.lens", B - 1, 700, ctx)]
    k, v = synth.kv_fill(SEED, "soak.kv", s, ctx)
    for b, n in enumerate(lens):
        g.load_kv(b, tr.to_device(np.ascontiguousarray(k[:, :, :n]), synth.BF16), tr.to_device(np.ascontiguousarray(v[:, :, :n]), synth.BF16))
    toks = synth.prompt_tokens(SEED, "soak.tok", B, s.vocab)
    slots = list(range(B))
    out = g.outputs(B, want_logits=True)
    first = None
    for rep in range(REPS):
        g.decode_step(slots, toks, out)
        got = (out.logits.clone(), out.hidden.clone(), out.score.clone())
        for b, n in enumerate(lens):
            g.seq_truncate(b, n)
        if first is None:
            first = got
        else:
            same = all(torch.equal(a, b) for a, b in zip(first, got))
            assert same, f"attention exchange: repetition {rep} differs from the first"
    # (2) router: 64 rows x 4 workgroups per row on the streaming tail (fp32 model, 256 hidden units)
    s = synth.TINY.with_(router_hidden=256)
    w = synth.make_weights(s, SEED + 10, bias_std=0.05)
    g = tr.Model(s.asdict(), w, 64, 8)
    x = torch.from_numpy(synth.hidden_rows(SEED, "soak.x", 64, s.d_model, False)).cuda()
    out = g.outputs(64)
    first = None
    for rep in range(REPS):
        g.tail(x, out)
        got = (out.score.clone(), out.flag.clone(), out.token.clone(), out.conf.clone())
        if first is None:
            first = got
        else:
            assert all(torch.equal(a, b) for a, b in zip(first, got)), f"router exchange: repetition {rep} differs from the first"
