"""tr_decode_step_active: the decode step of the sequences that device-side flags select (the large model's step on the
routed subset, with no trip of the flags to the host) against the oracle's plain loop, in which the HOST picks the subset from
the same flags and calls the ordinary decode step on it. Several calls are enqueued back to back with no synchronisation in
between; everything is checked afterwards."""
import numpy as np
import pytest
import torch

from paper_2504_07878_amd import synth
from parity import compare_outputs

pytestmark = pytest.mark.gpu
SEED = 7878

SHAPES = {
    # fused matrix-core path (d <= 896)
    "fused": synth.TINY.with_(name="act-fused", dtype=synth.BF16, kv_dtype=synth.BF16, vocab=5003),
    # wide model: every linear layer through split-K partials and finishing kernels (the large model's path)
    "split": synth.TINY.with_(name="act-split", d_model=1024, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ffn=2048, dtype=synth.BF16,
                              kv_dtype=synth.BF16, router_hidden=0, tie_lm_head=0),
}


@pytest.fixture(scope="module")
def tr():
    from paper_2504_07878_amd import tokroute
    tokroute.load_library()
    return tokroute


def _rows(h, idx):
    return type("O", (), {k: (None if getattr(h, k) is None else getattr(h, k)[idx]) for k in ("token", "conf", "score", "flag", "hidden", "logits")})()


@pytest.mark.parametrize("path", ["fused", "split"])
def test_device_selected_subset_equals_host_selected_subset(tr, tro, path):
    s = SHAPES[path]
    w = synth.make_weights(s, SEED, bias_std=0.05, gain_std=0.1)
    B, N_MAX, MAX_SEQ = 8, 4, 64
    g = tr.Model(s.asdict(), w, B, MAX_SEQ)
    o = tro.Model(s.asdict(), w, B, MAX_SEQ)
    lens = [5, 40, 17, 9, 33, 12, 26, 8]
    prompts = [synth.prompt_tokens(SEED, f"act.{path}.p{b}", n, s.vocab) for b, n in enumerate(lens)]
    g.prefill(list(range(B)), prompts)
    o.prefill(list(range(B)), prompts)
    rng = synth.rng(SEED, f"act.{path}.flags")
    calls = []
    cands = [list(range(B)), list(range(B)), list(range(B)), [6, 1, 3, 7, 2], list(range(B)), [4, 0, 5]]
    flag_sets = [None, np.zeros(B, np.int32), np.array([1, 1, 0, 1, 1, 1, 0, 1], np.int32), None, None, np.array([0, 5, 0], np.int32)]
    for k, (cand, fl) in enumerate(zip(cands, flag_sets)):
        if fl is None:
            fl = (rng.random(len(cand)) < 0.35).astype(np.int32)
        toks = synth.prompt_tokens(SEED, f"act.{path}.t{k}", len(cand), s.vocab)
        dev = dict(flags=torch.from_numpy(fl).cuda(), toks=torch.from_numpy(toks).cuda(), active=torch.full((2 + N_MAX,), -9, dtype=torch.int32, device="cuda"),
                   nxt=torch.full((len(cand),), -7, dtype=torch.int32, device="cuda"), out=g.outputs(N_MAX, want_logits=True))
        calls.append((cand, fl, toks, dev))
    for cand, fl, toks, dev in calls:            # all enqueued back to back: the host sees nothing in between
        g.decode_step_active(cand, dev["flags"], dev["toks"], N_MAX, dev["active"], dev["nxt"], dev["out"])
    torch.cuda.synchronize()
    exempt = stepped = 0
    for k, (cand, fl, toks, dev) in enumerate(calls):
        want = [i for i in range(len(cand)) if fl[i]][:N_MAX]           # the host's selection from the same flags
        act, nxt, go = dev["active"].cpu().numpy(), dev["nxt"].cpu().numpy(), dev["out"].cpu()
        assert act[0] == len(want) and act[1] == int((fl != 0).sum()), (k, act)
        assert act[2:2 + len(want)].tolist() == want and (act[2 + len(want):] == -1).all(), (k, act, want)
        pad = slice(len(want), N_MAX)
        assert (go.token[pad] == -1).all() and (go.flag[pad] == 0).all() and (go.conf[pad] == 0).all() and (go.score[pad] == 0).all()
        expect_next = np.full(len(cand), -7, np.int32)
        if want:
            oo = o.decode_step([cand[i] for i in want], toks[want], want_logits=True)
            exempt += compare_outputs(_rows(go, slice(0, len(want))), oo, s.dtype, s.threshold, f"{path} call {k}", joint=s.router_hidden > 0)
            expect_next[want] = go.token[:len(want)]
            stepped += len(want)
        assert np.array_equal(nxt, expect_next), (k, nxt, expect_next)
    assert exempt <= 1 and stepped >= 8
    for b in range(B):                           # lengths and counters followed the device's selection
        assert g.seq_len(b) == o.seq_len(b), b
        assert tuple(g.counters()[b]) == o.counters(b), b
    # and the ordinary step goes on from there
    toks = synth.prompt_tokens(SEED, f"act.{path}.after", B, s.vocab)
    go, oo = g.decode_step(list(range(B)), toks, want_logits=True).cpu(), o.decode_step(list(range(B)), toks, want_logits=True)
    assert compare_outputs(go, oo, s.dtype, s.threshold, f"{path} after", joint=s.router_hidden > 0) <= 1


def test_active_step_argument_and_capacity_errors(tr):
    s = SHAPES["fused"]
    w = synth.make_weights(s, SEED)
    g = tr.Model(s.asdict(), w, 4, 12)
    p = [synth.prompt_tokens(SEED, f"acte.{b}", 10, s.vocab) for b in range(4)]
    g.prefill([0, 1, 2, 3], p)
    z = lambda n, v=0: torch.full((n,), v, dtype=torch.int32, device="cuda")
    flags, toks, active = z(4), z(4, 3), z(6)
    with pytest.raises(tr.TokrouteError) as e:
        g.decode_step_active([0, 1, 2, 3], flags, toks, 2, z(4), None)              # fewer than 3 rows
    assert e.value.code == tr.ERR_INVALID_ARG
    with pytest.raises(tr.TokrouteError) as e:
        g.decode_step_active([0, 1, 1, 3], flags, toks, 4, active, None)            # duplicate candidate
    assert e.value.code == tr.ERR_INVALID_ARG
    flags[2] = 1
    g.decode_step_active([0, 1, 2, 3], flags, toks, 4, active, None)                # lengths 10 -> at most 11
    g.decode_step_active([0, 1, 2, 3], z(4), toks, 4, active, None)                 # at most 12 = max_seq: still fits
    with pytest.raises(tr.TokrouteError) as e:
        g.decode_step_active([0, 1, 2, 3], flags, toks, 4, active, None)            # every candidate may be full now
    assert e.value.code == tr.ERR_CAPACITY
    assert [g.seq_len(b) for b in range(4)] == [10, 10, 11, 10]                     # the host catches up here ...
    g.decode_step_active([0, 1, 2, 3], flags, toks, 4, active, None)                # ... and knows again that there is room
    assert [g.seq_len(b) for b in range(4)] == [10, 10, 12, 10]
    with pytest.raises(tr.TokrouteError) as e:
        g.decode_step_active([2], z(1, 1), z(1), 4, active, None)                   # slot 2 is full
    assert e.value.code == tr.ERR_CAPACITY
    t = synth.TINY                               # fp32 model: no matrix-core path
    gt = tr.Model(t.asdict(), synth.make_weights(t, SEED), 4, 16)
    gt.prefill([0], [synth.prompt_tokens(SEED, "acte.t", 4, t.vocab)])
    with pytest.raises(tr.TokrouteError) as e:
        gt.decode_step_active([0], z(1), z(1), 4, active, None)
    assert e.value.code == tr.ERR_SHAPE
    gp = tr.Model(s.asdict(), w, 4, 64, kv_page=32)      # paged cache: not served
    gp.prefill([0], [p[0]])
    with pytest.raises(tr.TokrouteError) as e:
        gp.decode_step_active([0], z(1), z(1), 4, active, None)
    assert e.value.code == tr.ERR_SHAPE
