"""The token-level routing loop end to end (Section 3.1, Figure 2): small model + router + large model on one GPU, against
the same loop written out with the CPU oracle in its plainest form — one sequence at a time, the large model re-run from
scratch over the whole prefix whenever it is called (what the paper's prototype does, Section 4.1)."""
import numpy as np
import pytest

from paper_2504_07878_amd import synth

pytestmark = pytest.mark.gpu
SEED = 7878


@pytest.fixture(scope="module")
def tr():
    from paper_2504_07878_amd import tokroute
    tokroute.load_library()
    return tokroute


def oracle_joint(tro, slm_shape, slm_w, llm_shape, llm_w, prompt, max_new, max_seq):
    slm = tro.Model(slm_shape.asdict(), slm_w, 1, max_seq)
    llm = tro.Model(llm_shape.asdict(), llm_w, 1, max_seq)
    seq = [int(x) for x in prompt]
    toks, routed, gaps = [], [], []
    o = slm.prefill([0], [seq], want_logits=True)
    for t in range(max_new):
        if o.flag[0]:
            lo = llm.prefill([0], [seq], want_logits=True)      # no cache: the whole prefix again
            tok, lg = int(lo.token[0]), lo.logits[0]
        else:
            tok, lg = int(o.token[0]), o.logits[0]
        top = np.sort(lg)[-2:]
        toks.append(tok); routed.append(bool(o.flag[0])); gaps.append(float(top[1] - top[0]))
        seq.append(tok)
        if t + 1 < max_new:
            o = slm.decode_step([0], [tok], want_logits=True)
    return toks, routed, gaps


@pytest.mark.parametrize("overlapped", [False, True])
@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
def test_joint_decoding_matches_the_plain_loop(tr, tro, dtype, overlapped):
    """overlapped: the schedule in which flagged sequences wait for the large model on a second stream while the others keep
    decoding; what each sequence emits must not depend on it."""
    from paper_2504_07878_amd import joint
    slm_shape = synth.TINY.with_(dtype=dtype, kv_dtype=dtype)
    llm_shape = synth.TINY.with_(name="tiny-large", n_layers=3, d_ffn=1536, router_hidden=0, tie_lm_head=0, dtype=dtype, kv_dtype=dtype)
    slm_w = synth.make_weights(slm_shape, SEED + 10, std=0.05, bias_std=0.05, gain_std=0.1)
    llm_w = synth.make_weights(llm_shape, SEED + 11, std=0.05, bias_std=0.05, gain_std=0.1)
    B, max_new, max_seq = 6, 24, 128
    prompts = [synth.prompt_tokens(SEED, f"joint.p{b}", n, slm_shape.vocab) for b, n in enumerate((5, 17, 40, 9, 64, 2))]
    slm = tr.Model(slm_shape.asdict(), slm_w, B, max_seq)
    llm = tr.Model(llm_shape.asdict(), llm_w, B, max_seq)
    tokens, routed = (joint.generate_overlapped if overlapped else joint.generate)(slm, llm, prompts, max_new)
    n_routed = 0
    for b in range(B):
        toks, rt, gaps = oracle_joint(tro, slm_shape, slm_w, llm_shape, llm_w, prompts[b], max_new, max_seq)
        for t in range(max_new):
            if tokens[b, t] != toks[t] or routed[b, t] != rt[t]:
                # free-running: the first difference must sit on a near-tie of the oracle (or of the router score, which
                # shows up as a routing difference); nothing after it can be compared
                assert dtype == synth.BF16 and (gaps[t] < 1e-3 or routed[b, t] != rt[t]), (b, t, tokens[b, t], toks[t], gaps[t])
                break
        n_routed += sum(rt)
    assert 0 < n_routed < B * max_new           # both models took part
    cnt = slm.counters()
    for b in range(B):
        assert cnt[b][0] == max_new and cnt[b][1] >= routed[b, 1:].sum()      # one small-model step per emitted token
