"""tr_tail_noalloc (the routing tail on the library's static device scratch, for callers that cannot allocate) against
tr_tail, through the C ABI: two calls in a row, the second on fewer rows, so that whatever the first call left in the shared
scratch array must not leak into the second."""
import numpy as np
import pytest
import torch

from paper_2504_07878_amd import synth
from parity import assert_rows_close

pytestmark = pytest.mark.gpu
SEED = 7878


@pytest.fixture(scope="module")
def tr():
    from paper_2504_07878_amd import tokroute
    tokroute.load_library()
    return tokroute


def _same_decisions(a, b, threshold):
    """token and flag identical unless the margin is below 1e-3 (top-2 logit gap / distance of the score to the threshold)"""
    for i in range(len(a.token)):
        if a.token[i] != b.token[i]:
            top = np.partition(b.logits[i].astype(np.float64), -2)
            assert top[-1] - top[-2] < 1e-3, i
        if a.flag[i] != b.flag[i]:
            assert abs(float(b.score[i]) - threshold) < 1e-3, i


@pytest.mark.parametrize("name", ["tiny_fp32", "small_bf16"])
def test_tail_on_static_scratch_equals_tr_tail_twice_in_a_row(tr, name):
    if name == "tiny_fp32":      # tr_tail runs the same streaming kernels: identical bits
        s = synth.TINY
    else:                        # tr_tail runs on the matrix cores: equal to the bf16 tolerance
        s = synth.TINY.with_(name="small-bf16", dtype=synth.BF16, kv_dtype=synth.BF16, vocab=5003)
    w = synth.make_weights(s, SEED, bias_std=0.05, gain_std=0.1)
    g = tr.Model(s.asdict(), w, 40, 8)
    for call, n in enumerate((37, 5)):               # the second call is smaller than the first
        x = torch.from_numpy(synth.hidden_rows(SEED, f"noalloc.{name}.{call}", n, s.d_model, False)).cuda()
        ref = g.tail(x, want_logits=True).cpu()
        out = g.outputs(n, want_logits=True)         # the caller's buffers exist before the call; the call allocates nothing
        before = torch.cuda.memory_allocated()
        got = g.tail_noalloc(x, out)
        assert torch.cuda.memory_allocated() == before
        got = got.cpu()
        if s.dtype == synth.F32:
            for k in ("token", "conf", "score", "flag", "hidden", "logits"):
                assert np.array_equal(getattr(got, k), getattr(ref, k)), (name, call, k)
        else:
            assert_rows_close(got.logits, ref.logits, 2e-2, f"{name} call {call} logits")
            assert_rows_close(got.hidden, ref.hidden, 2e-2, f"{name} call {call} hidden")
            assert np.allclose(got.conf, ref.conf, rtol=2e-2, atol=0) and np.allclose(got.score, ref.score, rtol=0, atol=2e-3)
            _same_decisions(got, ref, s.threshold)
        assert np.array_equal(got.flag, (got.score < np.float32(s.threshold)).astype(np.int32))


def test_sizes_beyond_the_static_scratch_are_refused(tr):
    s = synth.TINY
    g = tr.Model(s.asdict(), synth.make_weights(s, SEED), 80, 8)
    x = torch.zeros((65, s.d_model), dtype=torch.float32, device="cuda")
    with pytest.raises(tr.TokrouteError) as e:
        g.tail_noalloc(x, g.outputs(65))
    assert e.value.code == tr.ERR_CAPACITY
    g.tail_noalloc(x[:64], g.outputs(64)).cpu()      # the limit itself is served
