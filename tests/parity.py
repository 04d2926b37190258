"""Helpers shared by the GPU parity tests: tolerances and element-wise comparison against the oracle.

Tolerances (floating point): |gpu - oracle| <= rtol*|oracle| + rtol*rms(oracle row) for logits and hidden
state, with rtol 1e-4 for fp32 models and 2e-2 for bf16 models; the confidence uses the same rtol; the
router score is compared absolutely (1e-5 / 2e-3). Token and flag must be identical unless the oracle's
top-2 logit gap, or its score's distance to the threshold, is below 1e-3.
"""
import numpy as np

from paper_2504_07878_amd import synth


def rtol_of(dtype):
    return 1e-4 if dtype == synth.F32 else 2e-2


def score_atol_of(dtype):
    return 1e-5 if dtype == synth.F32 else 2e-3


def assert_rows_close(gpu, ref, rtol, what):
    gpu = np.asarray(gpu, np.float64); ref = np.asarray(ref, np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    rms = np.sqrt((ref * ref).mean(axis=-1, keepdims=True))
    bound = rtol * np.abs(ref) + rtol * rms
    err = np.abs(gpu - ref)
    bad = err > bound
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance; worst err {err.max():.3e} (bound there {bound.flat[err.argmax()]:.3e})"
    return float((err / (rms + 1e-30)).max())


def top2_gap(logits_row):
    part = np.partition(np.asarray(logits_row, np.float64), -2)
    return float(part[-1] - part[-2])


def compare_outputs(g, o, dtype, threshold, what, route_dir_below=True, joint=True, check_flag_rule=True):
    """g: GPU host outputs, o: oracle outputs (both with logits). Returns number of exempt near-ties."""
    rtol = rtol_of(dtype)
    n = len(o.token)
    exempt = 0
    if o.logits is not None and g.logits is not None:
        assert_rows_close(g.logits, o.logits, rtol, what + " logits")
    if o.hidden is not None and g.hidden is not None:
        assert_rows_close(g.hidden, o.hidden, rtol, what + " hidden")
    assert np.allclose(g.conf, o.conf, rtol=rtol, atol=0), (what, g.conf, o.conf)
    assert np.allclose(g.score, o.score, rtol=0, atol=score_atol_of(dtype)), (what, g.score, o.score)
    for i in range(n):
        if g.token[i] != o.token[i]:
            assert o.logits is not None and top2_gap(o.logits[i]) < 1e-3, f"{what}: row {i} token {g.token[i]} != {o.token[i]}"
            exempt += 1
        if g.flag[i] != o.flag[i]:
            assert abs(float(o.score[i]) - threshold) < 1e-3, f"{what}: row {i} flag {g.flag[i]} != {o.flag[i]} (score {o.score[i]})"
            exempt += 1
        if check_flag_rule:   # the flag is the comparison of the GPU's own score, exactly
            want = int(joint and ((g.score[i] < np.float32(threshold)) if route_dir_below else (g.score[i] > np.float32(threshold))))
            assert int(g.flag[i]) == want, (what, i, g.score[i], threshold, g.flag[i])
    return exempt
