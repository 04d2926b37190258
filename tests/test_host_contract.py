"""Host-side contract checks that need no GPU: the bench refuses more than one GPU with a message, the binding refuses to
run without a GPU instead of falling back to anything, and nothing in the product imports the oracle."""
import os
import re
import subprocess
import sys

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_several_gpus_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


@pytest.mark.skipif(torch.cuda.is_available(), reason="needs a machine without a GPU")
def test_binding_raises_without_a_gpu():
    from paper_2504_07878_amd import synth, tokroute
    s = synth.TINY
    with pytest.raises(RuntimeError, match="no CPU path"):
        tokroute.Model(s.asdict(), {}, 1, 8)


def test_product_sources_do_not_touch_the_oracle():
    """Only tests, the smoke check and the bench's cpu_baseline leg may use anything under oracle/."""
    use = re.compile(r"^\s*(from\s+oracle\b|import\s+oracle\b|#include\s+[\"<][^\">]*oracle)", re.M)
    pkg = os.path.join(ROOT, "paper_2504_07878_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp", ".c")):
                text = open(os.path.join(dirpath, f), errors="ignore").read()
                assert not use.search(text), f"{f} uses the oracle"
    bench = open(os.path.join(ROOT, "bench.py")).read()
    uses = [m.start() for m in use.finditer(bench)]
    assert uses, "the cpu_baseline leg times the oracle"
    for u in uses:   # every use sits inside cpu_baseline()
        enclosing = bench.rfind("\ndef ", 0, u)
        assert bench[enclosing:].startswith("\ndef cpu_baseline"), bench[enclosing:enclosing + 40]
