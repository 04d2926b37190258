"""Host bookkeeping of the paged cache, checked on the CPU: `tests/kv_pages_check.cpp` drives the page table with 20 000
random appends, rollbacks, forks and restarts per pool size against plain per-slot vectors (see its header)."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_page_table_bookkeeping_against_plain_vectors(tmp_path):
    exe = str(tmp_path / "kv_pages_check")
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-Werror", "-o", exe, os.path.join(ROOT, "tests", "kv_pages_check.cpp")], check=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout
    assert out.strip().endswith("OK"), out
