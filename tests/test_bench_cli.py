"""Host-side behaviour of the benchmark driver and the entry module (no GPU needed)."""
import os
import subprocess
import sys

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT,
                          capture_output=True, text=True, timeout=300)


@pytest.mark.parametrize("n", ["2", "8", "0"])
def test_more_than_one_gpu_is_refused_with_a_message(n):
    r = run_bench("--gpus", n)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and "--gpus must be 1" in r.stderr
    assert r.stdout.strip() == ""          # no JSON line that could be mistaken for a result


@pytest.mark.skipif(torch.cuda.is_available(), reason="checks the behaviour without a GPU")
def test_without_a_gpu_the_bench_fails_loudly():
    r = run_bench()
    assert r.returncode == 2
    assert "needs a GPU" in r.stderr
    assert r.stdout.strip() == ""


def test_entry_module_has_build_and_smoke():
    sys.path.insert(0, ROOT)
    import __graft_entry__ as g
    assert callable(g.build) and callable(g.smoke)


@pytest.mark.skipif(torch.cuda.is_available(), reason="checks the behaviour without a GPU")
def test_product_path_fails_loudly_without_a_gpu():
    """The binding never falls back to the CPU: without a device the call raises."""
    from paper_2505_14201_amd import flashd
    q = torch.zeros(1, 1, 8, 64, dtype=torch.bfloat16)
    with pytest.raises(Exception):
        flashd.attn_fwd(q, q, q, torch.empty_like(q), False, 0.125)
