"""The C oracle built with AddressSanitizer and UndefinedBehaviorSanitizer (gcc, host only) runs
a driver over ragged, causal, grouped-head, row-subset, chunked-state and skip-count cases in
heap buffers of exact size; any invalid access or undefined operation stops it.  What it
prints must equal what the ordinary build returns for the same inputs."""
import os
import subprocess

import numpy as np
import pytest
import torch

from oracle import attention as oa

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRCS = [os.path.join(ROOT, "oracle", f) for f in ("attn_oracle.c", "skip_oracle.c", "state_oracle.c")]
SHAPES = [(1, 1, 1, 1, 1, 1, 0), (2, 4, 2, 5, 9, 8, 1), (1, 2, 1, 9, 5, 4, 1),
          (1, 3, 3, 7, 7, 16, 0), (1, 2, 2, 3, 70, 2, 1)]
SCALE = 0.75


def gen(n: int, salt: int) -> np.ndarray:
    """The driver's integer hash, repeated with 32-bit wrap-around."""
    m = np.uint64(0xFFFFFFFF)
    x = (np.arange(n, dtype=np.uint64) * np.uint64(2654435761) + np.uint64(salt * 40503)) & m
    x ^= x >> np.uint64(15)
    x = (x * np.uint64(2246822519)) & m
    x ^= x >> np.uint64(13)
    return (((x >> np.uint64(8)) & np.uint64(0xFFFF)).astype(np.int64) - 32768).astype(np.float32) / np.float32(8192)


@pytest.fixture(scope="module")
def sanitized_output(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("asan") / "oracle_sanitized")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan",
           "-o", exe, os.path.join(HERE, "oracle_sanitized_driver.c"), *SRCS, "-lm"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ, OMP_NUM_THREADS="2", ASAN_OPTIONS="detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    env.pop("LD_PRELOAD", None)      # the sanitizer runtime has to come first
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, f"sanitized oracle failed (rc {r.returncode}):\n{r.stderr[-3000:]}"
    assert r.stdout.strip().endswith("done")
    out = {}
    for line in r.stdout.splitlines():
        f = line.split()
        if f[0] == "skip":
            out[("skip", int(f[1]))] = tuple(int(x) for x in f[2:5])
        elif f[0] != "done":
            out.setdefault((f[0], int(f[1])), []).append(float.fromhex(f[3]))
    return out


@pytest.mark.parametrize("c", range(len(SHAPES)))
def test_sanitized_build_runs_clean_and_agrees_with_the_ordinary_build(sanitized_output, c):
    B, Hq, Hkv, Lq, Lk, d, causal = SHAPES[c]
    q = torch.from_numpy(gen(B * Hq * Lq * d, 3 * c + 1).reshape(B, Hq, Lq, d))
    k = torch.from_numpy(gen(B * Hkv * Lk * d, 3 * c + 2).reshape(B, Hkv, Lk, d))
    v = torch.from_numpy(gen(B * Hkv * Lk * d, 3 * c + 3).reshape(B, Hkv, Lk, d))
    for algo, name in enumerate(("definition", "alg1", "alg2", "alg3")):
        want = oa.attn(q, k, v, bool(causal), SCALE, name).ravel()
        got = np.array(sanitized_output[(f"attn{algo}", c)])
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-13, err_msg=name)
    rows = [(B - 1, Hq - 1, 0), (B - 1, Hq - 1, Lq - 1)]
    want = oa.attn(q, k, v, bool(causal), SCALE, rows=rows).ravel()
    np.testing.assert_allclose(np.array(sanitized_output[("rows", c)]), want, rtol=0, atol=1e-13)
    cut = Lk // 2 if Lk > 1 else 1
    st1 = oa.attn_state(q, k[:, :, :cut].contiguous(), v[:, :, :cut].contiguous(), bool(causal),
                        SCALE, shift=Lk - Lq)
    got1 = np.array(sanitized_output[("state1", c)])
    assert np.array_equal(np.isinf(got1), np.isinf(st1.ravel()))
    fin = np.isfinite(st1.ravel())
    np.testing.assert_allclose(got1[fin], st1.ravel()[fin], rtol=0, atol=1e-13)
    if Lk - cut >= 1:
        st2 = oa.attn_state(q, k[:, :, cut:].contiguous(), v[:, :, cut:].contiguous(),
                            bool(causal), SCALE, state_in=st1, shift=Lk - Lq - cut).ravel()
        got2 = np.array(sanitized_output[("state2", c)])
        fin = np.isfinite(st2)
        assert np.array_equal(np.isfinite(got2), fin)
        np.testing.assert_allclose(got2[fin], st2[fin], rtol=0, atol=1e-13)
    assert sanitized_output[("skip", c)] == oa.skip_stats(q, k, bool(causal), SCALE, -1.0, 1.5)
