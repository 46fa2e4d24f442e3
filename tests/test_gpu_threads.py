"""Host threads: the header promises that the automatic entry point may be called from
several host threads at once, each on a stream of its own, while its split-K cache grows.
Results are bitwise reproducible for fixed inputs, so every threaded result must equal the
one a single thread gets for the same problem (which the parity tests hold to the oracle)."""
import threading

import pytest
import torch

from paper_2505_14201_amd import flashd, synthetic

pytestmark = pytest.mark.gpu

# decode and short-query shapes whose automatic choice splits the keys; key counts grow, so
# each thread's cache is outgrown several times while other threads are inside the library
LKS = [700, 1500, 3100, 6300, 4000, 9000]


def problem(tid, step):
    Lk = LKS[step] + 37 * tid
    w = synthetic.small("threads", 2, 8, 2, 1 + (tid % 2), Lk, 128 if tid % 2 else 64,
                        "bf16" if tid < 2 else "f16", False, seed=7000 + 10 * tid + step)
    q, k, v, _ = synthetic.make_qkv(w)
    return w, q.cuda(), k.cuda(), v.cuda()


def test_concurrent_calls_on_private_streams_equal_serial_calls():
    n_threads = 4
    probs = [[problem(t, s) for s in range(len(LKS))] for t in range(n_threads)]
    assert any(flashd.auto_splits(w.B, w.Hq, w.Hkv, w.Lq, w.Lk, w.d, flashd._DTYPE[q.dtype]) > 1
               for row in probs for (w, q, _, _) in row)
    torch.cuda.synchronize()

    outs = [[None] * len(LKS) for _ in range(n_threads)]
    errors = []
    gate = threading.Barrier(n_threads)

    def worker(t):
        try:
            stream = torch.cuda.Stream()
            gate.wait(timeout=30)
            for s, (w, q, k, v) in enumerate(probs[t]):
                o = torch.full_like(q, float("nan"))
                stream.wait_stream(torch.cuda.default_stream())
                flashd.attn_fwd(q, k, v, o, w.causal, w.scale, stream=stream)
                outs[t][s] = o
            stream.synchronize()
        except Exception as e:          # noqa: BLE001 - reported by the main thread
            errors.append((t, repr(e)))

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(n_threads)]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=100)
    assert not any(th.is_alive() for th in threads), "a worker did not finish"
    assert not errors, errors
    torch.cuda.synchronize()

    for t in range(n_threads):
        for s, (w, q, k, v) in enumerate(probs[t]):
            ref = torch.full_like(q, float("nan"))
            flashd.attn_fwd(q, k, v, ref, w.causal, w.scale)
            torch.cuda.synchronize()
            assert torch.isfinite(ref.float()).all()
            assert torch.equal(outs[t][s], ref), f"thread {t} step {s} differs from the serial call"
