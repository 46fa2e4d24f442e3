"""The entry points that never allocate only enqueue kernels, so they can be recorded into a
HIP graph and replayed: each replay (with the program's own eager work and synchronisations
in between, and fresh input values in the same buffers) must reproduce the eager result bit
for bit."""
import pytest
import torch

from paper_2505_14201_amd import flashd, synthetic

pytestmark = pytest.mark.gpu


def fresh(w, seed):
    import dataclasses
    q, k, v, _ = synthetic.make_qkv(dataclasses.replace(w, seed=seed))
    return q.cuda(), k.cuda(), v.cuda()


@pytest.mark.parametrize("case", [
    ("prefill", 2, 8, 4, 300, 300, 128, "bf16", True, flashd.VARIANT_TILE, 1),
    ("prefill split", 1, 2, 2, 130, 900, 64, "f16", False, flashd.VARIANT_TILE, 3),
    ("decode", 4, 16, 4, 1, 3000, 128, "bf16", False, flashd.VARIANT_AUTO, 4),
    ("per key", 1, 2, 1, 40, 200, 64, "f32", True, flashd.VARIANT_PER_KEY, 2),
    ("prefill, 256 rows", 1, 4, 2, 512, 1100, 128, "bf16", True, flashd.VARIANT_TILE_256, 1),
])
def test_graph_replays_equal_eager(case):
    name, B, Hq, Hkv, Lq, Lk, d, dtype, causal, variant, splits = case
    w = synthetic.small(name, B, Hq, Hkv, Lq, Lk, d, dtype, causal, seed=40)
    dt = {"f32": 0, "f16": 1, "bf16": 2}[dtype]
    nbytes = flashd.workspace_bytes(B, Hq, Hkv, Lq, Lk, d, dt, variant, splits)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda")
    q, k, v = fresh(w, 40)
    o = torch.empty_like(q)
    cnt = torch.zeros(3, dtype=torch.int64, device="cuda")

    def work():
        flashd.attn_fwd_ex(q, k, v, o, causal, w.scale, variant, splits, ws)
        flashd.skip_stats(q, k, causal, w.scale, counts=cnt)

    # warm-up outside the capture, on a side stream as torch asks for
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        work()
    torch.cuda.current_stream().wait_stream(s)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        work()
    for rep in range(3):
        qn, kn, vn = fresh(w, 41 + rep)
        q.copy_(qn); k.copy_(kn); v.copy_(vn)
        o.fill_(float("nan")); cnt.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        got_o, got_c = o.clone(), cnt.clone()
        o.fill_(float("nan")); cnt.fill_(-1)
        work()                                     # eager, same buffers
        torch.cuda.synchronize()
        assert torch.equal(got_o, o), f"{name}: replay {rep} differs from eager"
        assert torch.equal(got_c, cnt), f"{name}: replay {rep} counters differ"
        assert torch.isfinite(o.float()).all()
