"""The seeded input generators: shapes, determinism and the planted structure (no GPU)."""
import numpy as np
import torch

from paper_2505_14201_amd import synthetic


def test_config_table_matches_the_stated_workloads():
    c = synthetic.CONFIGS
    assert [(w.B, w.Hq, w.Hkv, w.Lq, w.Lk, w.d, w.dtype, w.causal) for w in c] == [
        (1, 1, 1, 128, 128, 64, "f32", False),
        (4, 32, 32, 2048, 2048, 128, "bf16", True),
        (1, 32, 32, 16384, 16384, 128, "bf16", False),
        (64, 32, 8, 1, 8192, 128, "bf16", False),
        (2, 16, 16, 4096, 4096, 64, "f16", True)]
    assert c[1].flops() == 4 * 128 * 4 * 32 * (2048 * 2049 // 2)
    assert c[2].flops() == 4 * 128 * 32 * 16384 ** 2
    assert c[3].bytes_io() == 2 * (2 * 64 * 8 * 8192 * 128 + 2 * 64 * 32 * 128)
    assert abs(c[1].scale - 128 ** -0.5) < 1e-15


def test_visible_pairs_counts_the_bottom_right_mask():
    for Lq, Lk in [(5, 5), (3, 7), (7, 3), (1, 4)]:
        w = synthetic.small("t", 1, 1, 1, Lq, Lk, 8, "f32", True, 0)
        brute = sum(1 for i in range(Lq) for j in range(Lk) if j <= i + Lk - Lq)
        assert w.visible_pairs() == brute


def test_generation_is_deterministic_and_cast_once():
    w = synthetic.small("t", 2, 4, 2, 9, 11, 16, "bf16", False, seed=5)
    a = synthetic.make_qkv(w)
    b = synthetic.make_qkv(w)
    for x, y in zip(a[:3], b[:3]):
        assert x.dtype == torch.bfloat16 and torch.equal(x, y)
    assert a[0].shape == (2, 4, 9, 16) and a[1].shape == (2, 2, 11, 16) and a[2].shape == a[1].shape
    rng = np.random.default_rng(5)
    q32 = rng.standard_normal((2, 4, 9, 16), dtype=np.float32)
    assert torch.equal(a[0], torch.from_numpy(q32).to(torch.bfloat16))


def test_planted_keys_are_visible_and_exact():
    w = synthetic.small("t", 1, 3, 3, 200, 200, 8, "f16", True, seed=6, qk_std=4.0, plant_frac=0.05)
    q, k, v, planted = synthetic.make_qkv(w)
    assert 10 <= len(planted) <= 60
    last = {}
    for (b, h, i, j) in planted:
        assert 0 <= j <= i
        last[(b, h, j)] = i
    for (b, h, j), i in last.items():
        assert torch.equal(k[b, h, j].float(), q[b, h, i].float() * 8)
    assert 3.5 < q.float().std() < 4.5 and 0.9 < v.float().std() < 1.1


def test_sample_rows_cover_edges():
    w = synthetic.CONFIGS[1]
    rows = synthetic.sample_rows(w, 300, seed=1, must=[(3, 31, 2047)])
    assert rows.shape == (300, 3) and len({tuple(r) for r in rows}) == 300
    iset = set(rows[:, 2].tolist())
    for i in (0, 1, 63, 64, 127, 128, 255, 256, 2046, 2047):
        assert i in iset
    assert (3, 31, 2047) in {tuple(r) for r in rows}
