"""GPU parity at the full sizes of the benchmark configurations, through the entry point and
in the launch configuration bench.py times (flashd_attn_fwd, automatic variant and splits).
The oracle is evaluated on all rows of a few heads plus sampled rows everywhere (first and
last rows, tile-edge rows, a seeded remainder) and, for the stress configuration, on every
row that has a planted dominant key."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from paper_2505_14201_amd import flashd, synthetic
from tests.gpu_util import check

pytestmark = pytest.mark.gpu
DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def run_auto(q, k, v, w, variant=None):
    """variant=None: flashd_attn_fwd as bench.py times it; else that variant, unsplit."""
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    og = torch.full_like(qg, float("nan"))
    if variant is None:
        flashd.attn_fwd(qg, kg, vg, og, w.causal, w.scale)
    else:
        flashd.attn_fwd_ex(qg, kg, vg, og, w.causal, w.scale, variant, 1)
    torch.cuda.synchronize()
    out = og.cpu()
    del qg, kg, vg, og
    torch.cuda.empty_cache()
    return out


def compare_rows(got, q, k, v, w, rows, what):
    ref = oa.attn(q, k, v, w.causal, w.scale, "definition", rows)
    idx = torch.from_numpy(rows.astype(np.int64))
    sel = got[idx[:, 0], idx[:, 1], idx[:, 2], :]
    assert torch.isfinite(got).all(), what + ": non-finite output somewhere"
    return check(sel, ref, DT[w.dtype], what)


def rows_for(w, heads, n_extra, seed, must=()):
    must = list(must) + [(b, h, i) for (b, h) in heads for i in range(w.Lq)]
    return synthetic.sample_rows(w, len(must) + n_extra, seed=seed, must=must)


def test_causal_prefill_config_and_its_shifted_values_twin():
    w = synthetic.CONFIGS[1]
    q, k, v, _ = synthetic.make_qkv(w)
    rows = rows_for(w, [(0, 0), (w.B - 1, w.Hq - 1), (1, 7)], 8192, seed=21)
    compare_rows(run_auto(q, k, v, w), q, k, v, w, rows, w.name)
    # both prefill kernels by name (whichever the automatic choice takes, bench.py times the
    # other one beside it), the per-tile blend and the ablation
    for variant in (flashd.VARIANT_TILE, flashd.VARIANT_TILE_256, flashd.VARIANT_TILE_BLEND,
                    flashd.VARIANT_ONLINE_SOFTMAX):
        compare_rows(run_auto(q, k, v, w, variant), q, k, v, w, rows[::4],
                     f"{w.name} variant={variant}")
    # V + 1: outputs near 1, where the absolute bound of 2e-2 is a real constraint
    v1 = (v.float() + 1.0).to(v.dtype)
    compare_rows(run_auto(q, k, v1, w), q, k, v1, w, rows[::4], w.name + " (V + 1)")


def test_long_noncausal_prefill_config():
    w = synthetic.CONFIGS[2]
    q, k, v, _ = synthetic.make_qkv(w)
    rows = synthetic.sample_rows(w, 3072, seed=22)
    compare_rows(run_auto(q, k, v, w), q, k, v, w, rows, w.name)
    for variant in (flashd.VARIANT_TILE, flashd.VARIANT_TILE_256):
        compare_rows(run_auto(q, k, v, w, variant), q, k, v, w, rows[::4],
                     f"{w.name} variant={variant}")


def test_gqa_decode_config_in_full():
    w = synthetic.CONFIGS[3]
    q, k, v, _ = synthetic.make_qkv(w)
    got = run_auto(q, k, v, w)
    ref = oa.attn(q, k, v, w.causal, w.scale)
    check(got, ref, DT[w.dtype], w.name)


def test_stability_stress_config_with_every_planted_row():
    w = synthetic.CONFIGS[4]
    q, k, v, planted = synthetic.make_qkv(w)
    assert len(planted) > 1000
    rows = rows_for(w, [(0, 0), (1, 15)], 4096, seed=24,
                    must=[(b, h, i) for (b, h, i, _) in planted])
    compare_rows(run_auto(q, k, v, w), q, k, v, w, rows, w.name)
    # the per-tile blend and the ablation on the same input (the variants bench.py times)
    for variant in (flashd.VARIANT_TILE_BLEND, flashd.VARIANT_ONLINE_SOFTMAX):
        compare_rows(run_auto(q, k, v, w, variant), q, k, v, w, rows[::2],
                     f"{w.name} variant={variant}")
