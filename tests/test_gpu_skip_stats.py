"""GPU parity of the static skip statistics (Sec. III-C): integer counts, compared bit for
bit with the oracle, which fixes the same fp32 score arithmetic."""
import dataclasses

import pytest
import torch

from oracle import attention as oa
from paper_2505_14201_amd import flashd, synthetic

pytestmark = pytest.mark.gpu


def both(q, k, causal, scale, lo=-6.0, hi=11.0):
    got = flashd.skip_stats(q.cuda(), k.cuda(), causal, scale, lo, hi)
    ref = oa.skip_stats(q, k, causal, scale, lo, hi)
    return got, ref


# (B, Hq, Hkv, Lq, Lk, d): several 64-key steps with ragged tails, Lq != Lk, GQA, empty rows
SHAPES = [(1, 1, 1, 1, 1, 64), (1, 2, 1, 3, 65, 64), (2, 4, 2, 70, 200, 128),
          (1, 2, 2, 333, 200, 64), (1, 3, 1, 130, 517, 128), (5, 1, 1, 9, 64, 128)]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_counts_match_the_oracle_exactly(shape, causal, dtype):
    B, Hq, Hkv, Lq, Lk, d = shape
    w = synthetic.small("skip", B, Hq, Hkv, Lq, Lk, d, dtype, causal, seed=31 + Lq + Lk)
    w = dataclasses.replace(w, qk_std=4.0)          # score differences reach both thresholds
    q, k, _, _ = synthetic.make_qkv(w)
    got, ref = both(q, k, causal, w.scale)
    assert got == ref
    if Lk >= 64 and Lq >= 3:
        assert ref[1] > 0 and ref[2] > 0


def test_thresholds_are_inclusive_and_adjustable():
    vals = [0.0, -6.0, 5.0, 16.0, 15.0, 4.0, -2.0]
    k = torch.zeros(1, 1, len(vals), 64)
    k[0, 0, :, 0] = torch.tensor(vals)
    q = torch.zeros(1, 1, 1, 64)
    q[0, 0, 0, 0] = 1.0
    assert both(q, k, False, 1.0) == ((6, 3, 2), (6, 3, 2))
    assert both(q, k, False, 1.0, -6.5, 11.5) == ((6, 1, 0), (6, 1, 0))


def test_counts_buffer_is_overwritten_not_accumulated():
    w = synthetic.small("skip", 1, 2, 1, 40, 90, 64, "bf16", False, seed=77)
    q, k, _, _ = synthetic.make_qkv(dataclasses.replace(w, qk_std=4.0))
    qg, kg = q.cuda(), k.cuda()
    buf = torch.full((3,), 123456789, dtype=torch.int64, device="cuda")
    flashd.skip_stats(qg, kg, False, w.scale, counts=buf)
    flashd.skip_stats(qg, kg, False, w.scale, counts=buf)
    torch.cuda.synchronize()
    assert tuple(int(x) for x in buf.cpu()) == oa.skip_stats(q, k, False, w.scale)


def test_stress_config_rates():
    """The stability-stress configuration (Q, K ~ N(0, 4^2), planted dominant keys) on a
    reduced batch: about seven steps in ten fall outside the static range."""
    w = dataclasses.replace(synthetic.CONFIGS[4], B=1, Hq=2, Hkv=2, Lq=1024, Lk=1024)
    q, k, _, _ = synthetic.make_qkv(w)
    got, ref = both(q, k, w.causal, w.scale)
    assert got == ref
    steps, low, high = got
    assert 0.6 < (low + high) / steps < 0.8


def test_iid_unit_scores_rarely_leave_the_range():
    w = dataclasses.replace(synthetic.CONFIGS[1], B=1, Hq=4, Hkv=4, Lq=512, Lk=512)
    q, k, _, _ = synthetic.make_qkv(w)
    got, ref = both(q, k, w.causal, w.scale)
    assert got == ref
    steps, low, high = got
    assert (low + high) / steps < 1e-3
