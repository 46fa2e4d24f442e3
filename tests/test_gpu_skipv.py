"""Decode with the saturation skip of Sec. III-C on the V fetch (flashd_attn_fwd_skipv):
parity against the fp64 oracle at the usual bound, equality with the unskipped decode kernel
(variant TILE), and the counters that say how many 32-key blocks went without their V."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import attention as oa
from paper_2505_14201_amd import flashd, synthetic
from tests.gpu_util import Guarded, check

pytestmark = pytest.mark.gpu
DT = {"f16": torch.float16, "bf16": torch.bfloat16}


def run_both(w, splits):
    q, k, v, _ = synthetic.make_qkv(w)
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    dt = {"f16": 1, "bf16": 2}[w.dtype]
    nbytes = flashd.workspace_bytes(w.B, w.Hq, w.Hkv, w.Lq, w.Lk, w.d, dt, flashd.VARIANT_TILE,
                                    splits)
    ws = Guarded(nbytes) if nbytes else None
    base_g = Guarded(qg.numel() * qg.element_size())
    skip_g = Guarded(qg.numel() * qg.element_size())
    base, skip = base_g.view(qg.dtype, qg.shape), skip_g.view(qg.dtype, qg.shape)
    counts = torch.zeros(2, dtype=torch.int64, device="cuda")
    wsp = ws.payload if ws else None
    flashd.attn_fwd_ex(qg, kg, vg, base, w.causal, w.scale, flashd.VARIANT_TILE, splits, wsp)
    flashd.attn_fwd_skipv(qg, kg, vg, skip, w.causal, w.scale, splits, wsp, counts)
    torch.cuda.synchronize()
    assert base_g.intact() and skip_g.intact() and (ws is None or ws.intact())
    visited, skipped = (int(x) for x in counts.cpu())
    return q, k, v, base.cpu(), skip.cpu(), visited, skipped


# (B, Hq, Hkv, Lq, Lk, d, dtype, causal, splits)
# one query position per head: the planted key is built from the last position's queries
PEAKED_SHAPES = [
    (3, 32, 8, 1, 4096, 128, "bf16", False, 1),      # the GQA decode shape, shortened
    (2, 8, 2, 1, 3000, 128, "bf16", False, 0),       # automatic key splits, ragged tail
    (2, 8, 2, 1, 2000, 64, "f16", False, 1),         # d = 64, f16 (coefficients flush sooner)
    (1, 4, 4, 1, 1500, 64, "bf16", True, 3),         # no grouping, explicit splits
]
SHAPES = PEAKED_SHAPES + [
    (2, 8, 2, 4, 2000, 64, "f16", True, 1),          # several positions, causal
    (1, 4, 4, 7, 1500, 64, "bf16", True, 3),
]


@pytest.mark.parametrize("shape", PEAKED_SHAPES)
def test_peaked_scores_skip_value_blocks_and_keep_the_result(shape):
    B, Hq, Hkv, Lq, Lk, d, dtype, causal, splits = shape
    w = synthetic.small("peaked", B, Hq, Hkv, Lq, Lk, d, dtype, causal, seed=8100 + Lk,
                        qk_std=4.0, sink_gain=8.0)
    q, k, v, base, skip, visited, skipped = run_both(w, splits)
    ref = oa.attn(q, k, v, causal, w.scale)
    check(skip, ref, DT[dtype], f"{shape} skipv")
    check(base, ref, DT[dtype], f"{shape} tile")
    assert torch.equal(base.view(torch.int16), skip.view(torch.int16)), \
        f"{shape}: the skip changed a bit of the output"
    assert visited >= B * Hkv * ((Lk + 31) // 32)
    # After the dominant key of a group (one of the first Lk / 64) almost every block of the
    # workgroup that holds it can go.  Key splits are workgroups of their own and share no
    # bound: only the split with the dominant key skips.
    nsplits = splits if splits else flashd.auto_splits(B, Hq, Hkv, Lq, Lk, d,
                                                       {"f16": 1, "bf16": 2}[dtype])
    assert skipped > 0.3 * visited / nsplits, \
        f"{shape}: only {skipped} of {visited} blocks skipped ({nsplits} splits)"


@pytest.mark.parametrize("shape", SHAPES)
def test_ordinary_scores_skip_nothing_and_match_bit_for_bit(shape):
    B, Hq, Hkv, Lq, Lk, d, dtype, causal, splits = shape
    w = synthetic.small("plain", B, Hq, Hkv, Lq, Lk, d, dtype, causal, seed=8200 + Lk)
    q, k, v, base, skip, visited, skipped = run_both(w, splits)
    assert skipped == 0 and visited > 0
    assert torch.equal(base.view(torch.int16), skip.view(torch.int16))
    check(skip, oa.attn(q, k, v, causal, w.scale), DT[dtype], f"{shape} skipv, nothing to skip")


def test_a_dominant_key_late_in_the_sequence_is_not_lost():
    """The dominant key comes last: nothing before it may be skipped on its account, and what
    was accumulated before it must give way to it."""
    w = synthetic.small("late", 2, 8, 2, 1, 2048, 128, "bf16", False, seed=8300, qk_std=4.0)
    q, k, v, _ = synthetic.make_qkv(w)
    g = w.Hq // w.Hkv
    for b in range(w.B):
        for kvh in range(w.Hkv):
            grp = q[b, kvh * g:(kvh + 1) * g, 0, :].float().sum(dim=0)
            k[b, kvh, w.Lk - 1 - 40 * kvh, :] = (grp * (8.0 / g)).to(k.dtype)
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    o = torch.full_like(qg, float("nan"))
    counts = torch.zeros(2, dtype=torch.int64, device="cuda")
    flashd.attn_fwd_skipv(qg, kg, vg, o, False, w.scale, 1, None, counts)
    torch.cuda.synchronize()
    check(o.cpu(), oa.attn(q, k, v, False, w.scale), torch.bfloat16, "late dominant key")


def test_skipv_is_refused_where_it_does_not_apply():
    q = torch.zeros(1, 8, 64, 64, dtype=torch.bfloat16, device="cuda")     # 64 rows per kv head
    k = torch.zeros(1, 8, 256, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(flashd.FlashdError) as e:
        flashd.attn_fwd_skipv(q, k, k, torch.empty_like(q), False, 0.1)
    assert e.value.status == -10
    qf = torch.zeros(1, 8, 1, 64, device="cuda")
    kf = torch.zeros(1, 8, 256, 64, device="cuda")
    with pytest.raises(flashd.FlashdError) as e:
        flashd.attn_fwd_skipv(qf, kf, kf, torch.empty_like(qf), False, 0.1)
    assert e.value.status == -10
