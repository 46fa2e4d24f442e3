"""The entry point that allocates nothing (split-K partial states in a fixed array inside the
library) against flashd_attn_fwd, through the C ABI: two calls in a row, the second on a
smaller problem, so that the array still holds the first call's partial states."""
import numpy as np
import pytest
import torch

from paper_2505_14201_amd import synthetic

pytestmark = pytest.mark.gpu


def _both(w):
    from paper_2505_14201_amd import flashd
    q, k, v, _ = synthetic.make_qkv(w)
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    dt = {"f32": 0, "f16": 1, "bf16": 2}[w.dtype]
    splits = flashd.auto_splits(w.B, w.Hq, w.Hkv, w.Lq, w.Lk, w.d, dt)
    need = flashd.workspace_bytes(w.B, w.Hq, w.Hkv, w.Lq, w.Lk, w.d, dt)
    ref = torch.full_like(qg, float("nan"))
    got = torch.full_like(qg, float("nan"))
    flashd.attn_fwd(qg, kg, vg, ref, w.causal, w.scale)
    flashd.attn_fwd_static(qg, kg, vg, got, w.causal, w.scale)
    torch.cuda.synchronize()
    return q, k, v, ref.cpu(), got.cpu(), splits, need


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_static_scratch_matches_the_allocating_entry_point(dtype):
    from oracle import attention as oa
    from tests.gpu_util import check
    # decode shapes that the automatic choice splits; the second call is smaller in every
    # dimension and uses fewer splits, so stale partial states of the first lie behind its own
    big = synthetic.small("na_big", 2, 8, 2, 1, 4096, 128, dtype, False, seed=71)
    small = synthetic.small("na_small", 1, 4, 2, 1, 1500, 128, dtype, False, seed=72)
    for w in (big, small):
        q, k, v, ref, got, splits, need = _both(w)
        assert splits > 1 and need > 0, "the case must use the scratch array"
        assert torch.equal(ref.view(torch.uint8), got.view(torch.uint8)), w.name
        want = oa.attn(q, k, v, w.causal, w.scale)
        check(got, want, q.dtype, w.name)


def test_static_scratch_on_a_split_prefill_and_unsplit_shapes():
    # a causal prefill whose keys are split by the tile kernel, then one without splits
    for w in (synthetic.small("na_pf", 1, 2, 2, 512, 4096, 64, "bf16", True, seed=73),
              synthetic.small("na_one", 1, 2, 1, 200, 200, 64, "f16", True, seed=74)):
        q, k, v, ref, got, splits, need = _both(w)
        assert torch.equal(ref.view(torch.uint8), got.view(torch.uint8)), w.name


def test_static_scratch_refuses_what_does_not_fit():
    from paper_2505_14201_amd import flashd
    # many long heads, keys split in two: more partial states than the array holds
    B, Hq, Hkv, Lq, Lk, d = 1, 96, 96, 512, 4096, 128
    need = flashd.workspace_bytes(B, Hq, Hkv, Lq, Lk, d, flashd.BF16)
    if need <= flashd.STATIC_SCRATCH_BYTES:
        pytest.skip("the automatic choice does not split this shape")
    q = torch.zeros(B, Hq, Lq, d, dtype=torch.bfloat16, device="cuda")
    k = torch.zeros(B, Hkv, Lk, d, dtype=torch.bfloat16, device="cuda")
    o = torch.zeros_like(q)
    with pytest.raises(flashd.FlashdError) as e:
        flashd.attn_fwd_static(q, k, k, o, True, 0.1)
    assert e.value.status == -7
