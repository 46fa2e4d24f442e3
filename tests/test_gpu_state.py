"""GPU parity of flashd_attn_fwd_state: chunks of keys with the Alg. 3 state handed in and
out, against the fp64 oracle (the literal recurrence; only o and s - ln w are unique)."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from paper_2505_14201_amd import flashd, synthetic
from tests.gpu_util import Guarded, check

pytestmark = pytest.mark.gpu
DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def lam_of(state, d):
    return state[..., d] - state[..., d + 1]


def check_state(got, ref, d, dtype, what):
    """got: GPU state (CPU float32 tensor), ref: oracle state (fp64).  Compares the output
    part to the usual tolerance and s - ln w (the only other quantity later steps see)."""
    check(got[..., :d], ref[..., :d], dtype, what + " (o)")
    lg, lr = lam_of(got.double().numpy(), d), lam_of(ref, d)
    empty = np.isneginf(lr)
    assert np.array_equal(np.isneginf(lg), empty), what + ": rows without keys"
    err = np.abs(lg[~empty] - lr[~empty])
    # fp32 rounding of the score sums.  (For bf16 the matrix-core kernels normalise o by the sum
    # of the ROUNDED tile coefficients; where a state leaves the kernel they carry the sum of
    # the unrounded ones beside it, and that is what s - ln w is taken from.)
    bound = 2e-4 + 1e-5 * np.abs(lr[~empty])
    assert np.all(err <= bound), f"{what}: s - ln w off by {err.max():.3e}"


def run_chunks(q, k, v, causal, scale, cuts, in_place=False):
    """Feeds the keys in chunks [0,c1), [c1,c2), ...; returns the final o and state."""
    B, Hq, Lq, d = q.shape
    Lk = k.shape[2]
    qg = q.cuda()
    st = None
    # the output and every state buffer sit between canaries, checked after the launches
    guards = [Guarded(qg.numel() * qg.element_size())]
    o = guards[0].view(qg.dtype, qg.shape)
    k0 = 0
    for k1 in list(cuts) + [Lk]:
        kc, vc = k[:, :, k0:k1].contiguous().cuda(), v[:, :, k0:k1].contiguous().cuda()
        if in_place and st is not None:
            out = st
        else:
            guards.append(Guarded(B * Hq * Lq * (d + 2) * 4))
            out = guards[-1].view(torch.float32, (B, Hq, Lq, d + 2))
        flashd.attn_fwd_state(qg, kc, vc, causal, scale, o=o, state_in=st, state_out=out,
                              causal_shift=(Lk - Lq) - k0)
        st = out
        k0 = k1
    torch.cuda.synchronize()
    assert all(g.intact() for g in guards), "a kernel wrote outside the output or a state buffer"
    return o.cpu(), st.cpu()


# (B, Hq, Hkv, Lq, Lk, d, cuts)
CASES = [
    (1, 2, 1, 70, 300, 64, (64, 200)),
    (2, 4, 2, 200, 333, 128, (100,)),
    (1, 2, 2, 333, 200, 128, (64, 128)),        # causal: the first rows see no key at all
    (1, 8, 2, 1, 4000, 128, (1000, 2500)),      # one query row per head: the split-K decode path
    (2, 4, 4, 129, 129, 64, (1, 2, 65)),
]


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_chunks_with_state_passing_match_the_oracle(case, causal, dtype):
    B, Hq, Hkv, Lq, Lk, d, cuts = case
    w = synthetic.small("state", B, Hq, Hkv, Lq, Lk, d, dtype, causal, seed=500 + Lq + Lk)
    q, k, v, _ = synthetic.make_qkv(w)
    ref_state = oa.attn_state(q, k, v, causal, w.scale)
    o, st = run_chunks(q, k, v, causal, w.scale, cuts)
    what = f"{case} causal={causal} {dtype}"
    check(o, ref_state[..., :d], DT[dtype], what + " (final o)")
    check_state(st, ref_state, d, DT[dtype], what)
    # and one call over all keys gives the same state
    o1, st1 = run_chunks(q, k, v, causal, w.scale, ())
    check(o1, ref_state[..., :d], DT[dtype], what + " (one call)")
    check_state(st1, ref_state, d, DT[dtype], what + " (one call)")


def test_state_may_be_updated_in_place_and_outputs_are_optional():
    w = synthetic.small("state", 1, 4, 2, 150, 400, 128, "bf16", True, seed=901)
    q, k, v, _ = synthetic.make_qkv(w)
    ref = oa.attn_state(q, k, v, True, w.scale)
    o, st = run_chunks(q, k, v, True, w.scale, (128, 256), in_place=True)
    check_state(st, ref, 128, torch.bfloat16, "in place")
    # state only, then output only from a state
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    half = 200
    s1 = torch.empty(1, 4, 150, 130, dtype=torch.float32, device="cuda")
    flashd.attn_fwd_state(qg, kg[:, :, :half].contiguous(), vg[:, :, :half].contiguous(), True,
                          w.scale, state_out=s1, causal_shift=400 - 150)
    o2 = torch.full_like(qg, float("nan"))
    flashd.attn_fwd_state(qg, kg[:, :, half:].contiguous(), vg[:, :, half:].contiguous(), True,
                          w.scale, o=o2, state_in=s1, causal_shift=400 - 150 - half)
    torch.cuda.synchronize()
    check(o2.cpu(), ref[..., :128], torch.bfloat16, "output from a state")
    with pytest.raises(flashd.FlashdError):
        flashd.attn_fwd_state(qg, kg, vg, True, w.scale)        # neither o nor state_out


def test_dominant_keys_across_chunk_boundaries_stay_finite():
    """Score jumps of hundreds between chunks: the merge saturates instead of overflowing."""
    import dataclasses
    w = dataclasses.replace(synthetic.CONFIGS[4], B=1, Hq=2, Hkv=2, Lq=512, Lk=512)
    q, k, v, _ = synthetic.make_qkv(w)
    ref = oa.attn_state(q, k, v, True, w.scale)
    o, st = run_chunks(q, k, v, True, w.scale, (100, 101, 300))
    assert torch.isfinite(o).all()
    check(o, ref[..., :64], torch.float16, "stress chunks")


@pytest.mark.parametrize("shape", [(1, 2, 2, 200, 300, 128), (1, 8, 2, 2, 900, 64)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_extreme_causal_shifts_show_every_key_or_none(shape, dtype):
    """Any int is a valid shift: from Lk up every key is visible (the non-causal result),
    below -Lq none (zeros, the state of a row without keys)."""
    B, Hq, Hkv, Lq, Lk, d = shape
    w = synthetic.small("shift", B, Hq, Hkv, Lq, Lk, d, dtype, False, seed=930 + Lq)
    q, k, v, _ = synthetic.make_qkv(w)
    ref = oa.attn(q, k, v, False, w.scale)
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    for shift in (Lk, Lk + 5, 2 ** 31 - 1):
        o = torch.full_like(qg, float("nan"))
        flashd.attn_fwd_state(qg, kg, vg, True, w.scale, o=o, causal_shift=shift)
        torch.cuda.synchronize()
        check(o.cpu(), ref, DT[dtype], f"{shape} {dtype} shift={shift}")
    for shift in (-Lq, -Lq - 7, -2 ** 31):
        o = torch.full_like(qg, float("nan"))
        st = torch.full((B, Hq, Lq, d + 2), float("nan"), dtype=torch.float32, device="cuda")
        flashd.attn_fwd_state(qg, kg, vg, True, w.scale, o=o, state_out=st, causal_shift=shift)
        torch.cuda.synchronize()
        assert torch.count_nonzero(o) == 0, f"shift={shift}: rows without keys must be zeros"
        assert torch.isneginf(st[..., d] - st[..., d + 1]).all(), f"shift={shift}: empty state"


@pytest.mark.parametrize("causal", [False, True])
def test_state_passing_with_query_heads_run_as_one_head(causal):
    """Few positions per head and several query heads per kv head: the tile kernel packs the
    group's heads into one run of rows; the state layout must not notice."""
    B, Hq, Hkv, Lq, Lk, d = 2, 8, 2, 24, 400, 128
    w = synthetic.small("state", B, Hq, Hkv, Lq, Lk, d, "bf16", causal, seed=940)
    q, k, v, _ = synthetic.make_qkv(w)
    ref_state = oa.attn_state(q, k, v, causal, w.scale)
    o, st = run_chunks(q, k, v, causal, w.scale, (130, 257))
    check(o, ref_state[..., :d], torch.bfloat16, f"packed state causal={causal} (o)")
    check_state(st, ref_state, d, torch.bfloat16, f"packed state causal={causal}")
