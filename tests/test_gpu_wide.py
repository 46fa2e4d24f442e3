"""GPU parity of variant TILE_256, the 256-row prefill kernel (one wavefront per SIMD, matrix
and vector work interleaved by hand, operands and accumulators in fixed registers), against
the oracle, and against TILE where the call is one it cannot serve.

The shapes cover what the kernel distinguishes: row tiles with many interior blocks (the fused
steps), the first block and the diagonal blocks of a causal mask (plain steps), wavefronts that
stop early under the mask, a ragged key tail, both storage types, scores that grow (references
move: the fused steps hand the block to the plain ones), a negative scale (plain steps only)."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from paper_2505_14201_amd import flashd, synthetic
from tests.gpu_util import check, run_flashd

pytestmark = pytest.mark.gpu
DT = {"f16": torch.float16, "bf16": torch.bfloat16}
WIDE = flashd.VARIANT_TILE_256


def sampled(got, q, k, v, w, n_rows, seed, what, scale=None):
    rows = synthetic.sample_rows(w, n_rows, seed=seed)
    ref = oa.attn(q, k, v, w.causal, w.scale if scale is None else scale, "definition", rows)
    idx = torch.from_numpy(rows.astype(np.int64))
    sel = got[idx[:, 0], idx[:, 1], idx[:, 2], :]
    assert torch.isfinite(got).all(), what + ": non-finite output"
    check(sel, ref, DT[w.dtype], what)


#   (B, Hq, Hkv, Lq, Lk)
SHAPES = [
    (1, 2, 2, 256, 256),       # one row tile, four key tiles
    (1, 4, 2, 512, 1024),      # GQA, Lk > Lq: the causal diagonal sits in the middle of the keys
    (2, 2, 1, 768, 700),       # ragged key tail; causal rows that see few keys
    (1, 3, 3, 1024, 1000),
    (1, 1, 1, 256, 4160),      # long rows of keys: 65 tiles, the copy ring wraps many times
    (1, 2, 2, 300, 500),       # rows past the end of the last row tile: one wavefront's block, then whole wavefronts
    (2, 3, 1, 513, 1100),      # one row in the last row tile
    (1, 2, 2, 40, 2048),       # less than one wavefront of rows
]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_wide_kernel_against_the_oracle(shape, causal, dtype):
    B, Hq, Hkv, Lq, Lk = shape
    w = synthetic.small("wide", B, Hq, Hkv, Lq, Lk, 128, dtype, causal, seed=9300 + Lq + Lk)
    q, k, v, _ = synthetic.make_qkv(w)
    got = run_flashd(q, k, v, causal, w.scale, WIDE, 1)
    sampled(got, q, k, v, w, 768, 31, f"{shape} causal={causal} {dtype}")
    if causal and Lq > Lk:
        assert torch.count_nonzero(got[:, :, :Lq - Lk]) == 0, "rows without keys must be zeros"


@pytest.mark.parametrize("dtype,qk_std", [("bf16", 6.0), ("f16", 3.0), ("f16", 6.0)])
@pytest.mark.parametrize("causal", [False, True])
def test_wide_kernel_with_large_and_growing_scores(dtype, qk_std, causal):
    """Large scores: references move often (f16 above all: a coefficient may be at most 2^13),
    so blocks go back and forth between the fused and the plain steps."""
    w = synthetic.small("wide big", 1, 2, 2, 512, 2048, 128, dtype, causal, seed=9400,
                        qk_std=qk_std, plant_frac=0.05)
    q, k, v, _ = synthetic.make_qkv(w)
    got = run_flashd(q, k, v, causal, w.scale, WIDE, 1)
    sampled(got, q, k, v, w, 512, 32, f"{dtype} std={qk_std} causal={causal}")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_wide_kernel_staircase_of_scores(dtype):
    """Keys whose scores rise step by step along the key axis: every few blocks some row's
    reference has to move, in the middle of a run of fused steps."""
    torch.manual_seed(5)
    Lq, Lk, d = 256, 2048, 128
    q = torch.zeros(1, 1, Lq, d)
    q[..., 0] = 1.0
    q[..., 1:] = 0.05 * torch.randn(Lq, d - 1)
    k = 0.05 * torch.randn(1, 1, Lk, d)
    k[0, 0, :, 0] = torch.arange(Lk) // 96 * 9.0          # steps of 9 nats every 96 keys
    v = torch.randn(1, 1, Lk, d)
    q, k, v = (t.to(DT[dtype]) for t in (q, k, v))
    got = run_flashd(q, k, v, False, 1.0, WIDE, 1)
    ref = oa.attn(q, k, v, False, 1.0)
    check(got, ref, DT[dtype], f"staircase {dtype}")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("level", [-40.0, -4.0, 30.0])
def test_wide_kernel_first_block_far_from_zero(dtype, causal, level):
    """The first block of a row tile takes a fused step with zero standing in for the rows'
    reference; scores that all lie far below zero (the coefficients would vanish), a little
    below (the sum falls short of the least that is trusted) or far above (they would overflow)
    must send it through the plain steps instead, and rows that see only a key or two must
    come out right either way."""
    torch.manual_seed(17)
    Lq, Lk, d = 512, 768, 128
    q = torch.zeros(1, 2, Lq, d)
    q[..., 0] = 1.0
    q[..., 1:] = 0.1 * torch.randn(2, Lq, d - 1)
    k = 0.1 * torch.randn(1, 2, Lk, d)
    k[..., 0] = level + 0.5 * torch.randn(2, Lk)
    v = torch.randn(1, 2, Lk, d)
    q, k, v = (t.to(DT[dtype]) for t in (q, k, v))
    got = run_flashd(q, k, v, causal, 1.0, WIDE, 1)
    ref = oa.attn(q, k, v, causal, 1.0)
    check(got, ref, DT[dtype], f"first block at {level} {dtype} causal={causal}")


@pytest.mark.parametrize("scale", [-0.09, 0.0])
def test_wide_kernel_negative_and_zero_scale(scale):
    w = synthetic.small("wide scale", 1, 2, 2, 256, 600, 128, "bf16", True, seed=9500)
    q, k, v, _ = synthetic.make_qkv(w)
    got = run_flashd(q, k, v, True, scale, WIDE, 1)
    sampled(got, q, k, v, w, 256, 33, f"scale={scale}", scale=scale)


@pytest.mark.parametrize("shape,dtype,d,splits", [
    ((1, 2, 2, 256, 512), "bf16", 64, 1),      # d = 64
    ((1, 2, 2, 256, 4096), "f16", 128, 2),     # split keys
])
def test_calls_the_wide_kernel_cannot_serve_run_as_tile(shape, dtype, d, splits):
    B, Hq, Hkv, Lq, Lk = shape
    w = synthetic.small("wide fallback", B, Hq, Hkv, Lq, Lk, d, dtype, True, seed=9600 + Lq)
    q, k, v, _ = synthetic.make_qkv(w)
    a = run_flashd(q, k, v, True, w.scale, WIDE, splits)
    b = run_flashd(q, k, v, True, w.scale, flashd.VARIANT_TILE, splits)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_wide_kernel_is_bitwise_reproducible_and_agrees_with_tile():
    w = synthetic.small("wide repro", 2, 4, 4, 512, 1536, 128, "bf16", True, seed=9700)
    q, k, v, _ = synthetic.make_qkv(w)
    a = run_flashd(q, k, v, True, w.scale, WIDE, 1)
    b = run_flashd(q, k, v, True, w.scale, WIDE, 1)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    t = run_flashd(q, k, v, True, w.scale, flashd.VARIANT_TILE, 1)
    # two roundings of the same row to bf16: a unit in the last place of the larger one apart
    assert (a.float() - t.float()).abs().max() <= 2.0 ** -7 * max(1.0, float(t.float().abs().max()))


def test_the_automatic_choice_takes_the_wide_kernel_where_it_says_so():
    """A shape flashd_auto_variant reports as TILE_256 (a workgroup per compute unit, 2048 keys,
    no mask): flashd_attn_fwd must return the 256-row kernel's bits, and they must agree with
    the oracle; short causal rows stay with the 128-row kernel."""
    w = synthetic.small("wide auto", 1, 64, 8, 1024, 2048, 128, "bf16", False, seed=9800)
    assert flashd.auto_variant(w.B, w.Hq, w.Hkv, w.Lq, w.Lk, w.d, flashd.BF16, False) == WIDE
    q, k, v, _ = synthetic.make_qkv(w)
    auto = run_flashd(q, k, v, False, w.scale, use_ex=False)
    wide = run_flashd(q, k, v, False, w.scale, WIDE, 1)
    assert torch.equal(auto.view(torch.int16), wide.view(torch.int16))
    sampled(auto, q, k, v, w, 1024, 37, "automatic choice, 256-row kernel")
    # under a causal mask: short queries late in a longer context (rows see 1792 keys on average)
    w = synthetic.small("wide auto causal", 8, 32, 8, 512, 2048, 128, "f16", True, seed=9802)
    assert flashd.auto_variant(w.B, w.Hq, w.Hkv, w.Lq, w.Lk, w.d, flashd.F16, True) == WIDE
    q, k, v, _ = synthetic.make_qkv(w)
    auto = run_flashd(q, k, v, True, w.scale, use_ex=False)
    wide = run_flashd(q, k, v, True, w.scale, WIDE, 1)
    assert torch.equal(auto.view(torch.int16), wide.view(torch.int16))
    sampled(auto, q, k, v, w, 1024, 38, "automatic choice under a causal mask, 256-row kernel")
    w = synthetic.small("wide auto no", 1, 8, 8, 1024, 1024, 128, "bf16", True, seed=9801)
    assert flashd.auto_variant(w.B, w.Hq, w.Hkv, w.Lq, w.Lk, w.d, flashd.BF16, True) == flashd.VARIANT_TILE
    q, k, v, _ = synthetic.make_qkv(w)
    auto = run_flashd(q, k, v, True, w.scale, use_ex=False)
    tile = run_flashd(q, k, v, True, w.scale, flashd.VARIANT_TILE, 0)
    assert torch.equal(auto.view(torch.int16), tile.view(torch.int16))
