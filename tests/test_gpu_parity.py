"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on the
same seeded inputs -- small shapes that span several tiles with ragged tails, every
variant and split count, and the edge cases of the method."""
import math

import numpy as np
import pytest
import torch

from oracle import attention as oa
from paper_2505_14201_amd import flashd, synthetic
from tests.gpu_util import check, run_flashd

pytestmark = pytest.mark.gpu

TILE, PER_KEY, ONLINE, BLEND = 1, 2, 3, 4
DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def oracle(q, k, v, causal, scale, rows=None):
    return oa.attn(q, k, v, causal, scale, "definition", rows)


# (B, Hq, Hkv, Lq, Lk): several 128-row and 64-key tiles, ragged tails, Lq != Lk, GQA
SHAPES = [
    (1, 1, 1, 1, 1),
    (1, 2, 1, 1, 300),
    (2, 4, 2, 5, 70),
    (1, 2, 2, 128, 128),
    (1, 4, 1, 200, 333),
    (1, 2, 2, 333, 200),      # causal: the first 133 rows see no key
    (1, 1, 1, 257, 515),
    (2, 8, 2, 64, 64),
]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("variant", [TILE, PER_KEY, ONLINE, BLEND])
def test_small_shapes_half(shape, causal, d, dtype, variant):
    B, Hq, Hkv, Lq, Lk = shape
    w = synthetic.small("t", B, Hq, Hkv, Lq, Lk, d, dtype, causal, seed=1000 + Lq * 7 + Lk + d)
    q, k, v, _ = synthetic.make_qkv(w)
    ref = oracle(q, k, v, causal, w.scale)
    got = run_flashd(q, k, v, causal, w.scale, variant, 1)
    check(got, ref, DT[dtype], f"{shape} causal={causal} d={d} {dtype} variant={variant}")


@pytest.mark.parametrize("shape,causal,variant,splits", [
    ((1, 8, 1, 1, 300001), False, TILE, 0),        # decode kernel, automatic splits, ragged tail
    ((1, 8, 1, 1, 300001), False, TILE, 64),       # the most splits the boundary takes
    ((1, 2, 1, 130, 200003), True, TILE, 0),       # tile kernel, Lk >> Lq, bottom-right mask
    ((1, 2, 1, 130, 200003), False, ONLINE, 7),
    ((1, 1, 1, 3, 100000), True, PER_KEY, 0),
])
def test_very_long_key_ranges(shape, causal, variant, splits):
    """Hundreds of thousands of keys per row (thousands of key tiles, ragged last tile): the
    carried state has to stay accurate over the whole run."""
    B, Hq, Hkv, Lq, Lk = shape
    w = synthetic.small("t", B, Hq, Hkv, Lq, Lk, 64, "bf16", causal, seed=4242 + Lk)
    q, k, v, _ = synthetic.make_qkv(w)
    ref = oracle(q, k, v, causal, w.scale)
    got = run_flashd(q, k, v, causal, w.scale, variant, splits)
    check(got, ref, torch.bfloat16, f"{shape} causal={causal} variant={variant} splits={splits}")


@pytest.mark.parametrize("scale", [-0.11, 0.0])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("variant,dtype", [(TILE, "bf16"), (ONLINE, "f16"), (PER_KEY, "f32"),
                                           (TILE, "f16")])
def test_negative_and_zero_scale(scale, causal, variant, dtype):
    """The boundary takes any scale: a negative one turns the ranking of the keys round, zero
    makes every visible key weigh the same; masks and ragged tiles must not care."""
    w = synthetic.small("t", 1, 4, 2, 200, 333, 128, dtype, causal, seed=77)
    q, k, v, _ = synthetic.make_qkv(w)
    ref = oracle(q, k, v, causal, scale)
    for splits in (1, 3):
        got = run_flashd(q, k, v, causal, scale, variant, splits)
        check(got, ref, DT[dtype], f"scale={scale} causal={causal} {dtype} variant={variant} "
                                   f"splits={splits}")
    # decode shape (the split-K decode kernel)
    wd = synthetic.small("t", 2, 8, 2, 1, 300, 128, dtype, False, seed=78)
    q, k, v, _ = synthetic.make_qkv(wd)
    got = run_flashd(q, k, v, False, scale, variant, 2)
    check(got, oracle(q, k, v, False, scale), DT[dtype], f"decode scale={scale} {dtype}")


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128])
def test_small_shapes_f32(shape, causal, d):
    B, Hq, Hkv, Lq, Lk = shape
    w = synthetic.small("t", B, Hq, Hkv, Lq, Lk, d, "f32", causal, seed=2000 + Lq * 7 + Lk + d)
    q, k, v, _ = synthetic.make_qkv(w)
    ref = oracle(q, k, v, causal, w.scale)
    got = run_flashd(q, k, v, causal, w.scale, PER_KEY, 1)
    check(got, ref, torch.float32, f"{shape} causal={causal} d={d} f32")
    got = run_flashd(q, k, v, causal, w.scale, use_ex=False)
    check(got, ref, torch.float32, f"{shape} causal={causal} d={d} f32 auto")


@pytest.mark.parametrize("variant", [TILE, PER_KEY, ONLINE, BLEND])
@pytest.mark.parametrize("splits", [2, 3, 7, 0])
@pytest.mark.parametrize("causal", [False, True])
def test_split_k_partials_merge_to_the_same_result(variant, splits, causal):
    for (B, Hq, Hkv, Lq, Lk, d, dtype) in [(2, 4, 2, 1, 1000, 128, "bf16"),
                                           (1, 2, 2, 150, 700, 64, "f16"),
                                           (1, 8, 1, 3, 64, 128, "bf16")]:
        w = synthetic.small("t", B, Hq, Hkv, Lq, Lk, d, dtype, causal, seed=3000 + Lk + splits)
        q, k, v, _ = synthetic.make_qkv(w)
        ref = oracle(q, k, v, causal, w.scale)
        got = run_flashd(q, k, v, causal, w.scale, variant, splits)
        check(got, ref, DT[dtype], f"splits={splits} variant={variant} Lq={Lq} Lk={Lk}")


@pytest.mark.parametrize("variant", [TILE, ONLINE, BLEND])
@pytest.mark.parametrize("splits", [1, 2, 5, 0])
def test_decode_shapes(variant, splits):
    """(Hq / Hkv) * Lq <= 32 query rows per kv head take the split-K decode kernel."""
    for (B, Hq, Hkv, Lq, Lk, d, dtype, causal) in [
            (3, 32, 8, 1, 3000, 128, "bf16", False),     # the GQA decode shape, shortened
            (1, 8, 1, 4, 500, 128, "bf16", True),        # exactly 32 rows, causal positions
            (2, 4, 4, 7, 333, 64, "f16", True),          # no GQA, several positions
            (1, 16, 2, 2, 31, 64, "bf16", False),        # less than one 32-key block
            (1, 2, 2, 9, 5, 128, "f16", True)]:          # Lq > Lk: rows without any key
        w = synthetic.small("t", B, Hq, Hkv, Lq, Lk, d, dtype, causal, seed=3300 + Lk + splits)
        q, k, v, _ = synthetic.make_qkv(w)
        ref = oracle(q, k, v, causal, w.scale)
        if splits > Lk:
            continue
        got = run_flashd(q, k, v, causal, w.scale, variant, splits)
        check(got, ref, DT[dtype], f"decode splits={splits} variant={variant} Lq={Lq} Lk={Lk}")


def test_split_k_f32_and_more_splits_than_tiles():
    w = synthetic.small("t", 1, 2, 1, 4, 130, 64, "f32", False, seed=3100)
    q, k, v, _ = synthetic.make_qkv(w)
    ref = oracle(q, k, v, False, w.scale)
    for splits in (2, 64):
        check(run_flashd(q, k, v, False, w.scale, PER_KEY, splits), ref, torch.float32)
    wb = synthetic.small("t", 1, 2, 1, 4, 130, 64, "bf16", True, seed=3101)
    q, k, v, _ = synthetic.make_qkv(wb)
    ref = oracle(q, k, v, True, wb.scale)
    for variant in (TILE, ONLINE, PER_KEY, BLEND):
        check(run_flashd(q, k, v, True, wb.scale, variant, 64), ref, torch.bfloat16)


def test_auto_entry_point_uses_cached_workspace_repeatedly():
    """flashd_attn_fwd with split-K shapes of growing then shrinking size on one stream."""
    for Lk in (600, 5000, 900):
        w = synthetic.small("t", 2, 8, 2, 1, Lk, 128, "bf16", False, seed=3200 + Lk)
        q, k, v, _ = synthetic.make_qkv(w)
        ref = oracle(q, k, v, False, w.scale)
        check(run_flashd(q, k, v, False, w.scale, use_ex=False), ref, torch.bfloat16, f"Lk={Lk}")


# ------------------------------------------------------------ method invariants ---

@pytest.mark.parametrize("variant,dtype", [(TILE, "bf16"), (TILE, "f16"), (PER_KEY, "f32"),
                                           (PER_KEY, "bf16"), (ONLINE, "bf16"), (BLEND, "bf16"),
                                           (BLEND, "f16")])
def test_single_key_returns_its_value_bitwise(variant, dtype):
    w = synthetic.small("t", 1, 2, 2, 70, 1, 64, dtype, False, seed=4000)
    q, k, v, _ = synthetic.make_qkv(w)
    got = run_flashd(q, k, v, False, w.scale, variant, 1)
    want = v[:, :, 0:1, :].expand(-1, -1, 70, -1)
    assert torch.equal(got, want)


@pytest.mark.parametrize("variant,dtype", [(TILE, "bf16"), (PER_KEY, "f32"), (ONLINE, "f16"),
                                           (BLEND, "bf16"), (BLEND, "f16")])
def test_uniform_scores_give_the_mean_of_values(variant, dtype):
    w = synthetic.small("t", 1, 2, 1, 40, 333, 128, dtype, False, seed=4001)
    q, k, v, _ = synthetic.make_qkv(w)
    q = torch.zeros_like(q)
    got = run_flashd(q, k, v, False, w.scale, variant, 1)
    mean = v.double().mean(dim=2, keepdim=True).expand(-1, 2, 40, -1).numpy()
    check(got, mean, DT[dtype])
    check(got, oracle(q, k, v, False, w.scale), DT[dtype])


@pytest.mark.parametrize("variant,dtype", [(TILE, "bf16"), (PER_KEY, "f32"), (PER_KEY, "f16"),
                                           (BLEND, "f16")])
def test_key_permutation_invariance(variant, dtype):
    w = synthetic.small("t", 1, 2, 2, 130, 300, 64, dtype, False, seed=4002)
    q, k, v, _ = synthetic.make_qkv(w)
    perm = torch.from_numpy(np.random.default_rng(1).permutation(300))
    a = run_flashd(q, k, v, False, w.scale, variant, 1)
    b = run_flashd(q, k[:, :, perm].contiguous(), v[:, :, perm].contiguous(), False, w.scale,
                   variant, 1)
    ref = oracle(q, k, v, False, w.scale)
    check(a, ref, DT[dtype])
    check(b, ref, DT[dtype])


@pytest.mark.parametrize("variant,dtype,d", [(TILE, "f16", 64), (TILE, "bf16", 128),
                                             (PER_KEY, "f32", 64), (PER_KEY, "f16", 64),
                                             (ONLINE, "f16", 64), (BLEND, "f16", 64),
                                             (BLEND, "bf16", 128)])
@pytest.mark.parametrize("splits", [1, 3])
def test_huge_scores_and_dominant_keys_stay_finite_and_right(variant, dtype, d, splits):
    """Scaled scores of +-hundreds with planted dominant keys (jumps of ~ +-1000 between
    consecutive scores): no max subtraction on the FLASH-D paths, yet no overflow."""
    w = synthetic.small("t", 1, 2, 2, 300, 300, d, dtype, True, seed=4003, qk_std=4.0,
                        plant_frac=0.1)
    q, k, v, planted = synthetic.make_qkv(w)
    assert len(planted) > 20
    ref = oracle(q, k, v, True, w.scale)
    got = run_flashd(q, k, v, True, w.scale, variant, splits)
    check(got, ref, DT[dtype], f"stress variant={variant} {dtype}")


@pytest.mark.parametrize("dtype,step_nats", [("f16", 12.0), ("f16", 30.0), ("bf16", 45.0),
                                             ("bf16", 60.0), ("bf16", 90.0), ("f16", 90.0)])
@pytest.mark.parametrize("Lq", [1, 160])
def test_staircase_scores(dtype, step_nats, Lq):
    """Scores that climb in steps every 96 keys: each step lifts the scores by step_nats above
    everything before it -- past what the rounded coefficients can hold (2^14 for f16, 2^60 for
    bf16, in powers of two; a nat is 1.44 of them) but, for the smaller steps, not past fp32,
    which is the case the reference shift serves; the largest steps overflow fp32 as well.
    The keys of a level share the weight, so the result is the mean of that level's values
    (plus a little of the level below), not a single key."""
    Lk, d = 96 * 6 + 40, 64
    rng = np.random.default_rng(int(step_nats) + Lq)
    level = (np.arange(Lk) // 96).astype(np.float64)
    q = torch.zeros(1, 2, Lq, d)
    q[..., 0] = 1.0
    q[..., 1:] = torch.from_numpy(0.05 * rng.standard_normal((1, 2, Lq, d - 1))).float()
    k = torch.from_numpy(0.5 * rng.standard_normal((1, 1, Lk, d))).float()
    k[0, 0, :, 0] = torch.from_numpy(step_nats * level).float()
    v = torch.from_numpy(rng.standard_normal((1, 1, Lk, d))).float()
    qq, kk, vv = (t.to(DT[dtype]) for t in (q, k, v))
    for causal in (False, True):
        ref = oracle(qq, kk, vv, causal, 1.0)
        for variant, splits in ((TILE, 1), (TILE, 2), (PER_KEY, 1), (BLEND, 1), (BLEND, 2)):
            got = run_flashd(qq, kk, vv, causal, 1.0, variant, splits)
            check(got, ref, DT[dtype], f"staircase {dtype} step={step_nats} Lq={Lq} "
                                       f"causal={causal} variant={variant} splits={splits}")


def test_score_ramps():
    """s_j = +-c*j: an ascending ramp keeps only the last key, a descending one the first."""
    L, d = 200, 64
    for sign in (+1.0, -1.0):
        q = torch.zeros(1, 1, 1, d)
        q[..., 0] = 1.0
        k = torch.zeros(1, 1, L, d)
        k[0, 0, :, 0] = sign * 40.0 * torch.arange(L)
        v = torch.from_numpy(np.random.default_rng(2).standard_normal((1, 1, L, d))).float()
        for dtype, variant in ((torch.float32, PER_KEY), (torch.bfloat16, TILE),
                               (torch.bfloat16, PER_KEY)):
            qq, kk, vv = q.to(dtype), k.to(dtype), v.to(dtype)
            got = run_flashd(qq, kk, vv, False, 1.0, variant, 1)
            want = vv[0, 0, -1 if sign > 0 else 0]
            if dtype == torch.float32:      # o + (v - o) * 1 may differ from v by an ulp
                assert torch.allclose(got[0, 0, 0], want, rtol=3e-7, atol=1e-7)
            else:
                assert torch.equal(got[0, 0, 0], want)


# ----------------------------------------------------------------- mask and heads ---

@pytest.mark.parametrize("variant,dtype", [(TILE, "bf16"), (PER_KEY, "f32"), (PER_KEY, "bf16"),
                                           (ONLINE, "bf16")])
def test_causal_mask_is_bit_exact_under_junk_in_masked_positions(variant, dtype):
    Lq, Lk, d = 200, 230, 64            # off = 30
    w = synthetic.small("t", 1, 2, 1, Lq, Lk, d, dtype, True, seed=4004)
    q, k, v, _ = synthetic.make_qkv(w)
    base = run_flashd(q, k, v, True, w.scale, variant, 1)
    for jstar in (31, 64, 100, 191, 229):
        k2, v2 = k.clone(), v.clone()
        k2[:, :, jstar:, :] = 3.0e4 if dtype != "f16" else 6.0e4
        v2[:, :, jstar:, :] = -2.5e4
        junk = run_flashd(q, k2, v2, True, w.scale, variant, 1)
        first_seeing = jstar - (Lk - Lq)            # row i sees key j iff j <= i + 30
        assert torch.equal(junk[:, :, :first_seeing], base[:, :, :first_seeing])
        assert not torch.equal(junk[:, :, first_seeing:], base[:, :, first_seeing:])


@pytest.mark.parametrize("variant,dtype", [(TILE, "bf16"), (PER_KEY, "f32"), (ONLINE, "f16")])
@pytest.mark.parametrize("Lq,Lk", [(64, 64), (40, 64), (64, 40)])
def test_identity_values_expose_the_weight_row(variant, dtype, Lq, Lk):
    d = 64
    w = synthetic.small("t", 1, 1, 1, Lq, Lk, d, dtype, True, seed=4005)
    q, k, v, _ = synthetic.make_qkv(w)
    v = torch.zeros_like(v)
    v[0, 0, :, :Lk] = torch.eye(Lk, dtype=v.dtype)
    got = run_flashd(q, k, v, True, w.scale, variant, 1)[0, 0].double().numpy()
    ref = oracle(q, k, v, True, w.scale)[0, 0]
    for i in range(Lq):
        for j in range(Lk):
            if j > i + (Lk - Lq):
                assert got[i, j] == 0.0 and ref[i, j] == 0.0
    assert np.array_equal(got != 0, ref != 0) or dtype == "f16"     # tiny weights may flush
    check(torch.from_numpy(got), ref, DT[dtype])


@pytest.mark.parametrize("variant,dtype", [(TILE, "bf16"), (PER_KEY, "f32"), (ONLINE, "bf16")])
def test_gqa_head_mapping(variant, dtype):
    w = synthetic.small("t", 2, 8, 2, 33, 90, 128, dtype, False, seed=4006)
    q, k, v, _ = synthetic.make_qkv(w)
    v[:, 1] = 3.25
    got = run_flashd(q, k, v, False, w.scale, variant, 1).float()
    assert torch.all((got[:, 4:] - 3.25).abs() <= (0.0 if dtype == "f32" else 0.02))
    assert not torch.any((got[:, :4] - 3.25).abs() < 1e-2)
    if dtype == "f32":
        assert torch.all((got[:, 4:] - 3.25).abs() < 1e-5)


def test_output_is_bitwise_reproducible():
    w = synthetic.small("t", 2, 4, 2, 300, 500, 128, "bf16", True, seed=4007)
    q, k, v, _ = synthetic.make_qkv(w)
    for variant, splits in ((TILE, 1), (TILE, 3), (PER_KEY, 2), (ONLINE, 1)):
        a = run_flashd(q, k, v, True, w.scale, variant, splits)
        b = run_flashd(q, k, v, True, w.scale, variant, splits)
        assert torch.equal(a, b)


def test_first_config_in_full():
    w = synthetic.CONFIGS[0]
    q, k, v, _ = synthetic.make_qkv(w)
    ref = oracle(q, k, v, w.causal, w.scale)
    got = run_flashd(q, k, v, w.causal, w.scale, use_ex=False)
    err = check(got, ref, torch.float32, "config 1")
    assert err <= 1e-5 * max(1.0, float(np.abs(ref).max()))
    assert math.isfinite(err)


# Shapes with more row tiles than the GPU has workgroup slots: the tile kernel then walks
# several row tiles per workgroup (under a causal mask a long and a short one as a pair,
# with a lone middle tile when their number is odd) and orders them per XCD.  Checked on all
# rows of a few heads plus sampled rows everywhere.
#   (B, Hq, Hkv, Lq, Lk, d, dtype, causal)
SCHEDULE_SHAPES = [
    (2, 64, 64, 1152, 1152, 128, "bf16", True),     # 9 row tiles: pairs + middle tile
    (2, 64, 16, 1100, 1300, 128, "f16", True),      # ragged, Lq != Lk, GQA
    (1, 40, 40, 2048, 2048, 128, "bf16", False),    # no mask, units a multiple of 8
    (1, 36, 12, 2000, 1000, 128, "bf16", False),    # units not a multiple of 8, ragged
    (2, 64, 64, 2048, 2048, 64, "f16", True),       # d = 64: more resident workgroups
    (1, 96, 96, 1280, 1280, 64, "bf16", False),
]


@pytest.mark.parametrize("shape", SCHEDULE_SHAPES)
@pytest.mark.parametrize("variant", [TILE, ONLINE])
def test_many_row_tiles_per_workgroup(shape, variant):
    B, Hq, Hkv, Lq, Lk, d, dtype, causal = shape
    w = synthetic.small("sched", B, Hq, Hkv, Lq, Lk, d, dtype, causal, seed=7000 + Lq + Hq)
    q, k, v, _ = synthetic.make_qkv(w)
    got = run_flashd(q, k, v, causal, w.scale, variant, 1)
    heads = [(0, 0), (B - 1, Hq - 1), (B // 2, Hq // 2 + 1)]
    must = [(b, h, i) for (b, h) in heads for i in range(Lq)]
    rows = synthetic.sample_rows(w, len(must) + 4096, seed=7001, must=must)
    ref = oracle(q, k, v, causal, w.scale, rows)
    idx = torch.from_numpy(rows.astype(np.int64))
    sel = got[idx[:, 0], idx[:, 1], idx[:, 2], :]
    check(sel, ref, DT[dtype], f"{shape} variant={variant}")


# Grouped-query attention with few positions per head: the tile kernel runs the g query
# heads of a kv head as one head of g * Lq rows (the causal rule then goes by the row index
# modulo Lq).  Head boundaries inside a wavefront's 32 rows, inside a row tile and across
# row tiles; more positions than keys (rows without keys in every head); key splits.
#   (B, Hq, Hkv, Lq, Lk)
PACKED_SHAPES = [
    (2, 8, 2, 16, 500),       # 4 x 16 rows: half a row tile
    (1, 8, 1, 40, 300),       # 320 rows in 3 row tiles instead of 8
    (1, 6, 2, 130, 200),      # 390 rows, boundaries at 130 and 260
    (2, 4, 2, 100, 260),
    (1, 16, 2, 9, 1000),      # 72 rows: boundaries every 9 rows
    (1, 8, 2, 50, 30),        # causal: the first 20 positions of every head see no key
    (1, 12, 4, 33, 33),
]


@pytest.mark.parametrize("shape", PACKED_SHAPES)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("variant,dtype,d", [(TILE, "bf16", 128), (TILE, "f16", 64),
                                             (ONLINE, "bf16", 64)])
@pytest.mark.parametrize("splits", [1, 3])
def test_query_heads_of_a_kv_group_run_as_one_head(shape, causal, variant, dtype, d, splits):
    B, Hq, Hkv, Lq, Lk = shape
    w = synthetic.small("pack", B, Hq, Hkv, Lq, Lk, d, dtype, causal, seed=8800 + Lq + Lk)
    q, k, v, _ = synthetic.make_qkv(w)
    ref = oracle(q, k, v, causal, w.scale)
    got = run_flashd(q, k, v, causal, w.scale, variant, splits)
    check(got, ref, DT[dtype], f"{shape} causal={causal} {dtype} d={d} v={variant} s={splits}")
    if causal and Lq > Lk:
        assert torch.count_nonzero(got[:, :, :Lq - Lk]) == 0, "rows without keys must be zeros"


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f16", 64)])
def test_short_queries_take_many_splits_through_the_automatic_entry_point(dtype, d):
    """8 heads x 8 positions per kv head are too many rows for the decode kernel; the tile
    kernel runs them as one head, and with so few rows in all the automatic choice cuts the
    keys into many splits."""
    B, Hq, Hkv, Lq, Lk = 2, 8, 1, 8, 3000
    from paper_2505_14201_amd import flashd
    assert flashd.auto_splits(B, Hq, Hkv, Lq, Lk, d, flashd._DTYPE[DT[dtype]]) >= 8
    w = synthetic.small("short queries", B, Hq, Hkv, Lq, Lk, d, dtype, True, seed=8900 + d)
    q, k, v, _ = synthetic.make_qkv(w)
    ref = oracle(q, k, v, True, w.scale)
    got = run_flashd(q, k, v, True, w.scale, use_ex=False)
    check(got, ref, DT[dtype], f"short queries {dtype} d={d}")


@pytest.mark.parametrize("shape,variant,dtype", [
    ((2, 8, 2, 1, 5000), TILE, "bf16"),        # decode kernel, 64 partials per row
    ((1, 4, 4, 150, 4500), TILE, "f16"),       # tile kernel
    ((1, 8, 2, 12, 4100), ONLINE, "bf16"),     # heads of a kv group as one head
    ((1, 2, 1, 9, 4200), PER_KEY, "f32"),
    ((1, 2, 2, 3, 64), PER_KEY, "bf16"),       # one key per split
])
@pytest.mark.parametrize("causal", [False, True])
def test_maximum_number_of_splits(shape, variant, dtype, causal):
    """64 splits (FLASHD_MAX_SPLITS): every lane of the merging wavefront holds a partial;
    under a causal mask many of them are empty."""
    B, Hq, Hkv, Lq, Lk = shape
    w = synthetic.small("max splits", B, Hq, Hkv, Lq, Lk, 128, dtype, causal, seed=9100 + Lk)
    q, k, v, _ = synthetic.make_qkv(w)
    ref = oracle(q, k, v, causal, w.scale)
    got = run_flashd(q, k, v, causal, w.scale, variant, 64)
    check(got, ref, DT[dtype], f"{shape} {dtype} variant={variant} causal={causal}")


def test_cached_workspace_can_be_released_and_grows_again():
    """flashd_release_workspace frees the per-stream scratch (live and outgrown buffers); the
    next call that needs scratch allocates afresh and gives the same result."""
    w = synthetic.small("t", 2, 8, 2, 1, 3000, 128, "bf16", False, seed=3210)
    q, k, v, _ = synthetic.make_qkv(w)
    ref = oracle(q, k, v, False, w.scale)
    side = torch.cuda.Stream()
    for round_ in range(2):
        for Lk in (700, 3000):                   # grows once: one buffer retired
            a = run_flashd(q, k[:, :, :Lk].contiguous(), v[:, :, :Lk].contiguous(), False, w.scale,
                           use_ex=False)
        check(a, ref, torch.bfloat16, f"round {round_}")
        with torch.cuda.stream(side):
            qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
            og = torch.empty_like(qg)
            flashd.attn_fwd(qg, kg, vg, og, False, w.scale)
        torch.cuda.synchronize()
        check(og.cpu(), ref, torch.bfloat16, f"side stream, round {round_}")
        flashd.release_workspace()
    flashd.release_workspace()                   # nothing left: still fine
