"""Pins for the CPU oracle (no GPU).  Each test ties a part of the oracle to
something that is not the oracle: a hand-worked fixture, an exact closed form,
a library routine, a high-precision brute force, or an invariant the
mathematics fixes."""
import decimal
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

from oracle import attention as oa
from oracle import recurrence as rec

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ALGOS = ("definition", "alg1", "alg2", "alg3")


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, vals = line.split(":")
            out[key.strip()] = [float(Fraction(t)) for t in vals.split()]
    return out


def tensors_from_scores(s, V):
    """One query whose scaled scores against N keys are exactly fl32(s_j):
    d_qk = 1 would not carry V, so use d = max(dv, 1) with q = e_0, k_j = s_j e_0."""
    s = np.asarray(s, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    n, d = V.shape
    q = torch.zeros(1, 1, 1, d, dtype=torch.float32)
    q[0, 0, 0, 0] = 1.0
    k = torch.zeros(1, 1, n, d, dtype=torch.float32)
    k[0, 0, :, 0] = torch.from_numpy(s.astype(np.float32))
    v = torch.from_numpy(V.astype(np.float32)).reshape(1, 1, n, d)
    return q, k, v


# ---------------------------------------------------------------- fixtures ---

def test_golden_two_keys_recurrence():
    g = read_golden("worked_example_two_keys.txt")
    s = np.log(np.array(g["exp_s"]))
    V = np.array([g["v1"], g["v2"]])
    o, w = rec.flashd_row(s, V)
    np.testing.assert_allclose(w, g["w"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(o[0], g["o1"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(o[1], g["o2"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(rec.flashd_row_two_products(s, V)[1], g["o2"], atol=1e-15)


def test_golden_four_keys_recurrence():
    g = read_golden("incremental_softmax_four_keys.txt")
    s = np.log(np.array(g["exp_s"]))
    V = np.eye(4)
    o, w = rec.flashd_row(s, V)
    np.testing.assert_allclose(w, g["w"], rtol=0, atol=1e-15)
    for i in range(4):
        np.testing.assert_allclose(o[i], g[f"o{i + 1}"], rtol=0, atol=2e-16 * 4)
    o1, w1 = rec.fa1_row(s, V)
    np.testing.assert_allclose(w1, g["w"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(o1[3], g["o4"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(rec.fa2_row(s, V), g["o4"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(rec.weights_rational(s), g["w"], rtol=0, atol=1e-15)


@pytest.mark.parametrize("algo", ALGOS)
def test_golden_c_oracle(algo):
    # scores reach the C code as float32, so ln 2, ln 3 carry a 6e-8 relative rounding
    g = read_golden("incremental_softmax_four_keys.txt")
    q, k, v = tensors_from_scores(np.log(np.array(g["exp_s"])), np.eye(4))
    o = oa.attn(q, k, v, False, 1.0, algo)
    np.testing.assert_allclose(o[0, 0, 0], g["o4"], rtol=0, atol=2e-7)
    g2 = read_golden("worked_example_two_keys.txt")
    q, k, v = tensors_from_scores(np.log(np.array(g2["exp_s"])), np.array([g2["v1"], g2["v2"]]))
    o = oa.attn(q, k, v, False, 1.0, algo)
    np.testing.assert_allclose(o[0, 0, 0], g2["o2"], rtol=0, atol=2e-7)


def test_golden_rejects_minus_sign():
    """The algorithm box prints sigma(s_i - s_{i-1} - ln w_{i-1}); the fixtures must be
    able to tell that reading from the + of the boxed equation."""
    g = read_golden("incremental_softmax_four_keys.txt")
    s = np.log(np.array(g["exp_s"]))
    w = [1.0]
    for i in range(1, 4):
        w.append(rec.sigmoid(s[i] - s[i - 1] - math.log(w[-1])))
    assert abs(w[2] - g["w"][2]) > 0.1           # 0.692 instead of 0.5
    assert abs(rec.weights_sigmoid(s)[0][2] - g["w"][2]) < 1e-15


# ------------------------------------------------------------- brute force ---

def brute_force(q, k, v, causal, scale):
    """Definition of Sec. II-A in 60-digit decimal arithmetic, no max shift."""
    decimal.getcontext().prec = 60
    D = decimal.Decimal
    B, Hq, Lq, d = q.shape
    _, Hkv, Lk, _ = k.shape
    out = np.zeros((B, Hq, Lq, d))
    sc = D(float(np.float32(scale)))
    for b in range(B):
        for h in range(Hq):
            kh = h // (Hq // Hkv)
            for i in range(Lq):
                js = [j for j in range(Lk) if (not causal) or j <= i + (Lk - Lq)]
                if not js:
                    continue
                es = []
                for j in js:
                    dot = sum(D(float(q[b, h, i, t])) * D(float(k[b, kh, j, t])) for t in range(d))
                    es.append((sc * dot).exp())
                den = sum(es)
                for t in range(d):
                    out[b, h, i, t] = float(sum(e * D(float(v[b, kh, j, t]))
                                                for e, j in zip(es, js)) / den)
    return out


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("causal,Lq,Lk", [(False, 3, 5), (True, 4, 4), (True, 3, 6), (True, 5, 3)])
def test_brute_force_tiny(algo, causal, Lq, Lk):
    rng = np.random.default_rng(7 + Lq * 10 + Lk)
    q = torch.from_numpy(rng.standard_normal((2, 4, Lq, 3)).astype(np.float32)) * 2
    k = torch.from_numpy(rng.standard_normal((2, 2, Lk, 3)).astype(np.float32)) * 2
    v = torch.from_numpy(rng.standard_normal((2, 2, Lk, 3)).astype(np.float32))
    want = brute_force(q.numpy(), k.numpy(), v.numpy(), causal, 0.7)
    got = oa.attn(q, k, v, causal, 0.7, algo)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)
    if causal and Lq > Lk:   # rows that see no key at all are zero
        assert np.all(got[:, :, : Lq - Lk, :] == 0.0)


# ---------------------------------------------------------- library routines ---

@pytest.mark.parametrize("algo", ALGOS)
def test_against_scipy_softmax(algo):
    rng = np.random.default_rng(11)
    B, Hq, Hkv, Lq, Lk, d = 2, 4, 2, 37, 53, 16
    q = torch.from_numpy(rng.standard_normal((B, Hq, Lq, d)).astype(np.float32))
    k = torch.from_numpy(rng.standard_normal((B, Hkv, Lk, d)).astype(np.float32))
    v = torch.from_numpy(rng.standard_normal((B, Hkv, Lk, d)).astype(np.float32))
    scale = float(np.float32(1 / math.sqrt(d)))
    got = oa.attn(q, k, v, False, scale, algo)
    for b in range(B):
        for h in range(Hq):
            S = scale * (q[b, h].double().numpy() @ k[b, h // 2].double().numpy().T)
            want = scipy.special.softmax(S, axis=-1) @ v[b, h // 2].double().numpy()
            np.testing.assert_allclose(got[b, h], want, rtol=0, atol=1e-13)


@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("Lq,Lk", [(40, 40), (17, 40)])
def test_against_torch_sdpa_causal_gqa(algo, Lq, Lk):
    rng = np.random.default_rng(13)
    B, Hq, Hkv, d = 1, 6, 2, 8
    q = torch.from_numpy(rng.standard_normal((B, Hq, Lq, d)).astype(np.float32))
    k = torch.from_numpy(rng.standard_normal((B, Hkv, Lk, d)).astype(np.float32))
    v = torch.from_numpy(rng.standard_normal((B, Hkv, Lk, d)).astype(np.float32))
    scale = float(np.float32(0.3))
    i = torch.arange(Lq)[:, None]
    j = torch.arange(Lk)[None, :]
    mask = j <= i + (Lk - Lq)                      # bottom-right aligned
    g = Hq // Hkv
    want = torch.nn.functional.scaled_dot_product_attention(
        q.double(), k.double().repeat_interleave(g, dim=1), v.double().repeat_interleave(g, dim=1),
        attn_mask=mask, scale=scale).numpy()
    got = oa.attn(q, k, v, True, scale, algo)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


# ------------------------------------------------- closed forms & special cases ---

def test_weights_closed_form_every_step():
    """Sec. III-A: w_i = e^{s_i - m_i}/l_i = e^{s_i} / sum_{j<=i} e^{s_j}; 0 < w_i <= 1."""
    rng = np.random.default_rng(3)
    s = rng.standard_normal(200) * 3
    w, lnw = rec.weights_sigmoid(s)
    prefix_lse = np.logaddexp.accumulate(s)
    np.testing.assert_allclose(w, np.exp(s - prefix_lse), rtol=1e-13, atol=0)
    np.testing.assert_allclose(s - lnw, prefix_lse, rtol=0, atol=1e-12)
    assert np.all(w > 0) and np.all(w <= 1)
    np.testing.assert_allclose(rec.weights_rational(s), w, rtol=1e-12, atol=0)


def test_uniform_scores_give_running_mean():
    rng = np.random.default_rng(4)
    V = rng.standard_normal((9, 5))
    o, w = rec.flashd_row(np.full(9, 2.5), V)
    np.testing.assert_allclose(w, 1.0 / np.arange(1, 10), rtol=1e-15)
    for i in range(9):
        np.testing.assert_allclose(o[i], V[: i + 1].mean(axis=0), rtol=0, atol=1e-15)


@pytest.mark.parametrize("algo", ALGOS)
def test_zero_query_gives_mean_of_values(algo):
    rng = np.random.default_rng(5)
    k = torch.from_numpy(rng.standard_normal((1, 2, 33, 8)).astype(np.float32))
    v = torch.from_numpy(rng.standard_normal((1, 2, 33, 8)).astype(np.float32))
    q = torch.zeros(1, 4, 3, 8)
    got = oa.attn(q, k, v, False, 0.35, algo)
    for h in range(4):
        want = v[0, h // 2].double().numpy().mean(axis=0)
        for i in range(3):
            np.testing.assert_allclose(got[0, h, i], want, rtol=0, atol=1e-15)


@pytest.mark.parametrize("algo", ALGOS)
def test_single_key_returns_its_value_exactly(algo):
    rng = np.random.default_rng(6)
    q = torch.from_numpy(rng.standard_normal((1, 1, 4, 8)).astype(np.float32))
    k = torch.from_numpy(rng.standard_normal((1, 1, 1, 8)).astype(np.float32))
    v = torch.from_numpy(rng.standard_normal((1, 1, 1, 8)).astype(np.float32))
    got = oa.attn(q, k, v, False, 1.0, algo)
    for i in range(4):
        assert np.array_equal(got[0, 0, i], v[0, 0, 0].double().numpy())


def test_alg1_and_alg3_agree_at_every_step():
    """Sec. III-C: Alg. 3 is a one-to-one rewrite of Alg. 1, so every o_i matches."""
    rng = np.random.default_rng(8)
    s = rng.standard_normal(150) * 4
    V = rng.standard_normal((150, 6))
    o3, w3 = rec.flashd_row(s, V)
    o1, w1 = rec.fa1_row(s, V)
    np.testing.assert_allclose(o3, o1, rtol=0, atol=1e-13)
    np.testing.assert_allclose(w3, w1, rtol=1e-12, atol=0)
    np.testing.assert_allclose(rec.fa2_row(s, V), o3[-1], rtol=0, atol=1e-13)
    np.testing.assert_allclose(rec.flashd_row_two_products(s, V), o3, rtol=0, atol=1e-13)
    np.testing.assert_allclose(scipy.special.softmax(s) @ V, o3[-1], rtol=0, atol=1e-13)


def test_c_alg3_matches_python_alg3():
    rng = np.random.default_rng(9)
    s = (rng.standard_normal(64) * 5).astype(np.float32).astype(np.float64)
    V = rng.standard_normal((64, 4)).astype(np.float32).astype(np.float64)
    q, k, v = tensors_from_scores(s, V)
    got = oa.attn(q, k, v, False, 1.0, "alg3")[0, 0, 0]
    np.testing.assert_allclose(got, rec.flashd_row(s, V)[0][-1], rtol=0, atol=1e-14)


def test_weight_curves_of_fig2():
    """Fig. 2: with w_{i-1} = 0.99 the weight follows the plain sigmoid of s_i - s_{i-1};
    a smaller w_{i-1} moves the same curve to the right by -ln w_{i-1}."""
    for dlt in np.linspace(-12, 12, 49):
        w99 = rec.sigmoid(dlt + math.log(0.99))
        assert abs(w99 - rec.sigmoid(dlt)) < 0.0026
        for wprev in (0.5, 0.1, 0.01):
            shifted = rec.sigmoid((dlt - math.log(wprev)) + math.log(wprev))
            assert abs(shifted - rec.sigmoid(dlt)) < 1e-15
            assert rec.sigmoid(dlt + math.log(wprev)) < rec.sigmoid(dlt)


# ------------------------------------------------------------------ invariants ---

def test_only_s_minus_lnw_is_carried():
    rng = np.random.default_rng(10)
    s = rng.standard_normal(20)
    w, lnw = rec.weights_sigmoid(s)
    # restart the recurrence at step 10 from (s_9 + delta, ln w_9 + delta)
    for delta in (-3.0, 0.7, 40.0):
        sp, lp = s[9] + delta, lnw[9] + delta
        for i in range(10, 20):
            x = s[i] - sp + lp
            wi, lp, sp = rec.sigmoid(x), rec.log_sigmoid(x), s[i]
            assert abs(wi - w[i]) < 1e-13


def test_shift_invariance():
    rng = np.random.default_rng(12)
    s = rng.standard_normal(50) * 2
    w0, _ = rec.weights_sigmoid(s)
    w1, _ = rec.weights_sigmoid(s + 123.0)
    np.testing.assert_allclose(w1, w0, rtol=1e-11, atol=0)


def test_any_partition_into_groups_gives_the_same_state():
    rng = np.random.default_rng(14)
    n = 45
    s = rng.standard_normal(n) * 6
    V = rng.standard_normal((n, 7))
    want_o, want_l = rec.state_of_run(s, V)
    np.testing.assert_allclose(want_l, scipy.special.logsumexp(s), rtol=0, atol=1e-12)
    partitions = [[0, n], list(range(n + 1)), [0, 1, n], [0, n - 1, n], [0, 16, 32, n],
                  [0, 0, 5, 5, 5, 30, n, n]]
    for _ in range(5):
        cuts = sorted(rng.choice(np.arange(1, n), size=6, replace=False).tolist())
        partitions.append([0] + cuts + [n])
    for bounds in partitions:
        o, lam = rec.grouped_row(s, V, bounds)
        np.testing.assert_allclose(o, want_o, rtol=0, atol=1e-13)
        assert abs(lam - want_l) < 1e-12


def test_merge_is_associative_commutative_with_identity():
    rng = np.random.default_rng(15)
    runs = []
    for n in (3, 8, 1):
        runs.append(rec.state_of_run(rng.standard_normal(n) * 5, rng.standard_normal((n, 4))))
    a, b, c = runs
    left = rec.merge(rec.merge(a, b), c)
    right = rec.merge(a, rec.merge(b, c))
    swapped = rec.merge(c, rec.merge(b, a))
    for x in (right, swapped):
        np.testing.assert_allclose(x[0], left[0], rtol=0, atol=1e-14)
        assert abs(x[1] - left[1]) < 1e-13
    empty = (np.zeros(4), rec.EMPTY_LAMBDA)
    for x in (rec.merge(empty, a), rec.merge(a, empty)):
        assert np.array_equal(x[0], a[0]) and x[1] == a[1]


def test_runs_merged_one_after_the_other_end_with_softmax_weights_over_their_lambdas():
    """Sec. III-A's closed form w_i = e^{s_i} / sum_{j<=i} e^{s_j} applied to runs as keys:
    after all merges run p carries the weight e^{Lam_p - Lam_total}, Lam_total the fold of
    the Lam alone -- so the merged output is sum_p e^{Lam_p - Lam_total} o_p."""
    rng = np.random.default_rng(21)
    runs = []
    for n in (4, 1, 9, 0, 6, 2):
        runs.append(rec.state_of_run(rng.standard_normal(n) * 7, rng.standard_normal((n, 5))))
    st = (np.zeros(5), rec.EMPTY_LAMBDA)
    lam_only = (np.zeros(5), rec.EMPTY_LAMBDA)
    for r in runs:
        st = rec.merge(st, r)
        lam_only = rec.merge(lam_only, (np.zeros(5), r[1]))
    assert abs(st[1] - lam_only[1]) < 1e-13
    lams = np.array([r[1] for r in runs])
    np.testing.assert_allclose(st[1], scipy.special.logsumexp(lams[np.isfinite(lams)]),
                               rtol=0, atol=1e-12)
    weights = np.where(np.isfinite(lams), np.exp(lams - st[1]), 0.0)
    np.testing.assert_allclose(weights.sum(), 1.0, rtol=0, atol=1e-13)
    direct = sum(w * r[0] for w, r in zip(weights, runs))
    np.testing.assert_allclose(direct, st[0], rtol=0, atol=1e-13)


@pytest.mark.parametrize("algo", ALGOS)
def test_key_permutation_invariance(algo):
    rng = np.random.default_rng(16)
    q = torch.from_numpy(rng.standard_normal((1, 2, 5, 8)).astype(np.float32))
    k = torch.from_numpy(rng.standard_normal((1, 2, 40, 8)).astype(np.float32)) * 3
    v = torch.from_numpy(rng.standard_normal((1, 2, 40, 8)).astype(np.float32))
    perm = torch.from_numpy(rng.permutation(40))
    a = oa.attn(q, k, v, False, 0.5, algo)
    b = oa.attn(q, k[:, :, perm], v[:, :, perm], False, 0.5, algo)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)


# ------------------------------------------------------------------- stability ---

def test_huge_scores_stay_finite_without_max():
    """Sec. III-C: no max subtraction, yet nothing overflows."""
    V = np.arange(12.0).reshape(4, 3)
    s = np.array([0.0, 1000.0, -1000.0, 1000.0])
    o, w = rec.flashd_row(s, V)
    assert np.all(np.isfinite(o)) and np.all(np.isfinite(w))
    np.testing.assert_allclose(o[-1], 0.5 * (V[1] + V[3]), rtol=0, atol=1e-12)
    up = 100.0 * np.arange(30)
    V2 = np.random.default_rng(17).standard_normal((30, 3))
    np.testing.assert_allclose(rec.flashd_row(up, V2)[0][-1], V2[-1], rtol=0, atol=1e-12)
    np.testing.assert_allclose(rec.flashd_row(-up, V2)[0][-1], V2[0], rtol=0, atol=1e-12)
    st = rec.grouped_row(s, V, [0, 2, 4])
    np.testing.assert_allclose(st[0], o[-1], rtol=0, atol=1e-12)


@pytest.mark.parametrize("algo", ("alg1", "alg2", "alg3"))
def test_stress_inputs_with_dominant_keys(algo):
    from paper_2505_14201_amd import synthetic
    w = synthetic.small("stress", 1, 2, 2, 96, 96, 16, "f16", True, seed=99, qk_std=4.0,
                        plant_frac=0.2)
    q, k, v, planted = synthetic.make_qkv(w)
    assert len(planted) > 10
    a = oa.attn(q, k, v, True, w.scale, "definition")
    b = oa.attn(q, k, v, True, w.scale, algo)
    assert np.all(np.isfinite(b))
    np.testing.assert_allclose(b, a, rtol=0, atol=1e-12)
    # where a planted key's score beats every other visible score by > 40, the output
    # is that key's value row
    hits = 0
    for (bb, h, i, j) in planted:
        sc = w.scale * (k[bb, h, : i + 1].double() @ q[bb, h, i].double()).numpy()
        others = np.delete(sc, j)
        if others.size == 0 or sc[j] - others.max() > 40:
            np.testing.assert_allclose(a[bb, h, i], v[bb, h, j].double().numpy(), atol=1e-12)
            hits += 1
    assert hits > 5


# ------------------------------------------------------------ mask and mapping ---

@pytest.mark.parametrize("algo", ALGOS)
@pytest.mark.parametrize("Lq,Lk", [(6, 6), (4, 7), (7, 4)])
def test_causal_mask_with_identity_values(algo, Lq, Lk):
    """V = I makes the output row the weight row: exactly 0 where masked, > 0 elsewhere."""
    rng = np.random.default_rng(18)
    d = 8
    q = torch.from_numpy(rng.standard_normal((1, 1, Lq, d)).astype(np.float32))
    k = torch.from_numpy(rng.standard_normal((1, 1, Lk, d)).astype(np.float32))
    v = torch.zeros(1, 1, Lk, d)
    v[0, 0, :, :Lk] = torch.eye(Lk)
    got = oa.attn(q, k, v, True, 0.4, algo)[0, 0]
    for i in range(Lq):
        for j in range(Lk):
            if j <= i + (Lk - Lq):
                assert got[i, j] > 0
            else:
                assert got[i, j] == 0.0
        if i + (Lk - Lq) >= 0:
            assert abs(got[i].sum() - 1.0) < 1e-14


def test_gqa_head_mapping():
    rng = np.random.default_rng(19)
    q = torch.from_numpy(rng.standard_normal((2, 8, 3, 4)).astype(np.float32))
    k = torch.from_numpy(rng.standard_normal((2, 2, 9, 4)).astype(np.float32))
    v = torch.from_numpy(rng.standard_normal((2, 2, 9, 4)).astype(np.float32))
    v[:, 1] = 3.25
    got = oa.attn(q, k, v, False, 1.0)
    assert np.all(np.abs(got[:, 4:] - 3.25) < 1e-14)
    assert not np.any(np.abs(got[:, :4] - 3.25) < 1e-3)


def test_row_subset_matches_full():
    rng = np.random.default_rng(20)
    q = torch.from_numpy(rng.standard_normal((2, 4, 10, 8)).astype(np.float32))
    k = torch.from_numpy(rng.standard_normal((2, 2, 12, 8)).astype(np.float32))
    v = torch.from_numpy(rng.standard_normal((2, 2, 12, 8)).astype(np.float32))
    full = oa.attn(q, k, v, True, 0.5)
    rows = np.array([[0, 0, 0], [1, 3, 9], [0, 2, 5], [1, 1, 1]], dtype=np.int32)
    part = oa.attn(q, k, v, True, 0.5, rows=rows)
    for r, (b, h, i) in enumerate(rows):
        assert np.array_equal(part[r], full[b, h, i])
    with pytest.raises(ValueError):
        oa.attn(q, k, v, True, 0.5, rows=np.array([[0, 0, 10]]))


def test_storage_dtypes_are_widened_exactly():
    rng = np.random.default_rng(21)
    for dt in (torch.bfloat16, torch.float16):
        q = torch.from_numpy(rng.standard_normal((1, 1, 3, 8)).astype(np.float32)).to(dt)
        k = torch.from_numpy(rng.standard_normal((1, 1, 5, 8)).astype(np.float32)).to(dt)
        v = torch.from_numpy(rng.standard_normal((1, 1, 5, 8)).astype(np.float32)).to(dt)
        a = oa.attn(q, k, v, False, 0.5)
        b = oa.attn(q.float(), k.float(), v.float(), False, 0.5)
        assert np.array_equal(a, b)


def test_skip_rule_counts():
    lo, hi, n = rec.skip_counts([0.0, -6.0, 5.0, 16.0, 15.0, 4.0, 4.0 - 5.99])
    assert (lo, hi, n) == (2, 2, 6)


# ---- static skip statistics (Sec. III-C, Table I) --------------------------------------

def _skip_brute(q, k, causal, scale, lo=-6.0, hi=11.0, margin=1e-3):
    """Plain-Python count in fp64; also returns the smallest distance of a score difference
    from a threshold (the fp32 oracle must agree exactly when that is not tiny)."""
    q = q.double().numpy()
    k = k.double().numpy()
    B, Hq, Lq, d = q.shape
    _, Hkv, Lk, _ = k.shape
    steps = low = high = 0
    closest = float("inf")
    for b in range(B):
        for h in range(Hq):
            kh = k[b, h // (Hq // Hkv)]
            for i in range(Lq):
                nvis = min(max(i + (Lk - Lq) + 1, 0), Lk) if causal else Lk
                s = (kh[:nvis] @ q[b, h, i]) * float(np.float32(scale))
                dlt = np.diff(s)
                steps += len(dlt)
                low += int(np.sum(dlt <= lo))
                high += int(np.sum(dlt >= hi))
                if len(dlt):
                    closest = min(closest, float(np.min(np.abs(dlt - lo))),
                                  float(np.min(np.abs(dlt - hi))))
    return steps, low, high, closest


def test_skip_stats_worked_example_with_exact_scores():
    # q = e_0, scale 1: the scores are the first components of the keys, all exact
    vals = [0.0, -6.0, 5.0, 16.0, 15.0, 4.0, -2.0]     # differences -6, 11, 11, -1, -11, -6
    k = torch.zeros(1, 1, len(vals), 4)
    k[0, 0, :, 0] = torch.tensor(vals)
    q = torch.zeros(1, 1, 1, 4)
    q[0, 0, 0, 0] = 1.0
    assert oa.skip_stats(q, k, False, 1.0) == (6, 3, 2)       # thresholds are inclusive
    assert oa.skip_stats(q, k, False, 1.0, lo=-6.5, hi=11.5) == (6, 1, 0)
    # causal, one query per key: row i walks keys 0..i
    qc = q.expand(1, 1, len(vals), 4).contiguous()
    dl = np.diff(vals)
    exp = (sum(range(len(vals))), sum(int(np.sum(dl[:i] <= -6)) for i in range(len(vals))),
           sum(int(np.sum(dl[:i] >= 11)) for i in range(len(vals))))
    assert oa.skip_stats(qc, k, True, 1.0) == exp


@pytest.mark.parametrize("shape", [(1, 2, 2, 9, 9, 16), (2, 4, 2, 5, 12, 8), (1, 3, 1, 12, 5, 32)])
@pytest.mark.parametrize("causal", [False, True])
def test_skip_stats_match_brute_force(shape, causal):
    B, Hq, Hkv, Lq, Lk, d = shape
    rng = np.random.default_rng(99 + Lq)
    q = torch.from_numpy((4 * rng.standard_normal((B, Hq, Lq, d))).astype(np.float32))
    k = torch.from_numpy((4 * rng.standard_normal((B, Hkv, Lk, d))).astype(np.float32))
    scale = 1.0 / math.sqrt(d)
    steps, low, high, closest = _skip_brute(q, k, causal, scale)
    assert closest > 1e-3          # no difference sits on a threshold: fp32 and fp64 must agree
    assert low > 0 and high > 0    # the sample exercises both counters
    assert oa.skip_stats(q, k, causal, scale) == (steps, low, high)
    assert rec.skip_counts is not None


def test_skip_stats_rate_has_the_gaussian_closed_form():
    # q = a e_0 and iid N(0,1) first key components: s_j is N(0, sigma^2) with sigma = a * scale,
    # a step's difference N(0, 2 sigma^2), so P(low) = Phi(-6 / (sigma sqrt 2)) and
    # P(high) = Phi(-11 / (sigma sqrt 2)).
    rng = np.random.default_rng(5)
    n = 200001
    k = torch.zeros(1, 1, n, 2)
    k[0, 0, :, 0] = torch.from_numpy(rng.standard_normal(n).astype(np.float32))
    q = torch.tensor([[[[8.0, 0.0]]]])
    sigma = 8.0 * 0.5
    steps, low, high = oa.skip_stats(q, k, False, 0.5)
    p_low = 0.5 * math.erfc(6.0 / (sigma * math.sqrt(2.0)) / math.sqrt(2.0))
    p_high = 0.5 * math.erfc(11.0 / (sigma * math.sqrt(2.0)) / math.sqrt(2.0))
    assert steps == n - 1
    # neighbouring steps share a score, which at most doubles the binomial variance
    for cnt, pr in ((low, p_low), (high, p_high)):
        sd = math.sqrt(2.0 * steps * pr * (1.0 - pr))
        assert abs(cnt - steps * pr) < 5.0 * sd, (cnt, steps * pr, sd)


def test_skip_stats_storage_types_are_widened_exactly():
    rng = np.random.default_rng(6)
    for dt in (torch.bfloat16, torch.float16):
        q = torch.from_numpy((3 * rng.standard_normal((1, 2, 6, 16))).astype(np.float32)).to(dt)
        k = torch.from_numpy((3 * rng.standard_normal((1, 1, 40, 16))).astype(np.float32)).to(dt)
        assert oa.skip_stats(q, k, False, 0.25) == oa.skip_stats(q.float(), k.float(), False, 0.25)


# ---- Alg. 3 with the state handed in and out (Sec. III-C) ------------------------------

def _rand_qkv(rng, B, Hq, Hkv, Lq, Lk, d, std=1.0):
    mk = lambda *s: torch.from_numpy((std * rng.standard_normal(s)).astype(np.float32))
    return mk(B, Hq, Lq, d), mk(B, Hkv, Lk, d), mk(B, Hkv, Lk, d)


@pytest.mark.parametrize("causal", [False, True])
def test_state_of_a_run_is_output_and_log_sum_exp(causal):
    rng = np.random.default_rng(11)
    B, Hq, Hkv, Lq, Lk, d = 2, 4, 2, 7, 19, 8
    q, k, v = _rand_qkv(rng, B, Hq, Hkv, Lq, Lk, d, 2.0)
    st = oa.attn_state(q, k, v, causal, 0.3)
    ref = oa.attn(q, k, v, causal, 0.3)
    assert np.allclose(st[..., :d], ref, rtol=0, atol=1e-12)
    # s_last - ln w_last = ln sum_j e^{s_j} over the visible keys (weight equation, Sec. III-B)
    kk = k.double().repeat_interleave(Hq // Hkv, dim=1)
    s = (q.double() @ kk.transpose(-1, -2)).numpy() * float(np.float32(0.3))
    for i in range(Lq):
        nvis = min(i + (Lk - Lq) + 1, Lk) if causal else Lk
        lse = scipy.special.logsumexp(s[:, :, i, :nvis], axis=-1)
        assert np.allclose(st[:, :, i, d] - st[:, :, i, d + 1], lse, rtol=0, atol=1e-12)
        assert np.allclose(st[:, :, i, d], s[:, :, i, nvis - 1])         # s_last is literal


@pytest.mark.parametrize("cuts", [(5,), (1, 2), (7, 8, 18)])
def test_chunked_keys_with_state_passing_equal_one_pass(cuts):
    rng = np.random.default_rng(12)
    B, Hq, Hkv, Lq, Lk, d = 1, 2, 1, 6, 19, 4
    q, k, v = _rand_qkv(rng, B, Hq, Hkv, Lq, Lk, d, 3.0)
    for causal in (False, True):
        full = oa.attn_state(q, k, v, causal, 0.5)
        st, k0 = None, 0
        for k1 in list(cuts) + [Lk]:
            st = oa.attn_state(q, k[:, :, k0:k1].contiguous(), v[:, :, k0:k1].contiguous(), causal,
                               0.5, st, shift=(Lk - Lq) - k0)
            k0 = k1
        # the literal recurrence does the same steps in the same order either way
        assert np.allclose(st, full, rtol=0, atol=1e-13)


def test_state_in_only_enters_through_s_minus_ln_w():
    rng = np.random.default_rng(13)
    q, k, v = _rand_qkv(rng, 1, 1, 1, 3, 9, 4, 2.0)
    first = oa.attn_state(q, k[:, :, :4].contiguous(), v[:, :, :4].contiguous(), False, 1.0)
    moved = first.copy()
    moved[..., 4] += 0.75                      # (s, ln w) -> (s + delta, ln w + delta)
    moved[..., 5] += 0.75
    a = oa.attn_state(q, k[:, :, 4:].contiguous(), v[:, :, 4:].contiguous(), False, 1.0, first)
    b = oa.attn_state(q, k[:, :, 4:].contiguous(), v[:, :, 4:].contiguous(), False, 1.0, moved)
    assert np.allclose(a, b, rtol=0, atol=1e-13)


def test_rows_without_keys_carry_the_empty_state_through():
    rng = np.random.default_rng(14)
    q, k, v = _rand_qkv(rng, 1, 1, 1, 5, 3, 4)
    st = oa.attn_state(q, k, v, True, 1.0)                 # Lq > Lk: rows 0, 1 see nothing
    assert np.all(st[0, 0, :2, :4] == 0) and np.all(np.isneginf(st[0, 0, :2, 4]))
    nxt = oa.attn_state(q, k, v, True, 1.0, st, shift=1)   # a second chunk they do see
    alone = oa.attn_state(q, k, v, True, 1.0, None, shift=1)
    assert np.allclose(nxt[0, 0, :2], alone[0, 0, :2], rtol=0, atol=1e-13)


def test_state_matches_the_scalar_recurrence():
    rng = np.random.default_rng(15)
    q, k, v = _rand_qkv(rng, 1, 1, 1, 1, 6, 3, 2.0)
    st = oa.attn_state(q, k, v, False, 0.7)[0, 0, 0]
    s = (k[0, 0].double() @ q[0, 0, 0].double()).numpy() * float(np.float32(0.7))
    o, lam = rec.state_of_run(s, v[0, 0].double().numpy())
    assert np.allclose(st[:3], o, atol=1e-13) and abs((st[3] - st[4]) - lam) < 1e-12
    _, lnw = rec.weights_sigmoid(s)
    assert abs(st[3] - s[-1]) < 1e-13 and abs(st[4] - lnw[-1]) < 1e-12
