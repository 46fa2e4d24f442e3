"""Randomised GPU parity: seeded draws over shapes (ragged, Lq != Lk both ways, GQA), storage
types, variants, split counts and score ranges from ordinary to very peaked (one key takes
nearly all the weight, outputs of magnitude 4: where the rounding of the coefficients and of
the output leave the least room inside the bound), each against the fp64 oracle; the same for
chunked calls with the state handed on and for fp8 K/V.  A draw that fails prints its
parameters."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from paper_2505_14201_amd import flashd, synthetic
from tests.gpu_util import check, run_flashd
from tests.test_gpu_state import check_state, run_chunks

pytestmark = pytest.mark.gpu
DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def draw(rng, it, dtypes=("bf16", "f16", "f32"), p=(0.45, 0.45, 0.1)):
    dtype = str(rng.choice(dtypes, p=p))
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 3]))
    Hq = Hkv * int(rng.choice([1, 2, 4, 8]))
    B = int(rng.choice([1, 2]))
    Lq = int(rng.choice([1, 2, 3, 17, 64, 100, 128, 129, 200, 300, 513]))
    Lk = int(rng.choice([1, 5, 63, 64, 65, 127, 128, 200, 333, 512, 777, 1500]))
    causal = bool(rng.integers(2))
    qk_std = float(rng.choice([1.0, 1.0, 3.0, 6.0]))
    plant = float(rng.choice([0.0, 0.0, 0.1])) if (causal and Hq == Hkv) else 0.0
    if Lq * Lk * Hq * B > 3e6:
        Lq = min(Lq, 64)
    return synthetic.small("rnd", B, Hq, Hkv, Lq, Lk, d, dtype, causal, seed=7000 + it,
                           qk_std=qk_std, plant_frac=plant)


@pytest.mark.parametrize("seed", [101, 102, 103, 104])
def test_random_forward_calls(seed):
    rng = np.random.default_rng(seed)
    for it in range(150):
        w = draw(rng, 1000 * seed + it)
        variant = int(rng.choice([0, 1, 2, 3, 4])) if w.dtype != "f32" else int(rng.choice([0, 2]))
        splits = int(rng.choice([0, 1, 2, 5]))
        if splits > w.Lk:
            splits = 1
        q, k, v, _ = synthetic.make_qkv(w)
        what = f"seed={seed} it={it} {w} variant={variant} splits={splits}"
        ref = oa.attn(q, k, v, w.causal, w.scale)
        got = run_flashd(q, k, v, w.causal, w.scale, variant, splits)
        check(got, ref, DT[w.dtype], what)


@pytest.mark.parametrize("seed", [201, 202])
def test_random_chunked_calls_with_state(seed):
    rng = np.random.default_rng(seed)
    for it in range(60):
        w = draw(rng, 1000 * seed + it)
        if w.plant_frac:          # planted keys are placed for the whole key range
            w = synthetic.small("rnd", w.B, w.Hq, w.Hkv, w.Lq, w.Lk, w.d, w.dtype, w.causal,
                                seed=w.seed, qk_std=w.qk_std)
        ncuts = int(rng.integers(0, 4))
        cuts = tuple(sorted(set(int(c) for c in rng.integers(1, max(2, w.Lk), size=ncuts)
                                if 0 < c < w.Lk)))
        q, k, v, _ = synthetic.make_qkv(w)
        what = f"seed={seed} it={it} {w} cuts={cuts}"
        ref = oa.attn_state(q, k, v, w.causal, w.scale)
        o, st = run_chunks(q, k, v, w.causal, w.scale, cuts)
        check(o, ref[..., :w.d], DT[w.dtype], what + " (o)")
        if w.qk_std <= 1.0:       # s - ln w to the fp32 bound only where scores are ordinary
            check_state(st, ref, w.d, DT[w.dtype], what)


@pytest.mark.parametrize("seed", [301])
def test_random_fp8_kv_calls(seed):
    rng = np.random.default_rng(seed)
    for it in range(60):
        w = draw(rng, 1000 * seed + it, dtypes=("bf16", "f16"), p=(0.5, 0.5))
        if w.plant_frac or w.qk_std > 3.0:
            w = synthetic.small("rnd", w.B, w.Hq, w.Hkv, w.Lq, w.Lk, w.d, w.dtype, w.causal,
                                seed=w.seed, qk_std=min(w.qk_std, 3.0))
        q, k, v, _ = synthetic.make_qkv(w)
        kscale = float(rng.choice([2.0 ** -4, 0.0371, 2.0 ** -2]))
        vscale = float(rng.choice([2.0 ** -5, 0.0293]))
        k8 = (k.float() / kscale).to(torch.float8_e4m3fn)
        v8 = (v.float() / vscale).to(torch.float8_e4m3fn)
        og = torch.full_like(q, float("nan")).cuda()
        flashd.attn_fwd_kv8(q.cuda(), k8.cuda(), v8.cuda(), og, w.causal, w.scale, kscale, vscale)
        torch.cuda.synchronize()
        sc = float(np.float32(w.scale) * np.float32(kscale))
        ref = oa.attn(q, k8.float(), v8.float(), w.causal, sc) * float(np.float32(vscale))
        check(og.cpu(), ref, DT[w.dtype], f"seed={seed} it={it} {w} kscale={kscale} vscale={vscale}")
