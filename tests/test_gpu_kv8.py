"""GPU parity of flashd_attn_fwd_kv8 (K and V stored as fp8 e4m3): the oracle gets the fp8
values widened exactly, so the bound is that of the f16/bf16 path (K and V are widened
exactly inside the kernel too; only the coefficients are rounded to the storage type)."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from paper_2505_14201_amd import flashd, synthetic
from tests.gpu_util import check

pytestmark = pytest.mark.gpu
DT = {"f16": torch.float16, "bf16": torch.bfloat16}


def quantise(x, scale):
    """fp8 storage of x / scale (round to nearest even, as torch does it)."""
    return (x.float() / scale).to(torch.float8_e4m3fn)


def run_and_ref(w, kscale, vscale):
    q, k, v, _ = synthetic.make_qkv(w)
    k8, v8 = quantise(k, kscale), quantise(v, vscale)
    og = torch.full_like(q, float("nan")).cuda()
    flashd.attn_fwd_kv8(q.cuda(), k8.cuda(), v8.cuda(), og, w.causal, w.scale, kscale, vscale)
    torch.cuda.synchronize()
    # exact oracle inputs: fp8 values as floats; kscale joins the score scale (one fp32
    # product, as in the kernel), vscale the output
    sc = float(np.float32(w.scale) * np.float32(kscale))
    ref = oa.attn(q, k8.float(), v8.float(), w.causal, sc) * float(np.float32(vscale))
    return og.cpu(), ref


# (B, Hq, Hkv, Lq, Lk, d): decode shapes, (Hq / Hkv) * Lq <= 32; ragged key counts
SHAPES = [(1, 4, 1, 1, 1, 64), (2, 8, 2, 1, 1000, 128), (1, 32, 8, 1, 4133, 128),
          (3, 4, 4, 5, 333, 64), (1, 8, 1, 4, 2050, 128), (2, 16, 2, 3, 77, 64)]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_fp8_kv_decode_matches_the_oracle(shape, causal, dtype):
    B, Hq, Hkv, Lq, Lk, d = shape
    w = synthetic.small("kv8", B, Hq, Hkv, Lq, Lk, d, dtype, causal, seed=800 + Lk + Hq)
    got, ref = run_and_ref(w, 2.0 ** -5, 2.0 ** -5)
    check(got, ref, DT[dtype], f"{shape} causal={causal} {dtype}")


def test_scales_that_are_not_powers_of_two_and_every_fp8_code():
    w = synthetic.small("kv8", 1, 8, 2, 2, 512, 128, "bf16", False, seed=811)
    got, ref = run_and_ref(w, 0.0371, 0.0293)
    check(got, ref, torch.bfloat16, "odd scales")
    # all 254 finite codes as key and value elements
    codes = torch.tensor([c for c in range(256) if c not in (0x7f, 0xff)], dtype=torch.uint8)
    k8 = codes.repeat(64 * 254 // 254)[:64 * 128].reshape(1, 1, 64, 128).view(torch.float8_e4m3fn)
    v8 = k8.flip(2).contiguous()
    q = (torch.randn(1, 4, 1, 128, generator=torch.Generator().manual_seed(3)) * 0.01).to(
        torch.bfloat16)
    og = torch.empty_like(q).cuda()
    flashd.attn_fwd_kv8(q.cuda(), k8.cuda(), v8.cuda(), og, False, 0.05, 0.125, 0.0078125)
    torch.cuda.synchronize()
    ref = oa.attn(q, k8.float(), v8.float(), False,
                  float(np.float32(0.05) * np.float32(0.125))) * 0.0078125
    check(og.cpu(), ref, torch.bfloat16, "all codes")


# prefill shapes: K and V are widened into scratch memory first, then the tile kernel runs
PREFILL = [(1, 4, 2, 200, 333, 128), (2, 2, 2, 333, 200, 64), (1, 8, 8, 130, 130, 128),
           (1, 2, 1, 64, 2000, 64)]


@pytest.mark.parametrize("shape", PREFILL)
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_fp8_kv_prefill_matches_the_oracle(shape, causal, dtype):
    B, Hq, Hkv, Lq, Lk, d = shape
    w = synthetic.small("kv8p", B, Hq, Hkv, Lq, Lk, d, dtype, causal, seed=850 + Lq + Lk)
    got, ref = run_and_ref(w, 0.03, 0.045)
    check(got, ref, DT[dtype], f"{shape} causal={causal} {dtype}")


def test_fp8_entry_point_rejects_fp32_queries():
    q = torch.zeros(1, 4, 1, 64, dtype=torch.float32, device="cuda")
    k8 = torch.zeros(1, 1, 64, 64, dtype=torch.float8_e4m3fn, device="cuda")
    with pytest.raises(ValueError):
        flashd.attn_fwd_kv8(q, k8, k8, torch.empty_like(q), False, 1.0, 1.0, 1.0)
    rc = flashd.raw().flashd_attn_fwd_kv8(q.data_ptr(), k8.data_ptr(), k8.data_ptr(),
                                          q.data_ptr(), 1, 4, 1, 1, 64, 64, 0, 1.0, 1.0, 1.0,
                                          flashd.F32, None)
    assert rc == -10
