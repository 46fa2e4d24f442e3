"""Maximum sizes: tensors of 2^32 elements, so that element offsets pass 2^31 and byte
offsets 2^33 inside one launch.  The oracle checks whole (batch, head) units taken from the
start of the tensors, from either side of the 2^31-element line and from the very end; a
32-bit offset anywhere in the path would read (or write) the wrong unit there.

Inputs are seeded N(0, 1) draws made on the GPU (17 GB per case would take minutes through
the host generator); the oracle gets the same values, copied back unit by unit."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from paper_2505_14201_amd import flashd
from tests.gpu_util import check

pytestmark = pytest.mark.gpu

B, H, D, LONG = 16, 8, 128, 262144          # B * H * LONG * D = 2^32 elements
UNITS = [(0, 0), (7, 7), (8, 0), (15, 7)]   # (8, 0) starts exactly at element 2^31
SCALE = float(np.float32(1.0 / np.sqrt(D)))


def normal(shape, dtype, seed):
    gen = torch.Generator(device="cuda").manual_seed(seed)
    t = torch.empty(shape, dtype=dtype, device="cuda")
    for b in range(shape[0]):                # slab by slab: each draw stays below 2^31 elements
        t[b].normal_(generator=gen)
    return t


def need_memory(gib):
    free, _ = torch.cuda.mem_get_info()
    if free < gib * 2 ** 30:
        pytest.skip(f"needs {gib} GiB of free device memory")


@pytest.mark.parametrize("Lq", [1, 64], ids=["decode_kernel", "tile_kernel"])
def test_long_keys_offsets_beyond_32_bits(Lq):
    need_memory(24)
    k = normal((B, H, LONG, D), torch.bfloat16, 4101)
    v = normal((B, H, LONG, D), torch.bfloat16, 4102)
    q = normal((B, H, Lq, D), torch.bfloat16, 4103)
    assert k.numel() == 2 ** 32
    o = torch.full_like(q, float("nan"))
    flashd.attn_fwd(q, k, v, o, False, SCALE)
    torch.cuda.synchronize()
    assert torch.isfinite(o.float()).all()
    for (b, h) in UNITS:
        sl = (slice(b, b + 1), slice(h, h + 1))
        ref = oa.attn(q[sl].cpu(), k[sl].cpu(), v[sl].cpu(), False, SCALE)
        check(o[sl].cpu(), ref, torch.bfloat16, f"Lq={Lq} unit {(b, h)}")
    del k, v
    torch.cuda.empty_cache()


def test_long_queries_offsets_beyond_32_bits():
    need_memory(24)
    Lk = 64
    q = normal((B, H, LONG, D), torch.bfloat16, 4201)
    k = normal((B, H, Lk, D), torch.bfloat16, 4202)
    v = normal((B, H, Lk, D), torch.bfloat16, 4203)
    rows = [slice(0, 300), slice(LONG // 2 - 150, LONG // 2 + 150), slice(LONG - 300, LONG)]
    o = torch.full_like(q, float("nan"))
    flashd.attn_fwd(q, k, v, o, False, SCALE)         # every row sees the 64 keys
    torch.cuda.synchronize()
    assert torch.isfinite(o.float()).all()
    for (b, h) in UNITS:
        for r in rows:
            sl = (slice(b, b + 1), slice(h, h + 1), r)
            ref = oa.attn(q[sl].cpu(), k[b:b + 1, h:h + 1].cpu(), v[b:b + 1, h:h + 1].cpu(), False,
                          SCALE)
            check(o[sl].cpu(), ref, torch.bfloat16, f"unit {(b, h)} rows {r.start}..{r.stop}")
    o.fill_(float("nan"))
    flashd.attn_fwd(q, k, v, o, True, SCALE)          # causal: the last 64 rows see 1 .. 64 keys
    torch.cuda.synchronize()
    for (b, h) in UNITS:
        ku, vu = k[b:b + 1, h:h + 1].cpu(), v[b:b + 1, h:h + 1].cpu()
        for r in rows:
            sl = (slice(b, b + 1), slice(h, h + 1), r)
            # this block of rows under the bottom-right rule: row r.start + t sees the keys
            # j <= t + shift (the oracle's recurrence takes the shift as an argument)
            shift = (Lk - LONG) + r.start
            ref = oa.attn_state(q[sl].cpu(), ku, vu, True, SCALE, shift=shift)[..., :D]
            check(o[sl].cpu(), ref, torch.bfloat16, f"unit {(b, h)} rows {r.start}..{r.stop}")
            if r.stop <= LONG - Lk:
                assert torch.count_nonzero(o[sl]) == 0, "rows without a visible key are zeros"
    del q, o
    torch.cuda.empty_cache()


def test_long_keys_fp32_per_key_kernel():
    need_memory(40)
    k = normal((B, H, LONG, D), torch.float32, 4301)
    v = normal((B, H, LONG, D), torch.float32, 4302)
    q = normal((B, H, 1, D), torch.float32, 4303)
    o = torch.full_like(q, float("nan"))
    flashd.attn_fwd(q, k, v, o, False, SCALE)
    torch.cuda.synchronize()
    for (b, h) in UNITS:
        sl = (slice(b, b + 1), slice(h, h + 1))
        ref = oa.attn(q[sl].cpu(), k[sl].cpu(), v[sl].cpu(), False, SCALE)
        check(o[sl].cpu(), ref, torch.float32, f"f32 unit {(b, h)}")
    del k, v
    torch.cuda.empty_cache()
