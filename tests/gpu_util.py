"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI binding,
run the oracle, and compare to the stated tolerances."""
from __future__ import annotations

import numpy as np
import torch

# fp32: max-abs error <= 1e-5 relative to the output scale max(1, max|o_ref|).
# f16/bf16 storage with fp32 accumulation: max-abs error <= 2e-2 absolute, plus a relative
# RMS gate of 1e-2 (with iid inputs |o| itself is only a few 1e-2, so the absolute bound
# alone could not tell a right answer from zeros).
F32_REL = 1e-5
HALF_ABS = 2e-2
HALF_RMS = 1e-2


def to_gpu(*ts):
    return [t.cuda() for t in ts]


CANARY_BYTES = 4096
CANARY = 0xA5


class Guarded:
    """A device buffer of `nbytes` with CANARY_BYTES of a fixed byte pattern on either side;
    intact() tells whether a launch wrote outside the part it was given.  The payload starts
    256-byte aligned (CANARY_BYTES is a multiple of 256 and torch allocations are aligned)."""

    def __init__(self, nbytes: int, fill: int = 0xFF):
        self.nbytes = int(nbytes)
        self.raw = torch.empty(self.nbytes + 2 * CANARY_BYTES, dtype=torch.uint8, device="cuda")
        self.raw.fill_(CANARY)
        self.payload = self.raw[CANARY_BYTES:CANARY_BYTES + self.nbytes]
        self.payload.fill_(fill)           # 0xFF bytes: NaN in every storage type

    def view(self, dtype, shape):
        return self.payload.view(dtype).view(shape)

    def intact(self) -> bool:
        lo = self.raw[:CANARY_BYTES]
        hi = self.raw[CANARY_BYTES + self.nbytes:]
        return bool((lo == CANARY).all().item()) and bool((hi == CANARY).all().item())


def run_flashd(q, k, v, causal, scale, variant=0, splits=0, use_ex=True):
    """q, k, v: CPU tensors in storage dtype.  Returns the GPU result as a CPU tensor.  The
    output and the workspace sit between canaries that are checked after the launch."""
    from paper_2505_14201_amd import flashd
    qg, kg, vg = to_gpu(q, k, v)
    og_guard = Guarded(qg.numel() * qg.element_size())
    og = og_guard.view(qg.dtype, qg.shape)
    ws_guard = None
    if use_ex:
        B, Hq, Lq, d = q.shape
        _, Hkv, Lk, _ = k.shape
        dt = {torch.float32: 0, torch.float16: 1, torch.bfloat16: 2}[q.dtype]
        nbytes = flashd.workspace_bytes(B, Hq, Hkv, Lq, Lk, d, dt, variant, splits)
        ws_guard = Guarded(nbytes) if nbytes else None
        flashd.attn_fwd_ex(qg, kg, vg, og, causal, scale, variant, splits,
                           ws_guard.payload if ws_guard else None)
    else:
        flashd.attn_fwd(qg, kg, vg, og, causal, scale)
    torch.cuda.synchronize()
    assert og_guard.intact(), "a kernel wrote outside the output buffer"
    assert ws_guard is None or ws_guard.intact(), "a kernel wrote outside the workspace"
    return og.cpu()


def max_abs_score(q, k, scale) -> float:
    """Largest |scale * q.k| over all (query, key) pairs of matching heads (fp64, CPU)."""
    B, Hq, Lq, d = q.shape
    g = Hq // k.shape[1]
    kk = k.double().repeat_interleave(g, dim=1)
    return float((q.double() @ kk.transpose(-1, -2)).abs().max()) * float(scale)


def check(got: torch.Tensor, ref: np.ndarray, dtype: torch.dtype, what: str = ""):
    """fp32: 1e-5 relative to the output scale whatever the size of the scores (the fp32 path
    carries the dot product and s - ln w in fp64)."""
    g = got.double().numpy().reshape(ref.shape)
    assert np.all(np.isfinite(g)), f"{what}: non-finite output"
    err = np.abs(g - ref)
    if dtype == torch.float32:
        bound = F32_REL * max(1.0, float(np.abs(ref).max()))
        assert err.max() <= bound, f"{what}: max abs err {err.max():.3e} > {bound:.3e}"
    else:
        assert err.max() <= HALF_ABS, f"{what}: max abs err {err.max():.3e} > {HALF_ABS}"
        den = float(np.sqrt((ref ** 2).sum()))
        if den > 0:
            rms = float(np.sqrt((err ** 2).sum())) / den
            assert rms <= HALF_RMS, f"{what}: relative rms err {rms:.3e} > {HALF_RMS}"
    return float(err.max())
