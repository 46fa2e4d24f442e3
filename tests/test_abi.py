"""The C ABI without a GPU: the library loads, exports what the header declares, and
turns every invalid argument into its status code before touching the device."""
import ctypes
import os
import re

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

from paper_2505_14201_amd import flashd  # noqa: E402

OK, E_NULL, E_SHAPE, E_DTYPE, E_HEADDIM, E_GQA, E_ALIGN, E_WS, E_HIP, E_ARCH, E_VARIANT = \
    0, -1, -2, -3, -4, -5, -6, -7, -8, -9, -10

P = 0x1000          # a non-null, 16-byte aligned fake pointer; never dereferenced on these paths

# A call whose arguments are all valid goes on to launch a kernel where there is a GPU, and the
# fake pointers would then be dereferenced on the device: such calls are only made without one
# (they end in FLASHD_E_HIP there).
NO_GPU = not torch.cuda.is_available()


def fwd(q=P, k=P, v=P, o=P, B=1, Hq=4, Hkv=2, Lq=8, Lk=8, d=64, causal=0, scale=0.125,
        dtype=flashd.BF16):
    return flashd.raw().flashd_attn_fwd(q, k, v, o, B, Hq, Hkv, Lq, Lk, d, causal, scale, dtype,
                                        None)


def fwd_ex(variant=0, splits=0, ws=None, ws_bytes=0, **kw):
    a = dict(q=P, k=P, v=P, o=P, B=1, Hq=4, Hkv=2, Lq=8, Lk=512, d=64, causal=0, scale=0.125,
             dtype=flashd.BF16)
    a.update(kw)
    return flashd.raw().flashd_attn_fwd_ex(a["q"], a["k"], a["v"], a["o"], a["B"], a["Hq"],
                                           a["Hkv"], a["Lq"], a["Lk"], a["d"], a["causal"],
                                           a["scale"], a["dtype"], None, variant, splits, ws,
                                           ws_bytes)


def test_header_symbols_are_exported():
    text = open(os.path.join(ROOT, "include", "flashd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(flashd_[a-z0-9_]+)\s*\(", text))
    assert declared == set(flashd.EXPORTS)
    lib = ctypes.CDLL(flashd.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_header_constants_match_binding():
    text = open(os.path.join(ROOT, "include", "flashd.h")).read()
    enums = dict((k, int(v)) for k, v in re.findall(r"(FLASHD_[A-Z0-9_]+)\s*=\s*(-?\d+)", text))
    assert (enums["FLASHD_F32"], enums["FLASHD_F16"], enums["FLASHD_BF16"]) == \
        (flashd.F32, flashd.F16, flashd.BF16)
    assert enums["FLASHD_VARIANT_TILE"] == flashd.VARIANT_TILE
    assert enums["FLASHD_VARIANT_PER_KEY"] == flashd.VARIANT_PER_KEY
    assert enums["FLASHD_VARIANT_ONLINE_SOFTMAX"] == flashd.VARIANT_ONLINE_SOFTMAX
    assert int(re.search(r"#define FLASHD_MAX_SPLITS (\d+)", text).group(1)) == flashd.MAX_SPLITS
    for name, val in enums.items():
        if name.startswith("FLASHD_E_") or name == "FLASHD_OK":
            s = flashd.status_string(val)
            assert s and s != "unknown status"
    assert flashd.status_string(-99) == "unknown status"
    assert flashd.version() >= 100


def test_null_pointers():
    for name in ("q", "k", "v", "o"):
        assert fwd(**{name: None}) == E_NULL


def test_shape_errors():
    for name in ("B", "Hq", "Hkv", "Lq", "Lk"):
        assert fwd(**{name: 0}) == E_SHAPE
        assert fwd(**{name: -3}) == E_SHAPE
    assert fwd(B=70000) == E_SHAPE
    assert fwd(B=60000, Hq=60000, Hkv=60000, Lq=100000, Lk=8) == E_SHAPE   # element count overflow
    assert fwd(B=1, Hq=1, Hkv=1, Lq=8, Lk=2_000_000_000, d=64) == E_SHAPE      # 32-bit key indices
    assert fwd(B=1, Hq=1, Hkv=1, Lq=1_500_000_000, Lk=8, d=64) == E_SHAPE


def test_dtype_headdim_gqa_align():
    assert fwd(dtype=3) == E_DTYPE
    assert fwd(dtype=-1) == E_DTYPE
    for d in (0, 32, 96, 256, 65):
        assert fwd(d=d) == E_HEADDIM
    assert fwd(Hq=5, Hkv=2) == E_GQA
    for name in ("q", "k", "v", "o"):
        assert fwd(**{name: P + 8}) == E_ALIGN
    assert fwd_ex(ws=P + 4, ws_bytes=1 << 30, splits=2) == E_ALIGN


def test_error_precedence_is_null_shape_dtype_headdim_gqa_align():
    assert fwd(q=None, B=0, dtype=9, d=3, Hq=5) == E_NULL
    assert fwd(B=0, dtype=9, d=3, Hq=5) == E_SHAPE
    assert fwd(dtype=9, d=3, Hq=5) == E_DTYPE
    assert fwd(d=3, Hq=5, q=P + 2) == E_HEADDIM
    assert fwd(Hq=5, q=P + 2) == E_GQA


def test_variant_and_split_errors():
    assert fwd_ex(variant=6) == E_VARIANT
    assert fwd_ex(variant=flashd.VARIANT_TILE_BLEND, dtype=flashd.F32) == E_VARIANT
    assert fwd_ex(variant=flashd.VARIANT_TILE_256, dtype=flashd.F32) == E_VARIANT
    assert fwd_ex(variant=-1) == E_VARIANT
    assert fwd_ex(variant=flashd.VARIANT_TILE, dtype=flashd.F32) == E_VARIANT
    assert fwd_ex(variant=flashd.VARIANT_ONLINE_SOFTMAX, dtype=flashd.F32) == E_VARIANT
    assert fwd_ex(splits=-1) == E_VARIANT
    assert fwd_ex(splits=flashd.MAX_SPLITS + 1) == E_VARIANT
    assert fwd_ex(splits=9, Lk=8) == E_VARIANT


def test_workspace_errors_and_sizes():
    need = flashd.workspace_bytes(1, 4, 2, 8, 512, 64, flashd.BF16, flashd.VARIANT_PER_KEY, 4)
    assert need == 4 * 1 * 4 * 8 * (64 + 2) * 4
    assert flashd.workspace_bytes(1, 4, 2, 8, 512, 64, flashd.BF16, flashd.VARIANT_PER_KEY, 1) == 0
    assert fwd_ex(variant=flashd.VARIANT_PER_KEY, splits=4) == E_WS
    assert fwd_ex(variant=flashd.VARIANT_PER_KEY, splits=4, ws=P, ws_bytes=need - 1) == E_WS
    # invalid problems have no workspace size
    assert flashd.workspace_bytes(1, 5, 2, 8, 512, 64, flashd.BF16, 0, 4) == 0
    assert flashd.workspace_bytes(1, 4, 2, 8, 512, 48, flashd.BF16, 0, 4) == 0
    # the automatic choice never exceeds the documented limits
    for (B, Hq, Hkv, Lq, Lk, d, dt) in [(64, 32, 8, 1, 8192, 128, flashd.BF16),
                                        (1, 1, 1, 128, 128, 64, flashd.F32),
                                        (4, 32, 32, 2048, 2048, 128, flashd.BF16),
                                        (1, 8, 8, 1, 100, 64, flashd.F16)]:
        s = flashd.auto_splits(B, Hq, Hkv, Lq, Lk, d, dt)
        assert 1 <= s <= min(flashd.MAX_SPLITS, Lk)
        assert flashd.workspace_bytes(B, Hq, Hkv, Lq, Lk, d, dt, 0, 0) == \
            flashd.workspace_bytes(B, Hq, Hkv, Lq, Lk, d, dt, 0, s)


def test_automatic_splits_follow_the_size_of_the_partial_states():
    # few query rows in all: short key ranges per split are worth it
    assert flashd.auto_splits(4, 8, 1, 8, 4096, 128, flashd.BF16) >= 8
    # one row tile of partial states per 128 rows: a split must keep 2048 keys
    assert flashd.auto_splits(1, 32, 32, 1024, 1024, 128, flashd.BF16) == 1
    assert flashd.auto_splits(4, 32, 32, 2048, 2048, 128, flashd.BF16) == 1
    assert flashd.auto_splits(1, 32, 8, 128, 32768, 128, flashd.BF16) == 16
    # decode: 256 keys are enough, and one round of 512 workgroups is the aim
    assert flashd.auto_splits(1, 32, 8, 1, 32768, 128, flashd.BF16) == 64
    assert flashd.auto_splits(64, 32, 8, 1, 8192, 128, flashd.BF16) == 1


def test_automatic_choice_of_the_prefill_kernel():
    V, BF, F16 = flashd.auto_variant, flashd.BF16, flashd.F16
    T, W = flashd.VARIANT_TILE, flashd.VARIANT_TILE_256
    assert V(1, 32, 32, 16384, 16384, 128, BF, False) == W     # long, no mask
    assert V(4, 32, 32, 2048, 2048, 128, BF, False) == W       # 2048 keys are enough without a mask
    assert V(4, 32, 32, 2048, 2048, 128, BF, True) == W        # the headline shape: two whole rounds of pairs
    assert V(3, 32, 32, 2048, 2048, 128, BF, True) == T        # a round and a half
    assert V(1, 32, 32, 2048, 2048, 128, BF, True) == T        # half the compute units
    assert V(1, 32, 32, 4096, 4096, 128, BF, True) == W        # rows see 2048 keys on average
    assert V(2, 32, 32, 3072, 3072, 128, BF, True) == W        # 1536 on average
    assert V(8, 32, 8, 512, 2048, 128, BF, True) == W          # short queries late in a long context
    assert V(8, 32, 32, 1024, 1024, 128, BF, True) == T
    assert V(1, 32, 32, 8192, 8192, 128, F16, True) == W       # 8192 keys under a causal mask
    assert V(1, 8, 8, 8192, 8192, 128, BF, True) == T          # 256 workgroups: too few with a mask
    assert V(1, 8, 8, 8192, 8192, 128, BF, False) == W
    assert V(1, 16, 16, 2048, 2048, 128, BF, False) == T       # 128 workgroups
    assert V(1, 32, 32, 1024, 1024, 128, BF, False) == T       # short rows of keys
    assert V(4, 32, 32, 1536, 1536, 128, BF, False) == W
    assert V(2, 16, 16, 4096, 4096, 64, F16, False) == T       # d = 64
    assert V(1, 32, 32, 4000, 4096, 128, BF, False) == W       # Lq need not be a multiple of 256
    assert V(1, 4, 4, 128, 128, 64, flashd.F32, False) == flashd.VARIANT_PER_KEY
    assert V(64, 32, 8, 1, 8192, 128, BF, False) == T          # decode shape
    assert V(1, 32, 32, 0, 4096, 128, BF, False) == -1
    assert V(1, 32, 32, 4096, 4096, 128, 7, False) == -1


@pytest.mark.skipif(torch.cuda.is_available(), reason="only meaningful on a machine without a GPU")
def test_valid_arguments_without_a_gpu_report_hip_error():
    assert fwd() == E_HIP


def test_binding_rejects_cpu_tensors():
    q = torch.zeros(1, 1, 4, 64)
    with pytest.raises(ValueError):
        flashd.attn_fwd(q, q, q, q, False, 1.0)


def stats(q=P, k=P, counts=P, B=1, Hq=4, Hkv=2, Lq=8, Lk=512, d=64, dtype=flashd.BF16):
    return flashd.raw().flashd_skip_stats(q, k, B, Hq, Hkv, Lq, Lk, d, 0, 1.0, dtype, -6.0, 11.0,
                                          counts, None)


def test_skip_stats_argument_errors():
    for name in ("q", "k", "counts"):
        assert stats(**{name: None}) == E_NULL
    assert stats(Lk=0) == E_SHAPE
    assert stats(dtype=7) == E_DTYPE
    assert stats(d=80) == E_HEADDIM
    assert stats(Hq=5) == E_GQA
    assert stats(q=P + 8) == E_ALIGN
    assert stats(counts=P + 4) == E_ALIGN
    if NO_GPU:
        assert stats(counts=P + 8) == E_HIP        # 8-byte alignment is enough for the counters


def fwd_state(q=P, k=P, v=P, o=P, sin=None, sout=P, B=1, Hq=4, Hkv=2, Lq=8, Lk=512, d=64,
              dtype=flashd.BF16):
    return flashd.raw().flashd_attn_fwd_state(q, k, v, o, sin, sout, B, Hq, Hkv, Lq, Lk, d, 1, 0,
                                              1.0, dtype, None)


def test_state_entry_point_argument_errors():
    for name in ("q", "k", "v"):
        assert fwd_state(**{name: None}) == E_NULL
    assert fwd_state(o=None, sout=None) == E_NULL            # nothing to write
    if NO_GPU:
        assert fwd_state(o=None) == E_HIP and fwd_state(sout=None) == E_HIP
    assert fwd_state(Lq=0) == E_SHAPE
    assert fwd_state(d=96) == E_HEADDIM
    assert fwd_state(Hq=3) == E_GQA
    assert fwd_state(sin=P + 4) == E_ALIGN
    assert fwd_state(sout=P + 8) == E_ALIGN


def fwd_kv8(q=P, k=P, v=P, o=P, B=1, Hq=8, Hkv=2, Lq=1, Lk=512, d=128, dtype=flashd.BF16):
    return flashd.raw().flashd_attn_fwd_kv8(q, k, v, o, B, Hq, Hkv, Lq, Lk, d, 0, 1.0, 1.0, 1.0,
                                            dtype, None)


def test_fp8_entry_point_argument_errors():
    for name in ("q", "k", "v", "o"):
        assert fwd_kv8(**{name: None}) == E_NULL
    assert fwd_kv8(Lk=0) == E_SHAPE
    assert fwd_kv8(d=72) == E_HEADDIM
    assert fwd_kv8(Hq=7) == E_GQA
    assert fwd_kv8(k=P + 8) == E_ALIGN
    assert fwd_kv8(dtype=flashd.F32) == E_VARIANT            # q and o must be f16 or bf16
    if NO_GPU:
        assert fwd_kv8(Hq=8, Hkv=2, Lq=9) == E_HIP


def test_header_is_plain_c_and_links_from_a_c_program(tmp_path):
    """A C99 program (no C++, no HIP headers) includes flashd.h, links against the shared
    library and calls the entry points that need no GPU."""
    import subprocess
    src = tmp_path / "consumer.c"
    src.write_text(r'''
#include <stdio.h>
#include <string.h>
#include "flashd.h"
int main(void) {
    unsigned long long counts[3];
    if (flashd_version() < 100) return 1;
    if (strcmp(flashd_status_string(FLASHD_OK), flashd_status_string(FLASHD_E_NULL)) == 0) return 2;
    if (flashd_attn_fwd(NULL, NULL, NULL, NULL, 1, 1, 1, 1, 1, 64, 0, 1.0f, FLASHD_BF16, NULL)
        != FLASHD_E_NULL) return 3;
    if (flashd_skip_stats(NULL, NULL, 1, 1, 1, 1, 1, 64, 0, 1.0f, FLASHD_F32, -6.0f, 11.0f,
                          counts, NULL) != FLASHD_E_NULL) return 4;
    if (flashd_workspace_bytes(1, 4, 2, 8, 512, 64, FLASHD_BF16, FLASHD_VARIANT_PER_KEY, 4)
        != (size_t)4 * 4 * 8 * 66 * 4) return 5;
    printf("ok %d\n", flashd_version());
    return 0;
}
''')
    exe = tmp_path / "consumer"
    libdir = os.path.dirname(flashd.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic",
                    "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                    "-L", libdir, "-l:" + os.path.basename(flashd.LIB_PATH),
                    "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    assert out.startswith("ok ")
