"""Do the pins of the state oracle and of the skip-statistics oracle bite?  As for the
attention oracle: one plausible mistake is planted in a copy of the C source, the copy is
built on its own, and a reference written out here independently (torch's softmax and
logsumexp in fp64; exact integer arithmetic for the counts) must reject it, while the
unmodified source passes.  CPU only; nothing of the product is involved."""
import ctypes
import os
import subprocess

import numpy as np
import pytest
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE = os.path.join(os.path.dirname(HERE), "oracle")
STATE_SRC = os.path.join(ORACLE, "state_oracle.c")
SKIP_SRC = os.path.join(ORACLE, "skip_oracle.c")


def compile_copy(tmp_path, text, tag):
    src = tmp_path / f"{tag}.c"
    lib = tmp_path / f"lib{tag}.so"
    src.write_text(text)
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-fno-fast-math",
                    "-ffp-contract=off", "-o", str(lib), str(src), "-lm"], check=True)
    return ctypes.CDLL(str(lib))


# ---------------------------------------------------------------- state in / out

STATE_MUTANTS = [
    ("state handed in is ignored", "if (in[d] != -INFINITY) {", "if (0) {"),
    ("ln w of the state handed in is dropped", "lnw = in[d + 1];", "lnw = 0.0;"),
    ("s of the state handed in is dropped", "s_prev = in[d];", "s_prev = 0.0;"),
    ("o of the state handed in is dropped", "for (int t = 0; t < d; ++t) out[t] = in[t];",
     "for (int t = 0; t < d; ++t) out[t] = 0.0;"),
    ("causal shift ignored", "nvis = (long)i + (long)shift + 1;", "nvis = (long)i + 1;"),
    ("causal shift off by one", "nvis = (long)i + (long)shift + 1;",
     "nvis = (long)i + (long)shift;"),
    ("minus sign of the algorithm box", "const double x = s - s_prev + lnw;",
     "const double x = s - s_prev - lnw;"),
    ("ln w not carried", "lnw = lw;", "lnw = 0.0;"),
    ("previous score not updated", "                    s_prev = s;\n", ""),
    ("first key not taken whole", "for (int t = 0; t < d; ++t) out[t] = (double)vrow[t];",
     "for (int t = 0; t < d; ++t) out[t] = 0.5 * (double)vrow[t];"),
    ("keys of the wrong kv head", "const float *kh = k + ((size_t)b * Hkv + h / g)",
     "const float *kh = k + ((size_t)b * Hkv + h % Hkv)"),
    ("values of the wrong kv head", "const float *vh = v + ((size_t)b * Hkv + h / g)",
     "const float *vh = v + ((size_t)b * Hkv + h % Hkv)"),
    ("blend with the wrong sign", "out[t] += ((double)vrow[t] - out[t]) * w;",
     "out[t] += ((double)vrow[t] + out[t]) * w;"),
    ("ln sigma: dropped x on the negative side", "lw = x - log1p(e);", "lw = -log1p(e);"),
    ("sigma: wrong value on the negative side", "w = e / (1.0 + e);", "w = 1.0 / (1.0 + e);"),
    ("scale dropped", "const double s = sc * dot;", "const double s = dot;"),
    ("s and ln w swapped on the way out", "out[d] = s_prev;\n                out[d + 1] = lnw;",
     "out[d] = lnw;\n                out[d + 1] = s_prev;"),
]


def state_lib(tmp_path, text, tag):
    h = compile_copy(tmp_path, text, tag)
    h.oracle_attn_state.restype = ctypes.c_int
    h.oracle_attn_state.argtypes = [ctypes.c_void_p] * 5 + [ctypes.c_int] * 8 + [ctypes.c_float]
    return h


def state_cases():
    rng = np.random.default_rng(11)
    out = []
    # (B, Hq, Hkv, Lq, Lk, d, causal, cut): the keys are fed as [0, cut) and [cut, Lk)
    for (B, Hq, Hkv, Lq, Lk, d, causal, cut) in [(2, 4, 2, 5, 9, 8, True, 4),
                                                 (1, 4, 2, 7, 5, 6, True, 2),
                                                 (2, 6, 3, 3, 8, 5, False, 3)]:
        q = rng.standard_normal((B, Hq, Lq, d)).astype(np.float32)
        k = rng.standard_normal((B, Hkv, Lk, d)).astype(np.float32)
        v = rng.standard_normal((B, Hkv, Lk, d)).astype(np.float32)
        out.append((q, k, v, causal, np.float32(0.61), cut))
    return out


def state_reference(q, k, v, causal, scale):
    """(o, logsumexp of the visible scores, score of the last visible key) per row, fp64."""
    g = q.shape[1] // k.shape[1]
    qq = torch.from_numpy(q).double()
    kk = torch.from_numpy(k).double().repeat_interleave(g, dim=1)
    vv = torch.from_numpy(v).double().repeat_interleave(g, dim=1)
    s = float(scale) * qq @ kk.transpose(-1, -2)
    Lq, Lk = q.shape[2], k.shape[2]
    nvis = torch.full((Lq,), Lk)
    if causal:
        i = torch.arange(Lq)[:, None]
        j = torch.arange(Lk)[None, :]
        s = s.masked_fill(j > i + (Lk - Lq), float("-inf"))
        nvis = torch.clamp(torch.arange(Lq) + (Lk - Lq) + 1, 0, Lk)
    lse = torch.logsumexp(s, dim=-1)
    p = torch.nan_to_num(torch.softmax(s, dim=-1), nan=0.0)
    last = torch.full(s.shape[:-1], float("-inf"), dtype=torch.float64)
    for r in range(Lq):
        if nvis[r] > 0:
            last[..., r] = s[..., r, nvis[r] - 1]
    return (p @ vv).numpy(), lse.numpy(), last.numpy()


def state_worst_error(lib):
    worst = 0.0
    for q, k, v, causal, scale, cut in state_cases():
        B, Hq, Lq, d = q.shape
        _, Hkv, Lk, _ = k.shape
        k1, v1 = np.ascontiguousarray(k[:, :, :cut]), np.ascontiguousarray(v[:, :, :cut])
        k2, v2 = np.ascontiguousarray(k[:, :, cut:]), np.ascontiguousarray(v[:, :, cut:])
        st1 = np.full((B, Hq, Lq, d + 2), np.nan)
        st2 = np.full((B, Hq, Lq, d + 2), np.nan)
        rc = lib.oracle_attn_state(q.ctypes.data, k1.ctypes.data, v1.ctypes.data, None,
                                   st1.ctypes.data, B, Hq, Hkv, Lq, cut, d, int(causal),
                                   Lk - Lq, float(scale))
        assert rc == 0
        rc = lib.oracle_attn_state(q.ctypes.data, k2.ctypes.data, v2.ctypes.data,
                                   st1.ctypes.data, st2.ctypes.data, B, Hq, Hkv, Lq, Lk - cut, d,
                                   int(causal), Lk - Lq - cut, float(scale))
        assert rc == 0
        o, lse, last = state_reference(q, k, v, causal, scale)
        lam = st2[..., d] - st2[..., d + 1]
        with np.errstate(invalid="ignore"):    # -inf - -inf for rows without keys, masked out
            err = [np.abs(st2[..., :d] - o), np.abs(np.where(np.isneginf(lse), 0.0, lam - lse)),
                   (np.isneginf(lam) != np.isneginf(lse)).astype(float),
                   np.abs(np.where(np.isneginf(last), 0.0, st2[..., d] - last))]
        # the first chunk alone is attention over its keys: checks the state that is handed on
        o1, lse1, _ = state_reference(q, k1, v1, False, scale) if not causal else (None,) * 3
        if o1 is not None:
            err.append(np.abs(st1[..., :d] - o1))
            err.append(np.abs((st1[..., d] - st1[..., d + 1]) - lse1))
        for e in err:
            worst = max(worst, float(np.nan_to_num(e, nan=np.inf).max()))
    return worst


def test_unmodified_state_oracle_passes(tmp_path):
    assert state_worst_error(state_lib(tmp_path, open(STATE_SRC).read(), "state_orig")) < 1e-12


@pytest.mark.parametrize("name,old,new", STATE_MUTANTS, ids=[m[0] for m in STATE_MUTANTS])
def test_planted_mistake_in_the_state_oracle_is_caught(tmp_path, name, old, new):
    text = open(STATE_SRC).read()
    assert text.count(old) == 1, f"mutation site of '{name}' not found exactly once"
    lib = state_lib(tmp_path, text.replace(old, new), "state_mut")
    assert state_worst_error(lib) > 1e-6, f"'{name}' slips through"


# ---------------------------------------------------------------- skip statistics

SKIP_MUTANTS = [
    ("the first key counted as a step", "if (j > 0) {", "if (1) {"),
    ("low end of the range taken as open", "if (diff <= lo) ++low;", "if (diff < lo) ++low;"),
    ("high end of the range taken as open", "if (diff >= hi) ++high;", "if (diff > hi) ++high;"),
    ("difference taken the other way round", "const float diff = s - prev;",
     "const float diff = prev - s;"),
    ("previous score not updated", "                    prev = s;\n", ""),
    ("causal rule off by one", "((long)Lk - (long)Lq) + 1;", "((long)Lk - (long)Lq);"),
    ("causal rule aligned top-left", "nvis = (long)i + ((long)Lk - (long)Lq) + 1;",
     "nvis = (long)i + 1;"),
    ("keys of the wrong kv head", "h / g) * (size_t)Lk * d;", "h % Hkv) * (size_t)Lk * d;"),
    ("scale dropped", "const float s = acc * scale;", "const float s = acc;"),
    ("dot product one element short", "for (int t = 0; t < d; ++t) acc = fmaf",
     "for (int t = 1; t < d; ++t) acc = fmaf"),
    ("low steps counted as high", "if (diff <= lo) ++low;", "if (diff <= lo) ++high;"),
    ("steps not counted", "                        ++steps;\n", ""),
]


def skip_lib(tmp_path, text, tag):
    h = compile_copy(tmp_path, text, tag)
    h.oracle_skip_stats.restype = ctypes.c_int
    h.oracle_skip_stats.argtypes = [ctypes.c_void_p] * 2 + [ctypes.c_int] * 7 + \
        [ctypes.c_float] * 3 + [ctypes.c_void_p]
    return h


def skip_cases():
    """Small integers as inputs and scale 1/2: every product, sum and difference is exact in
    fp32, so exact integer arithmetic is a reference, and differences land exactly on the
    ends of the range (both ends must count, Sec. III-C)."""
    rng = np.random.default_rng(5)
    out = []
    for (B, Hq, Hkv, Lq, Lk, d, causal) in [(2, 4, 2, 6, 40, 4, True), (1, 6, 3, 9, 5, 3, True),
                                            (2, 2, 1, 4, 50, 4, False)]:
        q = rng.integers(-3, 4, (B, Hq, Lq, d))
        k = rng.integers(-3, 4, (B, Hkv, Lk, d))
        out.append((q, k, causal))
    return out


def skip_reference(q, k, causal, lo2, hi2):
    """Counts with twice the scores as integers (scale 1/2): (steps, low, high, hits on an end)."""
    B, Hq, Lq, d = q.shape
    _, Hkv, Lk, _ = k.shape
    g = Hq // Hkv
    steps = low = high = ends = 0
    for b in range(B):
        for h in range(Hq):
            for i in range(Lq):
                nvis = min(max(i + (Lk - Lq) + 1, 0), Lk) if causal else Lk
                s2 = [int(np.dot(q[b, h, i], k[b, h // g, j])) for j in range(nvis)]
                for j in range(1, nvis):
                    diff2 = s2[j] - s2[j - 1]
                    steps += 1
                    low += diff2 <= lo2
                    high += diff2 >= hi2
                    ends += diff2 in (lo2, hi2)
    return steps, low, high, ends


def skip_mismatch(lib):
    bad, ends = 0, 0
    for q, k, causal in skip_cases():
        B, Hq, Lq, d = q.shape
        _, Hkv, Lk, _ = k.shape
        qf, kf = q.astype(np.float32), k.astype(np.float32)
        counts = np.zeros(3, dtype=np.uint64)
        rc = lib.oracle_skip_stats(qf.ctypes.data, kf.ctypes.data, B, Hq, Hkv, Lq, Lk, d,
                                   int(causal), 0.5, -6.0, 11.0, counts.ctypes.data)
        assert rc == 0
        st, lo, hi, e = skip_reference(q, k, causal, -12, 22)
        bad += tuple(int(c) for c in counts) != (st, lo, hi)
        ends += e
    return bad, ends


def test_unmodified_skip_oracle_passes_and_the_cases_hit_both_ends(tmp_path):
    bad, _ = skip_mismatch(skip_lib(tmp_path, open(SKIP_SRC).read(), "skip_orig"))
    assert bad == 0
    lows = highs = 0
    for q, k, causal in skip_cases():
        lows += skip_reference(q, k, causal, -12, 10 ** 9)[3]
        highs += skip_reference(q, k, causal, -10 ** 9, 22)[3]
    assert lows > 0 and highs > 0, "the cases must land on both ends of the range"


@pytest.mark.parametrize("name,old,new", SKIP_MUTANTS, ids=[m[0] for m in SKIP_MUTANTS])
def test_planted_mistake_in_the_skip_oracle_is_caught(tmp_path, name, old, new):
    text = open(SKIP_SRC).read()
    assert text.count(old) == 1, f"mutation site of '{name}' not found exactly once"
    bad, _ = skip_mismatch(skip_lib(tmp_path, text.replace(old, new), "skip_mut"))
    assert bad > 0, f"'{name}' slips through"
