"""Do the pins bite?  Each case below plants one plausible mistake in a copy of the C oracle
(a dropped term, a wrong sign or index, swapped operands), builds that copy on its own and
checks that an independent fp64 reference (torch's softmax written out here, not the oracle)
rejects it -- and that the unmodified source passes the same checks.  CPU only; nothing of
the product is involved."""
import ctypes
import os
import subprocess

import numpy as np
import pytest
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "attn_oracle.c")

# (name, text in the source, its replacement, algos whose result must change)
MUTANTS = [
    ("causal off by one", "+ ((long)p->Lk - (long)p->Lq) + 1;", "+ ((long)p->Lk - (long)p->Lq);",
     (0, 1, 2, 3)),
    ("causal aligned top-left", "+ ((long)p->Lk - (long)p->Lq) + 1;", "+ 1;", (0, 1, 2, 3)),
    ("scale dropped", "return p->scale * acc;", "return acc;", (0, 1, 2, 3)),
    ("dot product one element short", "for (int t = 0; t < p->d; ++t) acc +=",
     "for (int t = 1; t < p->d; ++t) acc +=", (0, 1, 2, 3)),
    ("kv head of a query head", "((size_t)b * Hkv + h / g) * (size_t)Lk * d;\n            const float *V",
     "((size_t)b * Hkv + h % Hkv) * (size_t)Lk * d;\n            const float *V", (0, 1, 2, 3)),
    ("values of the wrong kv head", "const float *V = v + ((size_t)b * Hkv + h / g)",
     "const float *V = v + ((size_t)b * Hkv + h % Hkv)", (0, 1, 2, 3)),
    ("row index decoded with the wrong head count", "h = (int)((r / Lq) % Hq);",
     "h = (int)((r / Lq) % Hkv);", (0, 1, 2, 3)),
    ("definition: denominator misses the last key",
     "for (long j = 0; j < n; ++j) den += exp(s[j] - mx);",
     "for (long j = 0; j + 1 < n; ++j) den += exp(s[j] - mx);", (0,)),
    ("definition: weights not normalised", "double f = exp(s[j] - mx) / den;",
     "double f = exp(s[j] - mx);", (0,)),
    ("alg1: carry and fresh swapped",
     "out[t] = out[t] * (carry / ln) + (double)vr[t] * (fresh / ln);",
     "out[t] = out[t] * (fresh / ln) + (double)vr[t] * (carry / ln);", (1,)),
    ("alg1: running sum forgets its rescale", "double carry = l * exp(m - mn);",
     "double carry = l;", (1,)),
    ("alg2: output not rescaled", "out[t] = out[t] * resc + (double)vr[t] * fresh;",
     "out[t] = out[t] + (double)vr[t] * fresh;", (2,)),
    ("alg2: final division dropped", "for (int t = 0; t < d; ++t) out[t] /= l;",
     "for (int t = 0; t < d; ++t) out[t] /= 1.0;", (2,)),
    ("alg3: minus sign of the algorithm box", "double x = sj - s_prev + lnw;",
     "double x = sj - s_prev - lnw;", (3,)),
    ("alg3: ln w not carried", "lnw = log_sigmoid(x);", "lnw = 0.0;", (3,)),
    ("alg3: previous score not updated", "        s_prev = sj;\n    }\n}\n\nint oracle_attn",
     "    }\n}\n\nint oracle_attn", (3,)),
    ("alg3: blend with the wrong sign", "out[t] += ((double)vr[t] - out[t]) * w;",
     "out[t] += ((double)vr[t] + out[t]) * w;", (3,)),
    ("alg3: first weight not one", "            w = 1.0;\n            lnw = 0.0;",
     "            w = 0.5;\n            lnw = 0.0;", (3,)),
    ("ln sigma: dropped x on the negative side", "return x - log1p(exp(x));",
     "return -log1p(exp(x));", (3,)),
    ("sigma: wrong branch value", "return e / (1.0 + e);", "return 1.0 / (1.0 + e);", (3,)),
]


def build(tmp_path, text, tag):
    src = tmp_path / f"attn_{tag}.c"
    lib = tmp_path / f"liboracle_{tag}.so"
    src.write_text(text)
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-fno-fast-math",
                    "-o", str(lib), str(src), "-lm"], check=True)
    h = ctypes.CDLL(str(lib))
    h.oracle_attn.restype = ctypes.c_int
    h.oracle_attn.argtypes = [
        ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
        ctypes.c_int, ctypes.c_float, ctypes.c_void_p, ctypes.c_long]
    return h


def cases():
    """Small problems with GQA, Lq != Lk both ways, causal and not; scores of moderate size."""
    rng = np.random.default_rng(7)
    out = []
    for (B, Hq, Hkv, Lq, Lk, d, causal) in [(2, 4, 2, 5, 9, 8, True), (1, 4, 2, 7, 4, 6, True),
                                            (2, 6, 3, 3, 8, 5, False)]:
        q = rng.standard_normal((B, Hq, Lq, d)).astype(np.float32)
        k = rng.standard_normal((B, Hkv, Lk, d)).astype(np.float32)
        v = rng.standard_normal((B, Hkv, Lk, d)).astype(np.float32)
        out.append((q, k, v, causal, np.float32(0.37)))
    return out


def reference(q, k, v, causal, scale):
    """softmax(scale q k^T + mask) v in fp64 with torch, kv heads repeated for the query heads."""
    g = q.shape[1] // k.shape[1]
    qq = torch.from_numpy(q).double()
    kk = torch.from_numpy(k).double().repeat_interleave(g, dim=1)
    vv = torch.from_numpy(v).double().repeat_interleave(g, dim=1)
    s = float(scale) * qq @ kk.transpose(-1, -2)
    Lq, Lk = q.shape[2], k.shape[2]
    if causal:
        i = torch.arange(Lq)[:, None]
        j = torch.arange(Lk)[None, :]
        s = s.masked_fill(j > i + (Lk - Lq), float("-inf"))
    p = torch.softmax(s, dim=-1)
    p = torch.nan_to_num(p, nan=0.0)            # rows that see no key: zeros
    return (p @ vv).numpy()


def worst_error(lib, algo):
    worst = 0.0
    for q, k, v, causal, scale in cases():
        B, Hq, Lq, d = q.shape
        _, Hkv, Lk, _ = k.shape
        o = np.full((B, Hq, Lq, d), np.nan)
        rc = lib.oracle_attn(algo, q.ctypes.data, k.ctypes.data, v.ctypes.data, o.ctypes.data,
                             B, Hq, Hkv, Lq, Lk, d, int(causal), float(scale), None, 0)
        assert rc == 0
        err = np.abs(o - reference(q, k, v, causal, scale))
        worst = max(worst, float(np.nan_to_num(err, nan=np.inf).max()))
    return worst


def test_unmodified_source_passes(tmp_path):
    lib = build(tmp_path, open(SRC).read(), "orig")
    for algo in range(4):
        assert worst_error(lib, algo) < 1e-12, algo


@pytest.mark.parametrize("name,old,new,algos", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, name, old, new, algos):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site of '{name}' not found exactly once"
    lib = build(tmp_path, text.replace(old, new), "mut")
    for algo in algos:
        assert worst_error(lib, algo) > 1e-6, f"'{name}' slips through for algo {algo}"
