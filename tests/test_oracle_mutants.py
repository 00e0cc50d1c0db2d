"""The pins must be able to fail: plant plausible mistakes in a COPY of the oracle
source (on the CPU, in a temp dir), compile it, and check that at least one pin of
a compact battery rejects every mutant, while the unmodified source passes all."""
import os
import re
import subprocess

import numpy as np
import pytest
from scipy.special import softmax

import oracle
import workloads as wl

SRC = open(os.path.join(os.path.dirname(oracle.__file__), "attn_oracle.c")).read()

# (name, text to find, replacement)
MUTANTS = [
    ("no_scale", "score[c] = scale * dot;", "score[c] = dot;"),
    ("no_max_subtraction", "score[c] = exp(score[c] - m);", "score[c] = exp(score[c]);"),
    ("no_normalisation", "double p = score[c] / Z;", "double p = score[c];"),
    ("mask_transposed", "mask + ((size_t)bh * nb + (size_t)(r / block)) * nb : NULL;\n            attn_row(q + base + (size_t)r * D, k + base, v + base, mrow, block,\n                     kv_len, D, scale, score, out);\n        }\n        free(score);\n    }\n    return failed ? -7 : 0;\n}\n\n/*\n * Selected",
     "mask + ((size_t)bh * nb + (size_t)(r / block)) : NULL;\n            attn_row(q + base + (size_t)r * D, k + base, v + base, mrow, block,\n                     kv_len, D, scale, score, out);\n        }\n        free(score);\n    }\n    return failed ? -7 : 0;\n}\n\n/*\n * Selected"),
    ("mask_block_index_by_row", "(mask_row[c / block] != 0)", "(mask_row[c % block % 2] != 0)"),
    # every loop of the row routine runs over all N allocated keys (stays inside the arrays)
    ("pad_keys_included", "                     kv_len, D, scale, score, out);\n        }\n        free(score);\n    }\n    return failed ? -7 : 0;\n}\n\n/*\n * Selected",
     "                     N, D, scale, score, out);\n        }\n        free(score);\n    }\n    return failed ? -7 : 0;\n}\n\n/*\n * Selected"),
    ("k_transposed_index", "bf16_to_f64(k[(size_t)c * D + d]);", "bf16_to_f64(k[(size_t)d * D + c]);"),
    ("v_wrong_row", "out[d] += p * bf16_to_f64(v[(size_t)c * D + d]);", "out[d] += p * bf16_to_f64(v[(size_t)(c ^ 1) * D + d]);"),
    ("softmax_sign", "score[c] = exp(score[c] - m);", "score[c] = exp(m - score[c]);"),
    ("mask_after_softmax", "if (!allowed) { score[c] = -INFINITY; continue; }", "if (!allowed) { score[c] = -1e-300; continue; }"),
    ("head_stride_dropped", "const size_t base = (size_t)bh * N * D;", "const size_t base = (size_t)(bh / H) * H * N * D;"),
    ("bf16_low_half", "uint32_t w = ((uint32_t)bits) << 16;", "uint32_t w = ((uint32_t)bits) << 15;"),
    ("pad_query_not_zeroed", "if (r >= kv_len) { for (int d = 0; d < D; ++d) out[d] = 0.0; continue; }\n            const size_t base",
     "if (r > kv_len) { for (int d = 0; d < D; ++d) out[d] = 0.0; continue; }\n            const size_t base"),
]


def widen(bits):
    return wl.bf16_bits_to_f32(bits).astype(np.float64)


def brute(q, k, v, kv_len, mask, block):
    B, H, N, D = q.shape
    live = (np.arange(N) < kv_len)
    Q, K, V = (np.where(live[None, None, :, None], widen(x), 0.0) for x in (q, k, v))
    allowed = np.kron(mask, np.ones((block, block), np.uint8)).astype(bool) & live
    S = np.matmul(Q, K.transpose(0, 1, 3, 2)) / np.sqrt(D) + np.where(allowed, 0.0, -np.inf)
    empty = ~allowed.any(-1)
    S[empty] = 0.0
    O = np.matmul(softmax(S, axis=-1), V)
    O[empty] = 0.0
    O[:, :, kv_len:] = 0.0
    return O


def battery(lib):
    """Names of the pins that `lib` fails."""
    failed = []

    def check(name, ok):
        if not ok:
            failed.append(name)

    B, H, N, D, block, kv_len = 2, 2, 192, 64, 64, 150
    q, k, v = wl.make_qkv(B, H, N, D, kv_len, seed=41, pad_fill="nan")
    mask = wl.mask_bernoulli_diag(B, H, 3, 0.4, 5)
    mask[0, 0] = [[1, 0, 1], [1, 1, 0], [0, 0, 1]]          # asymmetric on purpose
    with np.errstate(all="ignore"):
        o = oracle.attention(q, k, v, kv_len, mask, block, lib=lib)
        check("P1 brute force", np.allclose(o, brute(q, k, v, kv_len, mask, block), atol=1e-12, rtol=0))
        v1 = np.full_like(v, wl.BF16_ONE)
        o1 = oracle.attention(q, k, v1, kv_len, mask, block, lib=lib)
        check("P3 rows sum to one", np.allclose(o1[:, :, :kv_len], 1.0, atol=1e-13))
        check("S8 pad rows zero", bool((o[:, :, kv_len:] == 0).all()))
        k2, v2 = k.copy(), v.copy()
        k2[0, 0, 64:128], v2[0, 0, 64:128] = wl.BF16_INF, wl.BF16_NAN
        m5 = mask.copy()
        m5[0, 0, :, 1] = 0
        a = oracle.attention(q, k, v, kv_len, m5, block, lib=lib)
        b = oracle.attention(q, k2, v2, kv_len, m5, block, lib=lib)
        check("P5 masked blocks ignored", np.array_equal(a, b))
        qp, kp, vp = wl.make_qkv(1, 1, 64, 64, seed=42, gain=24.0)
        op = oracle.attention(qp, kp, vp, lib=lib)
        check("P12 peaky finite", bool(np.isfinite(op).all())
              and np.allclose(op, brute(qp, kp, vp, 64, np.ones((1, 1, 1, 1), np.uint8), 64), atol=1e-12))
    return failed


def compile_variant(tmp_path, name, text):
    src = tmp_path / f"{name}.c"
    so = tmp_path / f"{name}.so"
    src.write_text(text)
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-o", str(so),
                    str(src), "-lm"], check=True)
    return oracle.load(str(so))


def test_unmodified_source_passes_battery(tmp_path):
    assert battery(compile_variant(tmp_path, "clean", SRC)) == []


@pytest.mark.parametrize("name,find,repl", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_mutant_is_caught(tmp_path, name, find, repl):
    assert SRC.count(find) >= 1, f"mutation site for {name} not found in oracle source"
    text = SRC.replace(find, repl, 1)
    assert text != SRC
    failed = battery(compile_variant(tmp_path, re.sub(r"\W", "_", name), text))
    assert failed, f"mutant {name} survived every pin"
