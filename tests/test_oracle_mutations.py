"""The pins must bite: plant one plausible mistake at a time in a *copy* of the oracle's C
source (CPU only), build it, and check that the core pins reject it."""
import os
import subprocess
import sys

import pytest

from tests.oracle_core_pins import core_pins

MUTATIONS = {
    "kv head = h % Hkv": ("const int g = h / G;", "const int g = h % p->Hkv;"),
    "scale dropped": ("scores[t] = p->scale * acc;", "scores[t] = acc;"),
    "score sign": ("scores[t] = exp(scores[t] - smax);", "scores[t] = exp(smax - scores[t]);"),
    "slot/dim transposed": ("* p->BS + slot) * (int64_t)p->D + d;", "* p->D + d) * (int64_t)p->BS + slot;"),
    "head/block transposed": ("((phys * p->Hkv + g) * p->BS", "(((int64_t)g * p->NB + phys) * p->BS"),
    "table row stride": ("p->block_tables[(int64_t)b * p->MB + t / p->BS];\n        if",
                         "p->block_tables[(int64_t)b * (p->MB - 1) + t / p->BS];\n        if"),
    "token to block by modulo": ("int64_t phys = p->block_tables[(int64_t)b * p->MB + t / p->BS];\n        double w",
                                 "int64_t phys = p->block_tables[(int64_t)b * p->MB + t % p->BS];\n        double w"),
    "last token dropped": ("for (int t = t_first; t < L; ++t) {\n        scores[t] = exp",
                           "for (int t = t_first; t < L - 1; ++t) {\n        scores[t] = exp"),
    "unnormalised": ("double w = scores[t] / denom;", "double w = scores[t];"),
    "v uses k scale": ("load_kv(p, p->v_cache, p->v_scale,", "load_kv(p, p->v_cache, p->k_scale,"),
    "e4m3 bias 8": ("(int)expo - 7);", "(int)expo - 8);"),
    "e4m3 subnormal exponent": ("ldexp((double)mant / 8.0, -6);", "ldexp((double)mant / 8.0, -7);"),
    "e4m3 has infinities": ("if (expo == 0xFu && mant == 0x7u)", "if (expo == 0xFu)"),
    "q head stride": ("(((int64_t)b * Q + i) * Hq + h) * D;", "(((int64_t)b * Q + i) * Hq + h) * (D / 2);"),
    "window: token and head axes of q swapped": ("(((int64_t)b * Q + i) * Hq + h) * D;",
                                                 "(((int64_t)b * Hq + h) * Q + i) * D;"),
    "window: query sees one token too few": ("int visible = context_lens[b] - Q + 1 + i;",
                                             "int visible = context_lens[b] - Q + i;"),
    "window: query sees one token too many": ("int visible = context_lens[b] - Q + 1 + i;",
                                              "int visible = context_lens[b] - Q + 2 + i;"),
    "window: no causal mask": ("int visible = context_lens[b] - Q + 1 + i;", "int visible = context_lens[b];"),
    "window: order of the window reversed": ("int visible = context_lens[b] - Q + 1 + i;",
                                             "int visible = context_lens[b] - i;"),
    "sliding window one token too wide": ("? visible - window : 0;", "? visible - window - 1 : 0;"),
    "sliding window one token too narrow": ("? visible - window : 0;", "? visible - window + 1 : 0;"),
    "sliding window counted from the end of the context": ("? visible - window : 0;",
                                                           "? context_lens[b] - window : 0;"),
    "sliding window ignored in the value pass": ("for (int t = t_first; t < L; ++t) {\n        int64_t phys = p->block_tables[(int64_t)b * p->MB + t / p->BS];\n        double w",
                                                 "for (int t = 0; t < L; ++t) {\n        int64_t phys = p->block_tables[(int64_t)b * p->MB + t / p->BS];\n        double w"),
    "append: window written from the wrong end": ("int32_t t = context_lens[b] - Q + i;",
                                                   "int32_t t = context_lens[b] - 1 - i;"),
    "append: token and head axes of the new rows swapped": ("int64_t src = (((int64_t)b * Q + i) * Hkv + g) * D + d;",
                                                            "int64_t src = (((int64_t)b * Hkv + g) * Q + i) * D + d;"),
    "table check: id equal to the pool size accepted": ("if (id < 0 || id >= NB)", "if (id < 0 || id > NB)"),
    "table check: window start rounded up to the next block": ("for (int32_t t = t_first - t_first % BS; t < L; t += BS) {",
                                                               "for (int32_t t = t_first + (BS - t_first % BS) % BS; t < L; t += BS) {"),
    "table check: blocks of a refused length still looked at": ("                first[3] = L;\n            }\n            continue;",
                                                                "                first[3] = L;\n            }"),
    "table check: an odd prefix block counted as shared": ("int32_t shared = 2 * (prefix_blocks / 2);", "int32_t shared = prefix_blocks;"),
}


def test_unmutated_oracle_passes_core_pins(oracle):
    oracle.lib()
    core_pins(oracle)


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(oracle, tmp_path, name):
    old, new = MUTATIONS[name]
    src = open(os.path.join(os.path.dirname(oracle.__file__), "pa_oracle.c")).read()
    assert src.count(old) >= 1, f"mutation anchor not found: {old!r}"
    c = tmp_path / "mutant.c"
    so = tmp_path / "mutant.so"
    c.write_text(src.replace(old, new, 1))
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", str(so), str(c), "-lm"])
    # a mutant may read out of bounds, so it runs in a process of its own; any failure
    # (assertion, error code, crash) counts as caught
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    rc = subprocess.run([sys.executable, "-m", "tests.oracle_core_pins", str(so)], cwd=root,
                        stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL).returncode
    assert rc != 0, f"planted mistake {name!r} passed the core pins"
