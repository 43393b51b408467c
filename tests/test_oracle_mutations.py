"""Planted mistakes: every single-line mistake below, made in a COPY of the oracle's source (CPU only, in a
temporary directory), must make at least one pin of tests/test_oracle_pins.py fail.  This is the evidence that the
pins would catch a dropped term, a wrong sign, index, operand order, tie rule or rounding in the oracle."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "slimdp_oracle.c")

CMP_DESC = """return (x->key > y->key) ? -1 : 1;
    if (x->idx != y->idx) return (x->idx < y->idx) ? -1 : 1;
    return 0;
}
static int cmp_key_asc"""

MUTANTS = [
    ("score: multiply and add instead of one fused operation", "float s = fmaf(c, fabsf(gi), fabsf(w[i]));\n        if (s != s) {\n            uint32_t qnan = 0x7FC00000u;\n            memcpy(&s, &qnan, 4);\n        }\n        S[i] = s;\n    }\n}\n\n/* ---", "float s = c * fabsf(gi) + fabsf(w[i]);\n        if (s != s) {\n            uint32_t qnan = 0x7FC00000u;\n            memcpy(&s, &qnan, 4);\n        }\n        S[i] = s;\n    }\n}\n\n/* ---"),
    ("score: sum of magnitudes instead of magnitude of the sum", "gi = gi + g[k][i];", "gi = fabsf(gi) + fabsf(g[k][i]);"),
    ("score: |w| dropped", "float s = fmaf(c, fabsf(gi), fabsf(w[i]));\n        if (s != s) {\n            uint32_t qnan = 0x7FC00000u;\n            memcpy(&s, &qnan, 4);\n        }\n        S[i] = s;\n    }\n}\n\n/* ---", "float s = fmaf(c, fabsf(gi), w[i]);\n        if (s != s) {\n            uint32_t qnan = 0x7FC00000u;\n            memcpy(&s, &qnan, 4);\n        }\n        S[i] = s;\n    }\n}\n\n/* ---"),
    ("core: ascending instead of descending", CMP_DESC, CMP_DESC.replace("(x->key > y->key)", "(x->key < y->key)")),
    ("core: ties to the higher index", CMP_DESC, CMP_DESC.replace("(x->idx < y->idx)", "(x->idx > y->idx)")),
    ("explorer: word index reversed", "return out[i & 3u];", "return out[3u - (i & 3u)];"),
    ("explorer: worker and iteration swapped in the counter", "{ i >> 2, worker, (uint32_t)iteration, (uint32_t)(iteration >> 32) }", "{ i >> 2, (uint32_t)iteration, worker, (uint32_t)(iteration >> 32) }"),
    ("explorer: core not excluded", "if (in_core[i]) continue;", "if (0) continue;"),
    ("explorer: largest words instead of smallest", "qsort(p, cnt, sizeof(pair_t), cmp_key_asc_idx_asc);", "qsort(p, cnt, sizeof(pair_t), cmp_key_desc_idx_asc);"),
    ("merge: sign", "w[i] = fmaf(-lr, scratch_acc[i], w[i]);", "w[i] = fmaf(lr, scratch_acc[i], w[i]);"),
    ("merge: two roundings", "w[i] = fmaf(-lr, scratch_acc[i], w[i]);", "w[i] = w[i] - lr * scratch_acc[i];"),
    ("merge: untouched entries written", "if (scratch_hit[i]) w[i] = fmaf", "w[i] = fmaf"),
    ("merge: explorer value replaces instead of adds", "scratch_acc[i] = scratch_acc[i] + expl_val[wk][j];", "scratch_acc[i] = expl_val[wk][j];"),
    ("philox: multipliers swapped", "uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;", "uint64_t p0 = (uint64_t)0xCD9E8D57u * (uint64_t)c0;"),
    ("pull: local model not overwritten at the explorer", "if (w_local) w_local[expl_idx[j]] = expl_out[j];", ";"),
    ("pack: explorer values read at a shifted index", "expl_val[j] = g_k[expl_idx[j]];", "expl_val[j] = g_k[expl_idx[j] ^ 1u];"),
    ("dense update: significance of the OLD model", "w[i] = fmaf(-lr, acc, w[i]);\n        float s = fmaf(c, fabsf(acc), fabsf(w[i]));", "float wo = w[i]; w[i] = fmaf(-lr, acc, w[i]);\n        float s = fmaf(c, fabsf(acc), fabsf(wo));"),
    ("signature: position not mixed in", "sig += oracle_splitmix64_mix((uint64_t)core_idx[j] + (j << 32));", "sig += oracle_splitmix64_mix((uint64_t)core_idx[j]);"),
    ("local step: sign of the step", "w_local[i] = fmaf(-eta, grad[i], w_local[i]);", "w_local[i] = fmaf(eta, grad[i], w_local[i]);"),
    ("local step: a new accumulation keeps the old one", "delta[i] = first ? grad[i] : delta[i] + grad[i];", "delta[i] = delta[i] + grad[i];"),
    ("local step: two roundings", "w_local[i] = fmaf(-eta, grad[i], w_local[i]);", "w_local[i] = w_local[i] - eta * grad[i];"),
    ("quantiser: rounds up when it should not", "level = (uint32_t)l + (u < frac ? 1u : 0u);", "level = (uint32_t)l + (u > frac ? 1u : 0u);"),
    ("quantiser: nearest instead of random rounding", "level = (uint32_t)l + (u < frac ? 1u : 0u);", "level = (uint32_t)l + (0.5f < frac ? 1u : 0u);"),
    ("quantiser: 128 levels", "#define ORACLE_QUANT_LEVELS 127.0f", "#define ORACLE_QUANT_LEVELS 128.0f"),
    ("quantiser: scale of the first bucket for all", "scale[j / ORACLE_QUANT_BUCKET];\n        float mag", "scale[0];\n        float mag"),
    ("quantiser: the explorer's random stream", "uint32_t key[2] = { (uint32_t)seed ^ 0x51534744u, (uint32_t)(seed >> 32) ^ kind };", "uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };"),
    ("quantiser: sign lost", "code[j] = (uint8_t)((signbit(v[j]) ? 0x80u : 0u) | level);", "code[j] = (uint8_t)level;"),
    ("quantiser: word of the neighbouring element", "return out[j & 3u];", "return out[(j + 1u) & 3u];"),
]


@pytest.mark.parametrize("desc,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, desc, old, new):
    src = open(SRC).read()
    assert src.count(old) == 1, "mutation site not unique: " + desc
    mutated = tmp_path / "mutant.c"
    mutated.write_text(src.replace(old, new))
    env = dict(os.environ, SLIMDP_ORACLE_SRC=str(mutated), SLIMDP_ORACLE_LIB=str(tmp_path / "libmutant.so"))
    proc = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                           "-p", "no:cacheprovider"], capture_output=True, text=True, env=env, cwd=ROOT)
    assert proc.returncode == 1 and " failed" in proc.stdout, "SURVIVED: %s\n%s" % (desc, proc.stdout[-800:])


def test_the_unmodified_copy_passes(tmp_path):
    copy = tmp_path / "copy.c"
    copy.write_text(open(SRC).read())
    env = dict(os.environ, SLIMDP_ORACLE_SRC=str(copy), SLIMDP_ORACLE_LIB=str(tmp_path / "libcopy.so"))
    proc = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                           "-p", "no:cacheprovider"], capture_output=True, text=True, env=env, cwd=ROOT)
    assert proc.returncode == 0, proc.stdout[-800:]
