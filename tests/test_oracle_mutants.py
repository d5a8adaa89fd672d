"""The pins are sharp: a plausible mistake planted anywhere in the oracle (on the CPU, in a
copy of its source) makes at least one of the oracle's own pin tests fail."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "lda_oracle.c")
PIN_TESTS = ["tests/test_oracle_philox.py", "tests/test_oracle_conditional.py",
             "tests/test_oracle_iteration.py"]

MUTANTS = [
    ("theta keeps the token's own count", "const int32_t th = n_d[k] - own;", "const int32_t th = n_d[k];"),
    ("phi keeps the token's own count", "const int32_t ph = n_w[k] - own;", "const int32_t ph = n_w[k];"),
    ("n_k keeps the token's own count", "const int32_t nk = n_k[k] - own;", "const int32_t nk = n_k[k];"),
    ("denominator without V", "const double beta_V = beta * (double)V;", "const double beta_V = beta;"),
    ("alpha dropped from p2", "p2[k] = alpha * (double)pstar;", "p2[k] = (double)pstar;"),
    ("weight not rounded to fp32",
     "const float pstar = (float)(((double)ph + beta) / ((double)nk + beta_V));",
     "const double pstar = (((double)ph + beta) / ((double)nk + beta_V));"),
    ("sparse search one entry late", "            if (prefix > x) return k;",
     "            if (prefix > x) return k + 1 < K ? k + 1 : k;"),
    ("dense search one entry late", "            if (prefix > y) return k;",
     "            if (prefix > y) return k + 1 < K ? k + 1 : k;"),
    ("buckets in the wrong order", "    if (x < S) {", "    if (x >= Q) {"),
    ("phi transposed", "n_wk[(size_t)word_ids[t] * (size_t)K + z[t]] += 1;",
     "n_wk[(size_t)z[t] * (size_t)V + word_ids[t]] += 1;"),
    ("Philox multipliers swapped", "uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;",
     "uint64_t p0 = (uint64_t)0xCD9E8D57u * (uint64_t)c0;"),
    ("Philox round count", "for (int r = 0; r < 10; ++r) {", "for (int r = 0; r < 7; ++r) {"),
    ("iteration in the wrong counter word",
     "uint32_t ctr[4] = {(uint32_t)token, (uint32_t)(token >> 32), iter, 0u};",
     "uint32_t ctr[4] = {(uint32_t)token, iter, (uint32_t)(token >> 32), 0u};"),
    ("initial topic range", "(oracle_uniform(seed, 0u, (uint64_t)t) * (double)K);",
     "(oracle_uniform(seed, 0u, (uint64_t)t) * (double)(K - 1));"),
    ("likelihood drops lgamma(alpha)",
     "if (n_d[k] > 0) doc_side += lgamma((double)n_d[k] + alpha) - lg_alpha;",
     "if (n_d[k] > 0) doc_side += lgamma((double)n_d[k] + alpha);"),
    ("likelihood uses alpha for K alpha",
     "doc_side += lgamma(k_alpha) - lgamma((double)len + k_alpha);",
     "doc_side += lgamma(alpha) - lgamma((double)len + k_alpha);"),
    ("likelihood word side sign",
     "word_side += lgamma(v_beta) - lgamma((double)n_k[k] + v_beta);",
     "word_side += lgamma(v_beta) + lgamma((double)n_k[k] + v_beta);"),
    ("theta rows keep zero counts", "            if (n_d[k] > 0) {\n                if (topics)",
     "            if (n_d[k] >= 0) {\n                if (topics)"),
    ("pass uses the wrong word's row", "n_wk + (size_t)word_ids[t] * (size_t)K, n_k,\n                    (int32_t)z[t], u, work, 0, 0);\n            }\n        }\n        free(n_d);\n        free(work);\n    }\n}",
     "n_wk + (size_t)word_ids[doc_ptr[d]] * (size_t)K, n_k,\n                    (int32_t)z[t], u, work, 0, 0);\n            }\n        }\n        free(n_d);\n        free(work);\n    }\n}"),
]


def run_pins(lib_path):
    env = dict(os.environ, LDA_ORACLE_LIB=lib_path, LDA_ORACLE_MUTATION_TEST="1", OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PIN_TESTS],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    return r.returncode, r.stdout[-400:]


def test_every_planted_mistake_is_caught(tmp_path):
    source = open(SRC).read()
    builds = []
    for i, (name, old, new) in enumerate(MUTANTS):
        assert source.count(old) == 1, f"mutant '{name}': pattern not found exactly once"
        c_file = tmp_path / f"mutant_{i}.c"
        so_file = tmp_path / f"mutant_{i}.so"
        c_file.write_text(source.replace(old, new))
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
                               "-fno-fast-math", "-o", str(so_file), str(c_file), "-lm"])
        builds.append((name, str(so_file)))
    with ThreadPoolExecutor(max_workers=6) as pool:
        results = list(pool.map(lambda b: run_pins(b[1]), builds))
    survivors = [name for (name, _), (rc, _) in zip(builds, results) if rc == 0]
    assert not survivors, f"mistakes no pin catches: {survivors}"
    # and the unmodified oracle passes the same command
    so_file = tmp_path / "intact.so"
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
                           "-fno-fast-math", "-o", str(so_file), SRC, "-lm"])
    rc, tail = run_pins(str(so_file))
    assert rc == 0, tail
