"""The pins must notice a plausible mistake anywhere in the oracle: each case below plants ONE
mistake in a private copy of ``oracle/laq_oracle.c`` (CPU only, nothing here touches a GPU),
rebuilds that copy and runs the pin suite on it; the suite has to fail."""
import os
import shutil
import subprocess
import sys

import pytest

MUTATIONS = [
    ("raw scores: wrong KV head for a query head",
     "const int g = h / G;\n        for (int w = 0; w < W; ++w) {", "const int g = h % Hkv;\n        for (int w = 0; w < W; ++w) {"),
    ("raw scores: 1/d instead of 1/sqrt(d)",
     "scale = 1.0 / sqrt((double)d);\n\n    double *qrow", "scale = 1.0 / (double)d;\n\n    double *qrow"),
    ("raw scores: trailing window one position early",
     "int last = q_pos ? q_pos[w] : L - W + w;", "int last = q_pos ? q_pos[w] : L - W + w - 1;"),
    ("raw scores: explicit position excludes its own key",
     "if (last > L - 1) last = L - 1;\n            const int vis = last + 1;", "if (last > L - 1) last = L - 1;\n            const int vis = last;"),
    ("max pool: window one short on the right",
     "int lo = j - half, hi = j + half;\n            if (lo < 0) lo = 0;", "int lo = j - half, hi = j + half - 1;\n            if (lo < 0) lo = 0;"),
    ("max pool: clipped at L instead of the prefix",
     "if (hi > P - 1) hi = P - 1;\n            double m = r[lo];", "if (hi > L - 1) hi = L - 1;\n            double m = r[lo];"),
    ("average pool: divides by the clipped window's size",
     "o[j] = acc / (double)pool;",
     "o[j] = acc / (double)((j + half < P ? j + half : P - 1) - (j - half > 0 ? j - half : 0) + 1);"),
    ("average pool: kept columns leak into the prefix",
     "if (i >= 0 && i < P) acc += r[i];", "if (i >= 0 && i < L) acc += r[i];"),
    ("select: ties to the higher index",
     "return (x->index > y->index) - (x->index < y->index);   /* then lower index */",
     "return (x->index < y->index) - (x->index > y->index);"),
    ("select: smallest scores first",
     "if (x->score > y->score) return -1;      /* larger score first */\n    if (x->score < y->score) return 1;",
     "if (x->score > y->score) return 1;\n    if (x->score < y->score) return -1;"),
    ("select: retained window starts one early", "out[ksel + w] = P + w;", "out[ksel + w] = P + w - 1;"),
    ("compact: source rows addressed with the output's head stride",
     "(const char *)src + ((size_t)g * L + j) * row_bytes, row_bytes);",
     "(const char *)src + ((size_t)g * Bk + j) * row_bytes, row_bytes);"),
    ("sink + recent: recent part starts one early", "out[s + t] = L - recent + t;", "out[s + t] = L - recent + t - 1;"),
    ("sink + recent: sinks not clamped to the budget", "const int s = n_sink < Bk ? n_sink : Bk;", "const int s = n_sink;"),
    ("overlap: every listed position counts", "count += in_gold[j];", "count += 1;"),
    ("overlap: membership not cleared between heads",
     "memset(in_gold, 0, (size_t)L);\n        for (int t = 0; t < n_gold; ++t) {", "for (int t = 0; t < n_gold; ++t) {"),
    ("decode: wrong KV head",
     "const int g = h / G;\n        double M = -INFINITY;\n        for (int j = 0; j < Bk; ++j) {",
     "const int g = h % Hkv;\n        double M = -INFINITY;\n        for (int j = 0; j < Bk; ++j) {"),
    ("decode: weights not normalised", "out[(size_t)h * d + c] = acc / Z;", "out[(size_t)h * d + c] = acc;"),
    ("decode: keys used as values",
     "acc += p[j] * load_elem(vc, dtype, ((size_t)g * Bk + j) * d + c);",
     "acc += p[j] * load_elem(kc, dtype, ((size_t)g * Bk + j) * d + c);"),
    ("Q-cache: step stored in the mirrored slot",
     "memcpy((char *)q_cache + ((size_t)h * W + t) * row,", "memcpy((char *)q_cache + ((size_t)h * W + (W - 1 - t)) * row,"),
]


@pytest.fixture(scope="module")
def oracle_copy(tmp_path_factory, repo_root):
    """A private tree with everything the pin suite imports (no built libraries, no GPU package use)."""
    root = tmp_path_factory.mktemp("mutated")
    for name in ("oracle", "laq_inputs", "tests"):
        shutil.copytree(os.path.join(repo_root, name), os.path.join(root, name),
                        ignore=shutil.ignore_patterns("_build", "__pycache__", "*.so", "test_oracle_mutations.py",
                                                      "test_gpu_parity.py", "test_abi.py"))
    return str(root), open(os.path.join(repo_root, "oracle", "laq_oracle.c")).read()


@pytest.mark.parametrize("what,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_the_pins(oracle_copy, what, old, new):
    root, source = oracle_copy
    assert source.count(old) == 1, "the place to plant the mistake has moved: " + what
    with open(os.path.join(root, "oracle", "laq_oracle.c"), "w") as fh:
        fh.write(source.replace(old, new))
    shutil.rmtree(os.path.join(root, "oracle", "_build"), ignore_errors=True)
    res = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p", "no:cacheprovider"],
                         cwd=root, capture_output=True, text=True, timeout=600)
    assert res.returncode != 0, "no pin noticed: " + what
    assert "failed" in res.stdout, res.stdout[-400:]
