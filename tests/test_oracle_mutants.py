"""Do the pins bite? Each case plants one plausible mistake in a copy of the oracle's C source (a
dropped term, a wrong sign or index, a transposed operand, an off-by-one), builds it, and runs
the oracle's pin tests against that build in a child process: at least one pin must fail. The
mistakes live in the oracle, on the CPU; nothing here touches the GPU path."""
import os
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "sts_oracle.c")
PIN_FILES = ["test_oracle_select.py", "test_oracle_attn.py", "test_oracle_blocks.py", "test_oracle_headmap.py"]

# (name, text in sts_oracle.c, replacement, pin files that must notice)
MUTANTS = [
    ("aggregate adds right to left",
     "for (int i = 0; i < Tq; ++i) {\n        float p = P[(size_t)i * N + n];",
     "for (int ii = 0; ii < Tq; ++ii) {\n        const int i_src = Tq - 1 - ii; const int i = ii;\n        float p = P[(size_t)i_src * N + n];",
     ["test_oracle_select.py"]),
    ("aggregate drops the last query row",
     "for (int i = 0; i < Tq; ++i) {\n        float p = P[(size_t)i * N + n];",
     "for (int i = 0; i < (Tq > 1 ? Tq - 1 : Tq); ++i) {\n        float p = P[(size_t)i * N + n];",
     ["test_oracle_select.py"]),
    ("normaliser added instead of subtracted",
     "p = expf(p - lse[(size_t)r * Tq + i]);", "p = expf(p + lse[(size_t)r * Tq + i]);",
     ["test_oracle_select.py"]),
    ("normaliser of the wrong row",
     "p = expf(p - lse[(size_t)r * Tq + i]);", "p = expf(p - lse[(size_t)r * Tq]);",
     ["test_oracle_select.py"]),
    ("ties go to the higher index",
     "return (p->n > q->n) - (p->n < q->n);", "return (p->n < q->n) - (p->n > q->n);",
     ["test_oracle_select.py"]),
    ("smallest scores selected",
     "if (p->a > q->a) return -1;\n  if (p->a < q->a) return 1;", "if (p->a > q->a) return 1;\n  if (p->a < q->a) return -1;",
     ["test_oracle_select.py"]),
    ("index list left in score order",
     "qsort(out, (size_t)c, sizeof(int32_t), by_int);", "(void)by_int;",
     ["test_oracle_select.py"]),
    ("budget off by one",
     "const int c = k < nb ? k : nb;\n    int32_t *out = sel", "const int c = (k < nb ? k : nb) > 1 ? (k < nb ? k : nb) - 1 : (k < nb ? k : nb);\n    int32_t *out = sel",
     ["test_oracle_select.py"]),
    ("valid length ignored by the selection",
     "const int nb = seq_lens ? seq_lens[b] : N;\n    const int c = k < nb ? k : nb;", "const int nb = N; (void)b;\n    const int c = k < nb ? k : nb;",
     ["test_oracle_select.py"]),
    ("block sum runs past the valid length",
     "for (int n = m * page; n < (m + 1) * page && n < nb; ++n) {", "for (int n = m * page; n < (m + 1) * page && n < N; ++n) {",
     ["test_oracle_blocks.py"]),
    ("block sum skips the block's first token",
     "for (int n = m * page; n < (m + 1) * page && n < nb; ++n) {", "for (int n = m * page + (page > 1); n < (m + 1) * page && n < nb; ++n) {",
     ["test_oracle_blocks.py"]),
    ("remap ignores the head map",
     "const int j = head_map[t];\n      memcpy(indices", "const int j = t % Hd;\n      memcpy(indices",
     ["test_oracle_select.py"]),
    ("query head reads the wrong KV head",
     "const int g = t / G;", "const int g = t % Hkv;",
     ["test_oracle_attn.py"]),
    ("scale dropped",
     "s[j] = (double)scale * dot;\n        if (s[j] > m) m = s[j];", "s[j] = dot;\n        if (s[j] > m) m = s[j];",
     ["test_oracle_attn.py"]),
    ("values read from K",
     "vr = Vg + row * stride_n;", "vr = Kg + row * stride_n;",
     ["test_oracle_attn.py"]),
    ("gathered row index ignored for V",
     "const size_t row = idx ? (size_t)idx[j] : (size_t)j;\n          vr =", "const size_t row = (size_t)j;\n          vr =",
     ["test_oracle_attn.py"]),
    ("output not normalised",
     "o[e] = (total > 0) ? (float)(acc[e] / l) : 0.0f;", "o[e] = (total > 0) ? (float)(acc[e]) : 0.0f;",
     ["test_oracle_attn.py"]),
    ("log-sum-exp with the wrong sign",
     "(float)(m + log(l))", "(float)(m - log(l))",
     ["test_oracle_attn.py"]),
    ("own tokens: row i misses token i",
     "const int nnew = k_new ? (causal ? i + 1 : Tq) : 0;", "const int nnew = k_new ? (causal ? i : Tq) : 0;",
     ["test_oracle_attn.py"]),
    ("own tokens of the wrong KV head",
     "const uint16_t *kr = k_new + (((size_t)b * Tq + j) * Hkv + g) * d;", "const uint16_t *kr = k_new + (((size_t)b * Tq + j) * Hkv) * d;",
     ["test_oracle_attn.py"]),
    ("dense attention ignores the valid length",
     "c = seq_lens ? seq_lens[b] : N;\n      if (c < 0 || c > N) {", "c = N;\n      if (c < 0 || c > N) {",
     ["test_oracle_attn.py"]),
    ("logits written with query row and head swapped",
     "logits_out[(((size_t)b * Hq + t) * Tq + i) * N + j]", "logits_out[(((size_t)b * Tq + i) * Hq + t) * N + j]",
     ["test_oracle_attn.py"]),
    ("log-sum-exp written with query row and head swapped",
     "lse_out[((size_t)b * Hq + t) * Tq + i] =", "lse_out[((size_t)b * Tq + i) * Hq + t] =",
     ["test_oracle_attn.py"]),
    ("token stride of the cache ignored",
     "const uint16_t *kr = Kg + row * stride_n;", "const uint16_t *kr = Kg + row * (size_t)d;",
     ["test_oracle_attn.py"]),
    ("head stride of the cache ignored",
     "const uint16_t *Kg = k + (size_t)b * stride_b + (size_t)g * stride_h;",
     "const uint16_t *Kg = k + (size_t)b * stride_b + (size_t)g * (size_t)N * d;",
     ["test_oracle_attn.py"]),
    ("query of the wrong row",
     "const uint16_t *qr = q + (((size_t)b * Tq + i) * Hq + t) * d;", "const uint16_t *qr = q + (((size_t)b * Tq) * Hq + t) * d;",
     ["test_oracle_attn.py"]),
    ("short rows padded with 0 instead of -1",
     "for (int i = 0; i < k; ++i) out[i] = -1;", "for (int i = 0; i < k; ++i) out[i] = 0;",
     ["test_oracle_select.py"]),
    ("counts report the budget, not what was kept",
     "cnt[r] = c;\n    if (c == 0) continue;", "cnt[r] = k;\n    if (c == 0) continue;",
     ["test_oracle_select.py"]),
    ("maximum over the query rows takes the minimum",
     "acc = (p > acc) ? p : acc;", "acc = (p < acc) ? p : acc;",
     ["test_oracle_select.py"]),
    ("natural exponential replaced by a power of two",
     "p = expf(p - lse[(size_t)r * Tq + i]);", "p = exp2f(p - lse[(size_t)r * Tq + i]);",
     ["test_oracle_select.py"]),
    ("remapped counts taken from the first draft head",
     "if (counts) counts[(size_t)b * Hq + t] = cnt[(size_t)b * Hd + j];", "if (counts) counts[(size_t)b * Hq + t] = cnt[(size_t)b * Hd];",
     ["test_oracle_select.py"]),
    ("own tokens, not causal: the last one is missed",
     "const int nnew = k_new ? (causal ? i + 1 : Tq) : 0;", "const int nnew = k_new ? (causal ? i + 1 : Tq - 1) : 0;",
     ["test_oracle_attn.py"]),
    ("head mapping counts the union instead of the intersection",
     "shared += (in_t[n] & in_d[n]);", "shared += (in_t[n] | in_d[n]);",
     ["test_oracle_headmap.py"]),
    ("head mapping: the last best draft head wins",
     "if (row[i] > row[where]) where = i;", "if (row[i] >= row[where]) where = i;",
     ["test_oracle_headmap.py"]),
    ("head mapping: overlap of the first row only",
     "for (int r = 0; r < R; ++r) {\n      const unsigned char *in_t", "for (int r = 0; r < 1; ++r) {\n      const unsigned char *in_t",
     ["test_oracle_headmap.py"]),
]


def _build(src_text, out_dir):
    c = os.path.join(out_dir, "sts_oracle.c")
    with open(c, "w") as f:
        f.write(src_text)
    lib = os.path.join(out_dir, "libmutant.so")
    subprocess.run(["gcc", "-std=c11", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-fPIC", "-shared",
                    "-I", os.path.join(ROOT, "oracle"), "-o", lib, c, "-lm"], check=True)
    return lib


def _run_pins(lib, files):
    env = dict(os.environ, STS_ORACLE_LIB=lib, OMP_NUM_THREADS="2")
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                           *[os.path.join(ROOT, "tests", f) for f in files]],
                          capture_output=True, text=True, env=env, cwd=ROOT, timeout=600)


def test_unmodified_copy_passes_every_pin():
    """The harness itself: the same source, built the same way, passes (so a failing mutant
    fails because of its mistake, not because of the detour through another library)."""
    with tempfile.TemporaryDirectory() as tmp:
        r = _run_pins(_build(open(SRC).read(), tmp), PIN_FILES)
        assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]


def _c_mutant(m):
    name, old, new, files = m
    src = open(SRC).read()
    if src.count(old) != 1:
        return ("missing", f"the text this mutant replaces must occur exactly once: {old!r}")
    with tempfile.TemporaryDirectory() as tmp:
        r = _run_pins(_build(src.replace(old, new), tmp), files)
        return (r.returncode, r.stdout[-1500:] + r.stderr[-1500:])


def _py_mutant(m):
    import shutil
    name, old, new, files = m
    src = open(PY_SRC).read()
    if src.count(old) != 1:
        return ("missing", f"the text this mutant replaces must occur exactly once: {old!r}")
    with tempfile.TemporaryDirectory() as tmp:
        pkg = os.path.join(tmp, "oracle")
        shutil.copytree(os.path.join(ROOT, "oracle"), pkg, ignore=shutil.ignore_patterns("__pycache__"))
        with open(os.path.join(pkg, "__init__.py"), "w") as f:
            f.write(src.replace(old, new))
        env = dict(os.environ, STS_ORACLE_PKG_DIR=tmp, OMP_NUM_THREADS="2")
        env.pop("STS_ORACLE_LIB", None)
        r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                            *[os.path.join(ROOT, "tests", f) for f in files]],
                           capture_output=True, text=True, env=env, cwd=ROOT, timeout=600)
        return (r.returncode, r.stdout[-1500:] + r.stderr[-1500:])


@pytest.fixture(scope="module")
def verdicts():
    """Every mutant built and judged once, a few at a time (each is a compiler run plus a pytest
    child process), so that the whole file takes well under a minute."""
    from concurrent.futures import ThreadPoolExecutor
    jobs = [("c", m) for m in MUTANTS] + [("py", m) for m in PY_MUTANTS]
    with ThreadPoolExecutor(max_workers=max(2, min(6, (os.cpu_count() or 2) - 1))) as ex:
        out = list(ex.map(lambda j: _c_mutant(j[1]) if j[0] == "c" else _py_mutant(j[1]), jobs))
    return {(kind, m[0]): v for (kind, m), v in zip(jobs, out)}


@pytest.mark.parametrize("name", [m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, verdicts):
    rc, tail = verdicts[("c", name)]
    assert rc != "missing", tail
    assert rc == 1 and " failed" in tail, f"no pin noticed: {name}\n{tail}"


# ---- the Python half of the oracle (block expansion, per-head budgets, the composition of the
# selection stages): same procedure on a copy of the package
PY_SRC = os.path.join(ROOT, "oracle", "__init__.py")
PY_MUTANTS = [
    ("block expansion not clipped at N",
     "row.extend(range(int(m) * page, min((int(m) + 1) * page, N)))", "row.extend(range(int(m) * page, (int(m) + 1) * page))",
     ["test_oracle_blocks.py"]),
    ("block expansion ignores the counts",
     "c = kb if counts is None else int(counts[b, t])", "c = kb",
     ["test_oracle_blocks.py"]),
    ("block count of a ragged length rounded down",
     "lens = None if seq_lens is None else (np.asarray(seq_lens, np.int64) + page - 1) // page",
     "lens = None if seq_lens is None else np.asarray(seq_lens, np.int64) // page",
     ["test_oracle_blocks.py"]),
    ("blocks ranked by their first token only",
     "src = block_scores(A, page, seq_lens)", "src = np.ascontiguousarray(A[:, :, ::page])",
     ["test_oracle_blocks.py"]),
    ("every head gets the first head's budget",
     "kj = int(k_head[j])", "kj = int(k_head[0])",
     ["test_oracle_select.py"]),
    ("reduction switch dropped on the way to the aggregation",
     "A = aggregate(scores, lse, kind, reduce)", "A = aggregate(scores, lse, kind)",
     ["test_oracle_select.py"]),
    ("valid lengths dropped on the way to the selection",
     "sel, cnt = pick(A, k, seq_lens)", "sel, cnt = pick(A, k, None)",
     ["test_oracle_select.py"]),
    ("union of the rows: a later row's bit replaces the earlier ones",
     "keep[int(n)] = keep.get(int(n), 0) | (1 << i)", "keep[int(n)] = (1 << i)",
     ["test_oracle_rows.py"]),
    ("union of the rows: the rows' counts are ignored",
     "c = k if row_cnt is None else int(row_cnt[b, j, i])", "c = k",
     ["test_oracle_rows.py"]),
    ("union of the rows: every target head reads draft head 0",
     "j = int(head_map[t])\n            keep = {}", "j = 0\n            keep = {}",
     ["test_oracle_rows.py"]),
    ("per-row selection ranks the first row for every row",
     "A = aggregate(scores[:, :, i:i + 1], None if lse is None", "A = aggregate(scores[:, :, 0:1], None if lse is None",
     ["test_oracle_rows.py"]),
    ("per-row attention: every row uses the first row's list",
     "r = attn(np.ascontiguousarray(q[:, i:i + 1]), k, v, scale, np.ascontiguousarray(row_idx[:, :, i]),",
     "r = attn(np.ascontiguousarray(q[:, i:i + 1]), k, v, scale, np.ascontiguousarray(row_idx[:, :, 0]),",
     ["test_oracle_rows.py"]),
]


@pytest.mark.parametrize("name", [m[0] for m in PY_MUTANTS])
def test_planted_mistake_in_the_python_half_is_caught(name, verdicts):
    rc, tail = verdicts[("py", name)]
    assert rc != "missing", tail
    assert rc == 1 and " failed" in tail, f"no pin noticed: {name}\n{tail}"
