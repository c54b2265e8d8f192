"""Mutation check of the oracle's pins (CPU only): each planted mistake is applied to a temporary copy of
oracle/mcsd_oracle.c, the copy is built, and the pin tests (tests/test_oracle_mask.py, test_oracle_attention.py,
test_oracle_verify.py) are run against it in a subprocess.  Every mutant must fail at least one pin; the unmodified
copy must pass them all.  The mistakes are the plausible ones: a dropped term, a wrong sign or index, a transposed
operand, a comparison made non-strict."""
import concurrent.futures as cf
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ["tests/test_oracle_mask.py", "tests/test_oracle_attention.py", "tests/test_oracle_verify.py"]

# (name, text in mcsd_oracle.c, replacement)
MUTANTS = [
    ("parent index a mod b", "(int32_t)(off_prev + a / b[l])", "(int32_t)(off_prev + a % (n / b[l]))"),
    ("mask without the diagonal", "for (int64_t j = i; j >= 0; j = parent[j])", "for (int64_t j = parent[i]; j >= 0; j = parent[j])"),
    ("slice with the wrong row stride", "out[i * n + j] = M[i * n_full + j];", "out[i * n + j] = M[i * n + j];"),
    ("soft-max scale dropped", "s[j] = scale * dot;", "s[j] = dot;"),
    ("tree keys ignore the mask", "vis[j] = tree ? M[(int64_t)i * mask_stride + jj] : 1;", "vis[j] = 1;"),
    ("mask transposed", "M[(int64_t)i * mask_stride + jj]", "M[(int64_t)jj * mask_stride + i]"),
    ("values read from the key cache", ": v_scale * load_elem(v_prefix, pre0 + jj * d + c, kv_dtype);",
     ": v_scale * load_elem(k_prefix, pre0 + jj * d + c, kv_dtype);"),
    ("head stride of the cache", "const int64_t pre0 = seq_base[b] + (int64_t)h * head_stride;",
     "const int64_t pre0 = seq_base[b] + (int64_t)h * d;"),
    ("accept test not strict", "if (u * ((double)qrow[x] * S) < r[x])", "if (u * ((double)qrow[x] * S) <= r[x])"),
    ("accept test without the residual's sum", "if (u * ((double)qrow[x] * S) < r[x])", "if (u * ((double)qrow[x]) < r[x])"),
    ("residual with the wrong sign", "fma(-S, (double)qrow[v], r[v])", "fma(S, (double)qrow[v], r[v])"),
    ("residual without the sum", "fma(-S, (double)qrow[v], r[v])", "fma(-1.0, (double)qrow[v], r[v])"),
    ("residual not clamped at zero", "r[v] = d > 0.0 ? d : 0.0;", "r[v] = d;"),
    ("sum not updated after a rejection", "S = tree_sum(r, P);", ";"),
    ("terminal distribution is the target row", "if (S > 0.0) memcpy(term, r, sizeof(double) * (size_t)P);",
     "if (0) memcpy(term, r, sizeof(double) * (size_t)P);"),
    ("bonus token from the wrong row", "const float *prow = p + (cur + 1) * (int64_t)V;\n    for (int64_t v = 0; v < P; ++v) term[v]",
     "const float *prow = p + (cur) * (int64_t)V;\n    for (int64_t v = 0; v < P; ++v) term[v]"),
    ("children of a context start at the wrong node", "*first = t->off[ctx_level] + a * t->b[ctx_level];", "*first = t->off[ctx_level] + a;"),
    ("ties go to the last level-1 node", "if (len > best_len) {", "if (len >= best_len) {"),
    ("target-initialised length without the level-1 node", "int32_t len = 1 + traverse(", "int32_t len = traverse("),
    ("sampler descends left on equality", "if (thr < left) {", "if (thr <= left) {"),
    ("sampler keeps the threshold", "thr = thr - left;", ";"),
    ("sum taken left to right", "return tree_node(a, lo, len / 2) + tree_node(a, lo + len / 2, len / 2);",
     "{double s=0; for(int64_t i=lo;i<lo+len;++i) s+=a[i]; return s;}"),
    ("one uniform for all new tokens", "u_smp[(int64_t)b * n_new + k]", "u_smp[(int64_t)b * n_new]"),
    ("draft row of the root for every context", "const float *qrow = q + (cur + 1) * (int64_t)V;",
     "const float *qrow = q + (cur + 1 > 0 ? 0 : 0) * (int64_t)V;"),
]


def _run_pins(work, source_text):
    shutil.rmtree(work, ignore_errors=True)
    os.makedirs(work)
    for d in ("tests", "workloads", "oracle"):
        shutil.copytree(os.path.join(ROOT, d), os.path.join(work, d), ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    with open(os.path.join(work, "oracle", "mcsd_oracle.c"), "w") as f:
        f.write(source_text)
    env = dict(os.environ, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PINS], cwd=work,
                       capture_output=True, text=True, env=env)
    return r.returncode, r.stdout[-2000:]


@pytest.fixture(scope="module")
def source():
    with open(os.path.join(ROOT, "oracle", "mcsd_oracle.c")) as f:
        return f.read()


def test_every_mutation_site_still_exists(source):
    missing = [name for name, a, _ in MUTANTS if a not in source]
    assert not missing, f"the oracle's text changed; update these mutants: {missing}"


def test_unmodified_copy_passes_and_every_mutant_is_caught(source, tmp_path):
    rc, out = _run_pins(str(tmp_path / "clean"), source)
    assert rc == 0, "the pins fail on an unmodified copy of the oracle:\n" + out

    def one(job):
        k, (name, a, b) = job
        rc, out = _run_pins(str(tmp_path / f"m{k}"), source.replace(a, b, 1))
        shutil.rmtree(str(tmp_path / f"m{k}"), ignore_errors=True)
        return name, rc

    with cf.ThreadPoolExecutor(4) as ex:
        results = list(ex.map(one, enumerate(MUTANTS)))
    survived = [name for name, rc in results if rc == 0]
    assert not survived, f"planted mistakes that no pin catches: {survived}"
