"""Do the oracle's pins notice a mistake?  Each case plants one plausible mistake (a dropped term, a wrong sign or
index, a swapped operand) in a COPY of the oracle's sources and runs the pin tests against the copy: they must fail.
The unchanged copy must pass (so a failure is the mistake's doing, not the copying's).  CPU only; every planted
mistake keeps all memory accesses in bounds."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = [os.path.join(ROOT, "tests", "test_oracle_pins.py"), os.path.join(ROOT, "tests", "test_oracle_properties.py")]

C, PY = "spd_oracle.c", "spd_oracle.py"
MISTAKES = [
    # (name, file, text, replacement)
    ("scale dropped", C, "return scale * acc;", "return acc;"),
    ("query channels reversed", C, "widen(q, dtype, q_off + c)", "widen(q, dtype, q_off + (d - 1 - c))"),
    ("query head to KV head by modulo", C, "const int kv = h / G;", "const int kv = h % Hkv;"),
    ("sign of the exponent, unsplit", C, "const double e = exp(s[at] - m);", "const double e = exp(m - s[at]);"),
    ("sign of the exponent, partial", C, "const double e = exp(s[i] - m);", "const double e = exp(m - s[i]);"),
    ("unsplit output not normalised", C, "y[c] /= gamma;", "y[c] /= 1.0;"),
    ("partial output not normalised", C, "a[c] /= gamma;", "a[c] /= 1.0;"),
    ("log of the denominator dropped", C, "lse[r] = m + log(gamma);", "lse[r] = m;"),
    ("values read from the key tensor", C, "row_offset(views[p], 1, u, i, kv, &vb)", "row_offset(views[p], 0, u, i, kv, &vb)"),
    ("partial values read from the key tensor", C, "row_offset(view, 1, u, lo + i, kv, &vb)", "row_offset(view, 0, u, lo + i, kv, &vb)"),
    ("paged mode ignores the KV head", C, "page * w->block_stride + (int64_t)kv * w->head_stride",
     "page * w->block_stride + 0 * w->head_stride"),
    ("page of a token taken from the token before", C, "+ i / w->block_size]", "+ (i > 0 ? i - 1 : 0) / w->block_size]"),
    ("only the first owner's cache is attended", C, "for (int p = 0; p < n_views; ++p)", "for (int p = 0; p < 1; ++p)"),
    ("partial ignores the start of its range", C, "score(q, dtype, q_off, view, u, lo + i, kv, d, scale)",
     "score(q, dtype, q_off, view, u, i, kv, d, scale)"),
    ("alpha inverted", C, "const double alpha = exp(m_out[r] - m_in[r]);", "const double alpha = exp(m_in[r] - m_out[r]);"),
    ("second coefficient uses alpha, not its inverse", C, "(alpha_inv * g_in[r] + g_out[r])", "(alpha * g_in[r] + g_out[r])"),
    ("coefficients swapped", C, "c_in * A_in[(int64_t)r * d + c] + c_out * A_out[(int64_t)r * d + c]",
     "c_out * A_in[(int64_t)r * d + c] + c_in * A_out[(int64_t)r * d + c]"),
    ("merged denominator not rescaled", C, "g += g_out[r] * exp(m_out[r] - mm);", "g += g_out[r];"),
    ("merge with an empty public part returns nothing", C, "c_in = 1.0, c_out = 0.0;", "c_in = 0.0, c_out = 0.0;"),
    ("bf16 widened with the wrong shift", C, "[idx] << 16;", "[idx] << 15;"),
    ("fp16 exponent bias", C, "e - 15);", "e - 16);"),
    ("fp16 subnormal scale", C, "ldexp((double)f, -24)", "ldexp((double)f, -25)"),
    ("fp16 fraction width", C, "(double)f / 1024.0", "(double)f / 2048.0"),
    ("log-sum-exp without the log", PY, "out = m + np.log(gamma)", "out = m + gamma"),
    ("n-way merge: weights not normalised", PY, "W[i, r] = e[i] / den", "W[i, r] = e[i]"),
    ("n-way merge: log-sum-exp without the shift", PY, "lse[r] = top + np.log(den)", "lse[r] = np.log(den)"),
    ("attention mass: maximum instead of minimum", PY, "mn = np.minimum(mn, w[step])", "mn = np.maximum(mn, w[step])"),
    ("attention mass: threshold compared the wrong way", PY, "(w[step] < float(threshold))", "(w[step] > float(threshold))"),
    ("attention mass: one step forgotten in the sum", PY, "sm = sm + w[step]", "sm = sm + (w[step] if step else 0.0)"),
]


def run_pins_against_copy(base, file=None, text=None, replacement=None):
    root = os.path.join(base, "copy")
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(root, "oracle"),
                    ignore=shutil.ignore_patterns("*.so", "__pycache__"))   # the copy compiles its own library
    if file is not None:
        path = os.path.join(root, "oracle", file)
        with open(path) as f:
            src = f.read()
        if text not in src:
            return None
        with open(path, "w") as f:
            f.write(src.replace(text, replacement))
    env = dict(os.environ, SPD_ORACLE_PACKAGE_ROOT=root, OMP_NUM_THREADS="2")
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *PINS],
                          cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=600)


@pytest.fixture(scope="module")
def outcomes(tmp_path_factory):
    """All copies at once, four pytest runs at a time (each is a few seconds of mostly single-threaded work)."""
    from concurrent.futures import ThreadPoolExecutor
    cases = [("unchanged", None, None, None)] + MISTAKES
    base = str(tmp_path_factory.mktemp("oracle_copies"))
    def one(numbered):
        i, case = numbered
        return run_pins_against_copy(os.path.join(base, str(i)), *case[1:])
    with ThreadPoolExecutor(max_workers=4) as pool:
        return dict(zip((c[0] for c in cases), pool.map(one, enumerate(cases))))


def test_unchanged_copy_passes(outcomes):
    res = outcomes["unchanged"]
    assert res.returncode == 0, res.stdout[-3000:]


@pytest.mark.parametrize("name", [m[0] for m in MISTAKES])
def test_pins_notice_a_planted_mistake(outcomes, name):
    res = outcomes[name]
    assert res is not None, f"{name}: the oracle no longer contains the text this case replaces - update the case"
    # 1 = tests ran and at least one failed (anything else - a crash, a collection error - is not a detection)
    assert res.returncode == 1, f"{name}: pytest exit code {res.returncode}\n{res.stdout[-3000:]}"
