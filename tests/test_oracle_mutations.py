"""Do the pins bite?  One plausible mistake at a time (a wrong sign, 255 vs 256, a dropped
widening, truncation for rounding, swapped operands, n-1 for n, a wrong sort direction ...) is
planted in a COPY of the oracle, and the pin suite is run on that copy in a child process: it has
to fail.  Everything here is CPU work on the oracle; the product library is not involved.

The mistakes are textual edits of oracle/qv2_oracle.c or oracle/reference.py; an edit that no
longer matches its source line fails the test too (the list has to follow the oracle)."""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

C, PY = "qv2_oracle.c", "reference.py"
MUTATIONS = [
    # (file, original text, planted text)
    (C, "float z = -128.0f - prod;", "float z = -128.0f + prod;"),                       # zero-point sign
    (C, "float s = range / 255.0f;", "float s = range / 256.0f;"),                       # N - 1 levels
    (C, "float s = absmax / 127.0f;", "float s = absmax / 128.0f;"),                     # 2^(b-1) - 1
    (C, "int64_t r = (int64_t)llrintf(t); ", "int64_t r = (int64_t)t; "),                # truncation for rne
    (C, "clamp_i32(r + (int64_t)zp, -128, 127)", "clamp_i32(r - (int64_t)zp, -128, 127)"),
    (C, "clamp_i32(r + (int64_t)zp, -128, 127)", "clamp_i32(r + (int64_t)zp, -127, 127)"),  # narrow range
    (C, "float k = (float)((int32_t)q[i] - zp);", "float k = (float)((int32_t)q[i] + zp);"),
    (C, "double e = v - (double)xhat[i];", "double e = v + (double)xhat[i];"),
    (C, "return 10.0 * log10(sum_x2 / sum_e2);", "return 20.0 * log10(sum_x2 / sum_e2);"),
    (C, "return 10.0 * log10(sum_x2 / sum_e2);", "return 10.0 * log10(sum_e2 / sum_x2);"),
    (C, "if (x[i] < mn) mn = x[i];", "if (x[i] <= mn && i < n-1) mn = x[i];"),          # last element skipped
    (C, "float lo = mn < 0.0f ? mn : 0.0f;", "float lo = mn;"),                          # range not widened to 0
    (C, "return acc / (double)n;", "return acc / (double)(n-1);"),                       # sample variance
    (C, "return sum_e2 / (double)n;", "return sqrt(sum_e2 / (double)n);"),               # RMSE for MSE
    (C, "xy += x * y;", "xy += x * x;"),                                                 # cosine cross term
    (C, "float f = floorf(t);", "float f = rintf(t);"),                                  # histogram bin rule
    (C, "float top = (float)(nbins - 1);", "float top = (float)nbins - 2;"),             # last bin lost
    (C, "float root = sqrtf(var[c]);", "float root = var[c];"),                          # BN fold: sigma^2
    (C, "float d = b - mean[c];", "float d = b + mean[c];"),                             # BN fold: B - mu
    (PY, "out[i] = (s[i] - s[i - 1]) / dl", "out[i] = (s[i - 1] - s[i]) / dl"),          # delta sign
    (PY, "out[i] = (s[i] - s[i - 1]) / dl", "out[i] = (s[i] - s[i - 1]) * dl"),          # position gap
    (PY, "if M[i] > cfg.mse_factor * mean:", "if M[i] >= cfg.mse_factor * mean:"),       # strict >
    (PY, "mean = total / n if n else 0.0", "mean = total / (n - 1) if n > 1 else 0.0"),
    (PY, "if not is_out[i]), key=lambda i: (G[i], i))", "if not is_out[i]), key=lambda i: (-G[i], i))"),    # list by descending score
    (PY, "if is_out[i]), key=lambda i: (-key[i], i))", "if is_out[i]), key=lambda i: (key[i], i))"),   # largest outlier last
    (PY, "mixed += (32.0 if k else 8.0) * float(m)", "mixed += (32.0 if k else 8.0) ** 2 / 32.0 * float(m)"),
    (PY, "if bops_reduction_pct(macs, keep) < target_pct:", "if bops_reduction_pct(macs, keep) <= target_pct:"),
    (PY, "return list(range(n - 1, -1, -1))", "return list(range(n))"),                  # InOrder direction
    (PY, "kl += pa * math.log(pa / qb_)", "kl += qb_ * math.log(qb_ / pa)"),             # KL(Q || P)
    (PY, 'lines.append(f"{i},{name},{32 if k else 8}")', 'lines.append(f"{i},{name},{8 if k else 32}")'),   # bit-widths swapped
    (PY, 'lines = ["layer,name,bits"]', 'lines = ["layer,bits,name"]'),                   # header line
    (PY, "out.extend(m for m in order if group_id[m] == g)", "out.extend(sorted(m for m in order if group_id[m] == g))"),
]


def _run_one(args):
    k, (fname, old, new), base = args
    d = os.path.join(base, f"m{k}")
    os.makedirs(os.path.join(d, "tests"))
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(d, "oracle"),
                    ignore=shutil.ignore_patterns("*.so", "__pycache__"))
    shutil.copytree(os.path.join(ROOT, "paper_2501_07161_amd"), os.path.join(d, "paper_2501_07161_amd"),
                    ignore=shutil.ignore_patterns("*.so", "__pycache__", "csrc"))
    for f in ("test_oracle_pins.py", "conftest.py"):
        shutil.copy(os.path.join(ROOT, "tests", f), os.path.join(d, "tests", f))
    golden = os.path.join(ROOT, "tests", "golden")
    if os.path.isdir(golden):
        shutil.copytree(golden, os.path.join(d, "tests", "golden"))
    path = os.path.join(d, "oracle", fname)
    src = open(path).read()
    if old not in src:
        return k, "stale", f"{fname}: text to replace not found: {old!r}"
    open(path, "w").write(src.replace(old, new))
    # the planted text must still be a program: a copy that does not compile proves nothing
    check = (["gcc", "-std=c11", "-fsyntax-only", "-Wall", "-Werror", path] if fname == C
             else [sys.executable, "-c", f"import ast,sys; ast.parse(open({path!r}).read())"])
    c = subprocess.run(check, capture_output=True, text=True)
    if c.returncode != 0:
        return k, "broken", c.stderr[-800:]
    env = dict(os.environ, PYTHONDONTWRITEBYTECODE="1")
    r = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=d, capture_output=True, text=True, env=env, timeout=600)
    shutil.rmtree(d, ignore_errors=True)
    if r.returncode == 0:
        return k, "survived", f"{fname}: {old!r} -> {new!r}"
    if " failed" not in r.stdout or "AssertionError" not in r.stdout and "assert" not in r.stdout:
        return k, "broken", r.stdout[-800:] + r.stderr[-800:]      # died of something other than a pin
    return k, "killed", ""


def test_unmodified_copy_passes_and_every_planted_mistake_is_caught(tmp_path):
    base = str(tmp_path)
    # control: the same copying and running, nothing planted, must pass
    k, verdict, info = _run_one((999, (C, "float z = -128.0f - prod;", "float z = -128.0f - prod;"), base))
    assert verdict == "survived", f"control run did not pass: {verdict} {info}"
    jobs = [(k, m, base) for k, m in enumerate(MUTATIONS)]
    with ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as pool:
        results = list(pool.map(_run_one, jobs))
    bad = [(k, v, info) for k, v, info in results if v != "killed"]
    assert not bad, "\n".join(f"mutation {k}: {v}: {info}" for k, v, info in bad)
