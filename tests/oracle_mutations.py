#!/usr/bin/env python3
"""Plants one mistake at a time in a temporary COPY of the CPU oracle and runs the oracle's pins
(tests/test_oracle_pins.py, tests/test_oracle_head.py, tests/test_oracle_object_weights.py)
against it: every planted mistake must make a pin fail.  CPU only, nothing in the tree is
touched; not collected by pytest (a run takes a few minutes):

    python tests/oracle_mutations.py            # all mistakes
    python tests/oracle_mutations.py adam relu  # those whose name contains one of the words

Exit status 1 if a mistake survives.  The mistakes are of the kinds a re-implementation from
the paper is prone to: a transposed kernel or confusion matrix, a dropped term, a wrong sign or
weight in the interpolation and its adjoint, the other tie rule, the other normalisation, a
missing ReLU or rounding point, Adam's constants, the comparisons of Algorithm 1.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ["tests/test_oracle_pins.py", "tests/test_oracle_head.py", "tests/test_oracle_object_weights.py"]


def nth(s, a, b, n):
    i = -1
    for _ in range(n):
        i = s.index(a, i + 1)
    return s[:i] + b + s[i + len(a):]


def swap(a, b):
    return lambda s: s.replace(a, b)


KW = "W[(((size_t)o * ci + i) * k + kh) * k + kw]"
KW_T = "W[(((size_t)o * ci + i) * k + kw) * k + kh]"
# (file, name, edit)
C = "oracle/st_oracle.c"
PY = "oracle/object_weights.py"
MISTAKES = [
    (C, "forward kernel transposed", lambda s: nth(s, KW, KW_T, 1)),
    (C, "data-gradient kernel transposed", lambda s: nth(s, KW, KW_T, 2)),
    (C, "weight gradient stored transposed", swap("dW[(((size_t)o * ci + i) * k + kh) * k + kw] = acc;",
                                                  "dW[(((size_t)o * ci + i) * k + kw) * k + kh] = acc;")),
    (C, "bias gradient drops a term", swap("for (int p = 0; p < h * w; ++p) acc += dyo[p];",
                                           "for (int p = 1; p < h * w; ++p) acc += dyo[p];")),
    (C, "relu derivative 1 at the kink", swap("if (!(a[i] > 0.0)) dy[i] = 0.0;", "if (!(a[i] >= 0.0)) dy[i] = 0.0;")),
    (C, "no half-pixel offset", swap("((double)d + 0.5) / (double)STO_UP - 0.5", "((double)d) / (double)STO_UP")),
    (C, "interpolation weights swapped along y", swap("Zp[(size_t)Y * Wd + X] = r0 + wy * (r1 - r0);",
                                                      "Zp[(size_t)Y * Wd + X] = r1 + wy * (r0 - r1);")),
    (C, "adjoint with a wrong weight", swap("gp[y0 * w + x1] += (1.0 - wy) * wx * v;",
                                            "gp[y0 * w + x1] += (1.0 - wy) * (1.0 - wx) * v;")),
    (C, "argmax ties to the highest class", swap("if (v > bv) { bv = v; best = c; }", "if (v >= bv) { bv = v; best = c; }")),
    (C, "loss value ignores the pixel weights", swap("acc += wp * (lse - zb[(size_t)y * P]);",
                                                     "acc += (lse - zb[(size_t)y * P]);")),
    (C, "weighted loss normalised by the pixel count", swap("w_sum += weights ? weights[q] : 1;", "w_sum += 1;")),
    (C, "confusion matrix transposed", swap("conf[(size_t)y * C + pred[p]] += 1;", "conf[(size_t)pred[p] * C + y] += 1;")),
    (C, "mean IoU over predicted classes too", swap("if (row == 0) continue;", "if (row + col == 0) continue;")),
    (C, "other momentum form", swap("vel[i] = mu * vel[i] + grad[i];", "vel[i] = mu * (vel[i] + grad[i]);")),
    (C, "adam without the second bias correction", swap("vhat = v[i] / bc2;", "vhat = v[i];")),
    (C, "adam eps inside the root", swap("(sqrt(vhat) + eps)", "sqrt(vhat + eps)")),
    (C, "adam step index off by one", swap("optim_step(opt, params, grad, s1, s2, (int64_t)np, it + 1);",
                                           "optim_step(opt, params, grad, s1, s2, (int64_t)np, it);")),
    (C, "second relu missing", swap("    sto_relu(s->a2, (int64_t)d->n * d->c2 * hw);\n", "")),
    (C, "relu mask of layer 1 missing", swap("        sto_relu_bwd(da1, s.a1, (int64_t)d->n * d->c1 * hw);\n", "")),
    (C, "bf16 mode: da2 not rounded", swap("        if (q) sto_round_bf16(da2, (int64_t)d->n * d->c2 * hw);\n", "")),
    (C, "bf16 mode: a1 not rounded", swap("    if (q) sto_round_bf16(s->a1, (int64_t)d->n * d->c1 * hw);\n", "")),
    (C, "bf16 mode: logit gradient not rounded", swap("double* gq = operand_copy(g, (size_t)d->n * C * hw, q);",
                                                      "double* gq = operand_copy(g, (size_t)d->n * C * hw, 0);")),
    (C, "best parameters on >=", swap("if (metric > bm) { bm = metric;", "if (metric >= bm) { bm = metric;")),
    (C, "training skipped on <=", swap("if (bm < threshold) {", "if (bm <= threshold) {")),
    (C, "break rules swapped", swap("strict_break ? metric > threshold : metric >= threshold",
                                    "strict_break ? metric >= threshold : metric > threshold")),
    (PY, "weight map: window one column short", swap("for dx in range(-radius, radius + 1):", "for dx in range(-radius, radius):")),
    (PY, "weight map: rows and columns exchanged",
     swap("obj[:, ya + dy:yb + dy, xa + dx:xb + dx]", "obj[:, ya + dx:yb + dx, xa + dy:xb + dy]")),
    (PY, "weight map: ignore value counts as an object", swap(" & (lab != ignore_index)", "")),
    (PY, "weight map: first non-class counts as an object", swap("(lab < n_classes)", "(lab <= n_classes)")),
    (PY, "weight map: background fixed to class 0", swap("(lab != background)", "(lab != 0)")),
]


def main(words):
    work = tempfile.mkdtemp(prefix="oracle_mutations_")
    try:
        for d in ("oracle", "workloads"):
            shutil.copytree(os.path.join(ROOT, d), os.path.join(work, d), ignore=shutil.ignore_patterns("*.so", "__pycache__"))
        os.makedirs(os.path.join(work, "tests", "golden"))
        for f in ["tests/conftest.py", *PINS]:
            shutil.copy(os.path.join(ROOT, f), os.path.join(work, f))
        for f in os.listdir(os.path.join(ROOT, "tests", "golden")):
            if f.endswith(".txt"):
                shutil.copy(os.path.join(ROOT, "tests", "golden", f), os.path.join(work, "tests", "golden", f))
        survivors = 0
        for rel, name, edit in MISTAKES:
            if words and not any(w in name for w in words):
                continue
            original = open(os.path.join(ROOT, rel)).read()
            mutated = edit(original)
            assert mutated != original, f"the mistake '{name}' no longer applies to {rel}"
            open(os.path.join(work, rel), "w").write(mutated)
            lib = os.path.join(work, "oracle", "libst_oracle.so")
            if os.path.exists(lib):
                os.remove(lib)
            t0 = time.time()
            r = subprocess.run([sys.executable, "-m", "pytest", *PINS, "-x", "-q", "-p", "no:cacheprovider"], cwd=work,
                               capture_output=True, text=True)
            where = [l for l in r.stdout.splitlines() if l.startswith("FAILED")][:1]
            caught = r.returncode != 0 and bool(where)
            survivors += 0 if caught else 1
            print(("caught   " if caught else "SURVIVED "), name, f"({time.time() - t0:.0f} s)", *where, flush=True)
            open(os.path.join(work, rel), "w").write(original)
        return 1 if survivors else 0
    finally:
        shutil.rmtree(work, ignore_errors=True)


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
