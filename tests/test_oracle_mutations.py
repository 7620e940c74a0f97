"""Do the oracle's pins have teeth?  Each planted mistake below -- a dropped term, a wrong sign, a
shifted step index, a misplaced epsilon, ... -- is applied to a COPY of oracle/page_adamw.c in a
temporary directory (the tracked source is never edited), built there, and the pin tests are run
against that build in a child process (ORACLE_LIBRARY selects it): they must fail for every
mistake, and pass for the unmodified copy."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "page_adamw.c")
PINS = ["tests/test_oracle_adamw_pins.py", "tests/test_oracle_bf16.py"]

UPDATE = ("double pi = p[i] * (1.0 - h->lr * h->weight_decay) - h->lr * mhat / (sqrt(vhat) + h->eps);")

# (what the mistake is, text in the source, its replacement)
MISTAKES = [
    ("momentum takes the whole gradient", "h->beta1 * m[i] + (1.0 - h->beta1) * g", "h->beta1 * m[i] + g"),
    ("variance of g instead of g^2", "(1.0 - h->beta2) * g * g", "(1.0 - h->beta2) * g"),
    ("no bias correction of m", "double mhat = mi / bc1", "double mhat = mi"),
    ("no bias correction of v", "double vhat = vi / bc2", "double vhat = vi"),
    ("epsilon inside the root", "(sqrt(vhat) + h->eps)", "sqrt(vhat + h->eps)"),
    ("decay coupled into the moment", UPDATE,
     "double pi = p[i] - h->lr * h->weight_decay * mi - h->lr * mhat / (sqrt(vhat) + h->eps);"),
    ("decay applied to the new parameter", UPDATE,
     "double pi = (p[i] - h->lr * mhat / (sqrt(vhat) + h->eps)) * (1.0 - h->lr * h->weight_decay);"),
    ("no decay at all", UPDATE, "double pi = p[i] - h->lr * mhat / (sqrt(vhat) + h->eps);"),
    ("step index off by one", "pow(h->beta1, (double)t)", "pow(h->beta1, (double)(t + 1))"),
    ("step index off by one in the second moment", "pow(h->beta2, (double)t)", "pow(h->beta2, (double)(t - 1))"),
    ("clip without its 1e-6", "norm + 1e-6", "norm"),
    ("clip scale not capped at 1", "if (s > 1.0) s = 1.0;", ""),
    ("minus zero counts as a gradient", "(g16[i] & 0x7FFFu) != 0", "g16[i] != 0"),
    ("cast rounds half up, not to even", "u + 0x7FFFu + ((u >> 16) & 1u)", "u + 0x8000u"),
    ("cast truncates", "(u + 0x7FFFu + ((u >> 16) & 1u)) >> 16", "u >> 16"),
    ("update with the wrong sign", "- h->lr * mhat /", "+ h->lr * mhat /"),
    ("gradient not scaled by the clip factor", "double g = s * bf16_to_double(g16[i]);",
     "double g = bf16_to_double(g16[i]);"),
    ("norm is the sum of squares, not its root", "double norm = sqrt(sumsq);", "double norm = sumsq;"),
    ("sum of |g| instead of g^2", "s += g * g;", "s += fabs(g);"),
    ("skipped page is updated all the same", "*norm_out = 0.0f;\n        return 0;", "*norm_out = 0.0f;"),
    ("p16 cast from the old parameter", "p[i] = pi;\n        float pf = (float)pi;",
     "float pf = (float)p[i];\n        p[i] = pi;"),
    ("p16 cast from the double, one rounding", "float pf = (float)pi;", "float pf = (float)pi;\n        "
     "{ double q = pi; uint64_t w; memcpy(&w, &q, 8); w &= ~0xFFFFFFFFFFull; memcpy(&q, &w, 8); pf = (float)q; }"),
]


def build_and_run(tmp, name, text):
    d = os.path.join(tmp, name)
    os.makedirs(d)
    c, so = os.path.join(d, "page_adamw.c"), os.path.join(d, "liboracle.so")
    with open(c, "w") as f:
        f.write(text)
    subprocess.run(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
                    "-o", so, c, "-lm"], check=True, capture_output=True)
    env = dict(os.environ, ORACLE_LIBRARY=so)
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        "-k", "not every_fp32_pattern"] + PINS, cwd=ROOT, env=env, capture_output=True, text=True)
    return r.returncode, r.stdout[-600:]


def test_every_planted_mistake_fails_a_pin_and_the_unmodified_copy_passes(tmp_path):
    text = open(SRC).read()
    jobs = [("unmodified", text)]
    for k, (what, old, new) in enumerate(MISTAKES):
        assert text.count(old) == 1, f"{what}: the text to damage occurs {text.count(old)} times in the oracle source"
        jobs.append((f"m{k:02d}", text.replace(old, new)))
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(lambda j: build_and_run(str(tmp_path), *j), jobs))
    rc0, out0 = results[0]
    assert rc0 == 0, "the pins must pass on an unmodified copy:\n" + out0
    missed = [MISTAKES[k][0] for k, (rc, _) in enumerate(results[1:]) if rc == 0]
    assert not missed, f"planted mistakes no pin caught: {missed}"
    for (rc, out), (what, _, _) in zip(results[1:], MISTAKES):
        assert rc == 1, f"{what}: the pin run did not fail on an assertion (exit {rc}):\n{out}"
    assert open(SRC).read() == text          # the tracked source is as it was
