"""Do the pins notice a mistake?  One plausible mistake at a time (a sign, an index, a dropped term, an
off-by-one) is planted in a COPY of the oracle's source; the pin tests are run against that copy in a
child process and must fail.  The oracle itself is never touched.  A sample of the planted mistakes is
kept here so that the whole CPU suite stays short."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "saap_ref.c")

MISTAKES = [
    ("assign_keys: exact ties go to the higher id",
     "if (b == 0 || t > best_t) { best_t = t; best = b; }", "if (b == 0 || t >= best_t) { best_t = t; best = b; }"),
    ("assign_keys: sign of the bias",
     "if (bias) t += (double)bias[(size_t)h * B + b];\n          if (b == 0", "if (bias) t -= (double)bias[(size_t)h * B + b];\n          if (b == 0"),
    ("append_keys: a full bucket is not noticed",
     "if (o[b] + l[b] >= o[b + 1]) { overflow = 1; continue; }\n      int j = o[b] + l[b];\n      idx[",
     "if (o[b] + l[b] > o[b + 1]) { overflow = 1; continue; }\n      int j = o[b] + l[b];\n      idx["),
    ("classify_queries: weight set of another head",
     "if (Hw == Hkv) return hq / (Hq / Hkv);", "if (Hw == Hkv) return hq % Hkv;"),
    ("classify_queries: second bias dropped", "if (b2) t += (double)b2[(size_t)w * B + b];", ""),
    ("select_buckets: first head of the group counted twice, last one never",
     "for (int i = 1; i < heads; ++i) g = g + scores[((size_t)s * Hq + (size_t)l * heads + i) * B + b];",
     "for (int i = 0; i < heads - 1; ++i) g = g + scores[((size_t)s * Hq + (size_t)l * heads + i) * B + b];"),
    ("attention: score scale dropped", "a[i] = t * scale;", "a[i] = t;"),
    ("attention: log-sum-exp without the maximum", "if (lse) *lse = amax + log(sum);", "if (lse) *lse = log(sum);"),
    ("sparse attention: per-head lists read as per-KV-head lists",
     "const int32_t* sel = mode == 1 ? selected + (size_t)t * nprobe : selected + u * nprobe;\n    long count = 0;",
     "const int32_t* sel = selected + u * nprobe;\n    long count = 0;"),
    ("windowed attention: recent window one key short",
     "if (n < n_sink || n >= Nt - n_recent ||", "if (n < n_sink || n > Nt - n_recent ||"),
    ("prefill attention: a token does not see its own key",
     "int L = pos0[s] + t + 1;", "int L = pos0[s] + t;"),
    ("prefill attention: every token reads the list of the block's first token",
     "const int32_t* sel = selected + (u * Tq + t) * nprobe;", "const int32_t* sel = selected + (u * Tq) * nprobe;"),
    ("window_push: displaced row taken from the neighbouring slot", "ix[dst] = ix[j];", "ix[dst] = ix[j > 0 ? j - 1 : j];"),
    ("recompact_index: resident run shrunk to its occupied slots",
     "if (resident) on[B + 1] = on[B] + (o[B + 1] - o[B]);", "if (resident) on[B + 1] = on[B] + l[B];"),
    ("update_centroids: sum not divided by the count", "{ c[e] /= (double)count; sq += c[e] * c[e]; }", "{ sq += c[e] * c[e]; }"),
    ("bucket_attention_mass: not normalised", "for (int b = 0; b < B; ++b) m[b] /= sum;", ""),
    ("fp8 encoder: ties away from zero instead of to even",
     "int q = (int)nearbyint((2.0 * f - 1.0) * 8.0);", "int q = (int)floor((2.0 * f - 1.0) * 8.0 + 0.5);"),
    ("fp8 scale: a maximum exactly on 448 * 2^e takes the next power",
     "int e = f <= 0.875f ? ex - 9 : ex - 8;", "int e = f < 0.875f ? ex - 9 : ex - 8;"),
]


@pytest.mark.parametrize("what,old,new", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_a_planted_mistake_fails_the_pins(tmp_path, what, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, "the oracle changed: update this pattern"
    copy = tmp_path / "saap_ref.c"
    copy.write_text(text.replace(old, new))
    env = dict(os.environ, SAAP_ORACLE_SRC=str(copy))
    pins = [os.path.join(ROOT, "tests", f) for f in sorted(os.listdir(os.path.join(ROOT, "tests")))
            if f.startswith("test_oracle_") and f.endswith(".py") and f != os.path.basename(__file__)]
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *pins], cwd=ROOT, env=env,
                       capture_output=True, text=True)
    assert r.returncode == 1, f"{what}: the pins passed (or did not run):\n{r.stdout[-2000:]}\n{r.stderr[-1000:]}"
