"""Do the oracle's pins notice a mistake?  Each case plants ONE plausible
mistake in a copy of the oracle's source (a dropped term, a wrong sign, a
swapped operand, a stale state), builds it, and runs the CPU pins against that
build in a child process: the pins must fail.  CPU only; the mistakes are
planted in the oracle, never in the HIP path."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "regtopk_oracle.cpp")
PINS = ["tests/test_oracle_steps.py", "tests/test_oracle_rounds.py", "tests/test_oracle_extensions.py"]

MUTATIONS = [
    ("weight dropped from the denominator of the distortion", "float den = w * a_now;", "float den = a_now;"),
    ("sign of the local term in the numerator", "g_before - w * a_before", "g_before + w * a_before"),
    ("numerator and denominator swapped", "float D = num / den;", "float D = den / num;"),
    ("1 - Delta instead of 1 + Delta", "std::fabs(1.0f + D)", "std::fabs(1.0f - D)"),
    ("multiplied by mu instead of divided", "float x = r / mu;", "float x = r * mu;"),
    ("higher index wins ties", "return i < j;", "return i > j;"),
    ("aggregate without the weight", "acc = acc + o->w[(size_t)n] * o->ghat[(size_t)n * d + j];\n        agg[j] = acc;\n    }\n    o->t += 1;\n}\n\n// Aggregation weights",
     "acc = acc + o->ghat[(size_t)n * d + j];\n        agg[j] = acc;\n    }\n    o->t += 1;\n}\n\n// Aggregation weights"),
    ("error not cleared on the mask", "e[j] = a[j] - gh[j];                             // eps^{t+1} = a - ghat", "e[j] = a[j];"),
    ("smallest scores selected", "if (score[i] != score[j]) return score[i] > score[j];", "if (score[i] != score[j]) return score[i] < score[j];"),
    ("signed value instead of magnitude in the prior", "float p = std::fabs(a);", "float p = a;"),
    ("previous accumulated gradient never updated", "std::memcpy(ap, a, sizeof(float) * (size_t)d);", ""),
    ("previous mask never updated", "std::memcpy(sp, s, (size_t)d);", ""),
    ("error feedback dropped from the accumulation", "a[j] = e[j] + g[j];                              // accumulate", "a[j] = g[j];"),
    ("regulariser applied to unsent entries too", "if (mu != 0.0f && sp[j])", "if (mu != 0.0f)"),
    ("likelihood from the current instead of the previous aggregate slot", "f = likelihood_sent(a[j], ap[j], gprev[j], w, mu, o->likelihood);",
     "f = likelihood_sent(a[j], a[j], gprev[j], w, mu, o->likelihood);"),
    ("per-worker k ignored", "topk_mask(sc, d, o->kn[(size_t)n], s);", "topk_mask(sc, d, k, s);"),
    ("sent value weighted by omega", "val[(size_t)n * k + c] = a[j]; ++c; }\n        }\n        for (; c < k; ++c)", "val[(size_t)n * k + c] = w * a[j]; ++c; }\n        }\n        for (; c < k; ++c)"),
    ("tanh replaced by the clipped line", "    return tanh32(x);\n}\n\n// Prior", "    return x < 1.0f ? x : 1.0f;\n}\n\n// Prior"),
    ("Gaussian likelihood evaluated with tanh", "if (kind == 2) return erf32(x);", "if (kind == 2) return tanh32(x);"),
    ("general exponent ignored", "const float pr = o->exponent != 1.0f ? prior_pow(a[j], o->exponent) : prior(a[j], o->sqrt_steps);", "const float pr = prior(a[j], o->sqrt_steps);"),
    ("one square root too many in the prior", "for (int i = 0; i < m; ++i) p = std::sqrt(p);", "for (int i = 0; i <= m; ++i) p = std::sqrt(p);"),
    ("global Top-k over the last worker's values instead of the aggregate", "mag[(size_t)j] = std::fabs(acc);", "mag[(size_t)j] = std::fabs(o->a[(size_t)(o->N - 1) * d + j]);"),
]


def _survives(args):
    i, (name, old, new), tmp = args
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation %r does not apply exactly once" % name
    src = os.path.join(tmp, "m%d.cpp" % i)
    lib = os.path.join(tmp, "m%d.so" % i)
    with open(src, "w") as f:
        f.write(text.replace(old, new))
    subprocess.check_call(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
                           src, "-o", lib])
    env = dict(os.environ, REGTOPK_ORACLE_LIB=lib)
    rc = subprocess.run([sys.executable, "-m", "pytest", *PINS, "-x", "-q", "-p", "no:cacheprovider"], cwd=ROOT, env=env,
                        stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL, timeout=900).returncode
    return name if rc == 0 else None


def test_every_planted_mistake_fails_a_pin(tmp_path):
    with ThreadPoolExecutor(max_workers=4) as pool:
        survivors = [s for s in pool.map(_survives, [(i, m, str(tmp_path)) for i, m in enumerate(MUTATIONS)]) if s]
    assert not survivors, "no pin noticed: %s" % survivors
