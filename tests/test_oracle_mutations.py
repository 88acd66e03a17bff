"""Do the pins bite?  Each case plants ONE plausible mistake in a copy of the oracle's C source
(a dropped term, a wrong sign or index, a fused or re-associated operation, a rounding taken in
the wrong precision), compiles the copy, and runs the pin files named for it in a fresh
interpreter against that copy: the run must fail.  The unaltered copy must pass the same files.
Everything happens on the CPU; the HIP library is not involved."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "q8_oracle.c")

OPTIM, QUANT, CODEBOOK = "tests/test_oracle_optim.py", "tests/test_oracle_quantize.py", "tests/test_oracle_codebook.py"
BF16, F16, GOLDEN = "tests/test_oracle_bf16.py", "tests/test_oracle_f16.py", "tests/test_oracle_golden.py"

DECAY_THEN_STEP = """    if (s->wd != 0.0f && (s->flags & ORACLE_FLAG_DECOUPLED_WD)) {
        float t7 = s->alpha_wd * wv;
        wv = wv - t7;
    }
    *w = wv - t6;"""
STEP_THEN_DECAY = """    float w_old = wv;
    wv = wv - t6;
    if (s->wd != 0.0f && (s->flags & ORACLE_FLAG_DECOUPLED_WD)) {
        float t7 = s->alpha_wd * w_old;
        wv = wv - t7;
    }
    *w = wv;"""

NOT_SEARCH = ["-k", "not argmin"]                       # skip the slow exhaustive search pins where the search is untouched
SEARCH = ["-k", "critical_points and signed"]

# (name, [(old, new), ...], pin files that must catch it [+ pytest selection])
MUTATIONS = [
    # --- extension flags (bias correction, decoupled decay)
    ("fused scaled root plus eps", [("float rs = root * s->isbc2;\n        d = rs + s->eps;",
                                     "d = fmaf(root, s->isbc2, s->eps);")], [OPTIM]),
    ("step before decay", [(DECAY_THEN_STEP, STEP_THEN_DECAY)], [OPTIM]),
    ("bias-correction scalars in binary32",
     [("double bc1 = 1.0 - pow((double)beta1, (double)t);", "float bc1 = 1.0f - powf(beta1, (float)t);"),
      ("double bc2 = 1.0 - pow((double)beta2, (double)t);", "float bc2 = 1.0f - powf(beta2, (float)t);"),
      ("s.alpha_t = (float)((double)alpha / bc1);", "s.alpha_t = alpha / bc1;"),
      ("s.isbc2 = (float)(1.0 / sqrt(bc2));", "s.isbc2 = 1.0f / sqrtf(bc2);")], [OPTIM]),
    ("second-moment correction dropped", [("s.isbc2 = (float)(1.0 / sqrt(bc2));", "s.isbc2 = 1.0f;")], [OPTIM]),
    ("decoupled decay as one factor", [("float t7 = s->alpha_wd * wv;\n        wv = wv - t7;",
                                        "wv = wv * (1.0f - s->alpha_wd);")], [OPTIM]),
    # --- Eq. adam / Eq. sgd as printed
    ("fma in the first moment", [("float m = t1 + t2;", "float m = fmaf(s->omb1, g, t1);")], [OPTIM]),
    ("second moment as (1-beta2)*(g*g)", [("float t5 = t4 * g;", "float t5 = s->omb2 * (g * g);")], [OPTIM]),
    ("second moment squares the wrong factor", [("float t5 = t4 * g;", "float t5 = t4 * t4;")], [OPTIM]),
    ("first moment sign", [("float m = t1 + t2;", "float m = t1 - t2;")], [OPTIM]),
    ("eps dropped", [("d = root + s->eps;", "d = root;")], [OPTIM]),
    ("weight step sign", [("    *w = wv - t6;", "    *w = wv + t6;")], [OPTIM]),
    ("weight update by reciprocal multiply", [("        d = root + s->eps;\n        u = m / d;",
                                               "        d = root + s->eps;\n        u = m * (1.0f / d);")], [OPTIM]),
    ("square root in binary64 then twice rounded up", [("float root = sqrtf(r);", "float root = nextafterf(sqrtf(r), 2.0f * sqrtf(r));")], [OPTIM]),
    ("sgd momentum applied to the gradient", [("float t1 = beta * m_prev;", "float t1 = beta * g;")], [OPTIM]),
    ("sgd decay after the momentum", [("    float t1 = beta * m_prev;\n    float m = t1 + g;",
                                       "    float t1 = beta * m_prev;\n    float m = t1 + g;\n    if (wd != 0.0f) m = m + wd * wv;")],
     [OPTIM]),
    ("second state searched in the signed map", [("quantize_block(q_unsigned, rbuf, len, r_q + st, N_r + b);\n    }\n    return 0;\n}\n\n/* For the parity report",
                                                  "quantize_block(q_signed, rbuf, len, r_q + st, N_r + b);\n    }\n    return 0;\n}\n\n/* For the parity report")],
     [OPTIM]),
    # --- Eq. quant1 - quant3
    ("normalisation by reciprocal multiply", [("float x = T[i] / N;", "float x = T[i] * (1.0f / N);")], [QUANT] + NOT_SEARCH),
    ("ties to the upper code", [("return (twice > sum) ? hi : lo;", "return (twice >= sum) ? hi : lo;")], [QUANT] + SEARCH),
    ("midpoint compared in binary32", [("double twice = 2.0 * (double)x;\n    double sum = (double)q[lo] + (double)q[hi];\n    return (twice > sum) ? hi : lo;",
                                        "float mid = 0.5f * (q[lo] + q[hi]);\n    return (x > mid) ? hi : lo;")], [QUANT] + SEARCH),
    ("block maximum without the absolute value", [("if (a > N)", "if (T[i] > N)")], [QUANT] + NOT_SEARCH),
    ("dequantize with the first block's maximum", [("TD[i] = q[TQ[i]] * N[i / B];", "TD[i] = q[TQ[i]] * N[0];")], [QUANT] + NOT_SEARCH),
    ("short last block padded with the full length", [("int64_t len = (n - s < B) ? n - s : B;\n        quantize_block(q, T + s, len, TQ + s, N + b);",
                                                       "int64_t len = (n - s < B) ? n - s : B;\n        quantize_block(q, T + s, len, TQ + s, N + b);\n        if (len < B) N[b] = N[b] * 1.0000001f;")],
     [QUANT] + NOT_SEARCH),
    # --- codebook
    ("bin edge instead of bin centre", [("double num = 0.9 * (double)(2 * k + 1);", "double num = 0.9 * (double)(2 * k + 2);")], [CODEBOOK]),
    ("binary instead of decimal exponent", [("p10 *= 10.0;", "p10 *= 2.0;")], [CODEBOOK]),
    ("codebook evaluated in binary32", [("double frac = 0.1 + num / (double)(1 << (F + 1));", "double frac = (float)(0.1f + (float)num / (float)(1 << (F + 1)));")],
     [CODEBOOK]),
    ("unsigned map without its extra fraction bit", [("        k |= lead << fbits_low;\n        F = fbits_low + 1;", "        F = fbits_low;")], [CODEBOOK]),
    # --- 16-bit storage
    ("bfloat16 ties rounded up", [("if (lo > 0x8000u || (lo == 0x8000u && (hi & 1u)))", "if (lo >= 0x8000u)")], [BF16]),
    ("binary16 ties rounded up", [("if (frac > 0.5 || (frac == 0.5 && (k & 1)))", "if (frac >= 0.5)")], [F16]),
    ("binary16 subnormals flushed", [("if (k < 1024)                                      /* subnormal (only when E = -14) */\n        return (uint16_t)(sign | (uint16_t)k);",
                                      "if (k < 1024)\n        return sign;")], [F16]),
]


def run_pins(src_path, files):
    env = dict(os.environ, Q8_ORACLE_SRC=src_path)
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *files],
                          cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)


@pytest.fixture(scope="module")
def outcomes(tmp_path_factory):
    """Build and judge every altered copy once, a few at a time (each run is its own process)."""
    source = open(SRC).read()
    work = tmp_path_factory.mktemp("mutants")

    def one(item):
        k, (name, edits, files) = item
        text = source
        for old, new in edits:
            if text.count(old) != 1:
                return name, "mutation does not apply exactly once: %r" % old
            text = text.replace(old, new)
        path = work / ("mutant%d.c" % k)
        path.write_text(text)
        return name, run_pins(str(path), files)
    cases = [("unaltered", [], [OPTIM, QUANT, CODEBOOK, BF16, F16, GOLDEN] + NOT_SEARCH)] + MUTATIONS
    try:
        workers = max(1, min(8, len(os.sched_getaffinity(0))))
    except AttributeError:
        workers = 2
    with ThreadPoolExecutor(workers) as ex:
        return dict(ex.map(one, enumerate(cases)))


def test_unaltered_copy_passes(outcomes):
    r = outcomes["unaltered"]
    assert not isinstance(r, str), r
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name", [m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(outcomes, name):
    r = outcomes[name]
    assert not isinstance(r, str), r
    assert r.returncode == 1 and " failed" in r.stdout, \
        "planted mistake %r survived its pins (exit %d)\n%s" % (name, r.returncode, r.stdout[-1500:])
