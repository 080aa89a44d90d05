"""The pins must notice a planted mistake: each case edits a copy of oracle.c, rebuilds it on the CPU and
expects tests/test_oracle_pins.py to fail against that copy.  The oracle itself is never modified."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "oracle.c")
SRC_EPILOGUE = os.path.join(ROOT, "oracle", "epilogue.c")
PIN_FILES = [os.path.join(ROOT, "tests", "test_oracle_pins.py"), os.path.join(ROOT, "tests", "test_oracle_epilogue.py")]

# (name, text in oracle.c, replacement, which occurrence)
MUTANTS = [
    ("second moment uses beta1 rate", "(1.0 - beta2) * gh * gh", "(1.0 - beta1) * gh * gh", 0),
    ("epsilon inside the root", "sqrt(v1) + eps", "sqrt(v1 + eps)", 0),
    ("no first-moment bias correction", "const double m1 = m_ / c1;", "const double m1 = m_;", 0),
    ("no second-moment bias correction", "const double v1 = v_ / c2;", "const double v1 = v_;", 0),
    ("update sign", "const double p_ = wi - lr * u;", "const double p_ = wi + lr * u;", 0),
    ("decoupled decay dropped", "if (adam_mode != 0) u += wd * wi;", "", 0),
    ("L2 decay dropped", "if (adam_mode == 0) gh += wd * wi;", "", 0),
    ("only the last rank is kept", "S += grad_f32 == 1 ?", "S = grad_f32 == 1 ?", 0),
    ("fp32 slices read as halves", "grad_f32 == 1 ? (double)((const float *)g[r])[i]", "0 ? (double)((const float *)g[r])[i]", 0),
    ("fp16 intermediate not rounded", "if (grad_f32 == 2) S = oracle_half_to_double(oracle_float_to_half((float)S));", "", 0),
    ("flag decided in double", "return !isfinite((float)S);", "return !isfinite(S);", 0),
    ("step off by one", "pow(beta1, (double)step)", "pow(beta1, (double)(step + 1))", 0),
    ("gradient not squared", "(double)v[i] * beta2 + (1.0 - beta2) * gh * gh;\n        const double m1", "(double)v[i] * beta2 + (1.0 - beta2) * gh;\n        const double m1", 0),
    ("loss scale multiplies", "double gh = S / div;", "double gh = S * div;", 0),
    ("average ignored", "(grad_average ? (double)R : 1.0)", "1.0", 0),
    ("flag ignores infinities", "return !isfinite((float)S);", "return isnan((float)S);", 0),
    ("guard keeps nothing", "if (guard_elements && sum_overflows(S)) {", "if (0) {", 0),
    ("trust ratio inverted", "norm_w / norm_u : 1.0", "norm_u / norm_w : 1.0", 0),
    ("trust ratio fallback", "norm_w / norm_u : 1.0", "norm_w / norm_u : 0.0", 0),
    ("norm of u without decay", "+ eps) + wd * wi;\n        sum_w2", "+ eps);\n        sum_w2", 0),
    ("LAMB applies no ratio", "wi - lr * ratio * u", "wi - lr * u", 0),
    ("LAMB second moment rate", "(1.0 - beta2) * gh * gh", "(1.0 - beta1) * gh * gh", 2),
    ("half subnormal scale", "ldexp((double)frac, -24)", "ldexp((double)frac, -25)", 0),
    ("half exponent bias", "expo - 25", "expo - 24", 0),
    ("half encode rounds ties up", "nearbyint(ldexp(fr, 11))", "floor(ldexp(fr, 11) + 0.5)", 0),
    ("half encode overflow threshold", "a >= 65520.0", "a > 65504.0", 0),
    ("skip emits no fp16", "w16_out[i] = oracle_float_to_half(w[i]);\n    }\n}", "w16_out[i] = 0;\n    }\n}", 0),
]


# planted in epilogue.c
EPILOGUE_MUTANTS = [
    ("philox multiplier", "0xD2511F53u", "0xD2511F55u", 0),
    ("philox key increment", "0x9E3779B9u", "0x9E3779B1u", 0),
    ("philox nine rounds", "round < 10", "round < 9", 0),
    ("philox lanes swapped", "n1 = lo1, n2 = hi0 ^ c[3] ^ k[1], n3 = lo0", "n1 = lo0, n2 = hi0 ^ c[3] ^ k[1], n3 = lo1", 0),
    ("wrong word of the block", "return w[index % 4];", "return w[(index + 1) % 4];", 0),
    ("block of two", "const uint64_t block = index / 4;", "const uint64_t block = index / 2;", 0),
    ("seed high half ignored", "(uint32_t)(seed >> 32)};", "0u};", 0),
    ("mask inverted", ">= threshold;", "< threshold;", 0),
    ("scale is 1-p", "1.0 / (1.0 - (double)p_f)", "(1.0 - (double)p_f)", 0),
    ("bias indexed by slice position", "bias[gi % hidden]", "bias[i % hidden]", 0),
    ("mask indexed by slice position", "oracle_dropout_word(seed, gi)", "oracle_dropout_word(seed, i)", 0),
    ("residual dropped too", "d + oracle_half_to_double(residual[i])", "keep ? d + oracle_half_to_double(residual[i]) : 0.0", 0),
    ("only one rank", "for (int r = 0; r < R; ++r) sum +=", "for (int r = 0; r < 1; ++r) sum +=", 0),
]


def _replace_nth(text, old, new, nth):
    pos = -1
    for _ in range(nth + 1):
        pos = text.find(old, pos + 1)
        assert pos >= 0, "mutation site not found: %r" % old
    return text[:pos] + new + text[pos + len(old):]


def _pins_fail_against(path_so):
    env = dict(os.environ, ORACLE_SO=path_so)
    r = subprocess.run([sys.executable, "-m", "pytest"] + PIN_FILES + ["-x", "-q", "-p", "no:cacheprovider"], cwd=ROOT, env=env,
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    return r.returncode != 0, r.stdout[-400:]


def test_every_planted_mistake_is_caught(tmp_path):
    src = {SRC: open(SRC).read(), SRC_EPILOGUE: open(SRC_EPILOGUE).read()}
    cases = [(SRC, m) for m in MUTANTS] + [(SRC_EPILOGUE, m) for m in EPILOGUE_MUTANTS]

    def run(case):
        i, (which, (name, old, new, nth)) = case
        c = tmp_path / ("mut%d.c" % i)
        so = tmp_path / ("mut%d.so" % i)
        c.write_text(_replace_nth(src[which], old, new, nth))
        other = SRC_EPILOGUE if which == SRC else SRC
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-w", "-o", str(so), str(c), other, "-lm"])
        failed, tail = _pins_fail_against(str(so))
        return name, failed, tail

    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(run, enumerate(cases)))
    missed = [name for name, failed, _ in results if not failed]
    assert not missed, "pins did not catch: %s" % missed


def test_unmodified_copy_passes(tmp_path):
    so = tmp_path / "same.so"
    subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-w", "-o", str(so), SRC, SRC_EPILOGUE, "-lm"])
    failed, tail = _pins_fail_against(str(so))
    assert not failed, tail
