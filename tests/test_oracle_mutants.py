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
    ("second moment uses beta1 rate", "(1.0 - k->beta2) * grad * grad", "(1.0 - k->beta1) * grad * grad", 0),
    ("second moment decays with beta1", "k->beta2 * second_moment", "k->beta1 * second_moment", 0),
    ("epsilon inside the root", "const double spread = sqrt(e.second_moment / k->unbias2);\n    e.direction = mean / (spread + k->eps);",
     "const double spread = sqrt(e.second_moment / k->unbias2 + k->eps);\n    e.direction = mean / spread;", 0),
    ("no first-moment bias correction", "e.first_moment / k->unbias1", "e.first_moment", 0),
    ("no second-moment bias correction", "e.second_moment / k->unbias2", "e.second_moment", 0),
    ("update sign", "(double)w[i] - k.lr * e.direction", "(double)w[i] + k.lr * e.direction", 0),
    ("decoupled decay dropped", "if (!k->decay_in_gradient) e.direction += k->decay * weight;", "", 0),
    ("L2 decay dropped", "if (k->decay_in_gradient) grad += k->decay * weight;", "", 0),
    ("decay modes swapped", "adam_mode == 0);", "adam_mode != 0);", 0),
    ("only the last rank is kept", "total += kind == SLICES_F32 ?", "total = kind == SLICES_F32 ?", 0),
    ("fp32 slices read as halves", "kind == SLICES_F32 ? (double)((const float *)slice[r])[i]", "0 ? (double)((const float *)slice[r])[i]", 0),
    ("fp16 intermediate not rounded", "if (kind == SLICES_F16_SUM_F16) total = oracle_half_to_double(oracle_float_to_half((float)total));", "", 0),
    ("flag decided in double", "return !isfinite((float)total);", "return !isfinite(total);", 0),
    ("step off by one", "pow(k.beta1, (double)step)", "pow(k.beta1, (double)(step + 1))", 0),
    ("second bias correction from beta1", "pow(k.beta2, (double)step)", "pow(k.beta1, (double)step)", 0),
    ("gradient not squared", "(1.0 - k->beta2) * grad * grad", "(1.0 - k->beta2) * grad", 0),
    ("loss scale multiplies", "double grad = total / k->grad_divisor;", "double grad = total * k->grad_divisor;", 0),
    ("average ignored", "(grad_average ? (double)R : 1.0)", "1.0", 0),
    ("flag ignores infinities", "return !isfinite((float)total);", "return isnan((float)total);", 0),
    ("guard keeps nothing", "if (guard_elements && sum_overflows(total)) {", "if (0) {", 0),
    ("state not rounded to fp32 before the fp16 copy", "*w16_out = oracle_float_to_half(*w_out);", "*w16_out = oracle_double_to_half(weight_new);", 0),
    ("trust ratio inverted", "weight_norm / direction_norm : 1.0", "direction_norm / weight_norm : 1.0", 0),
    ("trust ratio fallback", "weight_norm / direction_norm : 1.0", "weight_norm / direction_norm : 0.0", 0),
    ("LAMB takes L2 decay", "step, R, grad_average, 0);", "step, R, grad_average, 1);", 0),
    ("LAMB applies no ratio", "k.lr * trust * e.direction", "k.lr * e.direction", 0),
    ("weight norm not squared", "weight_squares += (double)w[i] * (double)w[i];", "weight_squares += fabs((double)w[i]);", 0),
    ("direction norm without the root", "direction_norm = sqrt(direction_squares)", "direction_norm = direction_squares", 0),
    ("LAMB moments not stored", "m_out[i] = (float)e.first_moment;\n        v_out[i] = (float)e.second_moment;\n        weight_squares",
     "m_out[i] = m[i];\n        v_out[i] = v[i];\n        weight_squares", 0),
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
