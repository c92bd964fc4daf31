"""Are the oracle's pins strong enough?  Each case plants ONE plausible mistake (a dropped term, a wrong
sign or index, a swapped operand, an off-by-one) in a copy of oracle/eco_oracle.c, builds it, and runs the
pin tests (tests/test_oracle_{codec,random,step,modes,bf16}.py) against the copy in a child process: the pins must
fail.  The unmodified copy must pass.  Everything here runs on the CPU."""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "eco_oracle.c")
PINS = ["tests/test_oracle_codec.py", "tests/test_oracle_random.py", "tests/test_oracle_step.py",
        "tests/test_oracle_modes.py", "tests/test_oracle_bf16.py"]

# (name, text in the oracle, what a mistaken author might have written)
MUTANTS = [
    ("adam injection: sign of (1 - 1/beta1)",
     "kap = (REAL)((bc1 / cfg->lr) * (1.0 - 1.0 / cfg->beta1));", "kap = (REAL)((bc1 / cfg->lr) * (1.0 / cfg->beta1 - 1.0));"),
    ("adam injection: bias correction dropped from kappa",
     "kap = (REAL)((bc1 / cfg->lr) * (1.0 - 1.0 / cfg->beta1));", "kap = (REAL)((1.0 / cfg->lr) * (1.0 - 1.0 / cfg->beta1));"),
    ("adam injection: the factor sqrt(v^)+eps dropped",
     "r_fma(kap * dd[j], e, mt[j])", "r_fma(kap, e, mt[j])"),
    ("sgdm injection: 1/eta dropped from alpha",
     "alpha = (REAL)((1.0 / cfg->lr) * (1.0 - 1.0 / cfg->beta1));", "alpha = (REAL)(1.0 - 1.0 / cfg->beta1);"),
    ("sgdm injection: 1 - beta instead of 1 - 1/beta",
     "alpha = (REAL)((1.0 / cfg->lr) * (1.0 - 1.0 / cfg->beta1));", "alpha = (REAL)((1.0 / cfg->lr) * (1.0 - cfg->beta1));"),
    ("error with the wrong sign", "e = th[j] - q;", "e = q - th[j];"),
    ("bias correction exponent off by one",
     "bc1 = 1.0 - pow(cfg->beta1, (double)cfg->step);", "bc1 = 1.0 - pow(cfg->beta1, (double)cfg->step + 1.0);"),
    ("second-moment bias correction off by one",
     "bc2 = 1.0 - pow(cfg->beta2, (double)cfg->step);", "bc2 = 1.0 - pow(cfg->beta2, (double)cfg->step + 1.0);"),
    ("eps inside the square root", "dd[j] = r_sqrt(vt * rbc2) + epsf;", "dd[j] = r_sqrt(vt * rbc2 + epsf);"),
    ("adam step size without the bias correction of the first moment", "c1 = (REAL)(cfg->lr / bc1);", "c1 = (REAL)(cfg->lr);"),
    ("second moment of g instead of g*g", "omb2 * (g * g)", "omb2 * g"),
    ("momentum without the (1 - beta) damping", "mt[j] = r_fma(b1, m[i], omb1 * g);", "mt[j] = r_fma(b1, m[i], g);"),
    ("update added instead of subtracted", "th[j] = w - u;", "th[j] = w + u;"),
    ("weight decay with the wrong sign", "w = w - wdf * w;", "w = w + wdf * w;"),
    ("scale from rho + 1", "s = a / (REAL)rho;", "s = a / ((REAL)rho + 1);"),
    ("E4M3 exponent bias off by one", "ldexp((double)(8u + M), (int)E - 10)", "ldexp((double)(8u + M), (int)E - 9)"),
    ("E4M3 subnormal spacing", "ldexp((double)M, -9)", "ldexp((double)M, -10)"),
    ("nearest rounding: ties away from zero", "(below == above && (lo & 1))", "(below == above)"),
    ("stochastic rounding: strict threshold", "up = (F + 16.0 * (double)r16 + 8.0 >= 1048576.0);", "up = (F + 16.0 * (double)r16 + 8.0 > 1048576.0);"),
    ("stochastic rounding: random bits not scaled", "up = (F + 16.0 * (double)r16 + 8.0 >= 1048576.0);", "up = (F + (double)r16 + 8.0 >= 1048576.0);"),
    ("stochastic rounding: truncating rule (pulls toward zero)", "up = (F + 16.0 * (double)r16 + 8.0 >= 1048576.0);", "up = (F + 16.0 * (double)r16 >= 1048576.0);"),
    ("stochastic rounding: rounds up where it should round down", "up = (F + 16.0 * (double)r16 + 8.0 >= 1048576.0);", "up = !(F + 16.0 * (double)r16 + 8.0 >= 1048576.0);"),
    ("INT4 nibbles transposed (read)", "return (i & 1) ? (unsigned)(codes[i >> 1] >> 4) : (unsigned)(codes[i >> 1] & 15u);",
     "return (i & 1) ? (unsigned)(codes[i >> 1] & 15u) : (unsigned)(codes[i >> 1] >> 4);"),
    ("INT4 negative codes not two's complement", "return (unsigned)(neg ? -mag : mag) & 15u;", "return (unsigned)(mag | (neg << 3)) & 15u;"),
    ("Philox multiplier", "0xCD9E8D57u", "0xCD9E8D59u"),
    ("Philox key bumped before the first round", "if (r > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }", "{ k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }"),
    ("Philox output words crossed", "n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;", "n0 = (uint32_t)(p0 >> 32) ^ c1 ^ k0;"),
    ("random field of odd and even elements swapped in the step",
     "r16 = (gi & 1) ? (word >> 16) : (word & 0xFFFFu);", "r16 = (gi & 1) ? (word & 0xFFFFu) : (word >> 16);"),
    ("element offset ignored by the random counter", "const uint64_t gi = cfg->elem_offset + i;", "const uint64_t gi = i;"),
    ("step missing from the random counter", "ctr[2] = (uint32_t)step;", "ctr[2] = 0;"),
    ("bf16 rounding keeps 9 bits", "ue = ex - 8; ", "ue = ex - 9; "),
    ("exact injection: coefficients swapped", "mh = r_fma(-cb, e, r_fma(ca, aux[i], mt[j]));", "mh = r_fma(-ca, e, r_fma(cb, aux[i], mt[j]));"),
    ("master weights: update applied to the de-quantized weights", "if (mode == MODE_MASTER) w = aux[i];\n      else if (quantized)", "if (quantized)"),
    ("master weights: momentum gets the injection too", "else mh = mt[j];", "else mh = adam ? r_fma(kap * dd[j], e, mt[j]) : r_fma(alpha, e, mt[j]);"),
    ("bf16 scales: codes relative to the unrounded scale", "if (scale_bf16) { s = bf16_round_(s); inv = (REAL)1 / s; }",
     "if (scale_bf16) { s = bf16_round_(s); inv = (REAL)rho / a; }"),
    ("bf16 state: denominator from the rounded second moment", "dd[j] = r_sqrt(vt * rbc2) + epsf;",
     "dd[j] = r_sqrt((cfg->state_bf16 ? bf16_round_(vt) : vt) * rbc2) + epsf;"),
    ("bf16 state: injection added onto the rounded first moment", "mh = adam ? r_fma(kap * dd[j], e, mt[j]) : r_fma(alpha, e, mt[j]);",
     "mh = adam ? r_fma(kap * dd[j], e, cfg->state_bf16 ? bf16_round_(mt[j]) : mt[j]) : r_fma(alpha, e, cfg->state_bf16 ? bf16_round_(mt[j]) : mt[j]);"),
    ("bf16 state: the momentum is stored unrounded", "m[i] = cfg->state_bf16 ? bf16_round_(mh) : mh;", "m[i] = mh;"),
    ("error measured against the unrounded scale", "q = decode(fmt, code) * s_new;", "q = decode(fmt, code) / inv;"),
    ("old scale of the neighbouring block", "decode(fmt, get_code(fmt, codes, i)) * scales[b];", "decode(fmt, get_code(fmt, codes, i)) * scales[b > 0 ? b - 1 : 0];"),
]


def run_pins(source, workdir):
    env = dict(os.environ, ECO_ORACLE_SOURCE=source, OMP_NUM_THREADS="1", PYTHONDONTWRITEBYTECODE="1")
    r = subprocess.run([sys.executable, "-m", "pytest", *PINS, "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)
    return r.returncode, r.stdout[-1500:]


def compile_ok(source):
    for ctype in ("float", "double"):
        r = subprocess.run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
                            f"-DREAL={ctype}", source, "-o", os.devnull, "-lm"], stdout=subprocess.PIPE, stderr=subprocess.STDOUT)
        if r.returncode != 0:
            return False
    return True


def test_the_pins_notice_every_planted_mistake(tmp_path):
    text = open(SRC).read()
    jobs = []
    control = tmp_path / "control"
    control.mkdir()
    shutil.copy(SRC, control / "eco_oracle.c")
    jobs.append(("control (no mistake)", str(control / "eco_oracle.c")))
    for k, (name, old, new) in enumerate(MUTANTS):
        assert text.count(old) >= 1, f"mutant '{name}': its anchor is no longer in the oracle"
        d = tmp_path / f"m{k:02d}"
        d.mkdir()
        src = d / "eco_oracle.c"
        src.write_text(text.replace(old, new))
        assert compile_ok(str(src)), f"mutant '{name}' does not compile"
        jobs.append((name, str(src)))
    with ThreadPoolExecutor(max_workers=max(2, min(8, os.cpu_count() or 4))) as ex:
        results = list(ex.map(lambda j: run_pins(j[1], None), jobs))
    rc0, out0 = results[0]
    assert rc0 == 0, "the pins fail on an unmodified copy of the oracle:\n" + out0
    survivors = [name for (name, _), (rc, _) in zip(jobs[1:], results[1:]) if rc == 0]
    assert not survivors, "no pin notices these planted mistakes: " + "; ".join(survivors)
    broken = [(name, out) for (name, _), (rc, out) in zip(jobs[1:], results[1:]) if rc not in (0, 1)]
    assert not broken, "pin run ended abnormally for: " + "; ".join(n for n, _ in broken) + "\n" + broken[0][1]
