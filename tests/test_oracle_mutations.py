"""The pins must notice a broken oracle: each case plants one plausible mistake in a copy of the oracle's C source
(a dropped rounding term, a wrong sign, a transposed index, ...), builds it, and runs the pin suite against it in a
subprocess.  The suite has to fail for every mutant (and pass for the unmodified source)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "tfhe_oracle.c")

MUTANTS = {
    "sample_extract_no_negation": ("lwe_out[(size_t)r * N + j] = (uint64_t)0 - acc[(size_t)r * N + N - j];",
                                   "lwe_out[(size_t)r * N + j] = acc[(size_t)r * N + N - j];"),
    "decompose_truncates": ("else            v = (x + ((uint64_t)1 << (63 - bits))) >> (64 - bits);",
                            "else            v = x >> (64 - bits);"),
    "digit_tie_goes_positive": ("if (d >= (B >> 1)) { sd -= (int64_t)B; v += 1; }", "if (d > (B >> 1)) { sd -= (int64_t)B; v += 1; }"),
    "digit_carry_dropped": ("if (d >= (B >> 1)) { sd -= (int64_t)B; v += 1; }", "if (d >= (B >> 1)) { sd -= (int64_t)B; }"),
    "modswitch_truncates": ("uint64_t y = (x + ((uint64_t)1 << (w - 1))) >> w;", "uint64_t y = x >> w;"),
    "monomial_sign": ("out[j] = negate ? (uint64_t)0 - v : v;", "out[j] = negate ? v : (uint64_t)0 - v;"),
    "cyclic_instead_of_negacyclic": ("else       out[c - N] -= term;", "else       out[c - N] += term;"),
    "cmux_adds_instead_of_subtracts": ("lam[(size_t)r * N + c] -= acc[(size_t)r * N + c];", "lam[(size_t)r * N + c] += acc[(size_t)r * N + c];"),
    "cmux_rows_transposed": ("const uint64_t *row = bsk_i + ((size_t)r * l + j) * glwe;", "const uint64_t *row = bsk_i + ((size_t)j * (k + 1) + r) * glwe;"),
    "keyswitch_adds": ("out[x] -= dj * row[x];", "out[x] += dj * row[x];"),
    "keyswitch_levels_reversed": ("const uint64_t *row = ksk + ((size_t)i * l + j) * (n + 1);", "const uint64_t *row = ksk + ((size_t)i * l + (l - 1 - j)) * (n + 1);"),
    "lut_not_rotated_by_half_box": ("uint32_t box = p->N / t, h = box / 2;", "uint32_t box = p->N / t, h = 0;"),
    "accumulator_rotated_the_wrong_way": ("orc_monomial_mul(lut, N, (2 * N - bt) % (2 * N), acc + (size_t)k * N);", "orc_monomial_mul(lut, N, bt, acc + (size_t)k * N);"),
    "gadget_on_wrong_component": ("ct[(size_t)r * N] += lwe_sk[i] << (64 - j * p->pbs_base_log);", "ct[(size_t)k * N] += lwe_sk[i] << (64 - j * p->pbs_base_log);"),
    "body_sign_in_encryption": ("for (uint32_t i = 0; i < dim; i++) { ct[i] = mask[i]; b += mask[i] * sk[i]; }", "for (uint32_t i = 0; i < dim; i++) { ct[i] = mask[i]; b -= mask[i] * sk[i]; }"),
    "lincomb_drops_sign_extension": ("uint64_t wj = (uint64_t)(int64_t)w[(size_t)j * O + o];", "uint64_t wj = (uint64_t)(uint32_t)w[(size_t)j * O + o];"),
}


def _run_pins(lib_path):
    env = dict(os.environ, TFHE_ORACLE_LIB=lib_path)
    return subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                           "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)


def _build(src_text, out):
    c = out + ".c"
    with open(c, "w") as f:
        f.write(src_text)
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", out, c])


def test_unmodified_source_passes(tmp_path):
    out = str(tmp_path / "orig.so")
    _build(open(SRC).read(), out)
    r = _run_pins(out)
    assert r.returncode == 0, r.stdout.decode()[-2000:]


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_mutant(tmp_path, name):
    old, new = MUTANTS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, "mutation site not found exactly once: %s" % name
    out = str(tmp_path / (name + ".so"))
    _build(text.replace(old, new), out)
    r = _run_pins(out)
    assert r.returncode != 0, "the pins did not notice: %s" % name
