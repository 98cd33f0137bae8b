"""The pins must be sharp: a plausible mistake planted in a copy of the
oracle's C source (on the CPU, never in GPU code) has to fail at least one
pin of tests/test_oracle_pins.py."""
import ctypes
import json
import os
import subprocess

import pytest

import oracle
import test_oracle_lowbit as lowbit
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "sketch_oracle.c")

MUTANTS = {
    "hash drops the additive constant":
        ("(uint64_t)A * (uint64_t)a + (uint64_t)C)", "(uint64_t)A * (uint64_t)a)"),
    "hash reduces with modulo instead of multiply-shift":
        ("(uint32_t)((t * (uint64_t)K) >> 24)", "(uint32_t)(t % K)"),
    "address is column-major inside the group":
        ("uint32_t a = jl * to + ol;  /* Addr(w): offset in the group */", "uint32_t a = ol * tj + jl;"),
    "query address is column-major inside the group":
        ("uint32_t a = jl * to + ol;\n                    uint16_t best", "uint32_t a = ol * tj + jl;\n                    uint16_t best"),
    "update keeps the larger magnitude":
        ("if (fabs(ora_half_to_double(*s)) > aw) *s = w;", "if (fabs(ora_half_to_double(*s)) < aw || *s == 0x7C00) *s = w;"),
    "update lets the later arrival win a tie":
        ("if (fabs(ora_half_to_double(*s)) > aw) *s = w;", "if (fabs(ora_half_to_double(*s)) >= aw) *s = w;"),
    "update compares signed values":
        ("double aw = fabs(ora_half_to_double(w));", "double aw = ora_half_to_double(w);"),
    "query takes the signed maximum":
        ("if (mc > mb) return cand;", "if (ora_half_to_double(cand) > ora_half_to_double(best)) return cand; else return best;"),
    "query tie goes to the negative value":
        ("(cand >> 15) == 0", "(cand >> 15) == 1"),
    "query tie goes to the first row":
        ("if (mc == mb && (cand >> 15) == 0) return cand;", ""),
    "query takes the minimum magnitude":
        ("if (mc > mb) return cand;", "if (mc < mb) return cand;"),
    "query skips the last row":
        ("for (uint32_t r = 1; r < d; ++r) {\n                        uint16_t cand", "for (uint32_t r = 1; r + 1 < d; ++r) {\n                        uint16_t cand"),
    "rows share the first row's table":
        ("uint16_t cand = S[(uint64_t)r * K + ora_select", "uint16_t cand = S[ora_select"),
    "signed query compares magnitudes":
        ("if (vc > vb) return cand;", "if (fabs(vc) > fabs(vb)) return cand;"),
    "signed query takes the minimum":
        ("if (vc > vb) return cand;", "if (vc < vb) return cand;"),
    "signed query lets -0 win the zero tie":
        ("if (vc == vb && (cand >> 15) == 0) return cand;", "if (vc == vb && (cand >> 15) == 1) return cand;"),
    "signed query keeps the first row on a zero tie":
        ("if (vc == vb && (cand >> 15) == 0) return cand;", ""),
    "query modes are swapped":
        ("best = mode == 1 ? signedmax_pick(best, cand)", "best = mode == 0 ? signedmax_pick(best, cand)"),
    "group base advances by one row only":
        ("base += (uint64_t)d * K;\n        }\n    return ORA_OK;\n}\n\nint ora_query(", "base += K;\n        }\n    return ORA_OK;\n}\n\nint ora_query("),
    "groups are numbered column-major":
        ("uint32_t K = width[(uint64_t)jb * g.n_ob + ob];\n            const uint16_t *S", "uint32_t K = width[(uint64_t)ob * g.n_jb + jb];\n            const uint16_t *S"),
    "linear reads W transposed":
        ("W_hat[(uint64_t)j * out + o]", "W_hat[(uint64_t)o * in + j]"),
    "linear accumulates in single precision":
        ("double acc = 0.0;", "float acc = 0.0f;"),
    "linear skips the last input channel":
        ("for (uint32_t j = 0; j < in; ++j) {", "for (uint32_t j = 0; j + 1 < in; ++j) {"),
    "half conversion mis-scales subnormals":
        ("v = ldexp((double)m, -24);", "v = ldexp((double)m, -25);"),
    "half conversion drops the hidden bit":
        ("ldexp((double)(m + 1024), e - 25)", "ldexp((double)(m), e - 25)"),
    "never-reached states are left at +inf":
        ("if (states[i] == 0x7C00) states[i] = 0x0000;", ""),
    "low-bit codes round half away from zero":
        ("nearbyint(ora_half_to_double(S[k]) * (double)qmax / sc)", "round(ora_half_to_double(S[k]) * (double)qmax / sc)"),
    "low-bit step divides by qmax + 1":
        ("(double)q * sc / (double)qmax", "(double)q * sc / (double)(qmax + 1)"),
    "low-bit scale is the first state of the row":
        ("if ((S[k] & 0x7FFF) > top) top = S[k] & 0x7FFF;", "if (k == 0) top = S[k] & 0x7FFF;"),
    "low-bit state is truncated to binary16":
        ("double q = nearbyint(a / step);", "double q = floor(a / step);"),
    "low-bit scale of the first row serves the whole group":
        ("double sc = ora_half_to_double(scales[g * d + r]);", "double sc = ora_half_to_double(scales[g * d]);"),
    "low-bit four-bit codes use the eight-bit range":
        ("return bits == 8 ? 127 : bits == 4 ? 7 : 0;", "return bits == 8 ? 127 : bits == 4 ? 127 : 0;"),
}

PIN_FUNCS = [
    "test_worked_example_select", "test_worked_example_update_query_linear",
    "test_half_to_double_all_patterns", "test_select_identity_special_case",
    "test_select_range_and_extremes", "test_update_matrix_form_eq8",
    "test_query_matrix_form_eq9_single_row", "test_query_signed_zero_tie",
    "test_invariants_on_cfg1", "test_row_order_invariance_and_more_rows_never_hurt",
    "test_linear_against_numpy_fp64_and_one_hot",
    "test_worked_example_signed_max_query", "test_signed_max_query_zero_tie_and_negative_candidates",
]


def _example():
    with open(os.path.join(pins.GOLD, "worked_example.json")) as f:
        e = json.load(f)
    e["A"] = [int(v, 16) for v in e["hash_a"]]
    e["C"] = [int(v, 16) for v in e["hash_c"]]
    return e


def _run_pins():
    failed = []
    ex = _example()
    calls = [(n, getattr(pins, n)) for n in PIN_FUNCS]
    for n, fn in calls:
        try:
            fn(ex) if "worked_example" in n else fn()
        except (AssertionError, ValueError, IndexError) as e:
            failed.append(n)
    for shape in [(8, 12, 4, 6, 3), (6, 16, 1, 16, 4)]:
        try:
            pins.test_update_equals_sort_brute_force(shape)
        except (AssertionError, ValueError, IndexError):
            failed.append("test_update_equals_sort_brute_force")
    for d in (2, 4):
        try:
            pins.test_query_multi_row_via_matrix_forms(d)
        except (AssertionError, ValueError, IndexError):
            failed.append("test_query_multi_row_via_matrix_forms")
    for d in (2, 3):
        try:
            pins.test_signed_max_query_via_matrix_forms_and_numpy_max(d)
        except (AssertionError, ValueError, IndexError):
            failed.append("test_signed_max_query_via_matrix_forms_and_numpy_max")
    try:
        pins.test_identity_hash_reproduces_W(2)
    except (AssertionError, ValueError, IndexError):
        failed.append("test_identity_hash_reproduces_W")
    for fn in (lowbit.test_hand_worked_codes_four_bit, lowbit.test_hand_worked_codes_eight_bit,
               lowbit.test_hand_worked_non_integer_step):
        try:
            fn()
        except (AssertionError, ValueError, IndexError):
            failed.append(fn.__name__)
    for bits in (8, 4):
        for fn in (lowbit.test_end_points_symmetry_and_order,
                   lowbit.test_scale_is_the_row_maximum_and_error_is_at_most_half_a_step):
            try:
                fn(bits)
            except (AssertionError, ValueError, IndexError):
                failed.append(fn.__name__)
    return failed


def test_unmutated_oracle_passes_the_pin_subset():
    assert _run_pins() == []


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name, tmp_path):
    old, new = MUTANTS[name]
    src = open(SRC).read()
    assert src.count(old) >= 1, f"mutation site not found: {name}"
    # mutate the first site only when the text occurs in both update and query
    mutated = src.replace(old, new, 1)
    c = tmp_path / "mut.c"
    so = tmp_path / "mut.so"
    c.write_text(mutated)
    subprocess.check_call(["gcc", "-O1", "-std=c11", "-fPIC", "-shared", "-w", "-o", str(so), str(c), "-lm"])
    good = oracle._load()
    try:
        oracle._lib = oracle._bind(ctypes.CDLL(str(so)))
        failed = _run_pins()
    finally:
        oracle._lib = good
    assert failed, f"no pin noticed: {name}"
