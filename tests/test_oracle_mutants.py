"""The pins must catch plausible mistakes: each mutant below is the oracle's C source with one
planted error (a dropped term, a wrong sign or index, a transposed operand ...), compiled on the
CPU and run through the pins of test_oracle_pins.py.  Every mutant must fail at least one pin."""
import ctypes
import importlib.util
import os
import subprocess
import sys

import pytest

import test_oracle_pins as pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "sphattn_oracle.c")

MUTANTS = [
    ("sum of |s| instead of s^2", "z += acc * acc;", "z += fabs(acc);"),
    ("missing square root", "double nrm = sqrt(z);", "double nrm = z;"),
    ("epsilon added under the root", "double nrm = sqrt(z);", "double nrm = sqrt(z + 1e-6);"),
    ("scores scaled by 1/sqrt(d) only in the numerator",
     "o[k] += s[j] * Vh[(size_t)j * d + k];\n    double nrm", "o[k] += s[j] / sqrt((double)d) * Vh[(size_t)j * d + k];\n    double nrm"),
    ("weights lose their sign", "            o[k] += s[j] * Vh[(size_t)j * d + k];\n    double nrm",
     "            o[k] += fabs(s[j]) * Vh[(size_t)j * d + k];\n    double nrm"),
    ("K indexed transposed", "acc += q[k] * (m ? m[j] * Kh[(size_t)j * d + k] : Kh[(size_t)j * d + k]);",
     "acc += q[k] * (m ? m[j] * Kh[(size_t)j * d + k] : Kh[((size_t)k * N + j) % ((size_t)N * d)]);"),
    ("last key dropped", "    for (int j = 0; j < N; ++j) {\n        double acc = 0.0;\n        for (int k = 0; k < d; ++k)\n            acc += q[k] * (m",
     "    for (int j = 0; j < N - (N > 1); ++j) {\n        double acc = 0.0;\n        for (int k = 0; k < d; ++k)\n            acc += q[k] * (m"),
    ("wrong head for K/V", "const size_t kvh = (size_t)b * H_kv + h / (H / H_kv);   /* K/V head of this query head */",
     "const size_t kvh = (size_t)b * H_kv + h % H_kv;"),
    ("multiplicity of the query gene instead of the key gene", "(m ? m[j] * Kh[(size_t)j * d + k]", "(m ? m[0] * Kh[(size_t)j * d + k]"),
    ("streamed loop forgets to carry z", "                z += dz;", "                z = dz;"),
    ("bf16 widened from the low half", "uint32_t u = (uint32_t)bits << 16;", "uint32_t u = (uint32_t)bits;"),
    ("e4m3 bias off by one", "v = ldexp(1.0 + (double)m / 8.0, e - 7);", "v = ldexp(1.0 + (double)m / 8.0, e - 8);"),
    ("accumulator sums x instead of x^2", "    z += x * x;\n                        for", "    z += x;\n                        for"),
    ("accumulator forgets the multiplicity", "x += q[k] * (m ? m[j] * Kh[(size_t)j * d + k] : Kh[(size_t)j * d + k]);\n                        z +=",
     "x += q[k] * Kh[(size_t)j * d + k];\n                        z +="),
    ("accumulator indexes K/V rows with N_q", "const double *m = mult ? mult + (size_t)b * N_k : NULL;", "const double *m = mult ? mult + (size_t)b * N_q : NULL;"),
    ("backward: the term through z has the wrong power of r", "double ds = r[i] * gv - delta[i] * r[i] * r[i] * s;\n                if (m)\n                    ds *= m[j];                      /* d s_ij",
     "double ds = r[i] * gv - delta[i] * r[i] * s;\n                if (m)\n                    ds *= m[j];                      /* d s_ij"),
    ("backward: multiplicity missing on the way from ds to dK", "                if (m)\n                    ds *= m[j];\n                for (int k = 0; k < d; ++k) {\n                    dv[k]",
     "                for (int k = 0; k < d; ++k) {\n                    dv[k]"),
    ("backward: K/V gradients of a group overwrite each other", "double *dk = dK + kvh * head + (size_t)j * d, *dv = dV + kvh * head + (size_t)j * d;\n            for (int i = 0; i < N; ++i) {",
     "double *dk = dK + kvh * head + (size_t)j * d, *dv = dV + kvh * head + (size_t)j * d;\n            for (int k = 0; k < d; ++k) dk[k] = dv[k] = 0.0;\n            for (int i = 0; i < N; ++i) {"),
    ("backward: dK built from k instead of q", "dk[k] += ds * q[k];", "dk[k] += ds * kj[k];"),
    ("backward: dV forgets the normalisation", "double w = r[i] * s;", "double w = s;"),
    ("softmax without max shift and with wrong scale", "double c = 1.0 / sqrt((double)d);", "double c = 1.0 / (double)d;"),
]


def _mutant_module(tmp_path, idx, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation site not found: {old!r}"
    csrc = tmp_path / f"mutant_{idx}.c"
    lib = tmp_path / f"mutant_{idx}.so"
    csrc.write_text(text.replace(old, new, 1))
    subprocess.run(["gcc", "-O1", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", str(lib), str(csrc), "-lm"],
                   check=True)
    spec = importlib.util.spec_from_file_location(f"oracle_mutant_{idx}", os.path.join(ROOT, "oracle", "__init__.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod._LIB = str(lib)
    mod.build = lambda force=False: str(lib)
    return mod


def _pin_calls(o):
    yield lambda: pins.test_hand_worked_example(o)
    for args in [(2, 3, 1), (5, 2, 2), (8, 4, 3)]:
        yield lambda a=args: pins.test_brute_force_rationals(o, *a)
    yield lambda: pins.test_unit_norm_weight_rows(o)
    yield lambda: pins.test_scale_and_sign_invariance(o)
    yield lambda: pins.test_single_key_closed_form(o)
    yield lambda: pins.test_orthonormal_keys_closed_form(o)
    yield lambda: pins.test_gram_matrix_closed_form(o)
    for chunk in (1, 7, 29):
        yield lambda c=chunk: pins.test_streaming_identity(o, c)
    yield lambda: pins.test_bag_invariances(o)
    yield lambda: pins.test_bf16_widening_all_codes(o)
    yield lambda: pins.test_e4m3fn_widening_all_codes(o)
    yield lambda: pins.test_softmax_twin_against_library(o)
    for hh in [(4, 2), (6, 1)]:
        yield lambda a=hh: pins.test_grn_variant_against_numpy_definition(o, *a)
    yield lambda: pins.test_grn_multiplicity_brute_force_rationals(o)
    yield lambda: pins.test_accumulator_brute_force_rationals_rectangular(o)
    yield lambda: pins.test_accumulator_single_key_closed_form(o)
    yield lambda: pins.test_accumulators_add_over_key_partitions_and_tail_gives_attention(o, (0, 16, 32, 37))
    yield lambda: pins.test_backward_against_central_differences(o)
    yield lambda: pins.test_backward_against_library_autograd(o)
    yield lambda: pins.test_backward_structure(o)
    yield lambda: pins.test_grn_backward_against_central_differences_and_autograd(o)


@pytest.mark.parametrize("idx", range(len(MUTANTS)))
def test_every_planted_mistake_is_caught(tmp_path, idx):
    name, old, new = MUTANTS[idx]
    mutant = _mutant_module(tmp_path, idx, old, new)
    caught = 0
    for call in _pin_calls(mutant):
        try:
            call()
        except AssertionError:
            caught += 1
    assert caught > 0, f"no pin noticed the mutant: {name}"
