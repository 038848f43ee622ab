"""The pins have teeth: plant one plausible mistake at a time in a COPY of the oracle's
source (on the CPU, in a temporary file), load it in place of the real oracle, and check
that at least one pin fails.  Nothing here touches the GPU or the committed oracle."""
import ctypes
import os
import subprocess
import tempfile

import pytest

import oracle
import test_oracle_pins as pins

SRC = open(os.path.join(os.path.dirname(oracle.__file__), "contraction_oracle.cpp")).read()

# (name, text to find, replacement); every `find` must occur in the source
MUTANTS = [
    ("conj_dropped", "return op == OP_CONJ ? std::conj(x) : x;", "return x;"),
    ("complex_mul_sign", "a.real() * b.real() - a.imag() * b.imag()", "a.real() * b.real() + a.imag() * b.imag()"),
    ("odometer_never_carries", "while (k < shape.size() && ++idx[k] == shape[k]) idx[k++] = 0;",
     "if (!shape.empty() && ++idx[0] == shape[0]) idx[0] = 0;"),
    ("beta_term_dropped", "if (read_c) d = d + mul(beta,", "if (false) d = d + mul(beta,"),
    ("repeated_label_last_stride_only", "if (t.label[i] == lab) s += t.stride[i];", "if (t.label[i] == lab) s = t.stride[i];"),
    ("B_addressed_with_A_strides", "const int64_t off_B = baseB + displacement(K, psB);", "const int64_t off_B = baseB + displacement(K, psA);"),
    ("opC_ignored", "Widen<Acc, T>::of(apply_op(C[off_D], opC))", "Widen<Acc, T>::of(C[off_D])"),
    ("C_read_at_linear_index", "mul(beta, Widen<Acc, T>::of(apply_op(C[off_D], opC)))", "mul(beta, Widen<Acc, T>::of(apply_op(C[lin], opC)))"),
    ("alpha_also_scales_C", "D[off_D] = Narrow<T, Acc>::of(d);", "D[off_D] = Narrow<T, Acc>::of(read_c ? mul(alpha, d) : d);"),
    ("hadamard_label_summed", "if (has_label(tD, lab)) continue;", "if (has_label(tD, lab) && !has_label(tB, lab)) continue;"),
    ("aliasing_check_off", "if (p.first <= span) return V_D_ALIASING;", "if (false) return V_D_ALIASING;"),
    ("label_only_in_B_left_out", "only_B.push_back(l);", ";"),
    ("reduction_in_B_never_moves", "l.sA = 0; l.sB = summed_stride(tB, lab); l.sD = 0;", "l.sA = 0; l.sB = 0; l.sD = 0;"),
    ("reduction_keeps_last_element", "sum = sum + x;", "sum = x;"),
    ("free_stride_of_A_dropped", "const int64_t baseA = displacement(I, dsA);", "const int64_t baseA = 0;"),
    ("complex_modulus_is_squared_norm", "return hypotl(x.real(), x.imag());", "return x.real() * x.real() + x.imag() * x.imag();"),
    ("complex_modulus_is_taxicab", "return hypotl(x.real(), x.imag());", "return fabsl(x.real()) + fabsl(x.imag());"),
    ("storage_complex_modulus_is_squared_norm", "return std::hypot(x.real(), x.imag());", "return x.real() * x.real() + x.imag() * x.imag();"),
    ("single_complex_modulus_is_squared_norm", "inline float modulus(std::complex<float> x) { return std::hypot(x.real(), x.imag()); }",
     "inline float modulus(std::complex<float> x) { return x.real() * x.real() + x.imag() * x.imag(); }"),
    ("real_modulus_keeps_sign", "inline long double modulus(long double x) { return fabsl(x); }", "inline long double modulus(long double x) { return x; }"),
    ("normaliser_uses_only_A", "if (S) s += ma * mb;", "if (S) s += ma;"),
    ("literal_mode_scales_C_by_alpha", "T running = mul(be, apply_op(C[off_D], opC));", "T running = mul(al, apply_op(C[off_D], opC));"),
    ("last_term_skipped", "for (int64_t k = 0; k < size_P; ++k) {", "for (int64_t k = 1; k < size_P; ++k) {"),
    ("half_rounding_truncates", "const long double n = nearbyintl(a / quantum);", "const long double n = floorl(a / quantum);"),
    ("half_ties_away_from_zero", "const long double n = nearbyintl(a / quantum);", "const long double n = roundl(a / quantum);"),
    ("half_subnormal_grid_too_fine", "if (e < -14) e = -14;", "if (e < -15) e = -15;"),
    ("half_exponent_bias_off_by_one", "else a = ldexpl((long double)(1024 + frac), ef - 25);", "else a = ldexpl((long double)(1024 + frac), ef - 24);"),
    ("bfloat16_rounding_truncates", "a = nearbyintl(a / quantum) * quantum;", "a = floorl(a / quantum) * quantum;"),
    ("bfloat16_ties_away_from_zero", "a = nearbyintl(a / quantum) * quantum;", "a = roundl(a / quantum) * quantum;"),
    ("bfloat16_subnormal_grid_too_fine", "if (e < -126) e = -126;", "if (e < -127) e = -127;"),
    ("bfloat16_exponent_bias_off_by_one", "else a = ldexpl((long double)(128 + frac), ef - 134);", "else a = ldexpl((long double)(128 + frac), ef - 133);"),
    ("bfloat16_fraction_keeps_hidden_bit", "(uint16_t)((long long)(a / ldexpl(1.0L, e2 - 7)) - 128);", "(uint16_t)((long long)(a / ldexpl(1.0L, e2 - 7)) - 127);"),
    ("half_overflow_limit_too_high", "if (a >= 65536.0L) { bits = sign | 0x7c00u; return; }", "if (a >= 131072.0L) { bits = sign | 0x7c00u; return; }"),
]


def _pins_to_run():
    calls = []
    for dt in ("f64", "c128"):
        for seed in range(12):
            calls.append((pins.test_brute_force_integer_inputs_exact, (dt, seed)))
    for dt in ("f64", "c128"):
        for seed in range(4):
            calls.append((pins.test_einsum_random_problems, (dt, seed)))
    for row in pins._paper_examples():
        calls.append((pins.test_paper_label_examples, (row,)))
    for dt in ("c128", "c64", "f64", "f32"):
        for mode in (pins.oracle.MODE_TRUTH, pins.oracle.MODE_TIMED):
            calls.append((pins.test_normaliser_on_exact_moduli, (dt, mode)))
    for seed in range(10):
        calls.append((pins.test_isolated_labels_brute_force, ("f64", seed)))
    calls.append((pins.test_half_from_double_rounds_to_nearest_even, ()))
    calls.append((pins.test_half_to_double_on_every_bit_pattern, ()))
    calls.append((pins.test_bfloat16_from_double_rounds_to_nearest_even, ()))
    calls.append((pins.test_bfloat16_to_double_on_every_bit_pattern, ()))
    calls += [(pins.test_case4_example_is_a_reduction_then_a_contraction, ()), (pins.test_case5_broadcasts_the_product, ())]
    calls += [(pins.test_repeated_label_equals_summed_stride, ()), (pins.test_validation_classes, ()),
              (pins.test_conjugation_symmetry_and_op_equals_preconjugated_copy, ()),
              (pins.test_delta_operand_reproduces_permutation, ("c128",)),
              (pins.test_linearity_in_alpha_and_beta, ("c128",)),
              (pins.test_degenerate_shapes, ()),
              (pins.test_config4_hslowest_is_batched_AhB, ())]
    for p in pins.W.configs_reduced():
        calls.append((pins.test_all_ones_gives_product_of_contracted_extents, (p,)))
    return calls


@pytest.mark.parametrize("mutant", MUTANTS, ids=lambda m: m[0])
def test_a_pin_catches_the_planted_mistake(mutant, monkeypatch):
    name, find, repl = mutant
    assert find in SRC, "mutant pattern no longer matches the oracle source"
    with tempfile.TemporaryDirectory() as tmp:
        src, lib = os.path.join(tmp, "m.cpp"), os.path.join(tmp, "m.so")
        with open(src, "w") as f:
            f.write(SRC.replace(find, repl))
        subprocess.check_call(["g++", "-O1", "-fopenmp", "-shared", "-fPIC", "-std=c++17", src, "-o", lib])
        bad = ctypes.CDLL(lib)
        bad.oracle_validate.restype = ctypes.c_int
        bad.oracle_contract.restype = ctypes.c_int
        bad.oracle_max_threads.restype = ctypes.c_int
        bad.oracle_half_from_double.restype = ctypes.c_uint16
        bad.oracle_half_from_double.argtypes = [ctypes.c_double]
        bad.oracle_half_to_double.restype = ctypes.c_double
        bad.oracle_half_to_double.argtypes = [ctypes.c_uint16]
        bad.oracle_bfloat16_from_double.restype = ctypes.c_uint16
        bad.oracle_bfloat16_from_double.argtypes = [ctypes.c_double]
        bad.oracle_bfloat16_to_double.restype = ctypes.c_double
        bad.oracle_bfloat16_to_double.argtypes = [ctypes.c_uint16]
        oracle._load()
        monkeypatch.setattr(oracle, "_lib", bad)
        caught = 0
        for fn, args in _pins_to_run():
            try:
                fn(*args)
            except AssertionError:
                caught += 1
                break
        assert caught, "no pin noticed mutant %s" % name


def test_unmutated_oracle_passes_the_same_pins():
    for fn, args in _pins_to_run():
        fn(*args)
