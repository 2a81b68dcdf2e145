"""The pins must be able to fail: each plausible mistake planted in a copy of the oracle's C source
(a wrong sign, index, operand, rounding, bit order, plane weight) has to trip at least one pin.
CPU only; the mutated copies are built in a temporary directory and never touch oracle/."""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "abq_oracle.c")

MUTATIONS = {
    "acc: weight row read backwards along K":
        ("s += (int64_t)A[(size_t)m * K + k] * (int64_t)W[(size_t)n * K + k];",
         "s += (int64_t)A[(size_t)m * K + k] * (int64_t)W[(size_t)n * K + (K - 1 - k)];"),
    "acc: dropped last term":
        ("            for (int k = 0; k < K; ++k)\n                s += (int64_t)A[(size_t)m * K + k] * (int64_t)W",
         "            for (int k = 0; k < K - 1; ++k)\n                s += (int64_t)A[(size_t)m * K + k] * (int64_t)W"),
    "centered: sign of the activation zero-point":
        ("s += ((int64_t)A[(size_t)m * K + k] - az[m]) * ((int64_t)W[(size_t)n * K + k] - wz[n]);\n            accc[(size_t)m * N + n] = s;",
         "s += ((int64_t)A[(size_t)m * K + k] + az[m]) * ((int64_t)W[(size_t)n * K + k] - wz[n]);\n            accc[(size_t)m * N + n] = s;"),
    "dequant: activation scale of row 0 for every row":
        ("(double)accc[(size_t)m * N + n] * (double)a_scale[m] * (double)w_scale[n]",
         "(double)accc[(size_t)m * N + n] * (double)a_scale[0] * (double)w_scale[n]"),
    "dequant: scales swapped":
        ("(double)accc[(size_t)m * N + n] * (double)a_scale[m] * (double)w_scale[n]",
         "(double)accc[(size_t)m * N + n] * (double)a_scale[n % M] * (double)w_scale[m % N]"),
    "half: truncation instead of round-to-nearest-even":
        ("double r = nearbyint(scaled);", "double r = floor(scaled);"),
    "half: overflow threshold":
        ("if (back >= 65520.0)", "if (back >= 65536.0 * 2)"),
    "planes: bit order inside a word":
        ("|= (uint32_t)1u << (k & 31);", "|= (uint32_t)1u << (31 - (k & 31));"),
    "bitplane: plane weight 2^(s*t)":
        ("y += yst * ((int64_t)1 << (s + t));", "y += yst * ((int64_t)1 << (s * t));"),
    "bitplane: OR instead of AND":
        ("yst += popcount32(ar[kw] & wr[kw]);", "yst += popcount32(ar[kw] | wr[kw]);"),
    "quantizer: zero-point not clamped":
        ("z = zf < 0.0f ? 0 : (zf > (float)qmax ? qmax : (int)zf);", "z = (int)zf + 1;"),
    "quantizer: truncation instead of rint":
        ("float r = nearbyintf(t);", "float r = truncf(t);"),
    "rmsnorm: sum instead of mean of the squares":
        ("const double mean = ss / (double)K;", "const double mean = ss;"),
    "rmsnorm: eps dropped":
        ("(float)(1.0 / sqrt(mean + (double)eps));", "(float)(1.0 / sqrt(mean));"),
    "rmsnorm: gain of channel 0 for every channel":
        ("volatile float u = t * half_to_float(gamma_half[k]);", "volatile float u = t * half_to_float(gamma_half[0]);"),
    "silu: sign of the exponent":
        ("volatile float t = -g * 0x1.715476p+0f;", "volatile float t = g * 0x1.715476p+0f;"),
    "silu: natural instead of binary exponent scaling":
        ("volatile float t = -g * 0x1.715476p+0f;", "volatile float t = -g;"),
    "silu: polynomial term dropped":
        ("    p = p + c2; p = p * f;\n", "    p = p * f;\n"),
    "silu: second operand not applied":
        ("volatile float h = sg * u;", "volatile float h = sg;"),
    "rmsnorm: low half of the exact sum dropped":
        ("((double)hi * 18446744073709551616.0 + (double)lo) *", "((double)hi * 18446744073709551616.0) *"),
    "grouped: zero-point of group 0 for every group":
        ("((int64_t)W[(size_t)n * K + k] - wz[(size_t)n * G + g]);", "((int64_t)W[(size_t)n * K + k] - wz[(size_t)n * G]);"),
    "grouped: scale of group 0 for every group":
        ("(double)half_to_float(w_scale_half[(size_t)n * G + g]) * (double)inner;", "(double)half_to_float(w_scale_half[(size_t)n * G]) * (double)inner;"),
    "grouped: short last group dropped":
        ("    const int G = (K + gs - 1) / gs;\n#pragma omp parallel for schedule(static)\n    for (int m = 0; m < M; ++m) {\n        for (int n = 0; n < N; ++n) {\n            double total = 0.0, size = 0.0;\n            for (int g = 0; g < G; ++g) {",
         "    const int G = (K + gs - 1) / gs;\n#pragma omp parallel for schedule(static)\n    for (int m = 0; m < M; ++m) {\n        for (int n = 0; n < N; ++n) {\n            double total = 0.0, size = 0.0;\n            for (int g = 0; g < K / gs; ++g) {"),
    "grouped: sign of the activation zero-point":
        ("inner += ((int64_t)A[(size_t)m * K + k] - az[m]) *", "inner += ((int64_t)A[(size_t)m * K + k] + az[m]) *"),
    "grouped: activation scale of row 0 for every row":
        ("const double v = (double)a_scale[m] * total;", "const double v = (double)a_scale[0] * total;"),
    "requant: zero-point dropped":
        ("            int c = (int)rn + z;", "            int c = (int)rn;"),
    "requant: step of row 0 for every row":
        ("volatile float delta = scale[m];\n        const int z = zero[m];", "volatile float delta = scale[0];\n        const int z = zero[m];"),
    "requant: ties away from zero":
        ("float rn = nearbyintf(t);", "float rn = roundf(t);"),
    "add: difference instead of sum":
        ("volatile float s = half_to_float(a_half[i]) + half_to_float(b_half[i]);", "volatile float s = half_to_float(a_half[i]) - half_to_float(b_half[i]);"),
    "add: second operand taken from the first":
        ("volatile float s = half_to_float(a_half[i]) + half_to_float(b_half[i]);", "volatile float s = half_to_float(a_half[i]) + half_to_float(a_half[i]);"),
}

CHECKS = [
    lambda: pins.test_exhaustive_k1_all_codes(3, 5),
    lambda: pins.test_bruteforce_random_small(2, 8, 33),
    lambda: pins.test_w8a8_equals_library_matmul(5, 33, 257),
    lambda: pins.test_operand_roles_not_transposed(),
    lambda: pins.test_closed_forms(2, 8),
    lambda: pins.test_plane_composition_and_padding_and_symmetry(),
    lambda: pins.test_centered_equals_four_term_expansion(6, 6, 7, 5, 333),
    lambda: pins.test_unit_scales_zero_points_give_exact_half(),
    lambda: pins.test_dequant_equals_dequantise_then_multiply_longdouble(),
    lambda: pins.test_dequant_scale_roles_not_swapped(),
    lambda: pins.test_half_rounding_matches_numpy(),
    lambda: pins.test_pack_unpack_planes(5, 2, 100),
    lambda: pins.test_quant_act_invariants(4),
    lambda: pins.test_quant_act_invariants(8),
    lambda: pins.test_requant_pins(4),
    lambda: pins.test_rmsnorm_matches_float64_definition(3, 1000, 1e-6),
    lambda: pins.test_rmsnorm_closed_forms(),
    lambda: pins.test_rmsnorm_invariances_are_bit_exact(),
    lambda: pins.test_silu_mul_matches_float64_definition(),
    lambda: pins.test_silu_mul_closed_forms_and_limits(),
    lambda: pins.test_add_half_matches_numpy_two_step_rounding_and_identities(),
    lambda: pins.test_grouped_one_group_is_the_per_channel_result(),
    lambda: pins.test_grouped_equals_dequantise_then_multiply(4, 8, 3, 5, 300, 128),
    lambda: pins.test_grouped_single_live_group_uses_that_groups_scale_and_zero(),
]


def _load(path):
    lib = ctypes.CDLL(path)
    lib.abq_oracle_threads.restype = ctypes.c_int
    lib.abq_oracle_half_bits.restype = ctypes.c_uint16
    lib.abq_oracle_half_bits.argtypes = [ctypes.c_double]
    return lib


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name, tmp_path, monkeypatch):
    old, new = MUTATIONS[name]
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation target must occur exactly once: {name}"
    src = tmp_path / "mut.c"
    src.write_text(text.replace(old, new, 1))
    lib = tmp_path / "libmut.so"
    subprocess.run(["gcc", "-std=c11", "-O1", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", str(src), "-o", str(lib), "-lm"],
                   check=True)
    oracle._load()
    monkeypatch.setattr(oracle, "_lib", _load(str(lib)))
    failures = 0
    for check in CHECKS:
        try:
            check()
        except AssertionError:
            failures += 1
    assert failures >= 1, f"no pin noticed: {name}"


def test_unmutated_oracle_passes_every_check():
    oracle._load()
    for check in CHECKS:
        check()
