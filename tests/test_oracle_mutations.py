"""The pins must be able to fail: each case plants one plausible mistake in a
copy of the oracle's source (on the CPU, never in the GPU library), builds the
copy, points the pin tests at it and expects at least one of them to fail.
"""
import os

import pytest

import oracle
import test_oracle_lstm_pins as lpins
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(os.path.abspath(oracle.__file__)), "ssrnn_oracle.cpp")

# (label, text in the source, replacement)
MUTATIONS = [
    ("sru: candidate weight uses f instead of 1-f", "ci = f * ci + (1.0 - f) * xh;", "ci = f * ci + f * xh;"),
    ("sru: forget gate not applied to old state", "ci = f * ci + (1.0 - f) * xh;", "ci = ci + (1.0 - f) * xh;"),
    ("sru: highway term dropped", "r * std::tanh(ci) + (1.0 - r) * xt;", "r * std::tanh(ci);"),
    ("sru: highway term uses r", "r * std::tanh(ci) + (1.0 - r) * xt;", "r * std::tanh(ci) + r * xt;"),
    ("sru: no tanh on the cell", "r * std::tanh(ci) + (1.0 - r) * xt;", "r * ci + (1.0 - r) * xt;"),
    ("sru: f and r row blocks swapped",
     "const double* Uf = U.data() + static_cast<size_t>(d) * nt;\n    const double* Ur = U.data() + static_cast<size_t>(2) * d * nt;",
     "const double* Ur = U.data() + static_cast<size_t>(d) * nt;\n    const double* Uf = U.data() + static_cast<size_t>(2) * d * nt;"),
    ("sru: biases swapped", "const double bf = bias ? static_cast<double>(bias[i]) : 0.0;\n      const double br = bias ? static_cast<double>(bias[d + i]) : 0.0;\n      double ci = c[i];\n      for (int t = 0; t < nt; ++t) {\n        const double xh",
     "const double br = bias ? static_cast<double>(bias[i]) : 0.0;\n      const double bf = bias ? static_cast<double>(bias[d + i]) : 0.0;\n      double ci = c[i];\n      for (int t = 0; t < nt; ++t) {\n        const double xh"),
    ("sigmoid sign", "return 1.0 / (1.0 + std::exp(-z));", "return 1.0 / (1.0 + std::exp(z));"),
    ("weights read transposed (square case)", "const double w = weight_at(W, wdt, static_cast<size_t>(3) * d, ncol, row, col);",
     "const double w = ncol == d ? weight_at(W, wdt, static_cast<size_t>(3) * d, ncol, (row / d) * d + col, row % d) : weight_at(W, wdt, static_cast<size_t>(3) * d, ncol, row, col);"),
    ("qrnn: lag blocks reversed", "X[(static_cast<size_t>(j) * d + m) * nt + t] = operand(x_at(t0 + t - j, m), round_operand);",
     "X[(static_cast<size_t>(k - 1 - j) * d + m) * nt + t] = operand(x_at(t0 + t - j, m), round_operand);"),
    ("qrnn: looks ahead instead of back", "= operand(x_at(t0 + t - j, m), round_operand);", "= operand(x_at(t0 + t + j < L ? t0 + t + j : L - 1, m), round_operand);"),
    ("rounding mode: rounds when not asked to", "return round_operand ? to_bf16_value(v) : v;", "return to_bf16_value(v);"),
    ("rounding mode: argument ignored", "return round_operand ? to_bf16_value(v) : v;", "return v;"),
    ("reverse: direction ignored", "return reverse ? L - 1 - tau : tau;", "return tau;"),
    ("reverse: off by one", "return reverse ? L - 1 - tau : tau;", "return reverse ? (tau == 0 ? L - 1 : L - tau) % L : tau;"),
    ("reverse: sru output written in walk order", "hout[time_of(t0 + t, L, reverse) * d + i] = r * std::tanh(ci) + (1.0 - r) * xt;", "hout[(t0 + t) * d + i] = r * std::tanh(ci) + (1.0 - r) * xt;"),
    ("reverse: sru highway term taken in walk order", "const double xt = xin[time_of(t0 + t, L, reverse) * d + i];", "const double xt = xin[(t0 + t) * d + i];"),
    ("reverse: qrnn output written in walk order", "hout[time_of(t0 + t, L, reverse) * d + i] = o * std::tanh(ci);", "hout[(t0 + t) * d + i] = o * std::tanh(ci);"),
    ("reverse: qrnn window read in time order", "if (s >= 0) return xin[time_of(s, L, reverse) * d + m];", "if (s >= 0) return xin[s * d + m];"),
    ("rounding mode: truncates instead of rounding to nearest even", "u = (u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u;", "u = u & 0xFFFF0000u;"),
    ("rounding mode: highway term rounded too", "const double xt = xin[time_of(t0 + t, L, reverse) * d + i];", "const double xt = operand(xin[time_of(t0 + t, L, reverse) * d + i], round_operand);"),
    ("rounding mode: qrnn window not rounded", "= operand(x_at(t0 + t - j, m), round_operand);", "= x_at(t0 + t - j, m);"),
    ("qrnn: candidate not squashed", "const double z = std::tanh(Uz[static_cast<size_t>(i) * nt + t] + bz);",
     "const double z = Uz[static_cast<size_t>(i) * nt + t] + bz;"),
    ("qrnn: output without tanh", "hout[time_of(t0 + t, L, reverse) * d + i] = o * std::tanh(ci);", "hout[time_of(t0 + t, L, reverse) * d + i] = o * ci;"),
    ("qrnn: history order reversed", "nh[static_cast<size_t>(j) * d + m] = x_at(L - 1 - j, m);",
     "nh[static_cast<size_t>(k - 2 - j) * d + m] = x_at(L - 1 - j, m);"),
    ("state not carried across blocks", "      c[i] = ci;\n    }\n  }\n}\n\n// One QRNN layer.", "    }\n  }\n}\n\n// One QRNN layer."),
    ("initial state ignored (sru)", "c[i] = c_init ? c_init[static_cast<size_t>(l) * d + i] : 0.0;\n    sru_layer", "c[i] = 0.0;\n    sru_layer"),
    ("bf16 widened with the wrong shift", "static_cast<uint32_t>(bits) << 16;", "static_cast<uint32_t>(bits) << 15;"),
    ("fp8: exponent bias 8 (the other 8-bit float format)", "v = std::ldexp(1.0 + m / 8.0, e - 7);", "v = std::ldexp(1.0 + m / 8.0, e - 8);"),
    ("fp8: subnormals given the hidden one", "else if (e == 0) v = std::ldexp(m / 8.0, 1 - 7);", "else if (e == 0) v = std::ldexp(1.0 + m / 8.0, 0 - 7);"),
    ("fp8: subnormal exponent off by one", "v = std::ldexp(m / 8.0, 1 - 7);", "v = std::ldexp(m / 8.0, 0 - 7);"),
    ("fp8: mantissa of 4 bits", "const int m = code & 7;", "const int m = code & 15;"),
    ("fp8: sign ignored", "return (code & 0x80) ? -v : v;", "return v;"),
    ("fp8: scale of the wrong row", "scale_offset + row * sizeof(float), sizeof scale);", "scale_offset + (row ^ 1) * sizeof(float), sizeof scale);"),
    ("fp8: scales taken to start right behind the codes", "const size_t scale_offset = (rows * ncol + 255) / 256 * 256;", "const size_t scale_offset = (rows * ncol + 3) / 4 * 4;"),
    ("fp8: scale dropped", "return static_cast<double>(scale) * value_e4m3(", "return value_e4m3("),
    ("stack: every layer reads the external input", "    cur.swap(nxt);\n  }\n  if (n) std::memcpy(h, cur.data(), n * sizeof(double));\n  return 0;\n}\n\n// Stacked QRNN",
     "    if (l == n_layers - 1) cur.swap(nxt);\n  }\n  if (n) std::memcpy(h, cur.data(), n * sizeof(double));\n  return 0;\n}\n\n// Stacked QRNN"),
    ("step function: bias dropped", "if (bias) { uf += bias[i]; ur += bias[d + i]; }", ""),
    ("lstm: input gate replaced by 1 - f", "c[i] = f * c[i] + in * chat;\n        hnew[i]", "c[i] = f * c[i] + (1.0 - f) * chat;\n        hnew[i]"),
    ("lstm: forget gate not applied", "c[i] = f * c[i] + in * chat;\n        hnew[i]", "c[i] = c[i] + in * chat;\n        hnew[i]"),
    ("lstm: candidate not squashed", "const double chat = std::tanh(pre[3]);", "const double chat = pre[3];"),
    ("lstm: output without tanh of the cell", "hnew[i] = o * std::tanh(c[i]);", "hnew[i] = o * c[i];"),
    ("lstm: input and output gate rows swapped", "const double in = sigma(pre[1]);\n        const double o = sigma(pre[2]);", "const double in = sigma(pre[2]);\n        const double o = sigma(pre[1]);"),
    ("lstm: forget and candidate rows swapped", "const double f = sigma(pre[0]);\n        const double in = sigma(pre[1]);\n        const double o = sigma(pre[2]);\n        const double chat = std::tanh(pre[3]);",
     "const double f = sigma(pre[3]);\n        const double in = sigma(pre[1]);\n        const double o = sigma(pre[2]);\n        const double chat = std::tanh(pre[0]);"),
    ("lstm: feedback term dropped", "pre[g] = A[row * nt + t] + u + (bias", "pre[g] = A[row * nt + t] + (bias"),
    ("lstm: feedback matrix read transposed", "u += static_cast<double>(U[row * d + col]) * hprev[col];", "u += static_cast<double>(U[(static_cast<size_t>(g) * d + col) * d + i]) * hprev[col];"),
    ("lstm: feedback uses the step's own partial output", "        hnew[i] = o * std::tanh(c[i]);\n      }", "        hnew[i] = o * std::tanh(c[i]);\n        hprev[i] = hnew[i];\n      }"),
    ("lstm: feedback frozen at the start of the block", "        hprev[i] = hnew[i];\n        hout[(t0 + t) * d + i] = hnew[i];", "        if (t == nt - 1) hprev[i] = hnew[i];\n        hout[(t0 + t) * d + i] = hnew[i];"),
    ("lstm: bias dropped", "+ u + (bias ? static_cast<double>(bias[row]) : 0.0);", "+ u;"),
    ("lstm: bias added twice", "+ u + (bias ? static_cast<double>(bias[row]) : 0.0);", "+ u + 2.0 * (bias ? static_cast<double>(bias[row]) : 0.0);"),
    ("lstm: input products of a block use the block's first input", "for (int t = 0; t < nt; ++t) acc[t] += w * xin[(t0 + t) * d + col];", "for (int t = 0; t < nt; ++t) acc[t] += w * xin[t0 * d + col];"),
    ("lstm: input matrix read transposed", "const double w = static_cast<double>(W[static_cast<size_t>(row) * d + col]);", "const double w = static_cast<double>(W[(static_cast<size_t>(row / d) * d + col) * d + row % d]);"),
    ("lstm: initial h ignored", "hp[i] = h_init ? h_init[static_cast<size_t>(l) * d + i] : 0.0;", "hp[i] = 0.0;"),
    ("lstm: initial c ignored", "c[i] = c_init ? c_init[static_cast<size_t>(l) * d + i] : 0.0;\n      hp[i]", "c[i] = 0.0;\n      hp[i]"),
    ("lstm: every layer reads the external input", "    cur.swap(nxt);\n  }\n  if (n) std::memcpy(h, cur.data(), n * sizeof(double));\n  return 0;\n}\n\n// Brute force: one LSTM layer",
     "    if (l == n_layers - 1) cur.swap(nxt);\n  }\n  if (n) std::memcpy(h, cur.data(), n * sizeof(double));\n  return 0;\n}\n\n// Brute force: one LSTM layer"),
    ("lstm step function: feedback of the forget gate dropped", "1.0 / (1.0 + std::exp(-(zf + yf + bf)));", "1.0 / (1.0 + std::exp(-(zf + bf)));"),
    ("lstm step function: input gate bias from the output gate", "1.0 / (1.0 + std::exp(-(zi + yi + bi)));", "1.0 / (1.0 + std::exp(-(zi + yi + bo)));"),
    ("projection transposed", "static_cast<double>(P[static_cast<size_t>(i) * d_in + j])", "static_cast<double>(P[(static_cast<size_t>(j) * d_out + i) % (static_cast<size_t>(d_in) * d_out)])"),
]

BATTERY = [
    lambda: [pins.test_sru_hand_example(n, T) for n in ("sru_d2_example_a.txt", "sru_d2_example_b.txt") for T in (1, 2, 4)],
    lambda: [pins.test_qrnn_hand_example(T) for T in (1, 2, 4)],
    pins.test_step_functions_hand_examples,
    lambda: pins.test_sru_blocked_equals_bruteforce_bitwise(2, 2, 5, 11, 4, False),
    lambda: pins.test_sru_blocked_equals_bruteforce_bitwise(5, 2, 6, 13, 5, True),
    lambda: pins.test_qrnn_blocked_equals_bruteforce_bitwise(13, 3, 4, 20, 16, 3, False),
    pins.test_sru_forget_zero_gives_candidate,
    pins.test_sru_forget_half_is_exponential_average,
    pins.test_sru_reset_zero_is_identity_through_a_stack,
    lambda: pins.test_sru_layer_against_library_product_and_solved_recurrence(41),
    lambda: pins.test_qrnn_layer_against_library_product_and_solved_recurrence(44, 3),
    pins.test_stack_feeds_h_to_next_layer,
    pins.test_chunk_chaining_equals_one_call,
    pins.test_bf16_weights_are_widened_exactly,
    pins.test_linear_projection_against_numpy,
    pins.test_future_inputs_do_not_change_past_outputs,
    pins.test_operand_rounding_mode_rounds_only_the_matrix_operand,
    pins.test_reverse_direction_is_the_forward_pass_over_the_reversed_sequence,
    pins.test_fp8_code_values_follow_the_format,
    pins.test_fp8_weights_equal_their_fp32_values_bitwise,
    pins.test_fp8_row_scales_are_applied_per_row,
    lambda: [lpins.test_lstm_hand_example(T) for T in (1, 2, 4)],
    lpins.test_lstm_step_hand_example,
    lambda: lpins.test_lstm_blocked_equals_bruteforce_bitwise(2, 2, 5, 11, 4, False),
    lambda: lpins.test_lstm_blocked_equals_bruteforce_bitwise(3, 3, 4, 20, 16, True),
    lpins.test_lstm_all_zero_weights_halve_the_cell,
    lpins.test_lstm_closed_input_gate_and_open_forget_gate_keep_the_cell,
    lpins.test_lstm_closed_forget_gate_and_open_input_gate_give_the_candidate,
    lpins.test_scalar_lstm_iterated_with_math_functions,
    lpins.test_lstm_without_feedback_against_library_product_and_solved_recurrence,
    lpins.test_lstm_feedback_products_against_library_product,
    lpins.test_lstm_stack_feeds_h_to_the_next_layer,
    lpins.test_lstm_chunk_chaining_equals_one_call,
]


def _battery_fails() -> bool:
    for check in BATTERY:
        try:
            check()
        except AssertionError:
            return True
    return False


def test_unmodified_oracle_passes_the_battery():
    oracle.use_library(None)
    assert not _battery_fails()


@pytest.mark.parametrize("label,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(tmp_path, label, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation '{label}' no longer matches the source"
    mutated = tmp_path / "mutant.cpp"
    mutated.write_text(text.replace(old, new, 1))
    lib = oracle.load_library(oracle.compile_source(str(mutated), str(tmp_path / "libmutant.so")))
    oracle.use_library(lib)
    try:
        assert _battery_fails(), f"no pin noticed: {label}"
    finally:
        oracle.use_library(None)
