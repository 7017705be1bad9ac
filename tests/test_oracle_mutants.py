"""Checks that the pins have teeth: plausible mistakes are planted in COPIES of the CPU oracle
(on the CPU only; the copies are compiled into a temporary directory) and every such mutant must be
rejected by at least one pin of tests/test_oracle_pins.py."""
import importlib.util
import os
import shutil

import pytest

import test_oracle_pins as pins
import test_oracle_pool2d_pins as pool_pins
import test_oracle_bias_relu_pins as br_pins
import test_oracle_dilated_pins as dil_pins
import test_oracle_requant_pins as rq_pins

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "sw_oracle.c")

# (name, text to find, replacement, which occurrence)
MUTANTS = [
    ("conv2d filter flipped", "w[((co * C_in + ci) * R + r) * S + s];", "w[((co * C_in + ci) * R + (R - 1 - r)) * S + (S - 1 - s)];", 0),
    ("conv2d padding sign", "const int64_t h = i * stride + r - pad;", "const int64_t h = i * stride + r + pad;", 0),
    ("conv2d stride ignored on rows", "const int64_t h = i * stride + r - pad;", "const int64_t h = i + r - pad;", 0),
    ("output extent one short", "return span / stride + 1;", "return span / stride;", 0),
    ("conv2d input channel reversed", "x[((n * C_in + ci) * H + h) * W + v];", "x[((n * C_in + (C_in - 1 - ci)) * H + h) * W + v];", 0),
    ("conv2d last tap column dropped", "for (int64_t s = 0; s < S; ++s) {", "for (int64_t s = 0; s < S - (S > 1); ++s) {", 0),
    ("conv2d magnitude sums signed products", "mag += fabs(p);", "mag += p;", 0),
    ("depthwise stride ignored on columns", "const int64_t v = j * stride + s - pad;", "const int64_t v = j + s - pad;", 1),
    ("depthwise filter of the wrong channel", "(double)w[(c * R + r) * S + s];", "(double)w[(((c + 1) % C) * R + r) * S + s];", 0),
    ("conv1d window runs backwards", "const int64_t t = i * stride + j - pad;", "const int64_t t = i * stride - j + pad;", 0),
    ("conv1d tap order reversed", "(double)w[j] * (double)x[row * len + t];", "(double)w[k - 1 - j] * (double)x[row * len + t];", 0),
    ("average divides by window - 1", "y[row * Lo + i] = acc / (double)window;", "y[row * Lo + i] = acc / (double)(window > 1 ? window - 1 : 1);", 0),
    ("maximum starts from zero", "double m = (double)p[0];", "double m = 0.0;", 0),
    ("pooling stride ignored", "const float *p = x + row * len + i * stride;", "const float *p = x + row * len + i;", 0),
    ("int8 read as unsigned", "acc += (int64_t)x[((n * C_in + ci) * H + h) * W + v] *", "acc += (int64_t)(uint8_t)x[((n * C_in + ci) * H + h) * W + v] *", 0),
    ("int8 accumulator 16 bits wide", "y[((n * C_out + co) * Ho + i) * Wo + j] = (int32_t)acc;", "y[((n * C_out + co) * Ho + i) * Wo + j] = (int32_t)(int16_t)acc;", 0),
    ("pool2d average divides by the positions inside", "y[o] = acc / (double)(R * S);", "y[o] = acc / (double)inside;", 0),
    ("pool2d padding takes part in the maximum", "if (inside == 0 || e > m) m = e;", "if (e > m) m = e;", 0),
    ("pool2d window transposed", "for (int64_t s = 0; s < S; ++s) {\n                        const int64_t v = j * stride + s - pad;\n                        if (v < 0 || v >= W) continue;\n                        const double e", "for (int64_t s = 0; s < R; ++s) {\n                        const int64_t v = j * stride + s - pad;\n                        if (v < 0 || v >= W) continue;\n                        const double e", 0),
    ("pool2d stride ignored on columns", "const int64_t v = j * stride + s - pad;\n                        if (v < 0 || v >= W) continue;\n                        const double e", "const int64_t v = j + s - pad;\n                        if (v < 0 || v >= W) continue;\n                        const double e", 0),
    ("pool2d padding sign", "const int64_t h = i * stride + r - pad;\n                    if (h < 0 || h >= H) continue;\n                    for (int64_t s = 0; s < S; ++s) {\n                        const int64_t v = j * stride + s - pad;\n                        if (v < 0 || v >= W) continue;\n                        const double e", "const int64_t h = i * stride + r + pad;\n                    if (h < 0 || h >= H) continue;\n                    for (int64_t s = 0; s < S; ++s) {\n                        const int64_t v = j * stride + s - pad;\n                        if (v < 0 || v >= W) continue;\n                        const double e", 0),
    ("requantisation rounds ties away from zero", "float r = nearbyintf(prod);", "float r = roundf(prod);", 0),
    ("requantisation truncates", "float r = nearbyintf(prod);", "float r = truncf(prod);", 0),
    ("requantisation multiplies in double", "const float prod = v * sc;\n                float r = nearbyintf(prod);", "const double prod = (double)t * (double)sc;\n                float r = (float)nearbyint(prod);", 0),
    ("requantisation ignores the bias", "const int64_t b = bias ? (int64_t)bias[co] : 0;", "const int64_t b = 0; (void)bias;", 0),
    ("requantisation: rectifier clamps at -128", "const float lo = relu ? 0.0f : -128.0f;", "const float lo = -128.0f; (void)relu;", 0),
    ("requantisation: scale of the neighbouring channel", "const float sc = scale[co];", "const float sc = scale[(co + 1) % C_out];", 0),
    ("requantisation: upper clamp at 128 wraps", "if (r > 127.0f) r = 127.0f;", "if (r > 128.0f) r = 128.0f;", 0),
    ("int8 overflow never reported", "return overflow ? 2 : 0;", "return 0;", 0),
    ("dilation ignored on columns", "const int64_t vd = j * stride + s * dil - pad;", "const int64_t vd = j * stride + s - pad;", 0),
    ("dilation multiplies the stride", "const int64_t hd = i * stride + r * dil - pad;", "const int64_t hd = (i * stride + r) * dil - pad;", 0),
    ("dilated extent taken from the undilated filter", "return oracle_out_dim(in, dil * (k - 1) + 1, stride, pad);", "return oracle_out_dim(in, k, stride, pad);", 0),
    ("dilated span one tap too long", "return oracle_out_dim(in, dil * (k - 1) + 1, stride, pad);", "return oracle_out_dim(in, dil * k, stride, pad);", 0),
    ("dilated depthwise reads every channel", "const int64_t ci_first = depthwise ? co : 0, ci_end = depthwise ? co + 1 : C_in;", "const int64_t ci_first = 0, ci_end = C_in;", 0),
    ("dilated depthwise takes the first filter", "const float *wf = depthwise ? w + co * R * S : w + (co * C_in + ci) * R * S;", "const float *wf = depthwise ? w : w + (co * C_in + ci) * R * S;", 0),
    ("bias of the neighbouring channel", "const double b = bias ? (double)bias[co] : 0.0;", "const double b = bias ? (double)bias[(co + 1) % C_out] : 0.0;", 0),
    ("bias subtracted", "double t = y[o] + b;", "double t = y[o] - b;", 0),
    ("rectifier before the bias", "double t = y[o] + b;\n                if (relu && t < 0.0) t = 0.0;", "double t = y[o];\n                if (relu && t < 0.0) t = 0.0;\n                t += b;", 0),
    ("rectifier always on", "if (relu && t < 0.0) t = 0.0;", "if (t < 0.0) t = 0.0;", 0),
    ("rectifier takes the magnitude", "if (relu && t < 0.0) t = 0.0;", "if (relu && t < 0.0) t = -t;", 0),
    ("bias left out of the magnitude sum", "d[o] += fabs(b);", "d[o] += 0.0;", 0),
]


def _replace_nth(text, old, new, nth):
    pos = -1
    for _ in range(nth + 1):
        pos = text.find(old, pos + 1)
        assert pos >= 0, f"mutation site not found: {old!r}"
    return text[:pos] + new + text[pos + len(old):]


def _load_mutant(tmpdir, idx, old, new, nth):
    src = _replace_nth(open(SRC).read(), old, new, nth)
    d = os.path.join(tmpdir, f"m{idx}")
    os.makedirs(d)
    shutil.copy(os.path.join(ROOT, "oracle", "__init__.py"), os.path.join(d, "__init__.py"))
    open(os.path.join(d, "sw_oracle.c"), "w").write(src)
    spec = importlib.util.spec_from_file_location(f"oracle_mutant_{idx}", os.path.join(d, "__init__.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)      # its _SRC/_LIB point into d: it compiles and loads the mutant
    mod.build()
    return mod


def _battery(o):
    """A cheap subset of the pins, run against oracle-like module `o`."""
    for case in pins.CASES_2D:
        pins.test_conv2d_matches_scatter_brute_force(o, case)
        pins.test_conv2d_s8_matches_scatter_brute_force(o, case)
    for case in [(2, 3, 7, 6, 3, 3, 1, 1), (1, 2, 7, 7, 3, 2, 2, 1), (1, 4, 5, 5, 5, 5, 1, 2)]:
        pins.test_depthwise_matches_scatter_brute_force(o, case)
    for k, st, pad in [(1, 1, 0), (3, 1, 0), (3, 2, 1), (4, 3, 2), (9, 1, 0), (5, 1, 4)]:
        pins.test_conv1d_matches_scatter_brute_force(o, k, st, pad)
    pins.test_hand_worked_examples(o)
    for pad in (0, 1, 2):
        pins.test_impulse_reproduces_the_filter_without_flip(o, pad)
    for R, S in [(3, 3), (7, 7), (2, 6)]:
        pins.test_all_ones_filter_equals_box_sums(o, R, S)
    pins.test_max_pool_semantics(o)
    pins.test_s8_extremes_and_agreement_with_float_oracle(o)
    pins.test_s8_overflow_is_refused(o)
    pins.test_out_dim_formula(o)
    pins.test_entry_points_agree_with_each_other(o)
    for case in pool_pins.CASES:
        pool_pins.test_average_matches_scatter_brute_force(o, case)
        pool_pins.test_maximum_matches_slices_of_a_minus_infinity_padded_copy(o, case)
    pool_pins.test_closed_forms(o)
    rq_pins.test_hand_worked_ties_and_saturation(o)
    rq_pins.test_two_channels_use_their_own_scale_and_bias(o)
    rq_pins.test_conversion_to_fp32_comes_before_the_product(o)
    rq_pins.test_identity_monotonicity_and_overflow(o)
    pool_pins.test_special_cases_reduce_to_the_other_entry_points(o)
    br_pins.test_hand_worked_example(o)
    dil_pins.test_hand_worked_example(o)
    for case in dil_pins.CASES:
        dil_pins.test_dilated_equals_plain_convolution_with_a_zero_stuffed_filter(o, case)
    br_pins.test_no_bias_and_no_rectifier_is_the_plain_convolution(o)


def test_unmutated_copy_passes_the_battery(tmp_path, oracle):
    _battery(oracle)
    same = _load_mutant(str(tmp_path), 999, "return span / stride + 1;", "return span / stride + 1;", 0)
    _battery(same)


@pytest.mark.parametrize("idx", range(len(MUTANTS)), ids=[m[0] for m in MUTANTS])
def test_every_mutant_is_caught(tmp_path, idx):
    name, old, new, nth = MUTANTS[idx]
    mutant = _load_mutant(str(tmp_path), idx, old, new, nth)
    with pytest.raises(BaseException) as caught:
        _battery(mutant)
    assert not isinstance(caught.value, (KeyboardInterrupt, SystemExit)), name
