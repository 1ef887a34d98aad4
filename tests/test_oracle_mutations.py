"""Do the oracle's pins bite?  Each case plants one plausible mistake in a copy of the oracle's C
source (a dropped term, a wrong sign or index, a transposed operand, a reversed bit order),
builds it on the side and runs ``tests/test_oracle_pins.py`` against that build in a child
process: the pins must fail.  The untouched source, built the same way, must pass.

CPU only; nothing here touches the GPU library, and every planted index stays inside its
array, so a broken build computes wrong values but reads nothing out of bounds.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "espresso_oracle.c")

# (name, function whose body is edited, text to find there, replacement)
MUTATIONS = [
    ("sign_f32_strict", "orc_sign_f32", "x[i] >= 0.0f", "x[i] > 0.0f"),
    ("sign_f64_strict", "orc_sign_f64", "x[i] >= 0.0", "x[i] > 0.0"),
    ("pack_msb_first", "orc_pm1_to_words", "<< (i % 64)", "<< (63 - i % 64)"),
    ("pack_zero_counts_as_plus", "orc_pm1_to_words", "s[r * k + i] > 0", "s[r * k + i] >= -1"),
    ("unpack_msb_first", "orc_words_to_pm1", ">> (i % 64)", ">> (63 - i % 64)"),
    ("mismatch_counts_matches", "orc_mismatches_words", "if (ba != bb)", "if (ba == bb)"),
    ("dense_transposed_b", "orc_dense_pm1", "b[n * K + k]", "b[k * N + n]"),
    ("dense_negated", "orc_dense_pm1", "c[m * N + n] = acc;", "c[m * N + n] = -acc;"),
    ("dense_dropped_term", "orc_dense_pm1", "for (int64_t k = 0; k < K; ++k)", "for (int64_t k = 1; k < K; ++k)"),
    ("dense_transposed_output", "orc_dense_pm1", "c[m * N + n] = acc;", "c[n * M + m] = acc;"),
    ("conv_flipped_filter", "orc_conv_pm1", "filt[((l2 * kh + dy) * kw + dx) * C + c]",
     "filt[((l2 * kh + (kh - 1 - dy)) * kw + (kw - 1 - dx)) * C + c]"),
    ("conv_pad_sign", "orc_conv_pm1", ": (int32_t)pad_value;", ": (int32_t)(-pad_value);"),
    ("conv_pad_offset_sign", "orc_conv_pm1", "const int64_t y = m * stride + dy - pad;",
     "const int64_t y = m * stride + dy + pad;"),
    ("conv_stride_ignored_in_x", "orc_conv_pm1", "const int64_t x = n * stride + dx - pad;",
     "const int64_t x = n + dx - pad;"),
    ("conv_channel_dropped", "orc_conv_pm1", "for (int64_t c = 0; c < C; ++c) {", "for (int64_t c = 1; c < C; ++c) {"),
    ("unroll_tap_order", "orc_unroll_pm1", "row[(dy * kw + dx) * C + c]", "row[(dx * kh + dy) * C + c]"),
    ("unroll_pad_sign", "orc_unroll_pm1", ": (int8_t)pad_value;", ": (int8_t)(-pad_value);"),
    ("bn_beta_sign", "orc_bn_value", "return q + (double)beta;", "return q - (double)beta;"),
    ("bn_mean_sign", "orc_bn_value", "x - (double)mean", "x + (double)mean"),
    ("bn_eps_dropped", "orc_bn_value", "sqrt((double)var + (double)eps)", "sqrt((double)var)"),
    ("bn_no_sqrt", "orc_bn_value", "sqrt((double)var + (double)eps)", "((double)var + (double)eps)"),
    ("bn_channel_index", "orc_bn_i32", "gamma[c], beta[c], mean[c], var[c]", "gamma[c], beta[c], mean[C - 1 - c], var[c]"),
    ("maxpool_is_min", "orc_maxpool_pm1", "int8_t best = -128;", "int8_t best = 127;\n#define ORC_MIN 1"),
    ("maxpool_window_column_ignored", "orc_maxpool_pm1", "n * stride + dx) * C + c]", "n * stride) * C + c]"),
    # window != stride: each of these equals the right answer when win == stride, and with
    # win >= stride (the pins' cases) none of them reads or writes outside its arrays
    ("maxpool_stride_taken_as_window", "orc_maxpool_pm1", "const int64_t H2 = (H - win) / stride + 1;",
     "stride = win;\n    const int64_t H2 = (H - win) / stride + 1;"),
    ("maxpool_output_size_from_window", "orc_maxpool_pm1", "const int64_t H2 = (H - win) / stride + 1;",
     "const int64_t H2 = (H - win) / win + 1;"),
    ("maxpool_row_origin_steps_by_window", "orc_maxpool_pm1", "(b * H + m * stride + dy) * W", "(b * H + m * win + dy) * W"),
    ("maxpool_column_origin_steps_by_window", "orc_maxpool_pm1", "W + n * stride + dx) * C + c]",
     "W + n * win + dx) * C + c]"),
    ("maxpool_window_extent_is_stride", "orc_maxpool_pm1", "for (int64_t dy = 0; dy < win; ++dy)",
     "for (int64_t dy = 0; dy < stride; ++dy)"),
    ("dense_f64_reversed_weights", "orc_dense_f64", "(double)w[n * K + k]", "(double)w[n * K + (K - 1 - k)]"),
    ("dense_f64_single_precision_sum", "orc_dense_f64", "acc += (double)x[m * K + k] * (double)w[n * K + k];",
     "acc = (double)(float)(acc + (double)x[m * K + k] * (double)w[n * K + k]);"),
    ("conv_f64_flipped_filter", "orc_conv_f64", "filt[((l2 * kh + dy) * kw + dx) * C + c]",
     "filt[((l2 * kh + (kh - 1 - dy)) * kw + (kw - 1 - dx)) * C + c]"),
    ("dense_u8_signed_input", "orc_dense_u8", "(int32_t)x[m * K + k]", "(int32_t)(int8_t)x[m * K + k]"),
    ("conv_u8_flipped_filter", "orc_conv_u8", "filt[((l2 * kh + dy) * kw + dx) * C + c]",
     "filt[((l2 * kh + (kh - 1 - dy)) * kw + (kw - 1 - dx)) * C + c]"),
]
# the min-pool case also needs its comparison turned round
_EXTRA = {"maxpool_is_min": ("if (v > best)", "if (v < best)"),
          "maxpool_output_size_from_window": ("const int64_t W2 = (W - win) / stride + 1;",
                                              "const int64_t W2 = (W - win) / win + 1;"),
          # an origin that steps by the window stays inside the input only if the output size
          # shrinks with it
          "maxpool_row_origin_steps_by_window": ("const int64_t H2 = (H - win) / stride + 1;",
                                                 "const int64_t H2 = (H - win) / win + 1;"),
          "maxpool_column_origin_steps_by_window": ("const int64_t W2 = (W - win) / stride + 1;",
                                                    "const int64_t W2 = (W - win) / win + 1;")}


def _function_span(src, func):
    start = src.index(" " + func + "(")
    start = src.rindex("\n", 0, start) + 1
    end = src.index("\n}\n", start) + 3
    return start, end


def _mutated(src, name, func, old, new):
    a, b = _function_span(src, func)
    body = src[a:b]
    assert body.count(old) == 1, (name, body.count(old))
    body = body.replace(old, new)
    if name in _EXTRA:
        o2, n2 = _EXTRA[name]
        assert body.count(o2) == 1
        body = body.replace(o2, n2)
    return src[:a] + body + src[b:]


def _build(text, path_c, path_so):
    with open(path_c, "w") as f:
        f.write(text)
    subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-o", path_so, path_c, "-lm"],
                   check=True)


def _pins_pass(lib):
    env = dict(os.environ, ESPRESSO_ORACLE_LIB=lib, OMP_NUM_THREADS="2")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, "tests", "test_oracle_pins.py"), "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                       text=True)
    return r.returncode == 0, r.stdout[-2000:]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    src = open(SRC).read()
    good = str(tmp_path / "good.so")
    _build(src, str(tmp_path / "good.c"), good)
    ok, out = _pins_pass(good)
    assert ok, "the untouched oracle must pass its pins when loaded from the side build:\n" + out

    def run(case):
        name, func, old, new = case
        lib = str(tmp_path / (name + ".so"))
        _build(_mutated(src, name, func, old, new), str(tmp_path / (name + ".c")), lib)
        return name, _pins_pass(lib)[0]

    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(run, MUTATIONS))
    survivors = [name for name, passed in results if passed]
    assert not survivors, "no pin noticed: %s" % survivors


def test_mutations_are_distinct_and_apply():
    src = open(SRC).read()
    seen = set()
    for name, func, old, new in MUTATIONS:
        text = _mutated(src, name, func, old, new)
        assert text != src and text not in seen, name
        seen.add(text)
