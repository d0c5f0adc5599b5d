"""The pins must be able to fail: every planted mistake below (a textual mutant of the C oracle,
compiled to a temporary library and swapped in for the real one) has to be caught by at least one
of the pin tests.  All of this runs on the CPU; the committed oracle is not modified."""
import ctypes
import os
import subprocess

import pytest

import oracle
import test_oracle_pins as pins

SRC = os.path.join(os.path.dirname(oracle.__file__), "dwconv_oracle.c")

# (name, text to replace, replacement, which occurrence: 0 = fwd, 1 = bwd_data, 2 = bwd_filter, None = all)
MUTANTS = [
    ("fwd_filter_flipped", "w[wat(L, O, K, o, kh, kw)] * x[", "w[wat(L, O, K, o, K - 1 - kh, K - 1 - kw)] * x[", 0),
    ("fwd_pad_sign", "int ih = oh * s - p + kh, iw = ow * s - p + kw;", "int ih = oh * s + p - kh, iw = ow * s + p - kw;", 0),
    ("fwd_taps_transposed", "int ih = oh * s - p + kh, iw = ow * s - p + kw;", "int ih = oh * s - p + kw, iw = ow * s - p + kh;", 0),
    ("fwd_drops_last_tap", "for (int kw = 0; kw < K; ++kw) {\n                            int ih", "for (int kw = 0; kw < K - (K > 1); ++kw) {\n                            int ih", 0),
    ("fwd_ignores_stride_in_w", "int ih = oh * s - p + kh, iw = ow * s - p + kw;", "int ih = oh * s - p + kh, iw = ow - p + kw;", 0),
    ("bwd_data_filter_flipped", "] += w[wat(L, O, K, o, kh, kw)] * g;", "] += w[wat(L, O, K, o, K - 1 - kh, K - 1 - kw)] * g;", None),
    ("bwd_data_pad_sign", "int ih = oh * s - p + kh, iw = ow * s - p + kw;", "int ih = oh * s + p - kh, iw = ow * s + p - kw;", 1),
    ("bwd_data_wrong_channel_group", "dx[at(L, C, H, W, n, o / m, ih, iw)] +=", "dx[at(L, C, H, W, n, o % C, ih, iw)] +=", None),
    ("bwd_filter_pad_sign", "int ih = oh * s - p + kh, iw = ow * s - p + kw;", "int ih = oh * s + p - kh, iw = ow * s + p - kw;", 2),
    ("bwd_filter_taps_transposed", "dw[wat(L, O, K, o, kh, kw)] = acc;", "dw[wat(L, O, K, o, kw, kh)] = acc;", None),
    ("bwd_filter_mean_over_batch", "dw[wat(L, O, K, o, kh, kw)] = acc;", "dw[wat(L, O, K, o, kh, kw)] = acc / N;", None),
    ("out_dim_ceil", "return span / s + 1;", "return (span + s - 1) / s + 1;", None),
    ("nhwc_filter_layout", "return ((size_t)kh * K + kw) * O + o;", "return ((size_t)o * K + kh) * K + kw;", None),
    ("multiplier_mapping", "x[at(L, C, H, W, n, o / m, ih, iw)]", "x[at(L, C, H, W, n, o % C, ih, iw)]", None),
]


def _replace_nth(text, old, new, nth):
    if nth is None:
        assert old in text, old
        return text.replace(old, new)
    pos = -1
    for _ in range(nth + 1):
        pos = text.index(old, pos + 1)
    return text[:pos] + new + text[pos + len(old):]


def _pins():
    """A cheap but wide subset of the pins, each as a zero-argument callable."""
    calls = []
    for case in pins.TINY:
        calls.append(lambda c=case: pins.test_fwd_equals_block_diagonal_dense_convolution(*c))
        calls.append(lambda c=case: pins.test_bwd_data_equals_transposed_dense_convolution(*c))
        calls.append(lambda c=case: pins.test_bwd_filter_equals_masked_dense_gradient(*c))
    for kind, kv, vals in pins._golden():
        calls.append(lambda a=(kind, kv, vals): pins.test_all_ones_golden(*a))
    calls.append(pins.test_off_centre_delta_filter_pins_the_shift_direction)
    calls.append(pins.test_k1_is_a_per_channel_scale_and_dot_product)
    return calls


@pytest.mark.parametrize("name,old,new,nth", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(tmp_path, monkeypatch, name, old, new, nth):
    src = open(SRC).read()
    mutated = _replace_nth(src, old, new, nth)
    assert mutated != src
    csrc = tmp_path / "mutant.c"
    csrc.write_text(mutated)
    lib_path = tmp_path / "libmutant.so"
    subprocess.check_call(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-o", str(lib_path), str(csrc)])
    real = oracle._load()
    lib = ctypes.CDLL(str(lib_path))
    for fn in ("oracle_dwconv_fwd", "oracle_dwconv_bwd_data", "oracle_dwconv_bwd_filter", "oracle_out_dims"):
        getattr(lib, fn).argtypes = getattr(real, fn).argtypes
        getattr(lib, fn).restype = getattr(real, fn).restype
    lib.oracle_threads_available.restype = ctypes.c_int
    monkeypatch.setattr(oracle, "_lib", lib)
    caught = 0
    for call in _pins():
        try:
            call()
        except (AssertionError, ValueError):
            caught += 1
    assert caught > 0, "no pin noticed the mutant %s" % name
