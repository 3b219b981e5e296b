"""The pins must be able to fail: plausible mistakes are planted in a COPY of the oracle's C
source (on the CPU), the copy is compiled, and at least one pin has to reject each of them."""
import ctypes
import itertools
import os
import subprocess
import tempfile

import pytest

import test_oracle_pins as pins
from conftest import read_golden
from oracle import build as oracle_build
from oracle import ref

MUTATIONS = {
    "spmm drops the last term of a row": ("p < row_ptr[m + 1]; ++p", "p < row_ptr[m + 1] - 1; ++p"),
    "spmm subtracts instead of adds": ("c[n] += a * b[n]", "c[n] -= a * b[n]"),
    "spmm reads the wrong row of B": ("B + (size_t)col_idx[p] * N", "B + (size_t)(col_idx[p] > 0 ? col_idx[p] - 1 : 0) * N"),
    "spmm scale without absolute value": ("s[n] += fabs(a) * fabs(b[n])", "s[n] += a * fabs(b[n])"),
    "conv flips the filter vertically": ("ih = oh + r - 1", "ih = oh - r + 1"),
    "conv flips the filter horizontally": ("iw = ow + s - 1;\n                                if", "iw = ow - s + 1;\n                                if"),
    "conv checks width against height": ("iw >= Wd) continue", "iw >= H) continue"),
    "conv transposes the taps": ("* 3 + r) * 3 + s]", "* 3 + s) * 3 + r]"),
    "conv drops the first image row": ("if (ih < 0 ||", "if (ih <= 0 ||"),
    "conv forgets the padding shift": ("ih = oh + r - 1", "ih = oh + r"),
    "im2col orders taps column-major": ("(c * 9 + r * 3 + s) * N", "(c * 9 + s * 3 + r) * N"),
    "im2col forgets zero fill": ("inside ? X[", "1 ? X["),
}


def _pin_suite():
    g = read_golden
    pins.test_hand_worked_spmm(g)
    for M, K in itertools.product((1, 3, 8), (2, 5, 17)):
        pins.test_brute_force_tiny(M, K)
    pins.test_identity_permutation_and_power_of_two_scaling_are_bit_exact()
    pins.test_linearity_is_exact_on_integers()
    pins.test_conv_all_ones_counts_taps(g)
    pins.test_conv_hand_shift(g)
    pins.test_conv_hand_two_channels(g)
    for r, s in itertools.product(range(3), range(3)):
        pins.test_conv_single_tap_is_a_zero_filled_shift(r, s)
    pins.test_conv_direct_equals_spmm_on_explicit_im2col()
    pins.test_conv_matches_library_cross_correlation()


def test_unmutated_oracle_passes_the_suite():
    _pin_suite()


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_pins_reject_a_planted_mistake(name, monkeypatch):
    old, new = MUTATIONS[name]
    src = open(oracle_build.SRC).read()
    assert src.count(old) >= 1, "mutation target not found: the oracle source changed"
    with tempfile.TemporaryDirectory() as tmp:
        cpath, sopath = os.path.join(tmp, "m.c"), os.path.join(tmp, "m.so")
        open(cpath, "w").write(src.replace(old, new, 1))
        subprocess.run(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                        "-o", sopath, cpath, "-lm"], check=True)
        good = ref._load()
        bad = ctypes.CDLL(sopath)
        for fn in ("oracle_spmm", "oracle_conv3x3", "oracle_im2col3x3", "oracle_max_threads"):
            getattr(bad, fn).argtypes = getattr(good, fn).argtypes
            getattr(bad, fn).restype = getattr(good, fn).restype
        monkeypatch.setattr(ref, "_lib", bad)
        with pytest.raises(AssertionError):
            _pin_suite()
