"""Host check of the constants behind the LOGITS-mode exponential (csrc/spec_accept.hip: exp_softmax): the kernel's
own numbers, read from its source, put through the same steps in numpy (rounding by the 1.5 * 2^52 sum, two-part
ln2, Horner, ldexp) must give exp to a few 1e-16, and must be the ones the generator script produces."""
import os
import re

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2604_20503_amd", "csrc", "spec_accept.hip")


def constants():
    text = open(SRC).read()
    body = text[text.index("ExpConsts exp_consts()"):]
    body = body[:body.index("return k;")]
    vals = {m.group(1): float(m.group(2)) for m in re.finditer(r"k\.(\w+) = (-?[0-9.eE+-]+);", body)}
    assert {"floor", "log2e", "nln2_hi", "nln2_lo", "magic"} <= set(vals) and all(f"c{i}" in vals for i in range(1, 11))
    return vals


def exp_like_the_kernel(x, k):
    x = np.maximum(x, k["floor"])
    t = x * k["log2e"] + k["magic"]
    kf = t - k["magic"]
    low_word = (t.view(np.uint64) & np.uint64(0xFFFFFFFF)).astype(np.uint32).view(np.int32)
    assert np.array_equal(low_word.astype(np.float64), kf)      # the integer really sits in the sum's low word
    r = (x + kf * k["nln2_hi"]) + kf * k["nln2_lo"]
    p = np.full_like(x, k["c10"])
    for i in range(9, 0, -1):
        p = p * r + k[f"c{i}"]
    p = p * r + 1.0
    return np.ldexp(p, low_word)


def test_kernel_constants_reproduce_exp():
    k = constants()
    rng = np.random.default_rng(0)
    x = np.concatenate([-rng.random(400000) * 60, -rng.random(100000) * 700, -rng.random(50000) * 1e-3,
                        rng.random(1000) * 5, [0.0, -0.34657359, -0.3465736, -707.9]])
    y, ref = exp_like_the_kernel(x, k), np.exp(x.astype(np.longdouble))
    assert float(np.max(np.abs(y.astype(np.longdouble) / ref - 1))) < 2e-15   # numpy has no fused multiply-add: a little above the kernel's 5e-16
    assert exp_like_the_kernel(np.array([0.0]), k)[0] == 1.0
    # far below the range: 0, also for -inf and for arguments past the clamp
    assert np.all(exp_like_the_kernel(np.array([-746.0, -800.0, -1e300, -np.inf]), k) == 0.0)
    # the two parts of ln2: the high part ends in 21 zero bits (so k * hi is exact for |k| < 2^21), together they are ln2
    hi, lo = -k["nln2_hi"], -k["nln2_lo"]
    assert (np.float64(hi).view(np.uint64) & np.uint64((1 << 21) - 1)) == 0
    assert abs((np.longdouble(hi) + np.longdouble(lo)) / np.log(np.longdouble(2)) - 1) < 1e-18
    assert k["magic"] == 1.5 * 2.0 ** 52 and abs(k["log2e"] * np.log(2.0) - 1) < 1e-15


def test_constants_are_what_the_generator_gives():
    import importlib.util
    spec = importlib.util.spec_from_file_location("gen", os.path.join(os.path.dirname(SRC), "exp_poly_coefficients.py"))
    gen = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(gen)
    c, k = gen.coefficients(), constants()
    assert c[0] == 1.0
    for i in range(1, 11):
        assert abs(c[i] / k[f"c{i}"] - 1) < 1e-12, i   # long double differs between libms in the last digits
    assert gen.max_relative_error(np.array([1.0] + [k[f"c{i}"] for i in range(1, 11)])) < 1e-15
