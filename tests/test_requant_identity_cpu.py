"""The identity behind the three-instruction requantization of the convolution kernels, checked on the CPU.

Definition (oracle, O-2.3 of the int8 student): y = float32(acc) * m, one IEEE single multiplication.  The kernels start
their accumulators at bias + 0x4B000000, read the int32 result as a float (exactly 2^23 + acc for 0 <= acc < 2^23) and
compute fma(that, m, -2^23 * m).  A fused multiply-add rounds the exact value (2^23 + acc) * m - 2^23 * m = acc * m
once, so both must be the same float; here the fused operation is carried out exactly in float64 (a 24-bit by 24-bit
product and its difference with another such product fit 53 bits) and rounded to float32 once.
"""
import numpy as np


def as_float(bits):
    return np.asarray(bits, np.int64).astype(np.uint32).view(np.float32)


def fma_form(acc, m):
    x = as_float(0x4B000000 + acc.astype(np.int64)).astype(np.float64)
    c = (m * np.float32(-8388608.0)).astype(np.float64)          # exact: a power of two times m
    return (x * m.astype(np.float64) + c).astype(np.float32)


def test_offset_accumulator_reads_as_2_pow_23_plus_acc():
    acc = np.array([0, 1, 2, 127, 8388607], np.int64)
    assert np.array_equal(as_float(0x4B000000 + acc).astype(np.float64), 8388608.0 + acc)


def test_fma_form_equals_the_definition_for_non_negative_accumulators():
    rng = np.random.default_rng(2211)
    acc = np.concatenate([rng.integers(0, 1 << 23, 200000), np.arange(0, 4096), (1 << 23) - 1 - np.arange(0, 4096)]).astype(np.int32)
    m = np.exp(rng.uniform(np.log(1e-7), np.log(1e-1), acc.size)).astype(np.float32)
    ref = acc.astype(np.float32) * m
    assert np.array_equal(fma_form(acc, m), ref)
    # values that land exactly on rounding ties of the final integer: acc * m = k + 0.5 with m a power of two
    acc2 = (2 * np.arange(0, 5000) + 1).astype(np.int32)
    m2 = np.full(acc2.size, 0.5, np.float32)
    assert np.array_equal(fma_form(acc2, m2), acc2.astype(np.float32) * m2)


def test_negative_accumulators_stay_negative():
    rng = np.random.default_rng(15023)
    acc = -rng.integers(1, 1 << 30, 100000).astype(np.int64)
    m = np.exp(rng.uniform(np.log(1e-7), np.log(1e-1), acc.size)).astype(np.float32)
    y = fma_form(acc, m)
    assert (y < 0).all()                                          # the clamp to [0, 127] returns 0, as for float(acc) * m
