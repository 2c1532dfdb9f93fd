"""The numerical bounds of the GPU-vs-oracle comparisons, in one place.

Loss of a batch: 1e-5 relative.  Embedding tables after an iteration:

  fp32 tables    |got - want| <= max(1e-5, 16 units in the last place of the fp32 value want):
                 1e-5 max-abs wherever |want| < 8 (every workload: embeddings stay below 1),
                 and 16 spacings of the stored value beyond that, where 1e-5 would be fewer
                 than ten spacings (degenerate test batches: a thousand terms on one row,
                 values of tens).  The kernels add a row's terms exactly; what is left is the
                 fp32 arithmetic before the sum (dot products, the sigmoid, the gradient of a
                 run of equal centres summed in fp32: a few units of the result).
  16-bit tables  every element within one step of the storage format of the oracle's value,
                 or within the fp32 bound above where a sum cancels to a value far smaller
                 than its operands; and all but HALF_FLIP_FRACTION of the elements bit-identical.
                 A coefficient computed in fp32 carries a relative error of about 1e-7, which
                 moves a sum across a rounding boundary of a format with p significand bits with
                 probability about 1e-7 * 2^p: 2.6e-5 for bfloat16 (p = 8; measured 2e-5), 2e-4
                 for binary16 (p = 11; measured 1.7e-4).  Allowed: 1e-4 and 1e-3.
"""
import numpy as np

LOSS_RTOL = 1e-5
EMB_ATOL = 1e-5
EMB_ULPS = 16
HALF_FLIP_FRACTION = {"bf16": 1e-4, "f16": 1e-3}


def emb_bound(want):
    """Element-wise bound for fp32 table values."""
    want = np.asarray(want, dtype=np.float32)
    return np.maximum(np.float32(EMB_ATOL), EMB_ULPS * np.spacing(np.abs(want)))


def assert_emb_close(got, want):
    got = np.asarray(got, dtype=np.float32)
    want = np.asarray(want, dtype=np.float32)
    excess = np.abs(got.astype(np.float64) - want.astype(np.float64)) - emb_bound(want)
    assert excess.max() <= 0, float(excess.max())


def half_values(bits, fmt):
    """fp32 values of 16-bit patterns (uint16 array), fmt in {"bf16", "f16"}."""
    bits = np.asarray(bits, dtype=np.uint16)
    if fmt == "bf16":
        return (bits.astype(np.uint32) << 16).view(np.float32)
    return bits.view(np.float16).astype(np.float32)


def assert_half_close(got_bits, want_bits, fmt, steps=1, flip_fraction=None):
    """16-bit tables: within `steps` of the format (or the fp32 bound), few elements off at all."""
    got_bits = np.asarray(got_bits, dtype=np.uint16)
    want_bits = np.asarray(want_bits, dtype=np.uint16)
    near = np.abs(got_bits.astype(np.int32) - want_bits.astype(np.int32)) <= steps
    gv, wv = half_values(got_bits, fmt), half_values(want_bits, fmt)
    assert (near | (np.abs(gv - wv) <= emb_bound(wv))).all()
    off = float((got_bits != want_bits).mean())
    assert off <= (HALF_FLIP_FRACTION[fmt] if flip_fraction is None else flip_fraction), off
