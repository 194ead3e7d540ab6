"""The acceptance rule for a bf16 OUTPUT, shared by the GPU parity tests (and pinned on the CPU by
tests/test_bf16_rule.py).

A bf16 output is a quantised code: rounding the exact result to 8 significant bits alone costs
1.5e-3..2e-3 rel-L2, so the 2e-3 bar cannot be asked of every short row.  Both sides take the
rounding decision the same way:
  1. the bf16 output must equal round-to-nearest-even of the implementation's own fp32 output,
     bit for bit;
  2. it must be within one bf16 ulp of round-to-nearest-even of the oracle everywhere (or within
     1e-4 of the row's rms for elements far below the row's scale);
  3. where it differs from that code, the oracle's value must lie within the fp32 path's own error
     (4 x 5e-5 of the row's rms) of the rounding boundary between the two codes;
  4. its rel-L2 over the whole tensor must be <= 2e-3 once the tensor has >= 2048 elements.
"""
import numpy as np
import torch

TOL_BF16, TOL_BF16_F32OUT = 2e-3, 5e-5


def bf16_ordinal(x):
    """Map bf16 values (given as float arrays holding exact bf16) to integers monotone in value."""
    bits = (np.asarray(x, np.float32).view(np.uint32) >> 16).astype(np.int64)
    return np.where(bits & 0x8000, -(bits & 0x7fff), bits & 0x7fff)


def check_bf16_output(out_b, out_f32, ref_out):
    rne = torch.from_numpy(np.ascontiguousarray(out_f32)).to(torch.bfloat16).float().numpy()
    np.testing.assert_array_equal(out_b, rne)
    ref_b = torch.from_numpy(np.ascontiguousarray(ref_out)).to(torch.bfloat16).float().numpy()
    ulp = np.abs(bf16_ordinal(out_b) - bf16_ordinal(ref_b))
    # elements far below the row's scale carry the row's absolute fp32 error, which is many of THEIR ulps
    rms = np.sqrt((ref_out ** 2).mean(axis=-1, keepdims=True))
    small = np.abs(out_b - ref_b) <= 1e-4 * rms
    assert ((ulp <= 1) | small).all()
    # a different code is legitimate only where the exact value sits on a rounding boundary
    boundary = 0.5 * (out_b.astype(np.float64) + ref_b)
    assert ((ulp == 0) | small | (np.abs(ref_out - boundary) <= 4 * TOL_BF16_F32OUT * rms)).all()
    if ref_out.size >= 2048:
        den = np.linalg.norm(ref_out)
        if den == 0.0:   # every sequence empty: the result is exactly zero, and 0 / 0 is not a verdict
            assert not out_b.any()
        else:
            assert np.linalg.norm(out_b - ref_out) / den <= TOL_BF16
