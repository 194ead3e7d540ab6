"""CPU pins of the bf16-output acceptance rule (tests/bf16_rule.py): what it must accept and what
it must refuse.  The rule is test infrastructure for the GPU parity tests; these cases freeze it."""
import numpy as np
import pytest
import torch

from bf16_rule import TOL_BF16_F32OUT, bf16_ordinal, check_bf16_output


def rne(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16).float().numpy()


def truncate(x):
    return (np.ascontiguousarray(x, dtype=np.float32).view(np.uint32) & 0xffff0000).view(np.float32)


def next_code(b, step=1):
    """The bf16 value `step` codes above b (b holds exact bf16 values)."""
    o = bf16_ordinal(b) + step
    bits = np.where(o < 0, 0x8000 | (-o), o).astype(np.uint32) << 16
    return bits.view(np.float32)


@pytest.fixture
def ref():
    g = np.random.default_rng(20240804)
    # rows like attention outputs at the benchmark shape: means of many N(0,1) values, scale ~ 3e-3
    return g.standard_normal((32, 128)) * 3e-3


def test_exact_result_rounded_to_nearest_even_passes(ref):
    f32 = ref.astype(np.float32)
    check_bf16_output(rne(f32), f32, ref)


def test_fp32_path_error_of_the_tested_size_passes(ref):
    g = np.random.default_rng(1)
    rms = np.sqrt((ref ** 2).mean(axis=-1, keepdims=True))
    f32 = (ref + g.standard_normal(ref.shape) * 2e-5 * rms).astype(np.float32)   # what the fp32 bar (5e-5 per row) allows
    check_bf16_output(rne(f32), f32, ref)


def test_one_ulp_bias_on_every_element_fails(ref):
    f32 = ref.astype(np.float32)
    biased = next_code(rne(f32))
    # even if the implementation's own fp32 output agreed with the biased codes (clause 1 satisfied) ...
    with pytest.raises(AssertionError):
        check_bf16_output(biased, biased.copy(), ref)
    # ... and of course when it does not
    with pytest.raises(AssertionError):
        check_bf16_output(biased, f32, ref)


def test_single_flip_in_the_middle_of_a_rounding_interval_fails(ref):
    f32 = ref.astype(np.float32)
    good = rne(f32)
    # pick an element of ordinary size whose exact value sits near the CENTRE of its code's interval
    rms = np.sqrt((ref ** 2).mean(axis=-1, keepdims=True))
    centre_dist = np.abs(ref - good) / np.abs(next_code(good) - good)          # 0 = centre, 0.5 = boundary
    cand = np.argwhere((centre_dist < 0.05) & (np.abs(ref) > rms))
    assert len(cand) > 0
    i, j = cand[0]
    bad = good.copy()
    bad[i, j] = next_code(good)[i, j]
    with pytest.raises(AssertionError):
        check_bf16_output(bad, bad.copy(), ref)


def test_flip_exactly_at_a_rounding_boundary_is_accepted(ref):
    ref = ref.copy()
    f32 = ref.astype(np.float32)
    good = rne(f32)
    up = next_code(good)
    i, j = 3, 17
    ref[i, j] = 0.5 * (float(good[i, j]) + float(up[i, j])) * (1 - 1e-9)   # a hair below the boundary: RNE(ref) = good
    rms = np.sqrt((ref ** 2).mean(axis=-1, keepdims=True))
    assert abs(ref[i, j]) > rms[i, 0] * 0.05
    f32 = ref.astype(np.float32)
    f32[i, j] = np.float32(ref[i, j] * (1 + 2e-7))                          # an fp32 path a rounding error above it
    out_b = rne(f32)
    assert out_b[i, j] == up[i, j] or out_b[i, j] == good[i, j]
    check_bf16_output(out_b, f32, ref)


def test_truncation_instead_of_rounding_fails(ref):
    f32 = ref.astype(np.float32)
    trunc = truncate(f32)
    assert (trunc != rne(f32)).mean() > 0.3
    with pytest.raises(AssertionError):
        check_bf16_output(trunc, f32, ref)            # not RNE of its own fp32 output
    with pytest.raises(AssertionError):
        check_bf16_output(trunc, trunc.copy(), ref)   # an fp32 output that was itself truncated


def test_two_ulp_error_fails_even_on_one_element(ref):
    f32 = ref.astype(np.float32)
    bad = rne(f32)
    rms = np.sqrt((ref ** 2).mean(axis=-1, keepdims=True))
    i, j = np.argwhere(np.abs(ref) > rms)[0]
    bad[i, j] = next_code(bad, 2)[i, j]
    with pytest.raises(AssertionError):
        check_bf16_output(bad, bad.copy(), ref)


def test_whole_tensor_bar_applies_from_2048_elements(ref):
    # a uniformly scaled output (relative error 0.4 %, half a bf16 ulp) passes no clause on a large tensor
    f32 = (ref * 1.004).astype(np.float32)
    assert ref.size >= 2048 and TOL_BF16_F32OUT < 1e-3
    with pytest.raises(AssertionError):
        check_bf16_output(rne(f32), f32, ref)


def test_an_all_zero_reference_demands_exact_zeros():
    # every sequence of the batch empty: the whole result is zero, the relative error 0 / 0
    ref = np.zeros((2, 64, 64))
    zeros = np.zeros((2, 64, 64), np.float32)
    check_bf16_output(zeros.copy(), zeros, ref)
    bad = zeros.copy()
    bad[1, 3, 5] = 1e-30
    with pytest.raises(AssertionError):
        check_bf16_output(rne(bad), bad, ref)
