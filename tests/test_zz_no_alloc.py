"""ta_decode_noalloc: the workspace-free entry point against ta_decode.

Both run the same kernels with the same chunking, so the outputs must be
bit-identical; the oracle bar is checked as well.  Two calls in a row share
the library's device array, the second on a smaller input; then a ragged
batch (balanced launch: the array also holds the prefix table), several query
tokens, fp32, and a refusal of a problem whose partials exceed the array.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2408_04093_amd as ta
import ta_workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _lib():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    ta.load()


def noalloc(w, out_dtype):
    p = ta.make_problem(w.q, w.K, w.V, w.scale, w.valid_len, out_dtype)
    out = torch.full(tuple(w.q.shape), float("nan"), device=w.q.device,
                     dtype=torch.bfloat16 if out_dtype == ta.TA_BF16 else torch.float32)
    lse = torch.full(tuple(w.q.shape[:-1]), float("nan"), dtype=torch.float32, device=w.q.device)
    rc = ta.ta_decode_noalloc(p, w.q.data_ptr(), w.K.data_ptr(), w.V.data_ptr(), out.data_ptr(), lse.data_ptr(),
                              torch.cuda.current_stream().cuda_stream)
    assert rc == 0, ta.ta_status_string(rc)
    return out, lse


def same_as_decode_and_oracle(w, causal=False):
    for od in (ta.TA_F32, ta.TA_BF16):
        out, lse = noalloc(w, od)
        ref_out, ref_lse = ta.decode(w.q, w.K, w.V, w.scale, w.valid_len, od)
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16 if od == ta.TA_BF16 else torch.int32),
                           ref_out.view(torch.int16 if od == ta.TA_BF16 else torch.int32))
        assert torch.equal(lse.view(torch.int32), ref_lse.view(torch.int32))
    out, lse = noalloc(w, ta.TA_F32)
    torch.cuda.synchronize()
    vl = None if w.valid_len is None else w.valid_len.cpu().numpy()
    fn = oracle.decode_causal if causal else oracle.decode
    o_ref, l_ref = fn(w.q.cpu(), w.K.cpu(), w.V.cpu(), w.scale, vl)
    o = out.cpu().numpy().astype(np.float64)
    den = np.linalg.norm(o_ref, axis=-1)
    rel = np.linalg.norm(o - o_ref, axis=-1) / np.where(den > 0, den, 1.0)
    assert rel.max() <= (5e-5 if w.q.dtype == torch.bfloat16 else 1e-5)
    l = lse.cpu().numpy().astype(np.float64)
    fin = np.isfinite(l_ref)
    assert (np.isneginf(l) == np.isneginf(l_ref)).all() and np.abs(l[fin] - l_ref[fin]).max() <= 1e-4


def test_two_calls_in_a_row_the_second_on_a_smaller_input():
    big = W.make_qkv(2, 32, 8, 128, 40000, torch.bfloat16, seed=901, device="cuda:0")
    small = W.make_qkv(1, 8, 2, 128, 5000, torch.bfloat16, seed=902, device="cuda:0")
    same_as_decode_and_oracle(big)
    same_as_decode_and_oracle(small)
    same_as_decode_and_oracle(big)


def test_ragged_batch_several_tokens_and_fp32():
    w = W.make_qkv(6, 16, 4, 128, 20000, torch.bfloat16, seed=903, device="cuda:0")
    w.valid_len = torch.tensor([20000, 1, 0, 7777, 13, 4096], dtype=torch.int32, device="cuda:0")
    same_as_decode_and_oracle(w)
    m = W.make_multi(2, 5, 8, 2, 64, 3000, torch.bfloat16, 904, "cuda:0")
    same_as_decode_and_oracle(m, causal=True)
    f = W.make_qkv(1, 4, 2, 64, 9000, torch.float32, seed=905, device="cuda:0")
    same_as_decode_and_oracle(f)


def test_a_problem_beyond_the_array_is_refused():
    w = W.make_multi(1, 1024, 32, 8, 128, 8192, torch.bfloat16, 906, "cuda:0")
    p = ta.make_problem(w.q, w.K, w.V, w.scale, None, ta.TA_BF16)
    assert ta.ta_workspace_bytes(p, ta.ta_suggest_chunks(p)) > 16 << 20
    out = torch.empty_like(w.q)
    lse = torch.empty(tuple(w.q.shape[:-1]), dtype=torch.float32, device="cuda:0")
    assert ta.ta_decode_noalloc(p, w.q.data_ptr(), w.K.data_ptr(), w.V.data_ptr(), out.data_ptr(),
                                lse.data_ptr(), None) == 5
