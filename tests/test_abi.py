"""The C-ABI library: exported symbols and host-side argument checks (no GPU work).

Every check in the library runs before anything is launched, so the error
paths can be driven from a machine without a GPU using fake, never-dereferenced
device addresses.
"""
import ctypes
import os
import re

import pytest

import paper_2408_04093_amd as ta
from paper_2408_04093_amd import build as ta_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tree_attn.h")
FAKE = 0x1000  # 16-byte (and 256-byte) aligned, never dereferenced


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(ta.lib_path()):
        ta_build.build()
    return ta.load()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ta_[a-z_]+)\s*\(", text)))


def llama_problem():
    p = ta.Problem()
    p.B, p.Hq, p.Hkv, p.d, p.N = 1, 32, 8, 128, 131072
    p.k_stride_n = p.v_stride_n = 128
    p.k_stride_h = p.v_stride_h = 131072 * 128
    p.k_stride_b = p.v_stride_b = 8 * 131072 * 128
    p.qkv_dtype, p.out_dtype, p.scale = ta.TA_BF16, ta.TA_BF16, 128 ** -0.5
    return p


def test_header_declares_the_expected_entry_points():
    assert declared_functions() == sorted([
        "ta_status_string", "ta_suggest_chunks", "ta_workspace_bytes",
        "ta_decode_partial", "ta_tree_combine", "ta_decode", "ta_decode_noalloc", "ta_energy",
        "ta_decode_two_pass"])


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_struct_layout_matches_header():
    # 4 int32, 7 int64, 2 int32, float (+pad), pointer, int32 (+pad)
    assert ctypes.sizeof(ta.Problem) == 16 + 56 + 8 + 8 + 8 + 8
    assert ta.Problem.valid_len.offset == 88 and ta.Problem.scale.offset == 80 and ta.Problem.Sq.offset == 96


def test_status_strings(lib):
    names = [ta.ta_status_string(c) for c in range(8)]
    assert len(set(names)) == 8 and names[0] == "ok"
    assert ta.ta_status_string(99) == "unknown status"


def test_workspace_and_chunk_heuristic(lib):
    p = llama_problem()
    P = ta.ta_suggest_chunks(p)
    assert 32 <= P <= 512
    assert (p.B * p.Hkv * P) % 256 == 0       # whole rounds of one workgroup per compute unit
    assert ta.ta_workspace_bytes(p, P) >= 32 * P * 130 * 4
    assert ta.ta_workspace_bytes(p, P) % 256 == 0
    assert ta.ta_workspace_bytes(p, 0) == 0
    p.N = 64               # tiny: never more chunks than keys / 256, at least one
    assert ta.ta_suggest_chunks(p) == 1
    p.d = 96
    assert ta.ta_suggest_chunks(p) == 0 and ta.ta_workspace_bytes(p, 4) == 0
    p = llama_problem()
    p.Sq = 8                # 8 tokens x group of 4 = 32 rows in one pass, partials for 8 x 32 heads
    assert ta.ta_workspace_bytes(p, 16) >= 8 * 32 * 16 * 130 * 4
    assert (p.B * p.Hkv * ta.ta_suggest_chunks(p)) % 256 == 0
    # more (batch, kv head) groups than compute units: the fewest chunks that fill the last round
    for B, N, want in [(64, 8192, 1), (48, 16384, 2), (48, 2048, 1), (256, 1024, 1)]:
        p = llama_problem()
        p.B, p.N = B, N
        p.k_stride_h = p.v_stride_h = N * 128
        p.k_stride_b = p.v_stride_b = 8 * N * 128
        assert ta.ta_suggest_chunks(p) == want, (B, N)


@pytest.mark.parametrize("mutate,code", [
    (lambda p: setattr(p, "d", 96), 6),
    (lambda p: setattr(p, "Hq", 30), 2),
    (lambda p: setattr(p, "N", 0), 2),
    (lambda p: setattr(p, "qkv_dtype", 7), 3),
    (lambda p: setattr(p, "k_stride_n", 132), 4),    # rows no longer 16-byte aligned
    (lambda p: setattr(p, "v_stride_n", 64), 2),     # rows overlap
    (lambda p: setattr(p, "scale", float("nan")), 2),
    (lambda p: setattr(p, "N", 1 << 41), 6),
    (lambda p: setattr(p, "k_stride_n", 1 << 31), 6),   # a row of 4 GiB
    (lambda p: setattr(p, "Sq", -1), 2),
])
def test_bad_problems_are_refused_before_launch(lib, mutate, code):
    p = llama_problem()
    mutate(p)
    assert ta.ta_decode(p, FAKE, FAKE, FAKE, FAKE, 1 << 30, FAKE, FAKE, None) == code
    assert ta.ta_decode_partial(p, FAKE, FAKE, FAKE, 4, None, FAKE, FAKE, FAKE, None) == code


def test_null_alignment_and_workspace_errors(lib):
    p = llama_problem()
    need = ta.ta_workspace_bytes(p, ta.ta_suggest_chunks(p))
    assert ta.ta_decode(p, None, FAKE, FAKE, FAKE, need, FAKE, FAKE, None) == 1
    assert ta.ta_decode(p, FAKE, FAKE + 8, FAKE, FAKE, need, FAKE, FAKE, None) in (4,)
    assert ta.ta_decode(p, FAKE, FAKE, FAKE, FAKE + 16, need, FAKE, FAKE, None) == 4
    assert ta.ta_decode(p, FAKE, FAKE, FAKE, FAKE, need - 1, FAKE, FAKE, None) == 5
    assert ta.ta_decode_partial(p, FAKE, FAKE, FAKE, 0, None, FAKE, FAKE, FAKE, None) == 2
    assert ta.ta_decode_partial(p, FAKE, FAKE, FAKE, 4, None, None, FAKE, FAKE, None) == 1
    assert ta.ta_tree_combine(1, 32, 128, 4, FAKE, FAKE, None, FAKE, 0, FAKE, None) == 1
    assert ta.ta_tree_combine(1, 32, 96, 4, FAKE, FAKE, FAKE, FAKE, 0, FAKE, None) == 6
    assert ta.ta_tree_combine(1, 32, 128, 0, FAKE, FAKE, FAKE, FAKE, 0, FAKE, None) == 2
    assert ta.ta_tree_combine(1, 32, 128, 4, FAKE, FAKE, FAKE, FAKE, 5, FAKE, None) == 3


def test_noalloc_entry_point_checks_and_size_limit(lib):
    p = llama_problem()
    assert ta.ta_decode_noalloc(p, None, FAKE, FAKE, FAKE, FAKE, None) == 1
    p.d = 96
    assert ta.ta_decode_noalloc(p, FAKE, FAKE, FAKE, FAKE, FAKE, None) == 6
    # partials beyond the library's 16 MiB device array: refused before the array is looked up
    p = llama_problem()
    p.Sq, p.N = 1024, 8192
    assert ta.ta_workspace_bytes(p, ta.ta_suggest_chunks(p)) > 16 << 20
    assert ta.ta_decode_noalloc(p, FAKE, FAKE, FAKE, FAKE, FAKE, None) == 5


def test_energy_and_two_pass_argument_checks(lib):
    p = llama_problem()
    need = ta.ta_workspace_bytes(p, ta.ta_suggest_chunks(p))
    assert ta.ta_energy(p, FAKE, FAKE, FAKE, need, None, None) == 1
    assert ta.ta_energy(p, FAKE, FAKE, FAKE, need - 1, FAKE, None) == 5
    assert ta.ta_energy(p, FAKE, FAKE + 4, FAKE, need, FAKE, None) == 4
    assert ta.ta_decode_two_pass(p, FAKE, FAKE, None, FAKE, need, FAKE, FAKE, None) == 1
    assert ta.ta_decode_two_pass(p, FAKE, FAKE, FAKE, FAKE, need, FAKE + 1, FAKE, None) == 4   # checked before any launch
    assert ta.ta_decode(p, FAKE, FAKE, FAKE, FAKE, need, FAKE + 1, FAKE, None) == 4
    p.qkv_dtype, p.Sq = ta.TA_F32, 2      # fp32 K/V takes several query tokens too: same checks
    need = ta.ta_workspace_bytes(p, ta.ta_suggest_chunks(p))
    assert ta.ta_energy(p, FAKE, FAKE, FAKE, need - 1, FAKE, None) == 5
    assert ta.ta_decode_two_pass(p, FAKE, FAKE, FAKE, FAKE, need - 1, FAKE, FAKE, None) == 5


def test_chunk_heuristic_invariants_on_seeded_random_problems(lib):
    """For any valid problem: 1 <= P <= ceil(N / 256) (never chunks shorter than 256 keys), the
    workspace covers the chunked layout, and the launch grid stays below 2^31 workgroups."""
    import numpy as np
    rng = np.random.default_rng(31)
    for _ in range(400):
        p = ta.Problem()
        p.d = int(rng.choice([64, 128]))
        p.Hkv = int(rng.choice([1, 2, 4, 8, 16]))
        g = int(rng.choice([1, 2, 4, 7, 8, 16, 33, 71]))
        p.Hq = p.Hkv * g
        p.B = int(rng.choice([1, 2, 3, 5, 16, 48, 64, 300, 2049]))
        p.N = int(rng.choice([1, 255, 256, 257, 1000, 4096, 5000, 65536, 1 << 20]))
        bf16 = bool(rng.integers(0, 2))
        p.qkv_dtype = ta.TA_BF16 if bf16 else ta.TA_F32
        p.Sq = int(rng.choice([0, 1, 3, 17]))
        if p.N * p.d * (2 if bf16 else 4) >= 1 << 32:
            continue
        p.k_stride_n = p.v_stride_n = p.d
        p.k_stride_h = p.v_stride_h = p.N * p.d
        p.k_stride_b = p.v_stride_b = p.Hkv * p.N * p.d
        p.out_dtype, p.scale = ta.TA_F32, 0.1
        p.valid_len = FAKE if rng.integers(0, 2) else None
        P = ta.ta_suggest_chunks(p)
        assert 1 <= P <= -(-p.N // 256), (p.B, p.Hq, p.Hkv, p.d, p.N, p.Sq, P)
        sq = max(1, p.Sq)
        assert ta.ta_workspace_bytes(p, P) >= p.B * sq * p.Hq * P * (p.d + 2) * 4
        assert ta.ta_workspace_bytes(p, P) % 256 == 0
        slices = -(-sq * g // 64) if bf16 else sq * g   # fp32: at least one (token, head) row per workgroup
        assert p.B * p.Hkv * slices * P < 1 << 31


def test_ragged_problems_reserve_workspace_for_the_balanced_launch(lib):
    p = llama_problem()
    p.B = 16
    p.k_stride_b = p.v_stride_b = 8 * 131072 * 128
    plain = ta.ta_workspace_bytes(p, 1)
    p.valid_len = FAKE
    # 256 shares + 16 x 8 segments, 4 rows of 130 floats each, plus the prefix table
    assert ta.ta_workspace_bytes(p, 1) >= (256 + 128) * 4 * 130 * 4 + 17 * 8 > plain
    # many short sequences (more groups than compute units, capacity below 4096 keys): chunks, not shares
    p = llama_problem()
    p.B, p.N = 128, 1024
    p.k_stride_h = p.v_stride_h = 1024 * 128
    p.k_stride_b = p.v_stride_b = 8 * 1024 * 128
    plain = ta.ta_workspace_bytes(p, 1)
    p.valid_len = FAKE
    assert ta.ta_workspace_bytes(p, 1) == plain and ta.ta_suggest_chunks(p) == 1
    p.N = 8192                                   # long enough for the shares to pay: 1024 groups <= 4 per CU
    p.k_stride_h = p.v_stride_h = 8192 * 128
    p.k_stride_b = p.v_stride_b = 8 * 8192 * 128
    assert ta.ta_workspace_bytes(p, 1) >= (256 + 1024) * 4 * 130 * 4
    p.B = 129                                    # 1032 groups: beyond 4 per CU
    assert ta.ta_workspace_bytes(p, 1) == 129 * 32 * 130 * 4


def test_binding_refuses_host_tensors_and_wrong_length_tables():
    import torch
    q = torch.zeros((2, 8, 64), dtype=torch.bfloat16)
    K = torch.zeros((2, 2, 16, 64), dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="int32"):
        ta.make_problem(q, K, K, 1.0, torch.tensor([3, 4]))                      # int64 lengths
    with pytest.raises(ValueError, match="int32"):
        ta.make_problem(q, K, K, 1.0, torch.tensor([3, 4, 5], dtype=torch.int32))   # wrong shape
    with pytest.raises(ValueError, match="device tensors"):
        ta.make_problem(q, K, K, 1.0, torch.tensor([3, 4], dtype=torch.int32))   # host memory
    with pytest.raises(ValueError, match="disagree"):
        ta.make_problem(q, K.float(), K.float(), 1.0)


def test_size_check_does_not_overflow(lib):
    p = llama_problem()
    p.N = (1 << 62)
    assert ta.ta_decode(p, FAKE, FAKE, FAKE, FAKE, 1 << 30, FAKE, FAKE, None) == 6
    p.N, p.k_stride_n = 1 << 20, 1 << 45
    assert ta.ta_decode(p, FAKE, FAKE, FAKE, FAKE, 1 << 30, FAKE, FAKE, None) == 6


def test_head_slices_beyond_4_gib_get_enough_chunks(lib):
    # row offsets inside a chunk are 32-bit: a head slice of 8 GiB (2^25 keys of 256 bytes) needs >= 3 chunks
    p = llama_problem()
    p.B, p.Hq, p.Hkv, p.N = 1, 4, 1, 1 << 25
    p.k_stride_h = p.v_stride_h = p.k_stride_b = p.v_stride_b = p.N * 128
    P = ta.ta_suggest_chunks(p)
    assert P >= 3 and -(-p.N // P) * 256 < 1 << 32
    assert ta.ta_decode_partial(p, FAKE, FAKE, FAKE, 1, None, FAKE, FAKE, FAKE, None) == 6    # one chunk of 8 GiB
    assert ta.ta_decode_partial(p, FAKE, FAKE, FAKE, 2, None, FAKE, FAKE, FAKE, None) == 6    # two of 4 GiB
    assert ta.ta_decode_partial(p, FAKE, FAKE, FAKE, 64, FAKE, FAKE, FAKE, FAKE, None) == 6   # a table may hold any chunk
    # many sequences, more groups than compute units: still never one chunk per sequence
    p.B = 1024
    p.k_stride_b = p.v_stride_b = p.N * 128
    assert ta.ta_suggest_chunks(p) >= 3
    # ragged: the balanced launch (a piece may be a whole sequence) is not taken
    p.B, p.valid_len = 2, FAKE
    P = ta.ta_suggest_chunks(p)
    assert ta.ta_workspace_bytes(p, P) == -(-(2 * 4 * P * 130 * 4) // 256) * 256


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2408_04093_amd import _ffi
    monkeypatch.setattr(_ffi, "_lib", None)
    monkeypatch.setattr(_ffi, "_LIB_PATH", "/nonexistent/libtree_attn.so")
    with pytest.raises(ImportError, match="no CPU fallback"):
        _ffi.load()
