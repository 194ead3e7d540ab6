"""MI355X-native decode attention (Tree Attention hot path) -- Python binding.

Thin argument marshalling over the C ABI in include/tree_attn.h; every step of
the computation runs in the HIP kernels of libtree_attn.so.  There is no
fallback: if the library has not been built, loading raises.
"""
from ._ffi import (  # noqa: F401
    TA_BF16, TA_F32, TAError, Problem, lib_path, load,
    ta_status_string, ta_suggest_chunks, ta_workspace_bytes,
    ta_decode_partial, ta_tree_combine, ta_decode, ta_decode_noalloc, ta_energy, ta_decode_two_pass,
    make_problem, decode, decode_partial, tree_combine, energy, decode_two_pass,
)
