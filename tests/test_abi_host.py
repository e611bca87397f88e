"""Host-side checks that need no GPU: the shared library loads, exports every symbol the header
declares, sizes workspaces, and rejects bad arguments before anything could be launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2503_10501_amd", "libtokencarve.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libtokencarve.so not built (run __graft_entry__.build())")


def _binding():
    from paper_2503_10501_amd import binding
    binding.load_library()
    return binding


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "tokencarve.h")).read()
    declared = set(re.findall(r"TC_API\s+[\w\s\*]+?\b(tc_\w+)\s*\(", header))
    assert {"tc_attn_output", "tc_ipgs_score", "tc_select_topk", "tc_merge", "tc_compress"} <= declared
    lib = ctypes.CDLL(LIB)
    for name in declared:
        assert hasattr(lib, name), name
    tc = _binding()
    assert declared == set(tc.SYMBOLS)


def test_params_struct_matches_header_layout():
    tc = _binding()
    header = open(os.path.join(ROOT, "include", "tokencarve.h")).read()
    body = header[header.index("typedef struct {"):header.index("} tc_params;")]
    fields = re.findall(r"^\s*(?:int32_t|float)\s+(\w+);", body, flags=re.M)
    mine = [f[0].rstrip("_") for f in tc.tc_params._fields_]
    assert fields == mine
    assert ctypes.sizeof(tc.tc_params) == 4 * len(fields)


def test_workspace_size_and_status_strings():
    tc = _binding()
    from workloads import CONFIGS
    sizes = {n: tc.tc_workspace_bytes(tc.params_for(w)) for n, w in CONFIGS.items()}
    assert all(v > 0 and v % 256 == 0 for v in sizes.values())
    assert sizes["llava7b_b64"] > 50 * sizes["llava7b_b1"]
    # O + Gram + eigenvectors dominate: at least B*N*(2D + 8N + 4N) bytes (bf16 O, fp64 G, fp32 U)
    w = CONFIGS["llava7b_b64"]
    assert sizes["llava7b_b64"] >= w.batch * w.n_vis * (2 * w.hidden + 12 * w.n_vis)
    assert tc.tc_status_string(0) == "ok"
    assert len({tc.tc_status_string(-i) for i in range(8)}) == 8


@pytest.mark.parametrize("field,value,status", [
    ("n_vis", 0, -2), ("n_vis", 5000, -2), ("head_dim", 96, -2), ("hidden_dim", 100, -2), ("vis_start", 600, -2),
    ("dtype", 7, -3), ("eig_dtype", 3, -3), ("lambda_", 1.5, -4), ("lambda_", -0.1, -4), ("k_final", 0, -4),
    ("k_prune", 9999, -4), ("k_final", 1, -4), ("norm_mode", 9, -4), ("causal", 2, -4), ("sv_rtol", 1.0, -4), ("stream_groups", 5, -4),
    ("n_prompt_queries", -1, -4), ("n_prompt_queries", 9, -4),     # the tiny workload has 8 prompt tokens
])
def test_invalid_params_are_rejected_on_the_host(field, value, status):
    tc = _binding()
    from workloads import CONFIGS
    p = tc.params_for(CONFIGS["tiny"])
    setattr(p, field, value)
    assert tc.tc_workspace_bytes(p) == 0
    lib = tc.load_library()
    fake = 4096  # never dereferenced: the call must fail before any launch
    assert lib.tc_select_topk(ctypes.byref(p), fake, fake, fake, 1 << 30, None) == status


def test_null_alignment_and_workspace_errors():
    tc = _binding()
    from workloads import CONFIGS
    p = tc.params_for(CONFIGS["tiny"])
    lib = tc.load_library()
    need = tc.tc_workspace_bytes(p)
    fake = 4096
    assert lib.tc_select_topk(ctypes.byref(p), None, fake, fake, need, None) == -1
    assert lib.tc_select_topk(ctypes.byref(p), fake, fake, None, need, None) == -1
    assert lib.tc_select_topk(ctypes.byref(p), fake + 4, fake, fake, need, None) == -6
    assert lib.tc_select_topk(ctypes.byref(p), fake, fake, fake, need - 1, None) == -5
    assert lib.tc_merge(ctypes.byref(p), fake, fake, fake, fake, fake, None, fake, need, None) == -1
    assert lib.tc_ipgs_score(ctypes.byref(p), fake, None, fake, None, None, None, fake, need, None) == -1  # lambda>0 needs S
    assert lib.tc_attn_output(ctypes.byref(p), fake, fake, fake, fake, None, fake, need - 1, None) == -5
    assert lib.tc_compress(ctypes.byref(p), fake, fake, fake, fake, fake, fake, fake, None, None, None, None,
                           fake, need - 1, None) == -5
    assert lib.tc_compress(None, fake, fake, fake, fake, fake, fake, fake, None, None, None, None, fake, need,
                           None) == -1
    p.batch = 0   # an empty batch is valid and launches nothing
    assert lib.tc_select_topk(ctypes.byref(p), fake, fake, fake, 1 << 20, None) == 0
    assert lib.tc_select_topk(ctypes.byref(p), None, None, None, 0, None) == 0


def test_rank_and_sequence_entry_points_check_their_arguments_on_the_host():
    tc = _binding()
    from workloads import CONFIGS
    p = tc.params_for(CONFIGS["tiny"])
    lib = tc.load_library()
    need = tc.tc_workspace_bytes(p)
    fake = 4096
    c = ctypes.byref(p)
    assert lib.tc_info_rank(c, None, None, 0, 0.0, fake, None, None, fake, need, None) == -1
    assert lib.tc_info_rank(c, fake, None, 0, 0.0, None, None, None, fake, need, None) == -1
    assert lib.tc_info_rank(c, fake, fake, p.n_vis + 1, 0.0, fake, None, None, fake, need, None) == -2
    assert lib.tc_info_rank(c, fake, fake, -1, 0.0, fake, None, None, fake, need, None) == -2
    assert lib.tc_info_rank(c, fake, None, 0, 1e-9, fake, None, None, fake, need, None) == -4   # below what the Gram route resolves
    assert lib.tc_info_rank(c, fake, None, 0, 1.0, fake, None, None, fake, need, None) == -4
    assert lib.tc_info_rank(c, fake, None, 0, -0.5, fake, None, None, fake, need, None) == -4
    assert lib.tc_info_rank(c, fake, None, 0, 0.0, fake, None, None, fake, 16, None) == -5
    assert lib.tc_info_rank(c, fake, None, 0, 0.0, fake + 8, None, None, fake, need, None) == -6
    assert lib.tc_assemble_sequence(c, fake, fake, fake, None, fake, 10000.0, None, None, None) == -1
    assert lib.tc_assemble_sequence(c, fake, fake, fake, fake, fake, 10000.0, fake, None, None) == -1   # cos without sin
    assert lib.tc_assemble_sequence(c, fake, fake, fake, fake, fake, 1.0, fake, fake, None) == -4       # base must exceed 1
    assert lib.tc_assemble_sequence(c, fake, fake, fake, fake, fake + 2, 10000.0, None, None, None) == -6
    # host arithmetic: the paper's KV-cache column for 192 / 128 / 64 kept tokens at about 80 text tokens
    assert abs(100 * tc.tc_kv_cache_fraction(80, 576, 192, 32, 2) - 45.1) < 0.15
    assert abs(100 * tc.tc_kv_cache_fraction(80, 576, 128, 32, 2) - 36.0) < 0.15
    assert abs(100 * tc.tc_kv_cache_fraction(80, 576, 64, 32, 2) - 26.9) < 0.15
    assert tc.tc_kv_cache_fraction(80, 576, 600, 32, 2) == -1.0
    p.batch = 0
    assert lib.tc_info_rank(c, None, None, 0, 0.0, None, None, None, None, 0, None) == 0
    assert lib.tc_assemble_sequence(c, None, None, None, None, None, 0.0, None, None, None) == 0


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2503_10501_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        binding.load_library()
