"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares,
sizes workspaces and rejects bad arguments without touching a GPU."""
import ctypes
import os
import re

import pytest

import paper_2506_03566_amd as P
from synth import get_config, CONFIGS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lib():
    if not os.path.exists(P.LIB_PATH):
        pytest.skip("libposs.so not built (run __graft_entry__.build())")
    return P.load_library()


def test_exports_match_header():
    lib = _lib()
    header = open(os.path.join(ROOT, "include", "poss.h")).read()
    declared = set(re.findall(r"\b(poss_[a-z_]+)\s*\(", header))
    assert declared == set(P.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_layout_matches_header():
    # 7 ints, 2 floats, 11 ints = 80 bytes; the stats struct: 2 + 17 int64 + 3 doubles
    assert ctypes.sizeof(P.PossConfig) == 20 * 4
    assert ctypes.sizeof(P.PossStats) == 19 * 8 + 3 * 8


def test_workspace_bytes_and_config_validation():
    lib = _lib()
    for name, cfg in CONFIGS.items():
        assert lib.poss_workspace_bytes(ctypes.byref(P.make_config(cfg))) > 0, name
    big = lib.poss_workspace_bytes(ctypes.byref(P.make_config(get_config("c1_llama3_8b_3x2"))))
    assert 16e9 < big < 20e9          # ~17.6 GB of repacked bf16 weights + caches + scratch
    base = get_config("c0_tiny_f32")
    bad = [dict(top_k=0), dict(top_k=17), dict(depth=0), dict(depth=17), dict(total_tokens=0),
           dict(total_tokens=128), dict(total_tokens=85), dict(kv_page_tokens=48), dict(max_seq=100),
           dict(n_kv_heads=3), dict(dtype=3), dict(n_specialists=0), dict(positions_per_specialist=0),
           dict(top_k=4096), dict(dtype=1, head_dim=32), dict(dtype=1, d_model=260), dict(kv_page_order=2),
           dict(dtype=1, max_seq=500096)]          # beyond 256 attention splits of 64 blocks of 32 keys
    for over in bad:
        assert lib.poss_workspace_bytes(ctypes.byref(P.make_config(base.with_(**over)))) == 0, over
    assert lib.poss_workspace_bytes(ctypes.byref(P.make_config(base.with_(dtype=1, max_seq=499968)))) > 0
    assert lib.poss_workspace_bytes(None) == 0
    # several sequences per round: up to eight (passes whose stacked rows exceed a launch run in groups),
    # every sequence with caches and tree state of its own
    def ws(cfg, batch):
        return lib.poss_workspace_bytes(ctypes.byref(P.make_config(cfg, batch=batch)))
    c1 = get_config("c1_llama3_8b_3x2")
    assert ws(c1, 0) == ws(c1, 1) == big                    # 0 and 1 both mean one sequence
    assert big < ws(c1, 2) < ws(c1, 3) < ws(c1, 8)
    assert 0 < ws(base, 5) < ws(base, 6)
    assert ws(base, -1) == 0 and ws(base, 9) == 0


def test_null_arguments_are_rejected_before_any_gpu_work():
    lib = _lib()
    cfg = P.make_config(get_config("c0_tiny_f32"))
    out = ctypes.c_void_p()
    assert lib.poss_load(ctypes.byref(cfg), None, None, 0, None, ctypes.byref(out)) == P.E_INVALID_ARG
    assert b"null" in lib.poss_last_error(None)
    assert lib.poss_prefill(None, None, 0, None) == P.E_INVALID_ARG
    assert lib.poss_prefill_seq(None, 0, None, 0, None) == P.E_INVALID_ARG
    assert lib.poss_get_tree_seq(None, 0, None) == P.E_INVALID_ARG
    assert lib.poss_get_commit_seq(None, 0, None, None, None, None) == P.E_INVALID_ARG
    assert lib.poss_get_tokens_seq(None, 0, None, 0, None) == P.E_INVALID_ARG
    assert lib.poss_draft_tree(None, None) == P.E_INVALID_ARG
    assert lib.poss_verify_tree(None, None, None, None, None) == P.E_INVALID_ARG
    assert lib.poss_accept_and_commit(None, None, None, None, None) == P.E_INVALID_ARG
    assert lib.poss_get_stats(None, None) == P.E_INVALID_ARG
    assert lib.poss_debug_gemm_scratch_bytes(1, 0, 10, 10) == 0
    assert lib.poss_debug_gemm_scratch_bytes(1, 257, 10, 16) == 0
    lib.poss_free(None)
