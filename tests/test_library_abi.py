"""The C-ABI library loads and exports every symbol include/jakiro_verify.h declares;
host-only entry points behave (no GPU needed, no compute calls)."""
import ctypes
import os
import re

import pytest

import paper_2502_06282_amd as jk
from paper_2502_06282_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(jk.library_path()):
        from paper_2502_06282_amd import build
        build.build()
    return jk.lib()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "jakiro_verify.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(jk_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings_and_version(lib):
    assert jk.version() == "0.1"
    seen = {lib.jk_status_string(i).decode() for i in range(6)}
    assert len(seen) == 6 and lib.jk_status_string(99).decode() == "unknown status"


def test_validate_tree(lib):
    assert jk.validate_tree([-1, 0, 0, 1]) == 0
    assert jk.validate_tree([-1, -1, -1]) == 0
    assert jk.validate_tree([0]) == 2
    assert jk.validate_tree([-1, 1]) == 2
    assert jk.validate_tree([-2]) == 2
    assert jk.validate_tree([-1] * 129) == 1
    assert lib.jk_validate_tree(None, 3) == 1


def test_workspace_queries_are_host_only(lib):
    d = binding.AttnDesc(1, 60, 32, 8, 128, 0, 4096, 128, 0, 1024, 128, 0, 1024, 128, 0, 4096, 128, 0.0, 0)
    n = lib.jk_tree_verify_attention_workspace(ctypes.byref(d), 4096)
    assert n > 0 and n % 256 == 0
    d.head_dim = 96
    assert lib.jk_tree_verify_attention_workspace(ctypes.byref(d), 4096) == 0
    d.head_dim = 128; d.n_tree = 129
    assert lib.jk_tree_verify_attention_workspace(ctypes.byref(d), 4096) == 0
    assert lib.jk_tree_verify_attention_workspace(None, 4096) == 0
    g = lib.jk_accept_path_workspace(1, 60, 32000, 0)
    s = lib.jk_accept_path_workspace(1, 60, 32000, 1)
    assert 0 < g < s
    assert lib.jk_accept_path_workspace(1, 0, 32000, 0) == 0
    assert lib.jk_accept_path_workspace(1, 60, 32000, 7) == 0


def test_null_arguments_are_rejected_before_any_launch(lib):
    d = binding.AttnDesc(1, 4, 2, 2, 128, 0, 256, 128, 0, 256, 128, 0, 256, 128, 0, 256, 128, 0.0, 0)
    st = lib.jk_tree_verify_attention(ctypes.byref(d), None, None, None, None, None, None, None, 0, None, None, 0,
                                      None)
    assert st == 1
    st = lib.jk_accept_path(1, 4, 100, 4, None, None, None, 0, 1.0, None, None, None, None, None, None, 0, None)
    assert st == 1


def test_draft_layer_workspace_queries_and_argument_checks_are_host_only(lib):
    n = lib.jk_draft_heads_workspace(80, 4096, 128256)
    assert n > 0 and n % 256 == 0
    assert lib.jk_draft_heads_workspace(10, 4096, 128256) < n
    assert lib.jk_draft_heads_workspace(129, 4096, 128256) == 0      # too many rows
    assert lib.jk_draft_heads_workspace(10, 4000, 128256) == 0       # width not a multiple of 128
    assert lib.jk_draft_heads_workspace(10, 4096, 0) == 0
    d = binding.MoeDesc(10, 4096, 4096, 8)
    m = lib.jk_moe_experts_workspace(ctypes.byref(d))
    assert m > 0 and m % 256 == 0
    assert lib.jk_moe_experts_workspace(ctypes.byref(binding.MoeDesc(10, 4096, 4096, 1))) == 0   # no top-2 of one
    assert lib.jk_moe_experts_workspace(ctypes.byref(binding.MoeDesc(10, 4096, 1000, 8))) == 0
    assert lib.jk_moe_experts_workspace(None) == 0
    assert lib.jk_linear_workspace(10, 4096, 4096) > 0
    assert lib.jk_linear_workspace(300, 4096, 4096) == 0 and lib.jk_linear_workspace(10, 4096, 100) == 0
    # null pointers and bad shapes are rejected before any launch
    hd = binding.DraftHeadsDesc(10, 4096, 1000, 5, 0, 1.0, 0.0, 0.0)
    assert lib.jk_draft_heads(ctypes.byref(hd), None, None, None, None, None, None, None, None, 0, None) == 1
    assert lib.jk_moe_experts(ctypes.byref(d), None, None, None, None, None, None, None, None, None, None, 0, None) == 1
    assert lib.jk_linear(4, 8, 256, None, None, None, None, None, None, 0, None) == 1
    st = binding.TreeStateDesc(None, None, None, None, None, 64)
    assert lib.jk_tree_grow(ctypes.byref(st), 1, 1, 4, 4, 0, None, None, None, None, None) == 1
    assert lib.jk_tree_grow_tail(ctypes.byref(st), 1, 1, 4, 2, 2, 4, 0, None, None, None, None) == 1
    assert lib.jk_tree_finalize(ctypes.byref(st), 1, 8, None, None, None, None, None, None) == 1
    assert lib.jk_gather_draft_probs(1, 4, 100, None, 10, None, None, None) == 1


def test_static_fill_argument_checks_are_host_only(lib):
    st = binding.TreeStateDesc(None, None, None, None, None, 64)
    assert lib.jk_tree_fill_static(ctypes.byref(st), 1, 1, 4, 0, None, None, None, None, None, None, 4, None, 0, None,
                                   None, None) == 1


def test_attention_plans_of_the_workloads_are_host_only_and_stable(lib):
    """jk_tree_verify_attention_plan needs no device.  Without jk_init's placement check the merge inside the kernel is
    off, everything else is the plan the benchmarks run: this pins the planner's choices for the workload shapes (wave
    arrangement, tile pairing, row tiles, key splits), found by forced sweeps on an MI355X, against later edits of
    its cost table."""
    from workloads import CONFIGS
    want = {"c2_vicuna7b": (2, 2, 1, 1, 6), "c3_llama3_8b": (4, 1, 2, 2, 16), "c4_llama2_13b": (2, 2, 1, 1, 3),
            "c5_llama2_70b": (4, 1, 2, 7, 4), "c6_chain_sps": (2, 2, 1, 1, 1), "c7_static_tree": (2, 2, 1, 1, 4)}
    assert lib.jk_set_tuning(b"attn_fused", 0) == 0   # (as on a device whose placement has not been checked)
    try:
        _check_plans(lib, want, CONFIGS)
    finally:
        lib.jk_set_tuning(b"attn_fused", -1)


def _check_plans(lib, want, CONFIGS):
    for name, plan in want.items():
        c = CONFIGS[name]
        B, T, Hq, Hkv, D, L = c.batch, c.n_tree, c.n_q_heads, c.n_kv_heads, c.head_dim, c.prefix_len
        d = binding.AttnDesc(B, T, Hq, Hkv, D, T * Hq * D, Hq * D, D, L * Hkv * D, Hkv * D, D, T * Hkv * D, Hkv * D, D,
                             T * Hq * D, Hq * D, D, 0.0, 0)
        out = (ctypes.c_int32 * 6)()
        assert lib.jk_tree_verify_attention_plan(ctypes.byref(d), L, out) == 0
        assert tuple(out)[:5] == plan and out[5] == 0, (name, list(out))
        # the workspace query covers the plan with and without the merge inside the kernel
        rows = B * Hkv * plan[4] * plan[3] * 32 * plan[0]
        assert lib.jk_tree_verify_attention_workspace(ctypes.byref(d), L) >= rows * (D * 2 + 8) * (plan[4] > 1)


def _desc(B, T, Hq, Hkv, D, L, dtype=0):
    return binding.AttnDesc(B, T, Hq, Hkv, D, T * Hq * D, Hq * D, D, max(L, 1) * Hkv * D, Hkv * D, D, T * Hkv * D, Hkv * D, D,
                            T * Hq * D, Hq * D, D, 0.0, dtype)


def test_attention_plans_of_random_shapes_keep_their_invariants(lib):
    """Host-only: whatever the shape, a plan is one of the two wave arrangements with the row tiles that cover the
    T * G query rows, a split count within the library's limits (at most 64, at most 1024 tiles per split), and the
    workspace query covers its partials; forced arrangements and split counts are honoured; the fp32 path splits
    every 1024 keys.  Nothing here launches."""
    import random
    rng = random.Random(5)
    header = 32768
    try:
        for case in range(400):
            D = rng.choice([64, 128])
            Hkv = rng.choice([1, 2, 4, 8, 32, 40])
            G = rng.choice([1, 1, 2, 4, 8])
            B = rng.choice([1, 1, 2, 4, 8, 16, 64])
            T = rng.randint(1, 128)
            L = rng.choice([0, 1, 31, 32, 33, rng.randint(0, 5000), rng.randint(0, 200000), 1 << 20])
            force_arr = rng.choice([None, None, (4, 1), (2, 2)])
            force_s = rng.choice([0, 0, 0, 1, 2, 7, 16, 64])
            lib.jk_set_tuning(b"attn_fused", 0)
            lib.jk_set_tuning(b"attn_wm", force_arr[0] if force_arr else 0)
            lib.jk_set_tuning(b"attn_wn", force_arr[1] if force_arr else 0)
            lib.jk_set_tuning(b"attn_splits", force_s)
            d = _desc(B, T, Hkv * G, Hkv, D, L)
            out = (ctypes.c_int32 * 6)()
            what = (case, B, T, Hkv, G, D, L, force_arr, force_s)
            assert lib.jk_tree_verify_attention_plan(ctypes.byref(d), L, out) == 0, what
            wm, wn, kt, tiles, splits, fused = tuple(out)
            assert (wm, wn, kt) in ((4, 1, 2), (2, 2, 1)), what
            if force_arr:
                assert (wm, wn) == force_arr, what
            M = T * G
            assert tiles == (M + 32 * wm - 1) // (32 * wm), what
            n_tiles = (L + 31) // 32 + (T + 31) // 32
            s_min = (n_tiles + 1023) // 1024
            assert max(1, s_min) <= splits <= 64, what
            if force_s:
                assert splits == max(force_s, s_min), what
            else:
                assert splits <= max(1, s_min, n_tiles // (2 * wn * kt)), what   # at least two rounds per split
            assert fused == 0, what
            need = header + (B * Hkv * splits * tiles * 32 * wm * (D * 2 + 8) if splits > 1 else 0)
            assert lib.jk_tree_verify_attention_workspace(ctypes.byref(d), L) >= need, what
        for k in (b"attn_wm", b"attn_wn", b"attn_splits"):
            lib.jk_set_tuning(k, 0)
        # fp32 path: one workgroup per query row and 1024-key split; 64 splits at most
        for L, T in ((0, 1), (1000, 24), (1024, 1), (5000, 60), (65536 - 60, 60)):
            d = _desc(2, T, 8, 4, 64, L, dtype=1)
            out = (ctypes.c_int32 * 6)()
            assert lib.jk_tree_verify_attention_plan(ctypes.byref(d), L, out) == 0
            assert tuple(out) == (1, 1, 1, T * 2, (L + T + 1023) // 1024, 0)
        d = _desc(2, 60, 8, 4, 64, 65536, dtype=1)
        assert lib.jk_tree_verify_attention_plan(ctypes.byref(d), 65536, (ctypes.c_int32 * 6)()) != 0
        assert lib.jk_tree_verify_attention_workspace(ctypes.byref(d), 65536) == 0
        # bounds of the prefix length
        d = _desc(1, 8, 8, 8, 128, 64)
        assert lib.jk_tree_verify_attention_plan(ctypes.byref(d), -1, (ctypes.c_int32 * 6)()) != 0
        assert lib.jk_tree_verify_attention_plan(ctypes.byref(d), (1 << 24) + 1, (ctypes.c_int32 * 6)()) != 0
    finally:
        for k, v in ((b"attn_wm", 0), (b"attn_wn", 0), (b"attn_splits", 0), (b"attn_fused", -1)):
            lib.jk_set_tuning(k, v)
