"""GPU test of jk_accept_path_greedy_static, the entry point that takes no workspace and allocates nothing
(the greedy walk's partials live in a buffer inside the library's device image).  Its results must be those of
jk_accept_path in greedy mode, bit for bit, on two calls in a row that share the built-in buffer, the second
one smaller than the first (stale partials of the larger call stay behind it in the buffer)."""
import numpy as np
import pytest
import torch

import paper_2502_06282_amd as jk
from oracle import accept_path as oracle_accept
from workloads import CONFIGS, accept_inputs, tree_for_config

pytestmark = pytest.mark.gpu


def _inputs(cfg, seed):
    par = tree_for_config(cfg, seed=seed)
    a = accept_inputs(cfg, par, seed=seed)
    dev = torch.device("cuda")
    t = lambda v: torch.from_numpy(np.ascontiguousarray(v)).to(dev)
    return par, a, t(a["tokens"]), t(par.astype(np.int32)), t(a["logits"])


def test_static_scratch_greedy_equals_workspace_call_twice_in_a_row():
    big = CONFIGS["c4_llama2_13b"].with_(hit_prob=0.8)                 # 4 trees x 61 rows x 32 000 entries
    small = CONFIGS["c2_vicuna7b"].with_(vocab=5003, n_tree=23, hit_prob=0.8)  # 1 tree, ragged vocabulary
    for cfg, seed in ((big, 3), (small, 4)):
        par, a, tokens, parent, logits = _inputs(cfg, seed)
        B, depth = par.shape[0], cfg.depth
        ref_path, ref_len, ref_bonus = jk.accept_path(tokens, parent, logits, jk.JK_GREEDY, max_depth=depth)
        path = torch.full((B, depth), -7, dtype=torch.int32, device="cuda")
        alen = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        bonus = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        jk.accept_path_greedy_static(tokens, parent, logits, path, alen, bonus)
        torch.cuda.synchronize()
        assert torch.equal(path, ref_path) and torch.equal(alen, ref_len) and torch.equal(bonus, ref_bonus)
        for b in range(B):  # and both equal the oracle's walk
            r = oracle_accept(a["tokens"][b], par[b], a["logits"][b], "greedy", max_depth=depth)
            assert path[b, : int(alen[b])].cpu().tolist() == r.path and int(bonus[b]) == r.bonus_token
        assert int(alen.max()) >= 1


def test_static_scratch_rejects_inputs_beyond_its_limit():
    # 60 000 rows x 3 chunks x 8 bytes > 1 MiB: refused on the host, nothing launched, outputs untouched
    B, N, V = 2000, 29, 9000
    z = torch.zeros(1, dtype=torch.int32, device="cuda")
    fn = jk.lib().jk_accept_path_greedy_static
    import ctypes
    vp, i32 = ctypes.c_void_p, ctypes.c_int32
    fn.restype, fn.argtypes = i32, [i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    st = fn(B, N, V, 4, z.data_ptr(), z.data_ptr(), torch.zeros(4, device="cuda").data_ptr(), z.data_ptr(), z.data_ptr(),
            z.data_ptr(), None)
    assert st == 6 and b"scratch" in jk.lib().jk_status_string(st)
