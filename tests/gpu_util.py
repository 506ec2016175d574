"""Helpers shared by the GPU parity tests: move generated inputs to the device,
call the C-ABI through the binding, fetch results."""
import numpy as np
import torch

import paper_2502_06282_amd as jk
from oracle import tree_verify_attention as oracle_attention


_KNOBS = {"attn_wm": 0, "attn_wn": 0, "attn_splits": 0, "attn_fused": -1, "attn_deep": -1, "accept_single": 0, "spin_limit": -1}


def tune(name, value):
    """Force part of a launch plan (jk_set_tuning); the autouse fixture in conftest.py undoes it after the test."""
    jk.set_tuning(name, int(value))


def reset_tuning():
    for k, v in _KNOBS.items():
        jk.set_tuning(k, v)


def to_dev(x, dtype):
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    return {k: torch.from_numpy(np.ascontiguousarray(v)).cuda().to(tdt) for k, v in x.items()}


def gpu_attention(x, parent, prefix_len, dtype, scale=0.0, max_prefix_len=None):
    dv = to_dev(x, dtype)
    par = torch.from_numpy(np.ascontiguousarray(parent, dtype=np.int32)).cuda()
    pl = torch.tensor(list(prefix_len), dtype=torch.int32).cuda()
    out = jk.tree_verify_attention(dv["q"], dv["k_cache"], dv["v_cache"], dv["k_tree"], dv["v_tree"], par, pl,
                                   max_prefix_len=max_prefix_len, scale=scale)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64)


def check_attention(x, parent, prefix_len, dtype, tol, scale=None, rel_tol=None):
    ref = oracle_attention(**x, parent=parent, prefix_len=prefix_len, scale=scale)
    got = gpu_attention(x, parent, prefix_len, dtype, scale=0.0 if scale is None else scale)
    assert np.isfinite(got).all()
    err = np.abs(got - ref).max()
    assert err <= tol, f"max-abs error {err:.3e} > {tol}"
    if rel_tol is not None:
        nerr = err / np.abs(ref).max()
        assert nerr <= rel_tol, f"normalised error {nerr:.3e} > {rel_tol}"
    return got, ref
