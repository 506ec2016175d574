"""Pins for the paged-cache oracle: facts about the addressing that do not restate its two loops."""
import numpy as np

from oracle import gather_pages, scatter_rows, tree_verify_attention
from workloads import CONFIGS, attention_inputs, paged_layout, tree_for_config


def _case(page_size=32, L=150, seed=4):
    cfg = CONFIGS["c1_tiny"].with_(batch=2, prefix_len=L, n_q_heads=4, n_kv_heads=2, head_dim=16)
    par = tree_for_config(cfg, seed=seed)
    x = attention_inputs(cfg, seed=seed)
    pools, table = paged_layout(x["k_cache"], x["v_cache"], page_size, seed=seed)
    return cfg, par, x, pools, table


def test_layout_is_a_permutation_of_the_contiguous_cache():
    cfg, par, x, (kp, vp), table = _case()
    L = cfg.prefix_len
    # every page id is used at most once, and reading back in table order gives the cache
    used = table[:, : (L + 31) // 32].ravel()
    assert len(set(used.tolist())) == len(used)
    np.testing.assert_array_equal(gather_pages(kp, table, 32, L), x["k_cache"])
    np.testing.assert_array_equal(gather_pages(vp, table, 32, L), x["v_cache"])
    # slots the sequences do not own (tail of the last page, spare pages) are NaN: nothing else is stored
    assert np.isfinite(kp).sum() == x["k_cache"].size and np.isfinite(vp).sum() == x["v_cache"].size


def test_identity_table_is_a_reshape():
    cfg, par, x, _, _ = _case(L=128)
    B, L = 2, 128
    pool = x["k_cache"].reshape(B * 4, 32, 2, 16)            # 4 pages per sequence, in order
    table = np.arange(B * 4, dtype=np.int32).reshape(B, 4)
    np.testing.assert_array_equal(gather_pages(pool, table, 32, L), x["k_cache"])


def test_attention_is_invariant_under_relocating_pages():
    """Moving pages around physically (pool and table permuted together) cannot change attention."""
    cfg, par, x, (kp, vp), table = _case(page_size=64, L=150)
    L = cfg.prefix_len
    ref = tree_verify_attention(**x, parent=par, prefix_len=[L, L - 40])
    rng = np.random.default_rng(0)
    perm = rng.permutation(kp.shape[0])                      # new_id = perm[old_id]
    kp2, vp2 = np.empty_like(kp), np.empty_like(vp)
    kp2[perm], vp2[perm] = kp, vp
    table2 = perm[table].astype(np.int32)
    y = dict(x, k_cache=gather_pages(kp2, table2, 64, L), v_cache=gather_pages(vp2, table2, 64, L))
    got = tree_verify_attention(**y, parent=par, prefix_len=[L, L - 40])
    np.testing.assert_array_equal(got, ref)


def test_scatter_then_gather_round_trip_and_isolation():
    cfg, par, x, (kp, vp), table = _case(page_size=32, L=150)
    before = kp.copy()
    rows = np.full((3, 2, 16), 7.0)
    scatter_rows(kp, table, 32, 1, [30, 31, 32], rows)       # crosses a page boundary
    back = gather_pages(kp, table, 32, 150)
    np.testing.assert_array_equal(back[1, 30:33], rows)
    np.testing.assert_array_equal(back[0], gather_pages(before, table, 32, 150)[0])   # other sequence untouched
    changed = ~((kp == before) | (np.isnan(kp) & np.isnan(before)))
    assert changed.sum() == rows.size                                                  # exactly three rows were written
