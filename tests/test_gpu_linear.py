"""GPU parity: jk_linear (through the C ABI) against x w^T (+ residual), and Eq. 1 assembled from library
calls (projections -> tree attention over the draft layer's cache -> output projection + residual)
against the oracle's draft_attention_block."""
import numpy as np
import pytest
import torch

import paper_2502_06282_amd as jk
from oracle import draft_head as dh
from workloads import round_to_bf16

pytestmark = pytest.mark.gpu


def _bf(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(torch.bfloat16)


@pytest.mark.parametrize("m,n,k", [(1, 128, 128), (7, 300, 256), (33, 1000, 384), (80, 4096, 1024), (256, 513, 128),
                                   (10, 768, 4096)])
def test_exact_arithmetic_inputs_are_bit_exact(m, n, k):
    rng = np.random.default_rng(m + n)
    x = rng.integers(-2, 3, size=(m, k)).astype(np.float32)
    w = (rng.integers(-1, 2, size=(n, k)) * 0.125).astype(np.float32)
    r = rng.integers(-4, 5, size=(m, n)).astype(np.float32)
    got = jk.linear(_bf(x), _bf(w), out_dtype=torch.float32).cpu().numpy()
    np.testing.assert_array_equal(got.astype(np.float64), dh.linear(x, w))
    got = jk.linear(_bf(x), _bf(w), _bf(r), out_dtype=torch.float32).cpu().numpy()
    np.testing.assert_array_equal(got.astype(np.float64), dh.linear(x, w, r))
    got = jk.linear(_bf(x), _bf(w), _bf(r)).float().cpu().numpy()          # bf16 output: one rounding
    np.testing.assert_array_equal(got, round_to_bf16(dh.linear(x, w, r).astype(np.float32)))


def test_random_inputs_within_fp32_accumulation_error():
    rng = np.random.default_rng(1)
    m, n, k = 40, 2000, 2048
    x = round_to_bf16(rng.standard_normal((m, k), dtype=np.float32))
    w = round_to_bf16(rng.standard_normal((n, k), dtype=np.float32) / np.float32(np.sqrt(k)))
    got = jk.linear(_bf(x), _bf(w), out_dtype=torch.float32).cpu().numpy()
    ref = dh.linear(x, w)
    bound = k * 2.0 ** -23 * (np.abs(x).astype(np.float64) @ np.abs(w).astype(np.float64).T)
    assert (np.abs(got - ref) <= bound).all()


def test_eq1_block_from_library_calls():
    rng = np.random.default_rng(2)
    T, L, H, Hkv, D = 12, 300, 4, 2, 64
    d = H * D
    parent = np.array([-1, 0, 0, 1, 1, 2, 3, 3, 5, 6, 8, 8], dtype=np.int32)
    sc = np.float32(1.0 / np.sqrt(d))
    h = round_to_bf16(rng.standard_normal((T, d), dtype=np.float32))
    wq, wo = (round_to_bf16(rng.standard_normal((d, d), dtype=np.float32) * sc) for _ in range(2))
    wk, wv = (round_to_bf16(rng.standard_normal((Hkv * D, d), dtype=np.float32) * sc) for _ in range(2))
    kc, vc = (round_to_bf16(rng.standard_normal((L, Hkv, D), dtype=np.float32)) for _ in range(2))
    ref = dh.draft_attention_block(h, wq, wk, wv, wo, kc, vc, parent, H, Hkv)
    hd = _bf(h)
    q = jk.linear(hd, _bf(wq)).reshape(1, T, H, D)
    kt = jk.linear(hd, _bf(wk)).reshape(1, T, Hkv, D)
    vt = jk.linear(hd, _bf(wv)).reshape(1, T, Hkv, D)
    attn = jk.tree_verify_attention(q, _bf(kc)[None], _bf(vc)[None], kt, vt, torch.from_numpy(parent)[None].cuda(),
                                    torch.tensor([L], dtype=torch.int32).cuda())
    u = jk.linear(attn.reshape(T, d), _bf(wo), hd, out_dtype=torch.float32)
    torch.cuda.synchronize()
    err = np.abs(u.cpu().numpy() - ref).max()
    assert err <= 2e-2 * np.abs(ref).max(), err


def test_argument_errors():
    x = torch.zeros((4, 256), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((8, 256), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(jk.JakiroError) as e:
        jk.linear(x[:, :192].contiguous(), w[:, :192].contiguous())
    assert e.value.status == 3
    with pytest.raises(jk.JakiroError) as e:
        jk.linear(torch.zeros((257, 256), dtype=torch.bfloat16, device="cuda"), w)
    assert e.value.status == 3
    torch.cuda.synchronize()
