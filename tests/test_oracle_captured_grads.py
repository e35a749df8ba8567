"""Pins for the oracle's gradients of captured tensors (ALiBi bias, relative-bias table): central finite
differences of L = sum(O * dO) in the captured values, and autograd through a plain dense
implementation written with library ops."""
import math

import torch

from oracle import flex_oracle as fo


def setup(seed=5, B=2, Hq=4, Hkv=2, S=24, D=8, rel_len=6):
    g = torch.Generator().manual_seed(seed)
    r = lambda *s: torch.randn(*s, generator=g, dtype=torch.float64)
    return r(B, Hq, S, D), r(B, Hkv, S, D), r(B, Hkv, S, D), r(B, Hq, S, D), 0.3 * r(Hq), 0.5 * r(Hq, rel_len)


def loss(Q, K, V, dO, score_mod, mask_mod, scale):
    O, _ = fo.flex_attention(Q, K, V, score_mod, mask_mod, scale)
    return float((O * dO).sum())


def test_alibi_and_rel_bias_gradients_match_finite_differences():
    Q, K, V, dO, bias, table = setup()
    scale = 1.0 / math.sqrt(8)
    mask = fo.and_mask(fo.causal_mask, fo.sliding_window_mask(13))
    for cap in (None, 2.5):
        def mods(bias_v, table_v):
            sm = fo.Compose(fo.Alibi(bias_v), fo.RelBias(table_v))
            return sm if cap is None else fo.Compose(sm, fo.Softcap(cap))
        got = fo.flex_attention_backward_captured(Q, K, V, dO, mods(bias, table), mask, scale)
        eps = 1e-6
        for h in range(4):
            e = torch.zeros_like(bias)
            e[h] = eps
            fd = (loss(Q, K, V, dO, mods(bias + e, table), mask, scale)
                  - loss(Q, K, V, dO, mods(bias - e, table), mask, scale)) / (2 * eps)
            assert abs(fd - float(got["alibi_bias"][h])) < 1e-6 * max(1.0, abs(fd))
            for r in range(6):
                e = torch.zeros_like(table)
                e[h, r] = eps
                fd = (loss(Q, K, V, dO, mods(bias, table + e), mask, scale)
                      - loss(Q, K, V, dO, mods(bias, table - e), mask, scale)) / (2 * eps)
                assert abs(fd - float(got["rel_bias"][h, r])) < 1e-6 * max(1.0, abs(fd))


def test_gradients_match_autograd_through_dense_library_ops():
    Q, K, V, dO, bias, table = setup(seed=9, S=20)
    scale, S, G = 0.4, 20, 2
    bias_t, table_t = bias.clone().requires_grad_(True), table.clone().requires_grad_(True)
    q, kv = torch.arange(S).view(-1, 1), torch.arange(S).view(1, -1)
    rel = (q - kv).clamp(0, 5)
    s = torch.einsum("bhqd,bhkd->bhqk", Q, K.repeat_interleave(G, dim=1)) * scale
    s = s + bias_t.view(1, -1, 1, 1) * (q - kv).to(torch.float64) + table_t[:, rel].unsqueeze(0)
    s = s.masked_fill(kv > q, float("-inf"))
    O = torch.softmax(s, dim=-1) @ V.repeat_interleave(G, dim=1)
    (O * dO).sum().backward()
    got = fo.flex_attention_backward_captured(Q, K, V, dO, fo.Compose(fo.Alibi(bias), fo.RelBias(table)),
                                              fo.causal_mask, scale)
    assert torch.allclose(got["alibi_bias"], bias_t.grad, atol=1e-11, rtol=0)
    assert torch.allclose(got["rel_bias"], table_t.grad, atol=1e-11, rtol=0)


def test_mods_without_captured_tensors_give_nothing_and_masked_rows_add_nothing():
    Q, K, V, dO, bias, table = setup(S=16)
    assert fo.flex_attention_backward_captured(Q, K, V, dO, fo.Softcap(3.0), fo.causal_mask, 0.3) == {}
    # a mask that hides every key of some rows: those rows contribute exactly zero
    hide = lambda b, h, q_idx, kv_idx: (q_idx >= 8) & (kv_idx <= q_idx)
    got = fo.flex_attention_backward_captured(Q, K, V, dO, fo.Alibi(bias), hide, 0.3)
    assert torch.isfinite(got["alibi_bias"]).all()
    part = fo.flex_attention_backward_captured(Q[:, :, 8:], K, V, dO[:, :, 8:], fo.QOffset(fo.Alibi(bias), torch.tensor([8, 8])),
                                               fo.with_q_offset(fo.causal_mask, torch.tensor([8, 8])), 0.3)
    assert torch.allclose(got["alibi_bias"], part["alibi_bias"], atol=1e-12, rtol=0)
