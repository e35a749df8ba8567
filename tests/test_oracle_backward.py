"""Pins for the oracle's backward pass: finite differences, autograd of a library
formulation, and structural invariants (CPU only)."""
import math

import pytest
import torch

from oracle import flex_oracle as fo

F64 = torch.float64


def rand(*shape, seed=0):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(*shape, generator=g, dtype=F64)


def loss(Q, K, V, dO, score_mod, mask_mod, scale):
    O, _ = fo.flex_attention(Q, K, V, score_mod, mask_mod, scale)
    return float((O * dO).sum())


def central_difference(Q, K, V, dO, score_mod, mask_mod, scale, eps=1e-5):
    grads = []
    for which in range(3):
        tensors = [Q.clone(), K.clone(), V.clone()]
        g = torch.zeros_like(tensors[which])
        flat, gf = tensors[which].view(-1), g.view(-1)
        for i in range(flat.numel()):
            old = float(flat[i])
            flat[i] = old + eps
            up = loss(*tensors, dO, score_mod, mask_mod, scale)
            flat[i] = old - eps
            dn = loss(*tensors, dO, score_mod, mask_mod, scale)
            flat[i] = old
            gf[i] = (up - dn) / (2 * eps)
        grads.append(g)
    return grads


def _mods():
    doc = torch.tensor([[0, 0, 0, 0, 1, 1, 1, 1, 1, 1]], dtype=torch.int32)
    return {
        "causal_identity": (fo.Identity(), fo.causal_mask),
        "causal_softcap": (fo.Softcap(1.5), fo.causal_mask),
        "doc_causal_alibi": (fo.Alibi(torch.tensor([-0.3, -0.6, -0.9, -1.2], dtype=F64)),
                             fo.and_mask(fo.document_mask(doc), fo.causal_mask)),
        "swa_prefix_relbias": (fo.RelBias(rand(4, 5, seed=11)),
                               fo.or_mask(fo.and_mask(fo.causal_mask, fo.sliding_window_mask(3)), fo.prefix_mask(2))),
        "alibi_then_softcap": (fo.Compose(fo.Alibi(torch.tensor([-0.3, -0.6, -0.9, -1.2], dtype=F64)), fo.Softcap(2.0)),
                               fo.causal_mask),
    }


@pytest.mark.parametrize("name", list(_mods()))
def test_backward_matches_central_differences(name):
    score_mod, mask_mod = _mods()[name]
    # GQA (4 query heads on 2 KV heads) so the group sum of dK/dV is exercised too.
    Q, K, V, dO = rand(1, 4, 10, 4, seed=1), rand(1, 2, 10, 4, seed=2), rand(1, 2, 10, 4, seed=3), rand(1, 4, 10, 4, seed=4)
    scale = 0.6
    dQ, dK, dV = fo.flex_attention_backward(Q, K, V, dO, score_mod, mask_mod, scale)
    fQ, fK, fV = central_difference(Q, K, V, dO, score_mod, mask_mod, scale)
    for got, ref in ((dQ, fQ), (dK, fK), (dV, fV)):
        assert (got - ref).abs().max() <= 1e-8 * max(1.0, float(ref.abs().max()))


def test_backward_matches_autograd_of_library_sdpa():
    Q, K, V, dO = rand(2, 2, 17, 8, seed=1), rand(2, 2, 17, 8, seed=2), rand(2, 2, 17, 8, seed=3), rand(2, 2, 17, 8, seed=4)
    Qa, Ka, Va = (t.clone().requires_grad_(True) for t in (Q, K, V))
    out = torch.nn.functional.scaled_dot_product_attention(Qa, Ka, Va, is_causal=True)
    out.backward(dO)
    dQ, dK, dV = fo.flex_attention_backward(Q, K, V, dO, fo.Identity(), fo.causal_mask)
    assert torch.allclose(dQ, Qa.grad, atol=1e-12, rtol=0)
    assert torch.allclose(dK, Ka.grad, atol=1e-12, rtol=0)
    assert torch.allclose(dV, Va.grad, atol=1e-12, rtol=0)


def test_backward_softcap_matches_autograd_of_explicit_graph():
    # An independent statement of the same function with autograd doing the calculus.
    Q, K, V, dO = rand(1, 2, 12, 4, seed=1), rand(1, 1, 12, 4, seed=2), rand(1, 1, 12, 4, seed=3), rand(1, 2, 12, 4, seed=4)
    Qa, Ka, Va = (t.clone().requires_grad_(True) for t in (Q, K, V))
    s = (Qa @ Ka.transpose(-1, -2)) * 0.4
    s = 3.0 * torch.tanh(s / 3.0)
    keep = torch.tril(torch.ones(12, 12, dtype=torch.bool))
    p = torch.softmax(s.masked_fill(~keep, float("-inf")), dim=-1)
    (p @ Va).backward(dO)
    dQ, dK, dV = fo.flex_attention_backward(Q, K, V, dO, fo.Softcap(3.0), fo.causal_mask, 0.4)
    assert torch.allclose(dQ, Qa.grad, atol=1e-12, rtol=0)
    assert torch.allclose(dK, Ka.grad, atol=1e-12, rtol=0)
    assert torch.allclose(dV, Va.grad, atol=1e-12, rtol=0)


def test_gqa_gradients_are_group_sums():
    Q, K, V, dO = rand(1, 6, 9, 4, seed=1), rand(1, 2, 9, 4, seed=2), rand(1, 2, 9, 4, seed=3), rand(1, 6, 9, 4, seed=4)
    dQ, dK, dV = fo.flex_attention_backward(Q, K, V, dO, fo.Softcap(2.0), fo.causal_mask)
    Kr, Vr = K.repeat_interleave(3, dim=1), V.repeat_interleave(3, dim=1)
    dQm, dKm, dVm = fo.flex_attention_backward(Q, Kr, Vr, dO, fo.Softcap(2.0), fo.causal_mask)
    assert torch.allclose(dQ, dQm, atol=1e-14, rtol=0)
    assert torch.allclose(dK, dKm.view(1, 2, 3, 9, 4).sum(2), atol=1e-13, rtol=0)
    assert torch.allclose(dV, dVm.view(1, 2, 3, 9, 4).sum(2), atol=1e-13, rtol=0)


def test_shift_invariance_and_value_gradient_structure():
    # Softmax ignores a per-row constant, so d loss / d (row shift) = sum_kv dS' = 0.  With identity
    # score_mod and K = all-ones, dQ = scale * rowsum(dS) * 1 must vanish.
    Q, V, dO = rand(1, 1, 8, 4, seed=1), rand(1, 1, 8, 4, seed=3), rand(1, 1, 8, 4, seed=4)
    K = torch.ones(1, 1, 8, 4, dtype=F64)
    dQ, _, dV = fo.flex_attention_backward(Q, K, V, dO, fo.Identity(), fo.causal_mask)
    assert dQ.abs().max() < 1e-14
    # with K constant every row's P is uniform over its visible keys: dV[kv] = sum_{q>=kv} dO[q]/(q+1)
    ref = torch.zeros(8, 4, dtype=F64)
    for kv in range(8):
        for q in range(kv, 8):
            ref[kv] += dO[0, 0, q] / (q + 1)
    assert torch.allclose(dV[0, 0], ref, atol=1e-14, rtol=0)


def test_masked_keys_get_no_gradient():
    Q, K, V, dO = rand(1, 1, 8, 4, seed=1), rand(1, 1, 8, 4, seed=2), rand(1, 1, 8, 4, seed=3), rand(1, 1, 8, 4, seed=4)
    # only keys 0..2 are visible (prefix, no causal part): keys 3.. must get exactly zero dK, dV
    dQ, dK, dV = fo.flex_attention_backward(Q, K, V, dO, fo.Softcap(2.0), fo.prefix_mask(3))
    assert (dK[0, 0, 3:] == 0).all() and (dV[0, 0, 3:] == 0).all()
    assert dK[0, 0, :3].abs().min() > 0 and dV[0, 0, :3].abs().min() > 0


def test_backward_row_subset_matches_full():
    Q, K, V, dO = rand(1, 1, 40, 8, seed=1), rand(1, 1, 40, 8, seed=2), rand(1, 1, 40, 8, seed=3), rand(1, 1, 40, 8, seed=4)
    args = (Q[0, 0], K[0, 0], V[0, 0], dO[0, 0], fo.Softcap(2.0), fo.causal_mask, 0.4, 0, 0)
    dQ, dK, dV = fo.attention_head_backward(*args)
    rows = torch.tensor([39, 3, 17])
    dq, dk, dv = fo.attention_head_backward(*args, q_rows=rows)
    assert torch.allclose(dq, dQ[rows], atol=1e-13, rtol=0)
    # the remaining rows supply the rest of dK / dV
    rest = torch.tensor([i for i in range(40) if i not in (39, 3, 17)])
    _, dk2, dv2 = fo.attention_head_backward(*args, q_rows=rest, stripe=9)
    assert torch.allclose(dk + dk2, dK, atol=1e-13, rtol=0) and torch.allclose(dv + dv2, dV, atol=1e-13, rtol=0)
    # keys 30.. are seen only by rows 30.. under the causal mask
    _, dk3, dv3 = fo.attention_head_backward(*args, q_rows=torch.arange(30, 40))
    assert torch.allclose(dk3[30:], dK[30:], atol=1e-13, rtol=0) and torch.allclose(dv3[30:], dV[30:], atol=1e-13, rtol=0)
