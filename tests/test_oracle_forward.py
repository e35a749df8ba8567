"""Pins for the fp64 oracle's forward pass, masks and score mods (CPU only).

Each test checks the oracle against something other than itself: a scalar
pure-Python evaluation of Eq. 1, a library routine, a closed form, or an
invariant that a dropped term / wrong sign / transposed operand would break.
"""
import math

import pytest
import torch

from oracle import flex_oracle as fo

F64 = torch.float64


def rand(*shape, seed=0):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(*shape, generator=g, dtype=F64)


# ---- scalar re-statement of Eq. 1 with Python floats (tiny sizes only) ----
def scalar_flex(Q, K, V, score_fn, mask_fn, scale):
    B, Hq, Sq, D = Q.shape
    Hkv, Skv = K.shape[1], K.shape[2]
    G = Hq // Hkv
    O = torch.zeros(B, Hq, Sq, D, dtype=F64)
    LSE = torch.zeros(B, Hq, Sq, dtype=F64)
    for b in range(B):
        for h in range(Hq):
            for q in range(Sq):
                vals = []
                for kv in range(Skv):
                    s = sum(float(Q[b, h, q, d]) * float(K[b, h // G, kv, d]) for d in range(D)) * scale
                    s = score_fn(s, b, h, q, kv)
                    vals.append(s if mask_fn(b, h, q, kv) else None)
                live = [v for v in vals if v is not None]
                if not live:
                    LSE[b, h, q] = float("-inf")
                    continue
                m = max(live)
                den = math.fsum(math.exp(v - m) for v in live)
                LSE[b, h, q] = m + math.log(den)
                for d in range(D):
                    O[b, h, q, d] = math.fsum(math.exp(v - m) / den * float(V[b, h // G, kv, d])
                                              for kv, v in enumerate(vals) if v is not None)
    return O, LSE


CASES = {
    "causal_identity": (fo.Identity(), fo.causal_mask,
                        lambda s, b, h, q, kv: s, lambda b, h, q, kv: q >= kv),
    "swa_softcap": (fo.Softcap(2.5), fo.and_mask(fo.causal_mask, fo.sliding_window_mask(3)),
                    lambda s, b, h, q, kv: 2.5 * math.tanh(s / 2.5),
                    lambda b, h, q, kv: q >= kv and q - kv <= 3),
    "prefix_alibi": (fo.Alibi(torch.tensor([-0.5, -0.25, -0.125, -0.0625])),
                     fo.or_mask(fo.prefix_mask(4), fo.causal_mask),
                     lambda s, b, h, q, kv: s + [-0.5, -0.25, -0.125, -0.0625][h] * (q - kv),
                     lambda b, h, q, kv: kv < 4 or q >= kv),
}


@pytest.mark.parametrize("name", list(CASES))
def test_matches_scalar_definition(name):
    score_mod, mask_mod, score_fn, mask_fn = CASES[name]
    Q, K, V = rand(2, 4, 11, 5, seed=1), rand(2, 2, 13, 5, seed=2), rand(2, 2, 13, 5, seed=3)
    scale = 0.37
    O, LSE = fo.flex_attention(Q, K, V, score_mod, mask_mod, scale)
    O_ref, LSE_ref = scalar_flex(Q, K, V, score_fn, mask_fn, scale)
    assert torch.allclose(O, O_ref, atol=1e-12, rtol=0)
    assert torch.allclose(LSE, LSE_ref, atol=1e-12, rtol=0)


def test_rel_bias_and_document_match_scalar_definition():
    table = rand(4, 6, seed=9)
    doc = torch.tensor([[0, 0, 0, 1, 1, 1, 1, 2, 2, 2, 2, 2], [0, 0, 1, 1, 1, 1, 1, 1, 2, 2, 3, 3]], dtype=torch.int32)
    Q, K, V = rand(2, 4, 12, 3, seed=4), rand(2, 1, 12, 3, seed=5), rand(2, 1, 12, 3, seed=6)
    O, LSE = fo.flex_attention(Q, K, V, fo.RelBias(table), fo.and_mask(fo.document_mask(doc), fo.causal_mask), 0.5)
    O_ref, LSE_ref = scalar_flex(
        Q, K, V, lambda s, b, h, q, kv: s + float(table[h, min(max(q - kv, 0), 5)]),
        lambda b, h, q, kv: int(doc[b, q]) == int(doc[b, kv]) and q >= kv, 0.5)
    assert torch.allclose(O, O_ref, atol=1e-12, rtol=0)
    assert torch.allclose(LSE, LSE_ref, atol=1e-12, rtol=0)


def test_noop_equals_library_sdpa():
    Q, K, V = rand(2, 3, 40, 16, seed=1), rand(2, 3, 50, 16, seed=2), rand(2, 3, 50, 16, seed=3)
    O, LSE = fo.flex_attention(Q, K, V, fo.Identity(), fo.no_mask)
    ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V)
    assert torch.allclose(O, ref, atol=1e-12, rtol=0)
    lse_ref = torch.logsumexp(Q @ K.transpose(-1, -2) / math.sqrt(16), dim=-1)
    assert torch.allclose(LSE, lse_ref, atol=1e-12, rtol=0)


def test_causal_equals_library_sdpa_causal():
    Q, K, V = rand(1, 2, 33, 8, seed=1), rand(1, 2, 33, 8, seed=2), rand(1, 2, 33, 8, seed=3)
    O, _ = fo.flex_attention(Q, K, V, fo.Identity(), fo.causal_mask)
    ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V, is_causal=True)
    assert torch.allclose(O, ref, atol=1e-12, rtol=0)


def test_rows_sum_to_one():
    # With V = 1 everywhere the output is the row sum of P.
    Q, K = rand(1, 2, 64, 8, seed=1), rand(1, 2, 64, 8, seed=2)
    V = torch.ones(1, 2, 64, 8, dtype=F64)
    for mask in (fo.no_mask, fo.causal_mask, fo.and_mask(fo.causal_mask, fo.sliding_window_mask(5))):
        O, _ = fo.flex_attention(Q, K, V, fo.Softcap(3.0), mask)
        assert (O - 1.0).abs().max() < 1e-12


def test_causal_row0_is_v0():
    Q, K, V = rand(2, 4, 32, 8, seed=1), rand(2, 2, 32, 8, seed=2), rand(2, 2, 32, 8, seed=3)
    O, LSE = fo.flex_attention(Q, K, V, fo.Identity(), fo.causal_mask, 0.25)
    for h in range(4):
        assert torch.equal(O[:, h, 0], V[:, h // 2, 0])
        s00 = (Q[:, h, 0] * K[:, h // 2, 0]).sum(-1) * 0.25
        assert torch.allclose(LSE[:, h, 0], s00, atol=1e-14, rtol=0)


def test_document_mask_equals_independent_documents():
    lengths = [7, 12, 5, 8]
    doc = torch.repeat_interleave(torch.arange(4, dtype=torch.int32), torch.tensor(lengths)).view(1, -1)
    S = sum(lengths)
    Q, K, V = rand(1, 2, S, 8, seed=1), rand(1, 2, S, 8, seed=2), rand(1, 2, S, 8, seed=3)
    O, LSE = fo.flex_attention(Q, K, V, fo.Identity(), fo.document_mask(doc))
    pos = 0
    for L in lengths:
        sl = slice(pos, pos + L)
        o, l = fo.flex_attention(Q[:, :, sl], K[:, :, sl], V[:, :, sl], fo.Identity(), fo.no_mask)
        assert torch.allclose(O[:, :, sl], o, atol=1e-13, rtol=0)
        assert torch.allclose(LSE[:, :, sl], l, atol=1e-13, rtol=0)
        pos += L


def test_document_causal_alibi_equals_per_document_causal_alibi():
    # ALiBi depends on q - kv only, so packing documents must not change the result.
    lengths = [9, 4, 11]
    doc = torch.repeat_interleave(torch.arange(3, dtype=torch.int32), torch.tensor(lengths)).view(1, -1)
    S = sum(lengths)
    bias = -torch.tensor([0.5, 0.1])
    Q, K, V = rand(1, 2, S, 8, seed=1), rand(1, 2, S, 8, seed=2), rand(1, 2, S, 8, seed=3)
    O, _ = fo.flex_attention(Q, K, V, fo.Alibi(bias), fo.and_mask(fo.document_mask(doc), fo.causal_mask))
    pos = 0
    for L in lengths:
        sl = slice(pos, pos + L)
        o, _ = fo.flex_attention(Q[:, :, sl], K[:, :, sl], V[:, :, sl], fo.Alibi(bias), fo.causal_mask)
        assert torch.allclose(O[:, :, sl], o, atol=1e-13, rtol=0)
        pos += L


def test_alibi_penalises_distance():
    # Equal raw scores (Q = 0): under causal + ALiBi with negative bias the weights must decay
    # geometrically with distance: p(kv) ~ exp(bias * (q - kv)).
    S, slope = 6, 0.7
    Q = torch.zeros(1, 1, S, 4, dtype=F64)
    K = rand(1, 1, S, 4, seed=2)
    V = torch.eye(S, dtype=F64).view(1, 1, S, S)        # O[q] = the probability row itself
    O, _ = fo.flex_attention(Q, K, V, fo.Alibi(torch.tensor([-slope], dtype=F64)), fo.causal_mask)
    q = S - 1
    w = torch.tensor([math.exp(-slope * (q - kv)) for kv in range(S)], dtype=F64)
    assert torch.allclose(O[0, 0, q], w / w.sum(), atol=1e-14, rtol=0)


def test_softcap_bounded_and_limit():
    Q, K, V = 8 * rand(1, 2, 24, 8, seed=1), 8 * rand(1, 2, 24, 8, seed=2), rand(1, 2, 24, 8, seed=3)
    s = Q @ K.transpose(-1, -2)
    capped = fo.Softcap(5.0)(s, 0, 0, None, None)
    assert capped.abs().max() <= 5.0 and s.abs().max() > 50.0
    # cap -> infinity is the identity
    O_big, L_big = fo.flex_attention(Q, K, V, fo.Softcap(1e9), fo.causal_mask)
    O_id, L_id = fo.flex_attention(Q, K, V, fo.Identity(), fo.causal_mask)
    assert torch.allclose(O_big, O_id, atol=1e-9, rtol=0)
    assert torch.allclose(L_big, L_id, atol=1e-9, rtol=0)
    # LSE of capped scores can never exceed cap + ln(n_keys)
    _, L = fo.flex_attention(Q, K, V, fo.Softcap(5.0), fo.no_mask)
    assert L.max() <= 5.0 + math.log(24) + 1e-12


def test_softcap_grad_matches_central_difference():
    x = torch.linspace(-40, 40, 401, dtype=F64)
    sc = fo.Softcap(7.0)
    eps = 1e-6
    fd = (sc(x + eps, 0, 0, None, None) - sc(x - eps, 0, 0, None, None)) / (2 * eps)
    assert torch.allclose(sc.grad(x, 0, 0, None, None), fd, atol=1e-8, rtol=0)


def test_sliding_window_special_cases():
    S = 20
    Q, K, V = rand(1, 1, S, 4, seed=1), rand(1, 1, S, 4, seed=2), rand(1, 1, S, 4, seed=3)
    swa = lambda w: fo.and_mask(fo.causal_mask, fo.sliding_window_mask(w))
    O_c, L_c = fo.flex_attention(Q, K, V, fo.Identity(), fo.causal_mask)
    O_w, L_w = fo.flex_attention(Q, K, V, fo.Identity(), swa(S))
    assert torch.equal(O_c, O_w) and torch.equal(L_c, L_w)
    O_0, _ = fo.flex_attention(Q, K, V, fo.Identity(), swa(0))       # each row sees only itself
    assert torch.equal(O_0, V)
    # window w holds w + 1 keys (inclusive bound): with V = one-hot, count the non-zeros
    E = torch.eye(S, dtype=F64).view(1, 1, S, S)
    O_3, _ = fo.flex_attention(Q, K, E, fo.Identity(), swa(3))
    assert int((O_3[0, 0, 10] > 0).sum()) == 4 and O_3[0, 0, 10, 7] > 0 and O_3[0, 0, 10, 6] == 0
    # the paper's one-sided window alone lets every future key through
    O_one, _ = fo.flex_attention(Q, K, E, fo.Identity(), fo.sliding_window_mask(3))
    assert int((O_one[0, 0, 10] > 0).sum()) == 4 + (S - 11)


def test_prefix_special_cases():
    S = 24
    Q, K, V = rand(1, 1, S, 4, seed=1), rand(1, 1, S, 4, seed=2), rand(1, 1, S, 4, seed=3)
    swa = fo.and_mask(fo.causal_mask, fo.sliding_window_mask(5))
    a = fo.flex_attention(Q, K, V, fo.Identity(), fo.or_mask(swa, fo.prefix_mask(0)))
    b = fo.flex_attention(Q, K, V, fo.Identity(), swa)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    c = fo.flex_attention(Q, K, V, fo.Identity(), fo.or_mask(swa, fo.prefix_mask(S)))
    d = fo.flex_attention(Q, K, V, fo.Identity(), fo.no_mask)
    assert torch.equal(c[0], d[0]) and torch.equal(c[1], d[1])
    # prefix-LM: rows inside the prefix see the whole prefix (bidirectional), nothing after it
    E = torch.eye(S, dtype=F64).view(1, 1, S, S)
    O, _ = fo.flex_attention(Q, K, E, fo.Identity(), fo.or_mask(fo.prefix_mask(6), fo.causal_mask))
    assert int((O[0, 0, 2] > 0).sum()) == 6 and int((O[0, 0, 9] > 0).sum()) == 10


def test_rel_bias_constant_table_is_a_shift():
    Q, K, V = rand(1, 2, 16, 4, seed=1), rand(1, 2, 16, 4, seed=2), rand(1, 2, 16, 4, seed=3)
    table = torch.full((2, 8), 0.75, dtype=F64)
    O_b, L_b = fo.flex_attention(Q, K, V, fo.RelBias(table), fo.causal_mask)
    O_i, L_i = fo.flex_attention(Q, K, V, fo.Identity(), fo.causal_mask)
    assert torch.allclose(O_b, O_i, atol=1e-14, rtol=0)
    assert torch.allclose(L_b, L_i + 0.75, atol=1e-14, rtol=0)


def test_rel_bias_clamps_both_ends():
    table = torch.tensor([[1.0, 2.0, 3.0]], dtype=F64)
    q = torch.tensor([[0], [5]])
    kv = torch.tensor([[0, 1, 4, 5]])
    out = fo.RelBias(table)(torch.zeros(2, 4, dtype=F64), 0, 0, q, kv)
    # q=0: rel = 0,-1,-4,-5 -> all clamp to 0; q=5: rel = 5,4,1,0 -> 2,2,1,0
    assert out.tolist() == [[1.0, 1.0, 1.0, 1.0], [3.0, 3.0, 2.0, 1.0]]


def test_gqa_equals_mha_with_repeated_kv():
    Q, K, V = rand(2, 6, 10, 4, seed=1), rand(2, 2, 10, 4, seed=2), rand(2, 2, 10, 4, seed=3)
    bias = -torch.tensor([0.1, 0.2, 0.3, 0.4, 0.5, 0.6])
    O_g, L_g = fo.flex_attention(Q, K, V, fo.Alibi(bias), fo.causal_mask)
    Kr, Vr = K.repeat_interleave(3, dim=1), V.repeat_interleave(3, dim=1)
    O_m, L_m = fo.flex_attention(Q, Kr, Vr, fo.Alibi(bias), fo.causal_mask)
    assert torch.equal(O_g, O_m) and torch.equal(L_g, L_m)


def test_all_masked_row_convention():
    # ctx_len = 0 hides every key of sequence 1; window < 0 with causal hides every key everywhere.
    Q, K, V = rand(2, 2, 4, 4, seed=1), rand(2, 2, 6, 4, seed=2), rand(2, 2, 6, 4, seed=3)
    O, L = fo.flex_attention(Q, K, V, fo.Softcap(3.0), fo.ctx_len_mask(torch.tensor([4, 0])))
    assert torch.isfinite(O).all() and (O[1] == 0).all() and torch.isinf(L[1]).all() and (L[1] < 0).all()
    assert torch.isfinite(L[0]).all() and O[0].abs().sum() > 0
    dQ, dK, dV = fo.flex_attention_backward(Q, K, V, rand(2, 2, 4, 4, seed=4), fo.Softcap(3.0),
                                            fo.ctx_len_mask(torch.tensor([4, 0])))
    for g in (dQ, dK, dV):
        assert torch.isfinite(g).all() and (g[1] == 0).all()
    assert (dK[0, :, 4:] == 0).all() and (dV[0, :, 4:] == 0).all() and dQ[0].abs().sum() > 0


def test_q_rows_subset_matches_full():
    Q, K, V = rand(1, 1, 50, 8, seed=1), rand(1, 1, 50, 8, seed=2), rand(1, 1, 50, 8, seed=3)
    O, L = fo.flex_attention(Q, K, V, fo.Softcap(4.0), fo.causal_mask, 0.3)
    rows = torch.tensor([0, 7, 49, 13])
    o, l = fo.attention_head(Q[0, 0], K[0, 0], V[0, 0], fo.Softcap(4.0), fo.causal_mask, 0.3, 0, 0, q_rows=rows)
    assert torch.equal(o, O[0, 0, rows]) and torch.equal(l, L[0, 0, rows])
    o2, l2 = fo.attention_head(Q[0, 0], K[0, 0], V[0, 0], fo.Softcap(4.0), fo.causal_mask, 0.3, 0, 0, stripe=7)
    assert torch.allclose(o2, O[0, 0], atol=1e-14, rtol=0) and torch.allclose(l2, L[0, 0], atol=1e-14, rtol=0)
