"""Pins for the oracle's offset conversion (section 5.2) and multi-token paged attention (sections
5.1 + 5.2), against things other than itself: a scalar brute force, the dense textbook softmax on the
complete sequence, the one-token decode, and invariance under a permutation of the pool."""
import math

import torch

import flex_workloads as wlm
from oracle import flex_oracle as fo


def small_prefill(kv_lens, q_len, page=4, Hq=4, Hkv=2, D=8, slack=2, seed_shift=0):
    wl = wlm.CFG5.scaled(B=len(kv_lens), Hq=Hq, Hkv=Hkv, D=D, page_size=page,
                         max_pages=(max(kv_lens) + page - 1) // page + 1)
    return wlm.make_prefill_inputs(wl, kv_lens, q_len, slack_pages=slack)


def test_offset_conversion_shifts_only_the_query_index():
    off = torch.tensor([5, 0, 9], dtype=torch.int32)
    q, kv = torch.arange(4).view(-1, 1), torch.arange(16).view(1, -1)
    for b in range(3):
        got = fo.with_q_offset(fo.causal_mask, off)(b, 0, q, kv)
        want = torch.tensor([[k <= i + int(off[b]) for k in range(16)] for i in range(4)])
        assert torch.equal(got, want)
    # ALiBi: bias * (q + off - kv)
    bias = torch.tensor([-0.5, -0.25], dtype=torch.float64)
    s = torch.zeros(4, 16, dtype=torch.float64)
    got = fo.QOffset(fo.Alibi(bias), off)(s, 2, 1, q, kv)
    want = torch.tensor([[-0.25 * (i + 9 - k) for k in range(16)] for i in range(4)], dtype=torch.float64)
    assert torch.allclose(got, want, atol=0, rtol=0)


def test_paged_attention_matches_scalar_brute_force():
    inp = small_prefill([11, 6, 16], q_len=3)
    cap = 4.0
    slopes = torch.tensor([0.5, 0.25, 0.125, 0.0625], dtype=torch.float64)
    score = fo.Compose(fo.Alibi(-slopes), fo.Softcap(cap))
    mask = fo.and_mask(fo.causal_mask, fo.sliding_window_mask(6))
    O, LSE = fo.paged_attention(inp.Q, inp.K_pool, inp.V_pool, inp.page_table, inp.kv_lens, inp.q_offsets,
                                score, mask, inp.scale)
    P, G = 4, 2
    for b in range(3):
        n, off = int(inp.kv_lens[b]), int(inp.q_offsets[b])
        for h in range(4):
            for i in range(3):
                qpos = off + i
                w, acc = [], [0.0] * 8
                for t in range(n):
                    if not (t <= qpos and qpos - t <= 6):
                        continue
                    page, r = int(inp.page_table[b, t // P]), t % P
                    k = inp.K_pool[page, h // G, r].double()
                    s = float((inp.Q[b, h, i].double() * k).sum()) * inp.scale
                    s = s - float(slopes[h]) * (qpos - t)
                    s = cap * math.tanh(s / cap)
                    w.append((math.exp(s), page, r))
                tot = sum(x[0] for x in w)
                for e, page, r in w:
                    v = inp.V_pool[page, h // G, r].double()
                    for d in range(8):
                        acc[d] += e / tot * float(v[d])
                assert abs(float(LSE[b, h, i]) - math.log(tot)) < 1e-12
                assert max(abs(float(O[b, h, i, d]) - acc[d]) for d in range(8)) < 1e-12


def test_chunk_rows_equal_rows_of_dense_causal_attention_over_the_whole_sequence():
    # the cache holds the complete sequence; a chunk at offset o must reproduce rows o .. o + Lq of
    # ordinary causal attention, computed here with torch.softmax on the gathered sequence
    kv_lens, Lq, P = [23, 40, 8], 8, 4
    inp = small_prefill(kv_lens, Lq, slack=3)
    O, LSE = fo.paged_attention(inp.Q, inp.K_pool, inp.V_pool, inp.page_table, inp.kv_lens, inp.q_offsets,
                                fo.Identity(), fo.causal_mask, inp.scale)
    for b, n in enumerate(kv_lens):
        off = n - Lq
        Kc = torch.stack([inp.K_pool[int(inp.page_table[b, t // P]), :, t % P] for t in range(n)], dim=1).double()
        Vc = torch.stack([inp.V_pool[int(inp.page_table[b, t // P]), :, t % P] for t in range(n)], dim=1).double()
        for h in range(4):
            s = (inp.Q[b, h].double() @ Kc[h // 2].T) * inp.scale          # [Lq, n]
            qpos = torch.arange(off, n).view(-1, 1)
            s = s.masked_fill(torch.arange(n).view(1, -1) > qpos, float("-inf"))
            want = torch.softmax(s, dim=1) @ Vc[h // 2]
            assert torch.allclose(O[b, h], want, atol=1e-13, rtol=0)
            assert torch.allclose(LSE[b, h], torch.logsumexp(s, dim=1), atol=1e-13, rtol=0)


def test_one_token_chunk_is_the_decode_step():
    kv_lens = [13, 32, 1, 30]
    inp = small_prefill(kv_lens, q_len=1)
    score = fo.Softcap(5.0)
    O, LSE = fo.paged_attention(inp.Q, inp.K_pool, inp.V_pool, inp.page_table, inp.kv_lens, inp.q_offsets,
                                score, fo.causal_mask, inp.scale)
    O2, LSE2 = fo.paged_decode(inp.Q, inp.K_pool, inp.V_pool, inp.page_table, inp.kv_lens, score, inp.scale)
    assert torch.allclose(O, O2, atol=1e-14, rtol=0) and torch.allclose(LSE, LSE2, atol=1e-14, rtol=0)


def test_paged_attention_invariant_under_pool_permutation():
    inp = small_prefill([9, 20, 14], q_len=5)
    args = (inp.kv_lens, inp.q_offsets, fo.Identity(), fo.causal_mask, inp.scale)
    O, LSE = fo.paged_attention(inp.Q, inp.K_pool, inp.V_pool, inp.page_table, *args)
    n_pool = inp.K_pool.shape[0]
    perm = torch.randperm(n_pool, generator=torch.Generator().manual_seed(11))
    inv = torch.empty_like(perm)
    inv[perm] = torch.arange(n_pool)
    O2, LSE2 = fo.paged_attention(inp.Q, inp.K_pool[perm], inp.V_pool[perm],
                                  inv[inp.page_table.long()].to(torch.int32), *args)
    assert torch.equal(O, O2) and torch.equal(LSE, LSE2)


def test_tokens_past_kv_len_are_hidden_by_the_mask_not_the_slicing():
    # a non-causal chunk needs an explicit bound: without one the padding of the last page is visible
    inp = small_prefill([10], q_len=2, Hq=2, Hkv=1)
    bound = fo.ctx_len_mask(inp.kv_lens)
    O, _ = fo.paged_attention(inp.Q, inp.K_pool, inp.V_pool, inp.page_table, inp.kv_lens, inp.q_offsets,
                              fo.Identity(), bound, inp.scale)
    O_open, _ = fo.paged_attention(inp.Q, inp.K_pool, inp.V_pool, inp.page_table, inp.kv_lens, inp.q_offsets,
                                   fo.Identity(), fo.no_mask, inp.scale)
    assert not torch.allclose(O, O_open)
    Kc = torch.stack([inp.K_pool[int(inp.page_table[0, t // 4]), :, t % 4] for t in range(10)], dim=1).double()
    Vc = torch.stack([inp.V_pool[int(inp.page_table[0, t // 4]), :, t % 4] for t in range(10)], dim=1).double()
    for h in range(2):
        want = torch.softmax((inp.Q[0, h].double() @ Kc[0].T) * inp.scale, dim=1) @ Vc[0]
        assert torch.allclose(O[0, h], want, atol=1e-13, rtol=0)
