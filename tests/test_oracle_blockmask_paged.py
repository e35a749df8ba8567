"""Pins for the oracle's BlockMask builder, paged conversion and paged decode (CPU only)."""
import math

import pytest
import torch

import flex_workloads as wlm
from oracle import flex_oracle as fo

F64 = torch.float64


def lists(bm, name, b=0, h=0):
    num = bm[name.replace("indices", "num_blocks")][b, h]
    idx = bm[name][b, h]
    return [idx[i, :int(num[i])].tolist() for i in range(idx.shape[0])]


def dense_from_python(mask_fn, q_len, kv_len):
    return torch.tensor([[bool(mask_fn(q, kv)) for kv in range(kv_len)] for q in range(q_len)])


def test_cfg1_causal_closed_form():
    bm = fo.create_block_mask(fo.causal_mask, 1, 1, 256, 256, 64, 64)
    assert lists(bm, "kv_indices") == [[i] for i in range(4)]
    assert lists(bm, "full_kv_indices") == [list(range(i)) for i in range(4)]
    assert lists(bm, "q_indices") == [[j] for j in range(4)]
    assert lists(bm, "full_q_indices") == [list(range(j + 1, 4)) for j in range(4)]
    assert bm["stats"]["unmasked_pairs"] == 256 * 257 // 2
    # tail entries are zero
    assert bm["kv_indices"][0, 0, 0].tolist() == [0, 0, 0, 0]
    assert bm["full_kv_indices"][0, 0, 2].tolist() == [0, 1, 0, 0]


def test_cfg2_causal_closed_form_128x64():
    S = 8192
    bm = fo.create_block_mask(fo.causal_mask, 1, 1, S, S, 128, 64)
    for i in range(64):
        assert int(bm["kv_num_blocks"][0, 0, i]) == 2
        assert bm["kv_indices"][0, 0, i, :2].tolist() == [2 * i, 2 * i + 1]
        assert int(bm["full_kv_num_blocks"][0, 0, i]) == 2 * i
        assert bm["full_kv_indices"][0, 0, i, :2 * i].tolist() == list(range(2 * i))
    for j in range(128):
        assert int(bm["q_num_blocks"][0, 0, j]) == 1 and int(bm["q_indices"][0, 0, j, 0]) == j // 2
        assert int(bm["full_q_num_blocks"][0, 0, j]) == 63 - j // 2
        assert bm["full_q_indices"][0, 0, j, :63 - j // 2].tolist() == list(range(j // 2 + 1, 64))
    assert bm["stats"]["partial"] + bm["stats"]["full"] == 4160
    assert bm["stats"]["unmasked_pairs"] == S * (S + 1) // 2


@pytest.mark.parametrize("case", ["swa_prefix", "document", "one_sided_window", "ctx"])
def test_blocks_match_python_dense_mask(case):
    q_len, kv_len, Bq, Bk = 48, 64, 8, 4
    doc = torch.tensor([[0] * 10 + [1] * 23 + [2] * 31], dtype=torch.int32)
    if case == "swa_prefix":
        mod = fo.or_mask(fo.and_mask(fo.causal_mask, fo.sliding_window_mask(9)), fo.prefix_mask(6))
        fn = lambda q, kv: (q >= kv and q - kv <= 9) or kv < 6
    elif case == "document":
        mod = fo.and_mask(fo.document_mask(doc), fo.causal_mask)
        fn = lambda q, kv: int(doc[0, q]) == int(doc[0, kv]) and q >= kv
    elif case == "one_sided_window":
        mod = fo.sliding_window_mask(5)
        fn = lambda q, kv: q - kv <= 5
    else:
        mod = fo.ctx_len_mask(torch.tensor([37]))
        fn = lambda q, kv: kv < 37
    bm = fo.create_block_mask(mod, 1, 1, q_len, kv_len, Bq, Bk)
    dense = dense_from_python(fn, q_len, kv_len)
    NR, NC = q_len // Bq, kv_len // Bk
    part, full = lists(bm, "kv_indices"), lists(bm, "full_kv_indices")
    for i in range(NR):
        assert part[i] == sorted(part[i]) and full[i] == sorted(full[i])
        for j in range(NC):
            blk = dense[i * Bq:(i + 1) * Bq, j * Bk:(j + 1) * Bk]
            kind = "full" if blk.all() else ("partial" if blk.any() else "empty")
            assert (j in full[i]) == (kind == "full")
            assert (j in part[i]) == (kind == "partial")
    # transposed lists hold exactly the same block sets
    qpart, qfull = lists(bm, "q_indices"), lists(bm, "full_q_indices")
    assert {(i, j) for i in range(NR) for j in part[i]} == {(i, j) for j in range(NC) for i in qpart[j]}
    assert {(i, j) for i in range(NR) for j in full[i]} == {(i, j) for j in range(NC) for i in qfull[j]}
    assert all(l == sorted(l) for l in qpart + qfull)
    assert bm["stats"]["unmasked_pairs"] == int(dense.sum())


def test_broadcast_dims_and_per_batch_masks():
    doc = torch.tensor([[0] * 8 + [1] * 24, [0] * 20 + [1] * 12], dtype=torch.int32)
    bm = fo.create_block_mask(fo.document_mask(doc), 2, 1, 32, 32, 8, 8)
    assert bm["kv_indices"].shape == (2, 1, 4, 4) and bm["q_num_blocks"].shape == (2, 1, 4)
    assert lists(bm, "full_kv_indices", b=0) == [[0], [1, 2, 3], [1, 2, 3], [1, 2, 3]]
    assert lists(bm, "kv_indices", b=0) == [[], [], [], []]
    assert lists(bm, "kv_indices", b=1) == [[2], [2], [0, 1, 2, 3], [2]]
    assert lists(bm, "full_kv_indices", b=1) == [[0, 1], [0, 1], [], [3]]


def test_cfg4_counts_closed_form():
    # (0 <= q - kv <= W) or kv < P at S = 32768, W = 4096, P = 1024, 128x64 blocks.
    S, W, P = 32768, 4096, 1024
    mod = fo.or_mask(fo.and_mask(fo.causal_mask, fo.sliding_window_mask(W)), fo.prefix_mask(P))
    kinds, pairs = fo.block_kinds(mod, 1, 1, S, S, 128, 64)
    # rows q < P see P keys; P <= q < W + P see q + 1; later rows see the P prefix keys + W + 1 window keys
    closed = P * P + sum(q + 1 for q in range(P, W + P)) + (S - W - P) * (P + W + 1)
    assert pairs == closed == 155218944
    # block classes by pure integer reasoning on block corners
    n_full = n_part = 0
    for i in range(S // 128):
        q0, q1 = i * 128, i * 128 + 127
        for j in range(S // 64):
            k0, k1 = j * 64, j * 64 + 63
            if k1 < P:
                n_full += 1
                continue
            # window part only (columns >= P inside this block when k0 >= P; P is a multiple of 64)
            any_vis = (q1 >= k0) and (q0 - k1 <= W)
            all_vis = (q0 >= k1) and (q1 - k0 <= W)
            n_full += all_vis
            n_part += any_vis and not all_vis
    assert int((kinds == 2).sum()) == n_full and int((kinds == 1).sum()) == n_part


def test_ragged_lengths_round_up_and_the_outside_counts_as_masked():
    # causal, q_len = kv_len = 200, 64 x 64 blocks: 4 x 4 blocks; the last row / column holds 8 tokens
    S, B = 200, 64
    kinds, pairs = fo.block_kinds(fo.causal_mask, 1, 1, S, S, B, B)
    assert kinds.shape == (1, 1, 4, 4) and pairs == S * (S + 1) // 2
    want = torch.tensor([[1, 0, 0, 0], [2, 1, 0, 0], [2, 2, 1, 0], [1, 1, 1, 1]], dtype=torch.int8)
    assert torch.equal(kinds[0, 0], want)       # blocks of the last row are cut by the edge: never full
    # no mask at all, 100 x 150 with 64 x 64 blocks: the inner block is full, the edge blocks partial
    kinds, pairs = fo.block_kinds(fo.no_mask, 1, 1, 100, 150, 64, 64)
    assert pairs == 100 * 150 and kinds[0, 0].tolist() == [[2, 2, 1], [1, 1, 1]]
    # a multiple of the block size is unchanged by the rule, whatever lies beyond is simply absent
    a, _ = fo.block_kinds(fo.causal_mask, 1, 1, 256, 256, 64, 64)
    b, _ = fo.block_kinds(fo.causal_mask, 1, 1, 250, 250, 64, 64)
    assert torch.equal(a[0, 0, :3, :3], b[0, 0, :3, :3]) and b[0, 0, 3].tolist() == [1, 1, 1, 1]
    # scalar brute force on a tiny sliding-window case
    mod = fo.and_mask(fo.causal_mask, fo.sliding_window_mask(3))
    kinds, pairs = fo.block_kinds(mod, 1, 1, 10, 7, 4, 4)
    for i in range(3):
        for j in range(2):
            cnt = sum(1 for q in range(4 * i, 4 * i + 4) for k in range(4 * j, 4 * j + 4)
                      if q < 10 and k < 7 and k <= q and q - k <= 3)
            assert int(kinds[0, 0, i, j]) == (0 if cnt == 0 else (2 if cnt == 16 else 1))
    bm = fo.create_block_mask(mod, 1, 1, 10, 7, 4, 4)
    assert bm["kv_indices"].shape == (1, 1, 3, 2) and bm["q_indices"].shape == (1, 1, 2, 3)


def test_paged_conversion_and_phys2log():
    wl = wlm.CFG5.scaled(B=3, max_pages=8, page_size=4)
    inp = wlm.make_decode_inputs(wl, ctx_lens=[9, 32, 1], slack_pages=2)
    bm = fo.create_block_mask(fo.ctx_len_mask(inp.ctx_lens), 3, 1, 1, 32, 1, 4)
    assert bm["full_kv_num_blocks"][:, 0, 0].tolist() == [2, 8, 0]
    assert bm["kv_num_blocks"][:, 0, 0].tolist() == [1, 0, 1]
    n_pool = inp.K_pool.shape[0]
    for num_name, idx_name in (("kv_num_blocks", "kv_indices"), ("full_kv_num_blocks", "full_kv_indices")):
        phys, p2l = fo.convert_block_mask_paged(bm[num_name], bm[idx_name], inp.page_table, n_pool)
        for b in range(3):
            n = int(bm[num_name][b, 0, 0])
            for k in range(8):
                if k < n:
                    logical = int(bm[idx_name][b, 0, 0, k])
                    assert int(phys[b, 0, 0, k]) == int(inp.page_table[b, logical])
                    assert int(p2l[int(phys[b, 0, 0, k])]) == logical
                else:
                    assert int(phys[b, 0, 0, k]) == 0
    # converted mods evaluated at the physical token index agree with user mods at the logical index
    _, p2l_f = fo.convert_block_mask_paged(bm["full_kv_num_blocks"], bm["full_kv_indices"], inp.page_table, n_pool)
    _, p2l_p = fo.convert_block_mask_paged(bm["kv_num_blocks"], bm["kv_indices"], inp.page_table, n_pool)
    p2l = torch.maximum(p2l_f, p2l_p)
    user = fo.ctx_len_mask(inp.ctx_lens)
    for b in range(3):
        for logical_kv in range(int(inp.ctx_lens[b]) + 3):
            if logical_kv >= ((int(inp.ctx_lens[b]) + 3) // 4) * 4:
                break
            phys_kv = int(inp.page_table[b, logical_kv // 4]) * 4 + logical_kv % 4
            back = int(p2l[phys_kv // 4]) * 4 + phys_kv % 4
            assert back == logical_kv
            q, kv = torch.tensor([[0]]), torch.tensor([[back]])
            assert bool(user(b, 0, q, kv)) == (logical_kv < int(inp.ctx_lens[b]))


def test_paged_decode_equals_contiguous_attention():
    wl = wlm.CFG5.scaled(B=4, Hq=4, Hkv=2, D=8, max_pages=16, page_size=4)
    inp = wlm.make_decode_inputs(wl, ctx_lens=[13, 64, 1, 30], slack_pages=3)
    O, LSE = fo.paged_decode(inp.Q, inp.K_pool, inp.V_pool, inp.page_table, inp.ctx_lens, fo.Softcap(5.0), inp.scale)
    for b, n in enumerate([13, 64, 1, 30]):
        # gather the sequence token by token, independently of unpage()
        Kc = torch.stack([inp.K_pool[int(inp.page_table[b, t // 4]), :, t % 4] for t in range(n)], dim=1)
        Vc = torch.stack([inp.V_pool[int(inp.page_table[b, t // 4]), :, t % 4] for t in range(n)], dim=1)
        o, l = fo.flex_attention(inp.Q[b:b + 1].double(), Kc[None].double(), Vc[None].double(),
                                 fo.Softcap(5.0), fo.no_mask, inp.scale)
        assert torch.allclose(O[b], o[0], atol=1e-13, rtol=0) and torch.allclose(LSE[b], l[0], atol=1e-13, rtol=0)


def test_paged_decode_invariant_under_pool_permutation():
    wl = wlm.CFG5.scaled(B=3, Hq=4, Hkv=2, D=8, max_pages=8, page_size=4)
    inp = wlm.make_decode_inputs(wl, ctx_lens=[7, 32, 18])
    O, LSE = fo.paged_decode(inp.Q, inp.K_pool, inp.V_pool, inp.page_table, inp.ctx_lens, fo.Identity(), inp.scale)
    n_pool = inp.K_pool.shape[0]
    perm = torch.randperm(n_pool, generator=torch.Generator().manual_seed(5))
    inv = torch.empty_like(perm)
    inv[perm] = torch.arange(n_pool)
    K2, V2 = inp.K_pool[perm], inp.V_pool[perm]             # new page p holds old page perm[p]
    table2 = inv[inp.page_table.long()].to(torch.int32)
    O2, LSE2 = fo.paged_decode(inp.Q, K2, V2, table2, inp.ctx_lens, fo.Identity(), inp.scale)
    assert torch.equal(O, O2) and torch.equal(LSE, LSE2)


def test_paged_decode_empty_context():
    wl = wlm.CFG5.scaled(B=2, Hq=2, Hkv=1, D=8, max_pages=4, page_size=4)
    inp = wlm.make_decode_inputs(wl, ctx_lens=[0, 5])
    O, LSE = fo.paged_decode(inp.Q, inp.K_pool, inp.V_pool, inp.page_table, inp.ctx_lens, fo.Identity(), inp.scale)
    assert (O[0] == 0).all() and torch.isinf(LSE[0]).all() and torch.isfinite(LSE[1]).all()


def test_workload_generators_are_seeded_and_shaped():
    a = wlm.make_train_inputs(wlm.CFG1)
    b = wlm.make_train_inputs(wlm.CFG1)
    assert torch.equal(a.Q, b.Q) and a.Q.dtype == torch.bfloat16 and a.Q.shape == (1, 2, 256, 64) and a.dO is None
    c3 = wlm.make_train_inputs(wlm.CFG3.scaled(S=8192))
    assert sum(c3.doc_lengths[0]) == 8192 and all(1 <= L <= 4096 for L in c3.doc_lengths[0])
    assert all(L >= 256 for L in c3.doc_lengths[0][:-1])
    assert (c3.doc_ids[0][1:] >= c3.doc_ids[0][:-1]).all() and c3.doc_ids.dtype == torch.int32
    assert abs(float(c3.slopes[15]) - 2.0 ** -8) < 1e-9 and abs(float(c3.slopes[0]) - 2.0 ** -0.5) < 1e-7
    d = wlm.make_decode_inputs(wlm.CFG5.scaled(B=4, ctx_min=16, ctx_max=100, max_pages=8))
    used = [int(p) for b in range(4) for p in d.page_table[b, :(int(d.ctx_lens[b]) + 15) // 16]]
    assert len(set(used)) == len(used) == d.K_pool.shape[0]


def test_work_order_is_longest_first_and_a_permutation():
    """kv_order / q_order: per plane a permutation of the lines, descending number of listed blocks,
    ties by ascending index -- checked against a plain Python sort, and for the causal mask against
    the closed form (rows: last first; columns: first first)."""
    import random
    S, Bq, Bk = 1024, 128, 64
    bm = fo.create_block_mask(fo.causal_mask, 1, 1, S, S, Bq, Bk)
    NR, NC = S // Bq, S // Bk
    assert bm["kv_order"].tolist() == [[list(range(NR - 1, -1, -1))]]
    assert bm["q_order"][0, 0].tolist() == sorted(range(NC), key=lambda j: (-(NR - j // 2), j))
    rng = random.Random(5)
    doc = torch.tensor(sorted(rng.randrange(6) for _ in range(S)), dtype=torch.int32).view(1, S)
    mask = fo.and_mask(fo.document_mask(doc), fo.causal_mask)
    bm = fo.create_block_mask(mask, 1, 2, S, S, Bq, Bk)
    for name, num, full in (("kv_order", "kv_num_blocks", "full_kv_num_blocks"),
                            ("q_order", "q_num_blocks", "full_q_num_blocks")):
        for h in range(2):
            cnt = (bm[num][0, h] + bm[full][0, h]).tolist()
            assert bm[name][0, h].tolist() == sorted(range(len(cnt)), key=lambda i: (-cnt[i], i)), name
    # more lines than are sorted: the fixed orders
    long_rows = fo.work_order(torch.zeros(1, 1, fo.WORK_ORDER_MAX_LINES + 1, dtype=torch.int32), True)
    assert long_rows[0, 0, 0] == fo.WORK_ORDER_MAX_LINES and long_rows[0, 0, -1] == 0
    long_cols = fo.work_order(torch.zeros(1, 1, fo.WORK_ORDER_MAX_LINES + 1, dtype=torch.int32), False)
    assert long_cols[0, 0, 0] == 0 and long_cols[0, 0, -1] == fo.WORK_ORDER_MAX_LINES
