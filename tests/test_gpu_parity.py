"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle on identical seeded inputs.

BlockMask arrays must match bit for bit.  O (bf16) vs oracle: max abs <= 2e-2, mean abs <= 2e-3;
LSE <= 1e-2; gradients: max abs <= 2e-2 * max(1, max|ref|), mean abs <= 6e-3 * max(1, mean|ref|), and no
more than 3x (max) / 1.5x (mean) the error of an emulation that rounds only what a bf16 matrix-unit kernel must round
(helpers.check_grad, helpers.emulate_bf16_backward).
"""
import pytest
import torch

import flex_workloads as wlm
from oracle import flex_oracle as fo

from helpers import (assert_blockmask_equal, check_grad, check_output, emulate_bf16_backward, library_mods,
                     oracle_mods, run_backward, run_forward)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# Scaled-down versions of the benchmark workloads that the oracle finishes in seconds; each spans
# several BlockMask blocks per row, full + partial blocks and (for GQA) several heads per group.
SMALL = {
    "cfg1": wlm.CFG1,
    "cfg2_small": wlm.CFG2.scaled(B=2, Hq=2, Hkv=2, S=1024),
    "cfg3_small": wlm.CFG3.scaled(Hq=4, Hkv=4, S=2048, doc_len_min=100, doc_len_max=700),
    "cfg4_small": wlm.CFG4.scaled(B=1, Hq=8, Hkv=2, S=2048, window=300, prefix_len=128, rel_len=256),
    "noop_d64_64x64": wlm.Workload("noop", B=1, Hq=2, Hkv=2, S=512, D=64, Bq=64, Bk=64, mask="none",
                                   score="identity", seed=11),
    "causal_alibi_bk128": wlm.Workload("causal_alibi", B=1, Hq=4, Hkv=2, S=1024, D=128, Bq=64, Bk=128,
                                       mask="causal", score="alibi", seed=12),
    "swa_d64": wlm.Workload("swa", B=1, Hq=2, Hkv=1, S=1024, D=64, Bq=128, Bk=128, mask="swa_causal",
                            score="identity", seed=13, window=200),
    "prefix_lm_d128": wlm.Workload("prefix_lm", B=2, Hq=2, Hkv=2, S=768, D=128, Bq=128, Bk=64, mask="prefix_lm",
                                   score="identity", seed=14, prefix_len=200),
    "doc_causal_d128": wlm.Workload("doc", B=2, Hq=2, Hkv=1, S=1024, D=128, Bq=128, Bk=64, mask="doc_causal",
                                    score="identity", seed=15, doc_len_min=50, doc_len_max=400),
    # the variants of the paper's 16k-token benchmark (section 6.2) at head dimension 64, 128 x 64 blocks
    "noop_d64": wlm.Workload("noop128", B=1, Hq=2, Hkv=2, S=768, D=64, Bq=128, Bk=64, mask="none",
                             score="identity", seed=16),
    "causal_alibi_d64_gqa": wlm.Workload("alibi64", B=1, Hq=4, Hkv=1, S=1024, D=64, Bq=128, Bk=64, mask="causal",
                                         score="alibi", seed=17),
    "causal_softcap_d64": wlm.Workload("softcap64", B=1, Hq=2, Hkv=2, S=1024, D=64, Bq=128, Bk=64, mask="causal",
                                       score="softcap", seed=18, softcap=30.0),
    "prefix_lm_d64": wlm.Workload("prefix64", B=1, Hq=2, Hkv=1, S=1024, D=64, Bq=128, Bk=64, mask="prefix_lm",
                                  score="identity", seed=19, prefix_len=300),
    # compositions: a sliding window with a soft-cap; nested score_mods (bias, then soft-cap)
    "swa_softcap_d128": wlm.Workload("swa_cap", B=1, Hq=4, Hkv=2, S=1024, D=128, Bq=128, Bk=64, mask="swa_causal",
                                     score="softcap", seed=23, window=300, softcap=30.0),
    "causal_alibi_softcap_d64": wlm.Workload("alibi_cap", B=1, Hq=4, Hkv=4, S=768, D=64, Bq=128, Bk=64,
                                             mask="causal", score="alibi_softcap", seed=24, softcap=20.0),
    "doc_relbias_softcap_d128": wlm.Workload("rel_cap", B=2, Hq=2, Hkv=1, S=640, D=128, Bq=64, Bk=64,
                                             mask="doc_causal", score="rel_bias_softcap", seed=25, softcap=50.0,
                                             rel_len=96, doc_len_min=60, doc_len_max=300),
    "softcap_unbounded_d128": wlm.Workload("softcap_big", B=1, Hq=2, Hkv=2, S=512, D=128, Bq=128, Bk=64, mask="causal",
                                           score="softcap", seed=20, softcap=50.0),
}


@pytest.mark.parametrize("name", list(SMALL))
def test_forward_backward_small(name):
    wl = SMALL[name]
    inp = wlm.make_train_inputs(wl, with_dO=True)
    score, mask = oracle_mods(wl, inp)
    print(f"[case] {name} {wl}", flush=True)
    O, LSE, bm, ids = run_forward(wl, inp, DEV)
    ref_bm = fo.create_block_mask(mask, bm.Bm, 1, wl.S, wl.S, wl.Bq, wl.Bk)
    assert_blockmask_equal(bm, ref_bm)
    O_ref, LSE_ref = fo.flex_attention(inp.Q, inp.K, inp.V, score, mask, inp.scale)
    check_output(O, LSE, O_ref, LSE_ref)
    dQ, dK, dV = run_backward(wl, inp, DEV, O, LSE, bm, ids)
    dQ_ref, dK_ref, dV_ref = fo.flex_attention_backward(inp.Q, inp.K, inp.V, inp.dO, score, mask, inp.scale)
    dQ_em, dK_em, dV_em = emulate_bf16_backward(inp, score, mask)
    check_grad("dQ", dQ, dQ_ref, dQ_em)
    check_grad("dK", dK, dK_ref, dK_em)
    check_grad("dV", dV, dV_ref, dV_em)


# One BlockMask plane per query head (Hm = Hq): the kernels index the lists by the QUERY head, also
# under GQA where several query heads share a KV head (dK / dV walk one transposed list per head).
PER_HEAD = {
    "causal_softcap_d128_gqa": wlm.Workload("ph128", B=2, Hq=4, Hkv=2, S=640, D=128, Bq=128, Bk=64, mask="causal",
                                            score="softcap", seed=31, softcap=30.0),
    "swa_prefix_relbias_d64_gqa": wlm.Workload("ph64", B=1, Hq=6, Hkv=2, S=768, D=64, Bq=64, Bk=128,
                                               mask="swa_causal_or_prefix", score="rel_bias", seed=32, window=150,
                                               prefix_len=70, rel_len=64),
    "doc_alibi_d64": wlm.Workload("phdoc", B=2, Hq=4, Hkv=4, S=512, D=64, Bq=128, Bk=64, mask="doc_causal",
                                  score="alibi", seed=33, doc_len_min=40, doc_len_max=300),
}


@pytest.mark.parametrize("name", list(PER_HEAD))
def test_per_head_blockmask(name):
    wl = PER_HEAD[name]
    inp = wlm.make_train_inputs(wl, with_dO=True)
    score, mask = oracle_mods(wl, inp)
    print(f"[case] per-head BlockMask {name} {wl}", flush=True)
    O, LSE, bm, ids = run_forward(wl, inp, DEV, Hm=wl.Hq)
    assert bm.Hm == wl.Hq and bm.kv_indices.shape[1] == wl.Hq
    assert_blockmask_equal(bm, fo.create_block_mask(mask, bm.Bm, wl.Hq, wl.S, wl.S, wl.Bq, wl.Bk))
    O_ref, LSE_ref = fo.flex_attention(inp.Q, inp.K, inp.V, score, mask, inp.scale)
    check_output(O, LSE, O_ref, LSE_ref)
    dQ, dK, dV = run_backward(wl, inp, DEV, O, LSE, bm, ids)
    g_ref = fo.flex_attention_backward(inp.Q, inp.K, inp.V, inp.dO, score, mask, inp.scale)
    g_em = emulate_bf16_backward(inp, score, mask)
    for n, g, r, e in zip(("dQ", "dK", "dV"), (dQ, dK, dV), g_ref, g_em):
        check_grad(n, g, r, e)
    # the same call with the shared plane must give the same bits: the planes are identical
    O1, LSE1, bm1, _ = run_forward(wl, inp, DEV)
    assert torch.equal(O, O1) and torch.equal(LSE, LSE1)
    for a, b1 in zip((dQ, dK, dV), run_backward(wl, inp, DEV, O1, LSE1, bm1, ids)):
        assert torch.equal(a, b1)


def test_blockmask_without_full_blocks_gives_the_same_attention():
    """Listing every FULL block as PARTIAL (mask_mod evaluated everywhere, paper section 4.2) must not change
    the result beyond rounding: the tiles are merely visited in another order."""
    import paper_2412_05496_amd as fa
    wl = SMALL["cfg2_small"]
    inp = wlm.make_train_inputs(wl, with_dO=True)
    score, mask = oracle_mods(wl, inp)
    O, LSE, bm, ids = run_forward(wl, inp, DEV)
    mask_id, score_id, params, Q, K, V = ids
    bm2 = wlm.blockmask_all_partial(fa.alloc_blockmask, bm)
    assert int(bm2.full_kv_num_blocks.sum()) == 0 and int(bm2.full_q_num_blocks.sum()) == 0
    assert torch.equal(bm2.kv_num_blocks, bm.kv_num_blocks + bm.full_kv_num_blocks)
    O2, LSE2 = torch.empty_like(O), torch.empty_like(LSE)
    fa.flexattn_forward(Q, K, V, score_id, mask_id, params, bm2, inp.scale, O2, LSE2)
    O_ref, LSE_ref = fo.flex_attention(inp.Q, inp.K, inp.V, score, mask, inp.scale)
    check_output(O2, LSE2, O_ref, LSE_ref)
    dQ, dK, dV = run_backward(wl, inp, DEV, O2, LSE2, bm2, ids)
    dQ_ref, dK_ref, dV_ref = fo.flex_attention_backward(inp.Q, inp.K, inp.V, inp.dO, score, mask, inp.scale)
    check_grad("dQ", dQ, dQ_ref)
    check_grad("dK", dK, dK_ref)
    check_grad("dV", dV, dV_ref)


def test_work_order_changes_no_result():
    """The BlockMask's work order decides which workgroup takes which row / column of blocks, nothing
    else: with and without the order arrays every output is the same bit for bit."""
    import paper_2412_05496_amd as fa
    wl = SMALL["cfg3_small"]
    inp = wlm.make_train_inputs(wl, with_dO=True)
    O, LSE, bm, ids = run_forward(wl, inp, DEV)
    assert bm.kv_order is not None and bm.q_order is not None
    assert not torch.equal(bm.kv_order, torch.arange(bm.kv_order.shape[-1] - 1, -1, -1, device=DEV,
                                                     dtype=torch.int32).expand_as(bm.kv_order))
    grads = run_backward(wl, inp, DEV, O, LSE, bm, ids)
    grads_st = run_backward(wl, inp, DEV, O, LSE, bm, ids, stored=True)
    mask_id, score_id, params, Q, K, V = ids
    bm.kv_order, bm.q_order = None, None
    O2, LSE2 = torch.empty_like(O), torch.empty_like(LSE)
    fa.flexattn_forward(Q, K, V, score_id, mask_id, params, bm, inp.scale, O2, LSE2)
    torch.cuda.synchronize()
    assert torch.equal(O, O2) and torch.equal(LSE, LSE2)
    for g1, g2 in zip(grads, run_backward(wl, inp, DEV, O2, LSE2, bm, ids)):
        assert torch.equal(g1, g2)
    for g1, g2 in zip(grads_st, run_backward(wl, inp, DEV, O2, LSE2, bm, ids, stored=True)):
        assert torch.equal(g1, g2)


def test_causal_row0_is_v0_bit_exact():
    wl = wlm.CFG1
    inp = wlm.make_train_inputs(wl)
    O, LSE, _, _ = run_forward(wl, inp, DEV)
    assert torch.equal(O[:, :, 0].cpu(), inp.V[:, :, 0])


def test_all_masked_rows_give_zero_output_and_gradients():
    # sliding window with a negative window hides every key: O = 0, LSE = -inf, zero gradients
    wl = wlm.Workload("dead", B=1, Hq=2, Hkv=1, S=256, D=64, Bq=64, Bk=64, mask="swa_causal", score="identity",
                      seed=21, window=-1)
    inp = wlm.make_train_inputs(wl, with_dO=True)
    O, LSE, bm, ids = run_forward(wl, inp, DEV)
    assert int(bm.kv_num_blocks.sum()) == 0 and int(bm.full_kv_num_blocks.sum()) == 0
    assert (O == 0).all() and torch.isinf(LSE).all() and (LSE < 0).all()
    dQ, dK, dV = run_backward(wl, inp, DEV, O, LSE, bm, ids)
    assert (dQ == 0).all() and (dK == 0).all() and (dV == 0).all()


def test_rows_dead_inside_live_blocks():
    # document mask with every document alone except one: rows whose keys are all in *partial* blocks
    # and a prefix-only mask where later columns have no visible query at all (dK = dV = 0 there)
    wl = wlm.Workload("prefix_only", B=1, Hq=2, Hkv=2, S=512, D=64, Bq=64, Bk=64, mask="swa_causal_or_prefix",
                      score="rel_bias", seed=22, window=-1, prefix_len=70, rel_len=16)
    inp = wlm.make_train_inputs(wl, with_dO=True)
    score, mask = oracle_mods(wl, inp)
    O, LSE, bm, ids = run_forward(wl, inp, DEV)
    assert_blockmask_equal(bm, fo.create_block_mask(mask, 1, 1, wl.S, wl.S, wl.Bq, wl.Bk))
    O_ref, LSE_ref = fo.flex_attention(inp.Q, inp.K, inp.V, score, mask, inp.scale)
    check_output(O, LSE, O_ref, LSE_ref)
    dQ, dK, dV = run_backward(wl, inp, DEV, O, LSE, bm, ids)
    g_ref = fo.flex_attention_backward(inp.Q, inp.K, inp.V, inp.dO, score, mask, inp.scale)
    for n, g, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), g_ref):
        check_grad(n, g, r)
    assert (dK[:, :, 70:] == 0).all() and (dV[:, :, 70:] == 0).all()


def test_forward_is_deterministic_and_strided_inputs_work():
    wl = SMALL["cfg2_small"]
    inp = wlm.make_train_inputs(wl, with_dO=True)
    O1, L1, bm, ids = run_forward(wl, inp, DEV)
    O2, L2, _, _ = run_forward(wl, inp, DEV)
    assert torch.equal(O1, O2) and torch.equal(L1, L2)
    g1 = run_backward(wl, inp, DEV, O1, L1, bm, ids)
    g2 = run_backward(wl, inp, DEV, O1, L1, bm, ids)
    for a, b in zip(g1, g2):
        assert torch.equal(a, b)
    # same data laid out [B, S, H, D] in memory, viewed as [B, H, S, D]
    import paper_2412_05496_amd as fa
    mask_id, score_id, params, Q, K, V = ids
    Qs, Ks, Vs = (t.transpose(1, 2).contiguous().transpose(1, 2) for t in (Q, K, V))
    assert Qs.stride(2) != Q.stride(2)
    O3 = torch.empty_like(Qs)
    L3 = torch.empty_like(L1)
    fa.flexattn_forward(Qs, Ks, Vs, score_id, mask_id, params, bm, inp.scale, O3, L3)
    torch.cuda.synchronize()
    assert torch.equal(O3, O1) and torch.equal(L3, L1)


def test_backward_strided_layout_and_stages_agree():
    """[B, S, H, D] memory layout for every tensor of the backward, and the stages run one by one, give
    bit for bit what the dense single call gives."""
    import paper_2412_05496_amd as fa
    wl = SMALL["cfg2_small"].scaled(S=1000, Hq=4, Hkv=2)          # a cut last block and GQA as well
    inp = wlm.make_train_inputs(wl, with_dO=True)
    O, LSE, bm, ids = run_forward(wl, inp, DEV)
    dQ, dK, dV = run_backward(wl, inp, DEV, O, LSE, bm, ids)
    mask_id, score_id, params, Q, K, V = ids
    bshd = lambda t: t.transpose(1, 2).contiguous().transpose(1, 2)
    Qs, Ks, Vs, Os, dOs = (bshd(t) for t in (Q, K, V, O, inp.dO.to(DEV)))
    dQs, dKs, dVs = (bshd(torch.full_like(t, float("nan"))) for t in (Q, K, V))
    ws = torch.empty(fa.flexattn_backward_workspace_bytes(Q, K), dtype=torch.uint8, device=DEV)
    for stage in (fa.BWD_DELTA, fa.BWD_DQ, fa.BWD_DKDV):
        fa.flexattn_backward_stages(Qs, Ks, Vs, Os, dOs, LSE, score_id, mask_id, params, bm, inp.scale,
                                    dQs if stage == fa.BWD_DQ else None, dKs if stage == fa.BWD_DKDV else None,
                                    dVs if stage == fa.BWD_DKDV else None, ws, stage)
    torch.cuda.synchronize()
    assert torch.equal(dQs, dQ) and torch.equal(dKs, dK) and torch.equal(dVs, dV)


@pytest.mark.parametrize("mask_name", ["causal", "none"])
def test_dkdv_walk_longer_than_one_segment(mask_name):
    """A key column seen by more row blocks than the 1024 steps the dK/dV kernel lays out in LDS at a
    time: q_len = 66 560 in 64-row blocks against 128 keys, so each of the two key columns lists 1040
    (causal: 1 PARTIAL + 1039 FULL, resp. 1039 FULL) row blocks and the kernel walks them in two
    segments.  With so few keys the oracle evaluates every element."""
    import paper_2412_05496_amd as fa
    B, H, Sq, Skv, D, Bq, Bk = 1, 1, 66560, 128, 64, 64, 64
    gen = torch.Generator().manual_seed(41)
    Q, dO = wlm.randn_bf16(gen, B, H, Sq, D), wlm.randn_bf16(gen, B, H, Sq, D)
    K, V = wlm.randn_bf16(gen, B, H, Skv, D), wlm.randn_bf16(gen, B, H, Skv, D)
    scale = D ** -0.5
    mask_id, mask = {"causal": (fa.MASK_CAUSAL, fo.causal_mask), "none": (fa.MASK_NONE, fo.no_mask)}[mask_name]
    params = fa.ModParams()
    bm = fa.alloc_blockmask(1, 1, Sq, Skv, Bq, Bk, device=DEV)
    fa.flexattn_blockmask_build(mask_id, params, bm)
    assert_blockmask_equal(bm, fo.create_block_mask(mask, 1, 1, Sq, Skv, Bq, Bk))
    assert int((bm.q_num_blocks + bm.full_q_num_blocks).max()) > 1024
    Qd, Kd, Vd, dOd = (t.to(DEV) for t in (Q, K, V, dO))
    O = torch.full_like(Qd, float("nan"))
    LSE = torch.full((B, H, Sq), float("nan"), dtype=torch.float32, device=DEV)
    fa.flexattn_forward(Qd, Kd, Vd, fa.SCORE_IDENTITY, mask_id, params, bm, scale, O, LSE)
    dQ, dK, dV = (torch.full_like(t, float("nan")) for t in (Qd, Kd, Vd))
    fa.flexattn_backward(Qd, Kd, Vd, O, dOd, LSE, fa.SCORE_IDENTITY, mask_id, params, bm, scale, dQ, dK, dV)
    torch.cuda.synchronize()
    O_ref, LSE_ref = fo.flex_attention(Q, K, V, fo.Identity(), mask, scale)
    check_output(O, LSE, O_ref, LSE_ref)
    g_ref = fo.flex_attention_backward(Q, K, V, dO, fo.Identity(), mask, scale)
    for n, g, r in zip(("dQ", "dK", "dV"), (dQ, dK, dV), g_ref):
        check_grad(n, g, r)


@pytest.mark.parametrize("mask_name,D", [("causal", 128), ("none", 64)])
def test_running_maximum_that_moves_late_and_far(mask_name, D):
    """The forward moves a row's running maximum only when a block exceeds it by more than 2^8.  Keys whose
    scores grow along the sequence (small steps that stay below the threshold, then jumps far above it) and a
    first block of scores near -300 (whose 2^-max would overflow) must give the oracle's O and LSE."""
    import paper_2412_05496_amd as fa
    B, H, S = 1, 2, 1024
    gen = torch.Generator().manual_seed(4242 + D)
    Q = torch.randn(B, H, S, D, generator=gen)
    K = torch.randn(B, H, S, D, generator=gen)
    V = torch.randn(B, H, S, D, generator=gen)
    ramp = torch.cat([torch.linspace(0.02, 0.6, 512), torch.linspace(0.6, 0.7, 256), torch.linspace(3.0, 6.0, 256)])
    K = K * ramp.view(1, 1, S, 1)
    # head 1: every query has a positive mean, the first 32 keys a large negative one: scores of about -300 there
    Q[:, 1] = Q[:, 1] * 0.2 + 1.0
    K[:, 1, :32] = -300.0 / D
    Q, K, V = (t.to(torch.bfloat16).float() for t in (Q, K, V))
    scale = 1.0 / D ** 0.5 * 4.0
    mask = fo.causal_mask if mask_name == "causal" else fo.no_mask
    O_ref, LSE_ref = fo.flex_attention(Q, K, V, fo.Identity(), mask, scale)
    Qd, Kd, Vd = (t.to(torch.bfloat16).to(DEV) for t in (Q, K, V))
    mask_id = fa.MASK_CAUSAL if mask_name == "causal" else fa.MASK_NONE
    params = fa.ModParams()
    bm = fa.alloc_blockmask(1, 1, S, S, 128, 64, device=DEV)
    fa.flexattn_blockmask_build(mask_id, params, bm)
    O = torch.full_like(Qd, float("nan"))
    LSE = torch.full((B, H, S), float("nan"), dtype=torch.float32, device=DEV)
    fa.flexattn_forward(Qd, Kd, Vd, fa.SCORE_IDENTITY, mask_id, params, bm, scale, O, LSE)
    torch.cuda.synchronize()
    print(f"[case] lazy maximum {mask_name} D={D}: LSE range {float(LSE_ref.min()):.1f} .. {float(LSE_ref.max()):.1f}", flush=True)
    check_output(O, LSE, O_ref, LSE_ref)
