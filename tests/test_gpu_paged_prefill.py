"""GPU parity of the offset conversion (section 5.2) and of the paged forward for a chunk of query
tokens (sections 5.1 + 5.2) against the oracle, through the C ABI."""
import pytest
import torch

import flex_workloads as wlm
from oracle import flex_oracle as fo
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def build_and_convert(fa, dev, mask_id, params, nseq, q_len, kv_len_padded, Bq, page, page_table, n_pool):
    bm = fa.alloc_blockmask(nseq, 1, q_len, kv_len_padded, Bq, page, device=dev)
    fa.flexattn_blockmask_build(mask_id, params, bm)
    phys_kv, phys_full = torch.zeros_like(bm.kv_indices), torch.zeros_like(bm.full_kv_indices)
    p2l = torch.full((n_pool,), -1, dtype=torch.int32, device=dev)
    fa.flexattn_paged_convert_blockmask(bm.kv_num_blocks, bm.kv_indices, page_table, phys_kv, p2l)
    fa.flexattn_paged_convert_blockmask(bm.full_kv_num_blocks, bm.full_kv_indices, page_table, phys_full, p2l)
    return bm, phys_kv, phys_full, p2l


CASES = [
    # name, kv_lens, q_len, Bq, page, Hq, Hkv, D, mask, score, extra
    ("causal_d128", [700, 256, 1100], 256, 128, 64, 4, 2, 128, "causal", "identity", {}),
    ("causal_softcap_d128_p128", [1000, 384], 384, 128, 128, 4, 4, 128, "causal", "softcap", {"softcap": 30.0}),
    ("causal_alibi_d64_gqa", [900, 130, 64], 64, 64, 64, 8, 2, 64, "causal", "alibi", {}),
    ("swa_d64", [1500, 777], 128, 128, 64, 2, 2, 64, "swa_causal", "identity", {"window": 300}),
    ("softcap_unbounded_d128", [640, 320], 128, 64, 64, 2, 1, 128, "causal", "softcap", {"softcap": 50.0}),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_paged_chunk_matches_oracle(case):
    import paper_2412_05496_amd as fa
    name, kv_lens, q_len, Bq, page, Hq, Hkv, D, mask, score, extra = case
    dev = torch.device("cuda:0")
    nseq = len(kv_lens)
    max_pages = (max(kv_lens) + page - 1) // page
    wl = wlm.CFG5.scaled(name="prefill_" + name, B=nseq, Hq=Hq, Hkv=Hkv, D=D, page_size=page, max_pages=max_pages,
                         mask=mask, score=score, S=q_len, Bq=Bq, Bk=page, seed=3100 + len(name), **extra)
    inp = wlm.make_prefill_inputs(wl, kv_lens, q_len, slack_pages=3)
    slopes = wlm.alibi_slopes(Hq) if score == "alibi" else None

    # oracle: the user's mods, shifted inside paged_attention
    class Side:
        doc_ids = None
        rel_bias = None
    side = Side()
    side.slopes = slopes
    score_mod, mask_mod = hp.oracle_mods(wl, side)
    O_ref, LSE_ref = fo.paged_attention(inp.Q, inp.K_pool, inp.V_pool, inp.page_table, inp.kv_lens, inp.q_offsets,
                                        score_mod, mask_mod, inp.scale)

    mask_id, score_id, params, _ = hp.library_mods(wl, side, dev)
    params.q_offsets = inp.q_offsets.to(dev)
    page_table = inp.page_table.to(dev)
    n_pool = inp.K_pool.shape[0]
    bm, phys_kv, phys_full, p2l = build_and_convert(fa, dev, mask_id, params, nseq, q_len, max_pages * page, Bq, page,
                                                    page_table, n_pool)
    # BlockMask with offsets, bit for bit
    ref_bm = fo.create_block_mask(fo.with_q_offset(mask_mod, inp.q_offsets), nseq, 1, q_len, max_pages * page, Bq, page)
    hp.assert_blockmask_equal(bm, ref_bm)
    for phys, num, idx in ((phys_kv, "kv_num_blocks", "kv_indices"), (phys_full, "full_kv_num_blocks", "full_kv_indices")):
        want, _ = fo.convert_block_mask_paged(ref_bm[num], ref_bm[idx], inp.page_table, n_pool)
        assert torch.equal(phys.cpu(), want)

    Q = inp.Q.to(dev)
    O = torch.full_like(Q, float("nan"))
    LSE = torch.full(Q.shape[:3], float("nan"), dtype=torch.float32, device=dev)
    fa.flexattn_paged_forward(Q, inp.K_pool.to(dev), inp.V_pool.to(dev), score_id, mask_id, params, bm, phys_kv,
                              phys_full, inp.scale, O, LSE)
    torch.cuda.synchronize()
    hp.check_output(O, LSE, O_ref, LSE_ref)


def test_offset_conversion_in_the_contiguous_forward_and_backward():
    """q_offsets without paging: rows [off, off + Lq) of a longer causal problem, forward and backward."""
    import paper_2412_05496_amd as fa
    dev = torch.device("cuda:0")
    B, H, Lq, Lkv, D = 2, 2, 128, 512, 64
    wl = wlm.CFG2.scaled(name="offset_contig", B=B, Hq=H, Hkv=H, S=Lkv, D=D, Bq=64, Bk=64, softcap=20.0, seed=3201)
    inp = wlm.make_train_inputs(wl, with_dO=True)
    offs = torch.tensor([384, 200], dtype=torch.int32)
    Q, dO = inp.Q[:, :, :Lq].contiguous(), inp.dO[:, :, :Lq].contiguous()
    score_mod, mask_mod = fo.QOffset(fo.Softcap(20.0), offs), fo.with_q_offset(fo.causal_mask, offs)
    O_ref, LSE_ref = fo.flex_attention(Q, inp.K, inp.V, score_mod, mask_mod, inp.scale)
    dQ_ref, dK_ref, dV_ref = fo.flex_attention_backward(Q, inp.K, inp.V, dO, score_mod, mask_mod, inp.scale)

    params = fa.ModParams(softcap=20.0, q_offsets=offs.to(dev))
    bm = fa.alloc_blockmask(B, 1, Lq, Lkv, 64, 64, device=dev)
    fa.flexattn_blockmask_build(fa.MASK_CAUSAL, params, bm)
    hp.assert_blockmask_equal(bm, fo.create_block_mask(mask_mod, B, 1, Lq, Lkv, 64, 64))
    Qd, Kd, Vd, dOd = Q.to(dev), inp.K.to(dev), inp.V.to(dev), dO.to(dev)
    O = torch.full_like(Qd, float("nan"))
    LSE = torch.full(Qd.shape[:3], float("nan"), dtype=torch.float32, device=dev)
    fa.flexattn_forward(Qd, Kd, Vd, fa.SCORE_SOFTCAP, fa.MASK_CAUSAL, params, bm, inp.scale, O, LSE)
    dQ, dK, dV = torch.full_like(Qd, float("nan")), torch.full_like(Kd, float("nan")), torch.full_like(Vd, float("nan"))
    fa.flexattn_backward(Qd, Kd, Vd, O, dOd, LSE, fa.SCORE_SOFTCAP, fa.MASK_CAUSAL, params, bm, inp.scale, dQ, dK, dV)
    torch.cuda.synchronize()
    hp.check_output(O, LSE, O_ref, LSE_ref)
    hp.check_grad("dQ", dQ, dQ_ref)
    hp.check_grad("dK", dK, dK_ref)
    hp.check_grad("dV", dV, dV_ref)


def test_wrong_page_entries_stay_inside_the_pool():
    """Converted entries outside the pool are clamped: the call completes and gives finite numbers."""
    import paper_2412_05496_amd as fa
    dev = torch.device("cuda:0")
    wl = wlm.CFG5.scaled(name="prefill_clamp", B=1, Hq=2, Hkv=2, D=64, page_size=64, max_pages=4, seed=3301)
    inp = wlm.make_prefill_inputs(wl, [256], 64)
    params = fa.ModParams(q_offsets=inp.q_offsets.to(dev))
    bm, phys_kv, phys_full, _ = build_and_convert(fa, dev, fa.MASK_CAUSAL, params, 1, 64, 256, 64, 64,
                                                  inp.page_table.to(dev), inp.K_pool.shape[0])
    phys_full.fill_(2 ** 30)
    phys_kv.fill_(-5)
    Q = inp.Q.to(dev)
    O = torch.full_like(Q, float("nan"))
    LSE = torch.full(Q.shape[:3], float("nan"), dtype=torch.float32, device=dev)
    fa.flexattn_paged_forward(Q, inp.K_pool.to(dev), inp.V_pool.to(dev), fa.SCORE_IDENTITY, fa.MASK_CAUSAL, params, bm,
                              phys_kv, phys_full, inp.scale, O, LSE)
    torch.cuda.synchronize()
    assert torch.isfinite(O.float()).all() and torch.isfinite(LSE).all()
