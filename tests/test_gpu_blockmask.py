"""GPU parity of the BlockMask builder and the paged conversion: bit-exact against the oracle's
brute force, at small sizes and at the full sizes of the benchmark workloads."""
import pytest
import torch

import flex_workloads as wlm
from oracle import flex_oracle as fo

from helpers import assert_blockmask_equal

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def build(mask_id, params, Bm, Hm, q_len, kv_len, Bq, Bk):
    import paper_2412_05496_amd as fa
    bm = fa.alloc_blockmask(Bm, Hm, q_len, kv_len, Bq, Bk, device=DEV)
    for name in ("kv_indices", "full_kv_indices", "q_indices", "full_q_indices"):
        getattr(bm, name).fill_(-7)            # the builder must overwrite every entry, tails included
    fa.flexattn_blockmask_build(mask_id, params, bm)
    torch.cuda.synchronize()
    return bm


def test_every_mask_small_odd_blocks():
    import paper_2412_05496_amd as fa
    q_len, kv_len, Bq, Bk = 96, 160, 8, 16        # rectangular, many blocks, non-square blocks
    doc = wlm.document_ids([23, 50, 7, 80])[None, :].contiguous()
    ctx = torch.tensor([37, 160, 0], dtype=torch.int32)
    cases = [
        (fa.MASK_NONE, fa.ModParams(), fo.no_mask, 1),
        (fa.MASK_CAUSAL, fa.ModParams(), fo.causal_mask, 1),
        (fa.MASK_SLIDING_WINDOW, fa.ModParams(window=11), fo.sliding_window_mask(11), 1),
        (fa.MASK_SWA_CAUSAL, fa.ModParams(window=30), fo.and_mask(fo.causal_mask, fo.sliding_window_mask(30)), 1),
        (fa.MASK_DOCUMENT, fa.ModParams(doc_ids=doc.to(DEV)), fo.document_mask(doc), 1),
        (fa.MASK_DOCUMENT_CAUSAL, fa.ModParams(doc_ids=doc.to(DEV)), fo.and_mask(fo.document_mask(doc), fo.causal_mask), 1),
        (fa.MASK_PREFIX_LM, fa.ModParams(prefix_len=45), fo.or_mask(fo.causal_mask, fo.prefix_mask(45)), 1),
        (fa.MASK_SWA_CAUSAL_OR_PREFIX, fa.ModParams(window=20, prefix_len=19),
         fo.or_mask(fo.and_mask(fo.causal_mask, fo.sliding_window_mask(20)), fo.prefix_mask(19)), 1),
        (fa.MASK_CTX_LEN, fa.ModParams(ctx_lens=ctx.to(DEV)), fo.ctx_len_mask(ctx), 3),
    ]
    for mask_id, params, mod, Bm in cases:
        print(f"[case] mask_id={mask_id:#x}", flush=True)
        bm = build(mask_id, params, Bm, 1, q_len, kv_len, Bq, Bk)
        assert_blockmask_equal(bm, fo.create_block_mask(mod, Bm, 1, q_len, kv_len, Bq, Bk))


def test_per_head_broadcast_dims():
    import paper_2412_05496_amd as fa
    bm = build(fa.MASK_CAUSAL, fa.ModParams(), 2, 3, 256, 256, 64, 64)
    ref = fo.create_block_mask(fo.causal_mask, 2, 3, 256, 256, 64, 64)
    assert_blockmask_equal(bm, ref)


@pytest.mark.parametrize("cfg", ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
def test_full_size_configs(cfg):
    import paper_2412_05496_amd as fa
    print(f"[case] {cfg}", flush=True)
    if cfg == "cfg1":
        wl = wlm.CFG1
        bm = build(fa.MASK_CAUSAL, fa.ModParams(), 1, 1, wl.S, wl.S, wl.Bq, wl.Bk)
        ref = fo.create_block_mask(fo.causal_mask, 1, 1, wl.S, wl.S, wl.Bq, wl.Bk)
    elif cfg == "cfg2":
        wl = wlm.CFG2
        bm = build(fa.MASK_CAUSAL, fa.ModParams(), 1, 1, wl.S, wl.S, wl.Bq, wl.Bk)
        ref = fo.create_block_mask(fo.causal_mask, 1, 1, wl.S, wl.S, wl.Bq, wl.Bk)
        assert bm.stats.cpu().tolist() == [128, 4032, 8192, wl.S * (wl.S + 1) // 2]
    elif cfg == "cfg3":
        wl = wlm.CFG3
        g = torch.Generator().manual_seed(wl.seed)
        doc = wlm.document_ids(wlm.document_lengths(g, wl.S, wl.doc_len_min, wl.doc_len_max))[None, :].contiguous()
        bm = build(fa.MASK_DOCUMENT_CAUSAL, fa.ModParams(doc_ids=doc.to(DEV)), 1, 1, wl.S, wl.S, wl.Bq, wl.Bk)
        ref = fo.create_block_mask(fo.and_mask(fo.document_mask(doc), fo.causal_mask), 1, 1, wl.S, wl.S, wl.Bq, wl.Bk)
    elif cfg == "cfg4":
        wl = wlm.CFG4
        bm = build(fa.MASK_SWA_CAUSAL_OR_PREFIX, fa.ModParams(window=wl.window, prefix_len=wl.prefix_len), 1, 1,
                   wl.S, wl.S, wl.Bq, wl.Bk)
        mod = fo.or_mask(fo.and_mask(fo.causal_mask, fo.sliding_window_mask(wl.window)), fo.prefix_mask(wl.prefix_len))
        ref = fo.create_block_mask(mod, 1, 1, wl.S, wl.S, wl.Bq, wl.Bk)
        assert bm.stats.cpu().tolist() == [928, 18480, 131072, 155218944]
    else:
        wl = wlm.CFG5
        inp = wlm.make_decode_inputs(wl.scaled(D=8, Hq=1, Hkv=1))       # only ctx_lens / page table matter here
        kv_len = wl.max_pages * wl.page_size
        bm = build(fa.MASK_CTX_LEN, fa.ModParams(ctx_lens=inp.ctx_lens.to(DEV)), wl.B, 1, 1, kv_len, 1, wl.page_size)
        ref = fo.create_block_mask(fo.ctx_len_mask(inp.ctx_lens), wl.B, 1, 1, kv_len, 1, wl.page_size)
    assert_blockmask_equal(bm, ref)


def test_paged_conversion_matches_oracle():
    import paper_2412_05496_amd as fa
    wl = wlm.CFG5.scaled(B=8, D=8, Hq=1, Hkv=1, ctx_min=1, ctx_max=1000, max_pages=64)
    inp = wlm.make_decode_inputs(wl, slack_pages=5)
    kv_len = wl.max_pages * wl.page_size
    bm = build(fa.MASK_CTX_LEN, fa.ModParams(ctx_lens=inp.ctx_lens.to(DEV)), wl.B, 1, 1, kv_len, 1, wl.page_size)
    n_pool = inp.K_pool.shape[0]
    pt = inp.page_table.to(DEV)
    for num_name, idx_name in (("kv_num_blocks", "kv_indices"), ("full_kv_num_blocks", "full_kv_indices")):
        phys = torch.full_like(getattr(bm, idx_name), -7)
        p2l = torch.full((n_pool,), -1, dtype=torch.int32, device=DEV)
        fa.flexattn_paged_convert_blockmask(getattr(bm, num_name), getattr(bm, idx_name), pt, phys, p2l)
        torch.cuda.synchronize()
        phys_ref, p2l_ref = fo.convert_block_mask_paged(getattr(bm, num_name).cpu(), getattr(bm, idx_name).cpu(),
                                                        inp.page_table, n_pool)
        assert torch.equal(phys.cpu(), phys_ref) and torch.equal(p2l.cpu(), p2l_ref)
        # counts are untouched by the conversion
        assert torch.equal(getattr(bm, num_name).cpu(), fo.create_block_mask(
            fo.ctx_len_mask(inp.ctx_lens), wl.B, 1, 1, kv_len, 1, wl.page_size)[num_name])
