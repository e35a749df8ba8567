"""GPU parity of the paged split-KV decode against the oracle (which un-pages the cache and applies
Eq. 1 with one query row).  O: max abs <= 2e-2, mean abs <= 2e-3; LSE <= 1e-2."""
import pytest
import torch

import flex_workloads as wlm
from oracle import flex_oracle as fo

from helpers import check_output

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_decode(inp, score_id=0, params=None, mask_id=None):
    import paper_2412_05496_amd as fa
    params = params or fa.ModParams()
    mask_id = fa.MASK_CTX_LEN if mask_id is None else mask_id
    Q = inp.Q.to(DEV)
    O = torch.full((Q.shape[0], Q.shape[1], Q.shape[3]), float("nan"), dtype=torch.bfloat16, device=DEV)
    LSE = torch.full((Q.shape[0], Q.shape[1]), float("nan"), dtype=torch.float32, device=DEV)
    fa.flexattn_paged_decode(Q, inp.K_pool.to(DEV), inp.V_pool.to(DEV), inp.page_table.to(DEV),
                             inp.ctx_lens.to(DEV), score_id, mask_id, params, inp.scale, O, LSE)
    torch.cuda.synchronize()
    return O, LSE


def compare(inp, O, LSE, score_mod, mask_mod=None):
    O_ref, LSE_ref = fo.paged_decode(inp.Q, inp.K_pool, inp.V_pool, inp.page_table, inp.ctx_lens, score_mod, inp.scale,
                                     mask_mod)
    check_output(O[:, :, None, :], LSE[:, :, None], O_ref, LSE_ref)


def test_ragged_lengths_and_edge_cases():
    # lengths around the page (16), tile (64) and split (512) boundaries, one empty sequence
    ctx = [0, 1, 15, 16, 17, 63, 64, 65, 511, 512, 513, 1023, 1500, 2048, 700, 33]
    wl = wlm.CFG5.scaled(B=len(ctx), max_pages=128)
    inp = wlm.make_decode_inputs(wl, ctx_lens=ctx, slack_pages=7)
    print(f"[case] ragged ctx={ctx}", flush=True)
    O, LSE = run_decode(inp)
    assert (O[0] == 0).all() and torch.isinf(LSE[0]).all()
    compare(inp, O, LSE, fo.Identity())


@pytest.mark.parametrize("D,G,page", [(128, 4, 16), (64, 1, 16), (128, 4, 32), (64, 2, 32), (128, 8, 64), (64, 4, 128),
                                      (128, 4, 256), (64, 2, 256), (128, 2, 512)])
def test_shapes_and_page_sizes(D, G, page):
    wl = wlm.CFG5.scaled(B=6, Hq=2 * G, Hkv=2, D=D, page_size=page, ctx_min=1, ctx_max=3000,
                         max_pages=(3000 + page - 1) // page + 1)
    inp = wlm.make_decode_inputs(wl, slack_pages=3)
    print(f"[case] D={D} G={G} page={page} ctx={inp.ctx_lens.tolist()}", flush=True)
    O, LSE = run_decode(inp)
    compare(inp, O, LSE, fo.Identity())


@pytest.mark.parametrize("window", [0, 5, 31, 32, 100, 511, 512, 1300, 5000])
def test_sliding_window_in_decode(window):
    """Decode with a q-dependent mask: the query sits at q_idx = ctx_len - 1, so the window keeps
    kv >= ctx_len - 1 - window; splits wholly below it are skipped by the kernel."""
    import paper_2412_05496_amd as fa
    ctx = [1, 17, 64, 511, 512, 513, 1024, 1500, 2047, 2600, 700, 33]
    wl = wlm.CFG5.scaled(B=len(ctx), Hq=8, Hkv=2, max_pages=192)
    inp = wlm.make_decode_inputs(wl, ctx_lens=ctx, slack_pages=5)
    print(f"[case] window={window} ctx={ctx}", flush=True)
    O, LSE = run_decode(inp, fa.SCORE_IDENTITY, fa.ModParams(window=window), fa.MASK_CTX_LEN_WINDOW)
    mask = fo.and_mask(fo.ctx_len_mask(inp.ctx_lens), fo.sliding_window_mask(window))
    compare(inp, O, LSE, fo.Identity(), mask)
    slopes = wlm.alibi_slopes(8)
    O, LSE = run_decode(inp, fa.SCORE_ALIBI, fa.ModParams(window=window, alibi_bias=(-slopes).to(DEV)),
                        fa.MASK_CTX_LEN_WINDOW)
    compare(inp, O, LSE, fo.Alibi(-slopes.double()), mask)


def test_score_mods_in_decode():
    import paper_2412_05496_amd as fa
    wl = wlm.CFG5.scaled(B=4, Hq=8, Hkv=2, ctx_min=100, ctx_max=2000, max_pages=128)
    inp = wlm.make_decode_inputs(wl)
    O, LSE = run_decode(inp, fa.SCORE_SOFTCAP, fa.ModParams(softcap=2.0))
    compare(inp, O, LSE, fo.Softcap(2.0))
    slopes = wlm.alibi_slopes(8)
    O, LSE = run_decode(inp, fa.SCORE_ALIBI, fa.ModParams(alibi_bias=(-slopes).to(DEV)))
    compare(inp, O, LSE, fo.Alibi(-slopes.double()))


def test_relative_bias_in_decode():
    import paper_2412_05496_amd as fa
    wl = wlm.CFG5.scaled(B=5, Hq=8, Hkv=2, ctx_min=50, ctx_max=2500, max_pages=160)
    inp = wlm.make_decode_inputs(wl)
    table = torch.randn(8, 256, generator=torch.Generator().manual_seed(9)) * 0.5
    O, LSE = run_decode(inp, fa.SCORE_REL_BIAS, fa.ModParams(rel_bias=table.to(DEV)))
    compare(inp, O, LSE, fo.RelBias(table.double()))


@pytest.mark.parametrize("nseq,Hkv,ctx_max", [(1, 8, 8192), (2, 1, 20000), (3, 2, 700)])
def test_small_batches_are_cut_into_short_splits(nseq, Hkv, ctx_max):
    """The split length follows nseq * Hkv * (longest addressable context), so a small batch is cut into
    128 ... 512-key splits and a (sequence, head) is combined from many more partials than config 5's."""
    wl = wlm.CFG5.scaled(B=nseq, Hq=4 * Hkv, Hkv=Hkv, ctx_min=max(ctx_max - 300, 1), ctx_max=ctx_max,
                         max_pages=(ctx_max + 15) // 16)
    inp = wlm.make_decode_inputs(wl, slack_pages=2)
    print(f"[case] small batch nseq={nseq} Hkv={Hkv} ctx={inp.ctx_lens.tolist()}", flush=True)
    O, LSE = run_decode(inp)
    compare(inp, O, LSE, fo.Identity())


def test_wrong_tables_never_leave_the_buffers():
    """Device-side values are not trusted: page ids outside the pool and context lengths beyond what the
    page table addresses (or negative) are clamped, so the call returns normally with finite numbers --
    wrong rows, never an access outside the table, the pools or the workspace."""
    wl = wlm.CFG5.scaled(B=6, Hq=8, Hkv=2, ctx_min=100, ctx_max=1500, max_pages=96)
    inp = wlm.make_decode_inputs(wl, slack_pages=1)
    good_O, good_LSE = run_decode(inp)
    pt = inp.page_table.clone()
    pt[0, 0] = 2 ** 30                      # far past the pool
    pt[1, 1] = -7                           # negative
    pt[2, :] = inp.K_pool.shape[0]          # one past the last page, everywhere
    ctx = inp.ctx_lens.clone()
    ctx[3] = 96 * 16 + 5000                 # longer than the page table can address
    ctx[4] = -3                             # negative: treated as empty
    bad = wlm.DecodeInputs(wl, inp.Q, inp.K_pool, inp.V_pool, pt.contiguous(), ctx.contiguous(), inp.scale)
    O, LSE = run_decode(bad)
    assert torch.isfinite(O.float()).all()
    assert torch.isfinite(LSE[[0, 1, 2, 3, 5]]).all()
    assert (O[4] == 0).all() and torch.isinf(LSE[4]).all()
    # the untouched sequence is unaffected, bit for bit
    assert torch.equal(O[5], good_O[5]) and torch.equal(LSE[5], good_LSE[5])
    # a clamped id reads the nearest valid page: the same result as a table that names that page
    fixed = pt.clone()
    fixed[0, 0] = inp.K_pool.shape[0] - 1
    fixed[1, 1] = 0
    fixed[2, :] = inp.K_pool.shape[0] - 1
    ctx_fixed = ctx.clone()
    ctx_fixed[3] = 96 * 16
    ctx_fixed[4] = 0
    O2, LSE2 = run_decode(wlm.DecodeInputs(wl, inp.Q, inp.K_pool, inp.V_pool, fixed.contiguous(),
                                           ctx_fixed.contiguous(), inp.scale))
    assert torch.equal(O, O2) and torch.equal(LSE, LSE2)


def test_full_config5():
    wl = wlm.CFG5
    inp = wlm.make_decode_inputs(wl)
    print(f"[case] cfg5 total tokens {int(inp.ctx_lens.sum())}", flush=True)
    O, LSE = run_decode(inp)
    compare(inp, O, LSE, fo.Identity())


def test_pool_permutation_invariance_bit_exact():
    wl = wlm.CFG5.scaled(B=5, ctx_min=10, ctx_max=1500, max_pages=128)
    inp = wlm.make_decode_inputs(wl)
    O1, L1 = run_decode(inp)
    n_pool = inp.K_pool.shape[0]
    perm = torch.randperm(n_pool, generator=torch.Generator().manual_seed(3))
    inv = torch.empty_like(perm)
    inv[perm] = torch.arange(n_pool)
    inp2 = wlm.DecodeInputs(wl, inp.Q, inp.K_pool[perm].contiguous(), inp.V_pool[perm].contiguous(),
                            inv[inp.page_table.long()].to(torch.int32).contiguous(), inp.ctx_lens, inp.scale)
    O2, L2 = run_decode(inp2)
    assert torch.equal(O1, O2) and torch.equal(L1, L2)
