"""GPU parity of the neighborhood-attention masks (appendix, Neighborhood Attention) in the three
token orders: BlockMask bit for bit, forward and backward against the oracle, through the C ABI."""
import pytest
import torch

import flex_workloads as wlm
from oracle import flex_oracle as fo
from tests import helpers as hp

pytestmark = pytest.mark.gpu

LAYOUT_ID = {"row_major": 0, "tiled": 1, "morton": 2}

CANVASES = [
    # W, H, K, layout, tile, Bq, Bk
    (32, 32, 7, "row_major", 0, 128, 64),
    (24, 16, 5, "row_major", 0, 64, 64),        # width not a power of two
    (24, 16, 5, "tiled", 8, 64, 64),            # three tiles per canvas row
    (48, 32, 9, "tiled", 4, 128, 64),
    (32, 32, 7, "tiled", 8, 128, 64),
    (32, 32, 7, "morton", 0, 128, 64),
    (16, 16, 15, "morton", 0, 64, 64),          # window almost the whole canvas
    (16, 16, 1, "row_major", 0, 64, 64),        # every pixel sees only itself
]


def na_params(fa, W, H, K, layout, tile):
    return fa.ModParams(na_width=W, na_height=H, na_kernel=K, na_layout=LAYOUT_ID[layout], na_tile=tile)


@pytest.mark.parametrize("canvas", CANVASES, ids=[f"{c[0]}x{c[1]}_k{c[2]}_{c[3]}{c[4] or ''}" for c in CANVASES])
def test_blockmask_bit_exact(canvas):
    import paper_2412_05496_amd as fa
    W, H, K, layout, tile, Bq, Bk = canvas
    dev = torch.device("cuda:0")
    S = W * H
    bm = fa.alloc_blockmask(1, 1, S, S, Bq, Bk, device=dev)
    fa.flexattn_blockmask_build(fa.MASK_NEIGHBORHOOD, na_params(fa, W, H, K, layout, tile), bm)
    torch.cuda.synchronize()
    ref = fo.create_block_mask(fo.neighborhood_mask(W, H, K, layout, tile), 1, 1, S, S, Bq, Bk)
    assert ref["stats"]["unmasked_pairs"] == S * K * K
    hp.assert_blockmask_equal(bm, ref)


@pytest.mark.parametrize("layout,tile", [("row_major", 0), ("tiled", 8), ("morton", 0)])
@pytest.mark.parametrize("D", [64, 128])
def test_forward_backward_match_oracle(layout, tile, D):
    import paper_2412_05496_amd as fa
    W = H = 32
    K = 7
    dev = torch.device("cuda:0")
    wl = wlm.CFG1.scaled(name=f"na_{layout}_d{D}", B=1, Hq=2, Hkv=1, S=W * H, D=D, Bq=128, Bk=64, mask="none",
                         score="identity", seed=3400 + D + len(layout), backward=True)
    inp = wlm.make_train_inputs(wl, with_dO=True)
    mask_mod = fo.neighborhood_mask(W, H, K, layout, tile)
    O_ref, LSE_ref = fo.flex_attention(inp.Q, inp.K, inp.V, fo.Identity(), mask_mod, inp.scale)
    dQ_ref, dK_ref, dV_ref = fo.flex_attention_backward(inp.Q, inp.K, inp.V, inp.dO, fo.Identity(), mask_mod, inp.scale)

    params = na_params(fa, W, H, K, layout, tile)
    bm = fa.alloc_blockmask(1, 1, wl.S, wl.S, wl.Bq, wl.Bk, device=dev)
    fa.flexattn_blockmask_build(fa.MASK_NEIGHBORHOOD, params, bm)
    Q, Kd, V, dO = inp.Q.to(dev), inp.K.to(dev), inp.V.to(dev), inp.dO.to(dev)
    O = torch.full_like(Q, float("nan"))
    LSE = torch.full(Q.shape[:3], float("nan"), dtype=torch.float32, device=dev)
    fa.flexattn_forward(Q, Kd, V, fa.SCORE_IDENTITY, fa.MASK_NEIGHBORHOOD, params, bm, inp.scale, O, LSE)
    dQ, dK, dV = torch.full_like(Q, float("nan")), torch.full_like(Kd, float("nan")), torch.full_like(V, float("nan"))
    fa.flexattn_backward(Q, Kd, V, O, dO, LSE, fa.SCORE_IDENTITY, fa.MASK_NEIGHBORHOOD, params, bm, inp.scale, dQ, dK, dV)
    torch.cuda.synchronize()
    hp.check_output(O, LSE, O_ref, LSE_ref)
    hp.check_grad("dQ", dQ, dQ_ref)
    hp.check_grad("dK", dK, dK_ref)
    hp.check_grad("dV", dV, dV_ref)


def test_bad_canvas_parameters_are_refused():
    import paper_2412_05496_amd as fa
    dev = torch.device("cuda:0")
    bm = fa.alloc_blockmask(1, 1, 1024, 1024, 128, 64, device=dev)
    bad = [dict(na_width=32, na_height=32, na_kernel=4),                                  # even kernel
           dict(na_width=32, na_height=32, na_kernel=33),                                 # larger than the canvas
           dict(na_width=32, na_height=16, na_kernel=3),                                  # not q_len tokens
           dict(na_width=64, na_height=16, na_kernel=3, na_layout=2),                     # Morton needs a square
           dict(na_width=32, na_height=32, na_kernel=3, na_layout=1, na_tile=6),          # tile not a power of two
           dict(na_width=32, na_height=32, na_kernel=3, na_layout=3)]
    for kw in bad:
        with pytest.raises(fa.FlexAttnError):
            fa.flexattn_blockmask_build(fa.MASK_NEIGHBORHOOD, fa.ModParams(**kw), bm)


@pytest.mark.parametrize("layout,tile", [("row_major", 0), ("tiled", 8), ("tiled", 32), ("morton", 0)])
def test_blockmask_on_a_large_canvas_sampled_blocks(layout, tile):
    """128 x 128 pixels (16384 tokens): the kind of 300 sampled blocks, and the unmasked-pair count of the
    whole mask, against the oracle's mask evaluated on those blocks only."""
    import paper_2412_05496_amd as fa
    W = H = 128
    K, Bq, Bk = 13, 128, 64
    S = W * H
    dev = torch.device("cuda:0")
    bm = fa.alloc_blockmask(1, 1, S, S, Bq, Bk, device=dev)
    fa.flexattn_blockmask_build(fa.MASK_NEIGHBORHOOD, na_params(fa, W, H, K, layout, tile), bm)
    torch.cuda.synchronize()
    stats = bm.stats.cpu().tolist()
    assert stats[3] == S * K * K and stats[2] == (S // Bq) * (S // Bk)
    num, idx = bm.kv_num_blocks.cpu()[0, 0], bm.kv_indices.cpu()[0, 0]
    fnum, fidx = bm.full_kv_num_blocks.cpu()[0, 0], bm.full_kv_indices.cpu()[0, 0]
    mask = fo.neighborhood_mask(W, H, K, layout, tile)
    g = torch.Generator().manual_seed(17)
    rows = torch.randint(0, S // Bq, (300,), generator=g).tolist()
    cols = torch.randint(0, S // Bk, (300,), generator=g).tolist()
    # bias the sample towards blocks that are not empty: half of them are taken from the lists
    for n, i in enumerate(rows[:150]):
        if int(num[i]) > 0:
            cols[n] = int(idx[i, n % int(num[i])])
    for i, j in zip(rows, cols):
        keep = mask(0, 0, torch.arange(i * Bq, (i + 1) * Bq).view(-1, 1), torch.arange(j * Bk, (j + 1) * Bk).view(1, -1))
        cnt = int(keep.sum())
        want = 0 if cnt == 0 else (2 if cnt == Bq * Bk else 1)
        got = 1 if j in idx[i, :int(num[i])].tolist() else (2 if j in fidx[i, :int(fnum[i])].tolist() else 0)
        assert got == want, (i, j, got, want)
