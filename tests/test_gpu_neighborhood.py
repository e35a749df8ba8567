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
