"""Pins for the oracle's neighborhood-attention masks (appendix, Neighborhood Attention): textbook
values of the three token layouts, the size and place of the neighborhoods by brute force, equality of
the attention output across layouts up to the permutation of the tokens, and the paper's qualitative
claim that the tiled and Morton layouts leave fewer blocks to compute."""
import torch

from oracle import flex_oracle as fo


def test_layouts_are_permutations_with_textbook_values():
    W = H = 8
    for layout, tile in (("row_major", 0), ("tiled", 4), ("morton", 0)):
        idx = sorted(fo.na_token_index(x, y, W, H, layout, tile) for y in range(H) for x in range(W))
        assert idx == list(range(W * H)), layout
    # Z-order curve: (x, y) = (1,0) (0,1) (1,1) (2,0) (3,1) (0,2) (7,7)
    z = lambda x, y: fo.na_token_index(x, y, 8, 8, "morton")
    assert [z(1, 0), z(0, 1), z(1, 1), z(2, 0), z(3, 1), z(0, 2), z(7, 7)] == [1, 2, 3, 4, 7, 8, 63]
    # 4 x 4 tiles on an 8-wide canvas: tile (1, 0) starts at 16, tile (0, 1) at 32; inside a tile row-major
    t = lambda x, y: fo.na_token_index(x, y, 8, 8, "tiled", 4)
    assert [t(0, 0), t(3, 0), t(0, 1), t(4, 0), t(0, 4), t(5, 6)] == [0, 3, 4, 16, 32, 48 + 2 * 4 + 1]
    xs, ys = fo.na_token_xy(8, 8, "tiled", 4)
    assert (int(xs[16]), int(ys[16])) == (4, 0) and (int(xs[57]), int(ys[57])) == (5, 6)


def test_every_query_sees_the_nearest_kernel_squared_pixels():
    W, H, K = 12, 8, 5
    mask = fo.neighborhood_mask(W, H, K)
    n = W * H
    keep = mask(0, 0, torch.arange(n).view(-1, 1), torch.arange(n).view(1, -1))
    assert (keep.sum(dim=1) == K * K).all()
    # interior pixel (6, 4): the window centred on it
    want = {(y * W + x) for y in range(2, 7) for x in range(4, 9)}
    assert set(torch.nonzero(keep[4 * W + 6]).flatten().tolist()) == want
    # corner (0, 0) and edge pixel (11, 3): the window moved inside the canvas
    assert set(torch.nonzero(keep[0]).flatten().tolist()) == {(y * W + x) for y in range(5) for x in range(5)}
    assert set(torch.nonzero(keep[3 * W + 11]).flatten().tolist()) == {(y * W + x) for y in range(1, 6) for x in range(7, 12)}
    # every key of a query is at least as near (Chebyshev) as every non-key, up to the shift at the border:
    # for interior queries the kept set is exactly the ball of radius K // 2
    for qy in range(2, H - 2):
        for qx in range(2, W - 2):
            row = keep[qy * W + qx].view(H, W)
            for y in range(H):
                for x in range(W):
                    assert bool(row[y, x]) == (max(abs(x - qx), abs(y - qy)) <= 2)
    # kernel as large as the canvas: nothing is masked
    full = fo.neighborhood_mask(7, 7, 7)(0, 0, torch.arange(49).view(-1, 1), torch.arange(49).view(1, -1))
    assert full.all()


def test_attention_is_the_same_in_every_layout_up_to_the_token_permutation():
    W = H = 8
    K, D = 3, 8
    n = W * H
    g = torch.Generator().manual_seed(77)
    Q, Kt, V = (torch.randn(1, 2, n, D, generator=g, dtype=torch.float64) for _ in range(3))
    O0, L0 = fo.flex_attention(Q, Kt, V, fo.Identity(), fo.neighborhood_mask(W, H, K), 0.35)
    for layout, tile in (("tiled", 4), ("tiled", 2), ("morton", 0)):
        # token i of this layout is the pixel that row-major token perm[i] holds
        xs, ys = fo.na_token_xy(W, H, layout, tile)
        perm = ys * W + xs
        O1, L1 = fo.flex_attention(Q[:, :, perm], Kt[:, :, perm], V[:, :, perm], fo.Identity(),
                                   fo.neighborhood_mask(W, H, K, layout, tile), 0.35)
        assert torch.allclose(O1, O0[:, :, perm], atol=1e-14, rtol=0), layout
        assert torch.allclose(L1, L0[:, :, perm], atol=1e-14, rtol=0), layout


def test_tiled_and_morton_layouts_leave_fewer_blocks_for_large_neighborhoods():
    # the paper's point (appendix, mask figures): the same neighborhoods touch fewer blocks once the
    # tokens of a 2-D patch are contiguous.  It holds once the neighborhood spans many canvas rows
    # (64 x 64 canvas, 13 x 13 kernel); a small kernel on a narrow canvas is already compact row by row.
    W = H = 64
    counts = {}
    for K in (13, 3):
        for layout, tile in (("row_major", 0), ("tiled", 8), ("morton", 0)):
            kinds, pairs = fo.block_kinds(fo.neighborhood_mask(W, H, K, layout, tile), 1, 1, W * H, W * H, 128, 64)
            assert pairs == W * H * K * K
            counts[K, layout] = int((kinds > 0).sum())
    assert counts[13, "tiled"] < counts[13, "row_major"] and counts[13, "morton"] < counts[13, "row_major"]
    assert counts[3, "row_major"] <= counts[3, "tiled"]
