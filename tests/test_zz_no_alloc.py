"""flexattn_paged_decode_static (the entry point that allocates nothing: its workspace is an array in
the library's device image) against flexattn_paged_decode on a caller-owned workspace: same kernels,
so O and LSE must agree bit for bit -- on two calls in a row, the second with a smaller input, so that
what the first call left in the shared array is seen not to matter."""
import pytest
import torch

import flex_workloads as wlm

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def both(inp, score_id, params):
    import paper_2412_05496_amd as fa
    Q, Kp, Vp = inp.Q.to(DEV), inp.K_pool.to(DEV), inp.V_pool.to(DEV)
    pt, ctx = inp.page_table.to(DEV), inp.ctx_lens.to(DEV)
    out = []
    for fn in (fa.flexattn_paged_decode, fa.flexattn_paged_decode_static):
        O = torch.full((Q.shape[0], Q.shape[1], Q.shape[3]), float("nan"), dtype=torch.bfloat16, device=DEV)
        LSE = torch.full((Q.shape[0], Q.shape[1]), float("nan"), dtype=torch.float32, device=DEV)
        fn(Q, Kp, Vp, pt, ctx, score_id, fa.MASK_CTX_LEN, params, inp.scale, O, LSE)
        torch.cuda.synchronize()
        out.append((O, LSE))
    return out


def test_static_workspace_decode_matches_the_workspace_call_twice_in_a_row():
    import paper_2412_05496_amd as fa
    assert fa.flexattn_paged_decode_static_capacity() == 40 << 20
    big = wlm.make_decode_inputs(wlm.CFG5.scaled(B=24, ctx_min=200, ctx_max=9000, max_pages=600))
    small = wlm.make_decode_inputs(wlm.CFG5.scaled(B=3, Hq=8, Hkv=2, D=64, ctx_min=1, ctx_max=700, max_pages=48,
                                                   seed=77))
    for name, inp, score_id, params in (("large", big, fa.SCORE_IDENTITY, fa.ModParams()),
                                        ("small", small, fa.SCORE_SOFTCAP, fa.ModParams(softcap=20.0))):
        print(f"[case] static decode, {name}: ctx {inp.ctx_lens.tolist()}", flush=True)
        (O_ws, L_ws), (O_st, L_st) = both(inp, score_id, params)
        assert torch.isfinite(O_ws.float()).all() and torch.isfinite(L_ws).all()
        assert torch.equal(O_st, O_ws) and torch.equal(L_st, L_ws)


def test_static_workspace_decode_refuses_what_does_not_fit():
    import paper_2412_05496_amd as fa
    # 256 sequences x 32 heads x 32 splits x 130 floats = 136 MB of partials: over the 40 MiB array
    wl = wlm.CFG5.scaled(B=256, ctx_min=16, ctx_max=64)
    inp = wlm.make_decode_inputs(wl)
    Q = inp.Q.to(DEV)
    O = torch.zeros((Q.shape[0], Q.shape[1], Q.shape[3]), dtype=torch.bfloat16, device=DEV)
    assert fa.flexattn_paged_decode_workspace_bytes(Q, inp.K_pool.to(DEV), inp.page_table.to(DEV)) > 40 << 20
    with pytest.raises(fa.FlexAttnError) as e:
        fa.flexattn_paged_decode_static(Q, inp.K_pool.to(DEV), inp.V_pool.to(DEV), inp.page_table.to(DEV),
                                        inp.ctx_lens.to(DEV), fa.SCORE_IDENTITY, fa.MASK_CTX_LEN, fa.ModParams(),
                                        inp.scale, O)
    assert e.value.status == fa.ERR_WORKSPACE
