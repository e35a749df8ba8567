"""Glue for the parity tests: turns a synthetic workload into (a) the oracle's mods and (b) the
library's ids + device-side parameters.  The two descriptions are written separately on purpose:
nothing of the method's arithmetic is shared between them."""
from __future__ import annotations

import torch

import flex_workloads as wlm
from oracle import flex_oracle as fo

# tolerances (bf16 kernel output vs fp64 oracle)
O_MAX, O_MEAN, LSE_MAX = 2e-2, 2e-3, 1e-2


def oracle_mods(wl: wlm.Workload, inp):
    if wl.mask == "causal":
        mask = fo.causal_mask
    elif wl.mask == "none":
        mask = fo.no_mask
    elif wl.mask == "doc_causal":
        mask = fo.and_mask(fo.document_mask(inp.doc_ids), fo.causal_mask)
    elif wl.mask == "swa_causal":
        mask = fo.and_mask(fo.causal_mask, fo.sliding_window_mask(wl.window))
    elif wl.mask == "prefix_lm":
        mask = fo.or_mask(fo.causal_mask, fo.prefix_mask(wl.prefix_len))
    elif wl.mask == "swa_causal_or_prefix":
        mask = fo.or_mask(fo.and_mask(fo.causal_mask, fo.sliding_window_mask(wl.window)), fo.prefix_mask(wl.prefix_len))
    else:
        raise ValueError(wl.mask)
    if wl.score == "identity":
        score = fo.Identity()
    elif wl.score == "softcap":
        score = fo.Softcap(wl.softcap)
    elif wl.score == "alibi":
        score = fo.Alibi(-inp.slopes.double())          # score - slope_h * (q - kv)
    elif wl.score == "rel_bias":
        score = fo.RelBias(inp.rel_bias.double())
    else:
        raise ValueError(wl.score)
    return score, mask


def library_mods(wl: wlm.Workload, inp, dev):
    import paper_2412_05496_amd as fa
    mask_id = {"causal": fa.MASK_CAUSAL, "none": fa.MASK_NONE, "doc_causal": fa.MASK_DOCUMENT_CAUSAL,
               "swa_causal": fa.MASK_SWA_CAUSAL, "prefix_lm": fa.MASK_PREFIX_LM,
               "swa_causal_or_prefix": fa.MASK_SWA_CAUSAL_OR_PREFIX}[wl.mask]
    score_id = {"identity": fa.SCORE_IDENTITY, "softcap": fa.SCORE_SOFTCAP, "alibi": fa.SCORE_ALIBI,
                "rel_bias": fa.SCORE_REL_BIAS}[wl.score]
    params = fa.ModParams(window=wl.window, prefix_len=wl.prefix_len, softcap=wl.softcap)
    if inp.doc_ids is not None:
        params.doc_ids = inp.doc_ids.to(dev)
    if inp.slopes is not None:
        params.alibi_bias = (-inp.slopes).to(dev)
    if inp.rel_bias is not None:
        params.rel_bias = inp.rel_bias.to(dev)
    Bm = wl.B if wl.mask == "doc_causal" else 1
    return mask_id, score_id, params, Bm


BM_NAMES = ("kv_num_blocks", "kv_indices", "full_kv_num_blocks", "full_kv_indices",
            "q_num_blocks", "q_indices", "full_q_num_blocks", "full_q_indices")


def assert_blockmask_equal(bm, ref):
    for name in BM_NAMES:
        got = getattr(bm, name).cpu()
        assert got.dtype == torch.int32 and got.shape == ref[name].shape, name
        assert torch.equal(got, ref[name]), name
    if bm.stats is not None:
        st = bm.stats.cpu().tolist()
        assert st == [ref["stats"]["partial"], ref["stats"]["full"], ref["stats"]["total"],
                      ref["stats"]["unmasked_pairs"]], st


def run_forward(wl, inp, dev):
    """BlockMask build + forward through the C ABI.  Returns (O, LSE, bm, ids)."""
    import paper_2412_05496_amd as fa
    mask_id, score_id, params, Bm = library_mods(wl, inp, dev)
    bm = fa.alloc_blockmask(Bm, 1, wl.S, wl.S, wl.Bq, wl.Bk, device=dev)
    fa.flexattn_blockmask_build(mask_id, params, bm)
    Q, K, V = inp.Q.to(dev), inp.K.to(dev), inp.V.to(dev)
    O = torch.full_like(Q, float("nan"))
    LSE = torch.full(Q.shape[:3], float("nan"), dtype=torch.float32, device=dev)
    fa.flexattn_forward(Q, K, V, score_id, mask_id, params, bm, inp.scale, O, LSE)
    torch.cuda.synchronize()
    return O, LSE, bm, (mask_id, score_id, params, Q, K, V)


def run_backward(wl, inp, dev, O, LSE, bm, ids):
    import paper_2412_05496_amd as fa
    mask_id, score_id, params, Q, K, V = ids
    dO = inp.dO.to(dev)
    dQ = torch.full_like(Q, float("nan"))
    dK = torch.full_like(K, float("nan"))
    dV = torch.full_like(V, float("nan"))
    fa.flexattn_backward(Q, K, V, O, dO, LSE, score_id, mask_id, params, bm, inp.scale, dQ, dK, dV)
    torch.cuda.synchronize()
    return dQ, dK, dV


def check_output(O, LSE, O_ref, LSE_ref):
    err = (O.double().cpu() - O_ref).abs()
    assert torch.isfinite(O.float()).all()
    assert float(err.max()) <= O_MAX, f"O max abs err {float(err.max()):.3e}"
    assert float(err.mean()) <= O_MEAN, f"O mean abs err {float(err.mean()):.3e}"
    lerr = (LSE.double().cpu() - LSE_ref).abs()
    lerr = torch.where(torch.isinf(LSE_ref) & (LSE.double().cpu() == LSE_ref), torch.zeros_like(lerr), lerr)
    assert float(lerr.max()) <= LSE_MAX, f"LSE max abs err {float(lerr.max()):.3e}"


def check_grad(name, got, ref):
    """max|g - ref| <= 2e-2 * max(1, max|ref|) and mean|g - ref| <= 2e-3 * max(1, 10 * mean|ref|)."""
    got = got.double().cpu()
    assert torch.isfinite(got).all(), name
    err = (got - ref).abs()
    assert float(err.max()) <= 2e-2 * max(1.0, float(ref.abs().max())), \
        f"{name} max abs err {float(err.max()):.3e} (ref max {float(ref.abs().max()):.3e})"
    assert float(err.mean()) <= 2e-3 * max(1.0, 10.0 * float(ref.abs().mean())), \
        f"{name} mean abs err {float(err.mean()):.3e} (ref mean {float(ref.abs().mean()):.3e})"
