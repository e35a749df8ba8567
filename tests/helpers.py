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
    elif wl.score == "alibi_softcap":               # nested score_mods: the bias first, then the soft-cap
        score = fo.Compose(fo.Alibi(-inp.slopes.double()), fo.Softcap(wl.softcap))
    elif wl.score == "rel_bias_softcap":
        score = fo.Compose(fo.RelBias(inp.rel_bias.double()), fo.Softcap(wl.softcap))
    else:
        raise ValueError(wl.score)
    return score, mask


def library_mods(wl: wlm.Workload, inp, dev):
    import paper_2412_05496_amd as fa
    mask_id = {"causal": fa.MASK_CAUSAL, "none": fa.MASK_NONE, "doc_causal": fa.MASK_DOCUMENT_CAUSAL,
               "swa_causal": fa.MASK_SWA_CAUSAL, "prefix_lm": fa.MASK_PREFIX_LM,
               "swa_causal_or_prefix": fa.MASK_SWA_CAUSAL_OR_PREFIX}[wl.mask]
    score_id = {"identity": fa.SCORE_IDENTITY, "softcap": fa.SCORE_SOFTCAP, "alibi": fa.SCORE_ALIBI,
                "rel_bias": fa.SCORE_REL_BIAS, "alibi_softcap": fa.SCORE_ALIBI | fa.SCORE_SOFTCAP,
                "rel_bias_softcap": fa.SCORE_REL_BIAS | fa.SCORE_SOFTCAP}[wl.score]
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
ORDER_NAMES = ("kv_order", "q_order")


def assert_blockmask_equal(bm, ref):
    for name in BM_NAMES:
        got = getattr(bm, name).cpu()
        assert got.dtype == torch.int32 and got.shape == ref[name].shape, name
        assert torch.equal(got, ref[name]), name
    for name in ORDER_NAMES:
        if getattr(bm, name) is not None:
            got = getattr(bm, name).cpu()
            assert got.dtype == torch.int32 and got.shape == ref[name].shape, name
            assert torch.equal(got, ref[name]), name
    if bm.stats is not None:
        st = bm.stats.cpu().tolist()
        assert st == [ref["stats"]["partial"], ref["stats"]["full"], ref["stats"]["total"],
                      ref["stats"]["unmasked_pairs"]], st


def run_forward(wl, inp, dev, Hm=1):
    """BlockMask build + forward through the C ABI.  Returns (O, LSE, bm, ids).  Hm = 1 builds one
    BlockMask plane shared by all heads, Hm = wl.Hq one plane per query head."""
    import paper_2412_05496_amd as fa
    mask_id, score_id, params, Bm = library_mods(wl, inp, dev)
    bm = fa.alloc_blockmask(Bm, Hm, wl.S, wl.S, wl.Bq, wl.Bk, device=dev)
    fa.flexattn_blockmask_build(mask_id, params, bm)
    Q, K, V = inp.Q.to(dev), inp.K.to(dev), inp.V.to(dev)
    O = torch.full_like(Q, float("nan"))
    LSE = torch.full(Q.shape[:3], float("nan"), dtype=torch.float32, device=dev)
    fa.flexattn_forward(Q, K, V, score_id, mask_id, params, bm, inp.scale, O, LSE)
    torch.cuda.synchronize()
    return O, LSE, bm, (mask_id, score_id, params, Q, K, V)


def nonempty_blocks(bm):
    """PARTIAL + FULL blocks of all planes: the capacity the backward that keeps dS in memory asks for."""
    st = bm.stats.cpu().tolist()
    return int(st[0] + st[1])


def run_backward(wl, inp, dev, O, LSE, bm, ids, stored=False):
    """stored: through flexattn_backward_stored (dS kept in memory) instead of flexattn_backward."""
    import paper_2412_05496_amd as fa
    mask_id, score_id, params, Q, K, V = ids
    dO = inp.dO.to(dev)
    dQ = torch.full_like(Q, float("nan"))
    dK = torch.full_like(K, float("nan"))
    dV = torch.full_like(V, float("nan"))
    if stored:
        fa.flexattn_backward_stored(Q, K, V, O, dO, LSE, score_id, mask_id, params, bm, inp.scale, dQ, dK, dV,
                                    nonempty_blocks(bm))
    else:
        fa.flexattn_backward(Q, K, V, O, dO, LSE, score_id, mask_id, params, bm, inp.scale, dQ, dK, dV)
    torch.cuda.synchronize()
    return dQ, dK, dV


def _stats(err):
    return float(err.max()), float(err.mean()), float(err.pow(2).mean().sqrt())


def check_output(O, LSE, O_ref, LSE_ref):
    """O: max abs <= 2e-2, mean abs <= 2e-3; LSE: max abs <= 1e-2 (the stated tolerances).  Prints the
    measured max / mean / RMSE (the paper's own accuracy metric, section 6.3)."""
    err = (O.double().cpu() - O_ref).abs()
    lerr = (LSE.double().cpu() - LSE_ref).abs()
    lerr = torch.where(torch.isinf(LSE_ref) & (LSE.double().cpu() == LSE_ref), torch.zeros_like(lerr), lerr)
    print("  [err] O max %.3e mean %.3e rmse %.3e | LSE max %.3e mean %.3e rmse %.3e"
          % (_stats(err) + _stats(lerr)), flush=True)
    assert torch.isfinite(O.float()).all()
    assert float(err.max()) <= O_MAX, f"O max abs err {float(err.max()):.3e}"
    assert float(err.mean()) <= O_MEAN, f"O mean abs err {float(err.mean()):.3e}"
    assert float(lerr.max()) <= LSE_MAX, f"LSE max abs err {float(lerr.max()):.3e}"


# Gradient tolerance.  Absolute bound, relative to the gradient's own scale (a gradient element is a
# sum of thousands of products of bf16 operands, so its rounding error scales with the gradient, not
# with 1):  max|g - ref| <= 2e-2 * max(1, max|ref|)  and  mean|g - ref| <= 6e-3 * max(1, mean|ref|)
# (measured: <= 6.5e-3 resp. <= 3.6e-3 over every case of the suite; rounding the result to bf16
# alone costs a mean of 2.3e-3 * mean|ref|).
# Where the caller supplies `emul` -- the same gradient from emulate_bf16_backward(), i.e. exact
# arithmetic except for the roundings to bf16 that any kernel feeding bf16 matrix units must make --
# the kernel may be at most 3x (max) resp. 1.5x (mean) as far from the oracle as that emulation is
# (measured: <= 1.65x resp. <= 1.02x).
G_MAX, G_MEAN, EMUL_MAX, EMUL_MEAN = 2e-2, 6e-3, 3.0, 1.5


def check_grad(name, got, ref, emul=None, mean_tol=G_MEAN):
    got = got.double().cpu()
    assert torch.isfinite(got).all(), name
    err = (got - ref).abs()
    line = "  [err] %s max %.3e mean %.3e rmse %.3e (ref max %.3e mean %.3e)" % (
        (name,) + _stats(err) + (float(ref.abs().max()), float(ref.abs().mean())))
    if emul is not None:
        e_err = (emul - ref).abs()
        line += " | bf16 emulation max %.3e mean %.3e" % (float(e_err.max()), float(e_err.mean()))
    print(line, flush=True)
    assert float(err.max()) <= G_MAX * max(1.0, float(ref.abs().max())), \
        f"{name} max abs err {float(err.max()):.3e} (ref max {float(ref.abs().max()):.3e})"
    assert float(err.mean()) <= mean_tol * max(1.0, float(ref.abs().mean())), \
        f"{name} mean abs err {float(err.mean()):.3e} (ref mean {float(ref.abs().mean()):.3e})"
    if emul is not None:
        assert float(err.max()) <= EMUL_MAX * float(e_err.max()) + 1e-6, \
            f"{name} max abs err {float(err.max()):.3e} > {EMUL_MAX} x emulation {float(e_err.max()):.3e}"
        assert float(err.mean()) <= EMUL_MEAN * float(e_err.mean()) + 1e-7, \
            f"{name} mean abs err {float(err.mean()):.3e} > {EMUL_MEAN} x emulation {float(e_err.mean()):.3e}"


def _bf16(x):
    return x.to(torch.bfloat16).to(torch.float64)


def emulate_bf16_backward(inp, score, mask):
    """dQ, dK, dV of the oracle's formulas with ONLY the roundings a bf16 matrix-unit kernel cannot
    avoid: the forward output O, the probabilities P and the score gradients dS are rounded to bf16
    where they become matrix operands, and the three results are rounded to bf16; every sum is
    exact (fp64).  Its distance from the oracle is the yardstick for the kernel's."""
    B, Hq, S, D = inp.Q.shape
    Hkv = inp.K.shape[1]
    G = Hq // Hkv
    dQ = torch.empty(B, Hq, S, D, dtype=torch.float64)
    dK = torch.zeros(B, Hkv, S, D, dtype=torch.float64)
    dV = torch.zeros(B, Hkv, S, D, dtype=torch.float64)
    kv_idx = torch.arange(S).view(1, -1)
    for b in range(B):
        for h in range(Hq):
            Qh, Kh, Vh, dOh = (t.double() for t in (inp.Q[b, h], inp.K[b, h // G], inp.V[b, h // G], inp.dO[b, h]))
            q_idx = torch.arange(S)
            s, s_mod, keep = fo._modified_scores(Qh, Kh, score, mask, inp.scale, b, h, q_idx)
            P, _ = fo._softmax_rows(s_mod, keep)
            Pb = _bf16(P)
            delta = (dOh * _bf16(Pb @ Vh)).sum(dim=1, keepdim=True)
            g = score.grad(s, b, h, q_idx.view(-1, 1), kv_idx)
            dS = _bf16(torch.where(keep, P * (dOh @ Vh.T - delta) * g, torch.zeros_like(P)))
            dQ[b, h] = _bf16(inp.scale * (dS @ Kh))
            dK[b, h // G] += inp.scale * (dS.T @ Qh)
            dV[b, h // G] += Pb.T @ dOh
    return dQ, _bf16(dK), _bf16(dV)
