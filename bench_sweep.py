"""Sweep over the shapes of the paper's kernel benchmarks (section 6.2: head dimension 64, KV size fixed
at 256 MiB, causal attention from 1k to 64k tokens; seven variants at 16k tokens with and without GQA;
section 4.2: the full / partial split; section 6.2 / 6.4: decode from 1k to 132k tokens, small batches, page sizes 16 .. 256;
sections 5.1 + 5.2: a chunk of query tokens against a paged cache, beside the same chunk on a contiguous cache;
appendix: neighborhood attention in row-major, tiled and Morton token order over canvas and kernel sizes).

    python bench_sweep.py [--part train|variants|split|decode|batch|pages|prefill|na|all] [--iters N]

One JSON line per measured point (synthetic seeded inputs, bf16, one MI355X).  TFLOP/s count UNMASKED
FLOPs only (4 D per pair forward, 10 D backward); decode is HBM GB/s of the K/V bytes of the tokens read.
The comparison systems of the paper's figures are not part of this build; the lines give this
implementation's curves in the figures' shapes.  A summary of a run is kept under profiles/.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def event_ms(fn, iters):
    import torch
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):      # warm-up
        fn()
    torch.cuda.synchronize()
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / iters


def library_mods(fa, wl, inp, dev):
    mask_id = {"causal": fa.MASK_CAUSAL, "none": fa.MASK_NONE, "doc_causal": fa.MASK_DOCUMENT_CAUSAL,
               "swa_causal": fa.MASK_SWA_CAUSAL, "prefix_lm": fa.MASK_PREFIX_LM}[wl.mask]
    score_id = {"identity": fa.SCORE_IDENTITY, "softcap": fa.SCORE_SOFTCAP, "alibi": fa.SCORE_ALIBI}[wl.score]
    params = fa.ModParams(window=wl.window, prefix_len=wl.prefix_len, softcap=wl.softcap)
    if inp.doc_ids is not None:
        params.doc_ids = inp.doc_ids.to(dev)
    if inp.slopes is not None:
        params.alibi_bias = (-inp.slopes).to(dev)
    return mask_id, score_id, params, (wl.B if wl.mask == "doc_causal" else 1)


def stored_backward_ms(fa, args, n_blocks, iters):
    """The same backward through flexattn_backward_stored (dS kept in memory); args as for flexattn_backward,
    n_blocks = PARTIAL + FULL blocks of the BlockMask."""
    import torch
    Q, K, bm = args[0], args[1], args[9]
    ws = torch.empty(fa.flexattn_backward_stored_workspace_bytes(Q, K, bm, n_blocks), dtype=torch.uint8, device=Q.device)
    t = event_ms(lambda: fa.flexattn_backward_stored(*args, n_blocks, ws), iters)
    del ws
    return t


def train_point(fa, wlm, wl, iters, tag, dev, force_partial=False):
    import torch
    inp = wlm.make_train_inputs(wl, with_dO=True)
    mask_id, score_id, params, Bm = library_mods(fa, wl, inp, dev)
    bm = fa.alloc_blockmask(Bm, 1, wl.S, wl.S, wl.Bq, wl.Bk, device=dev)
    fa.flexattn_blockmask_build(mask_id, params, bm)
    torch.cuda.synchronize()
    stats = bm.stats.cpu().tolist()
    pairs = stats[3] * (wl.B // Bm) * wl.Hq
    if force_partial:
        bm = wlm.blockmask_all_partial(fa.alloc_blockmask, bm)
    Q, K, V, dO = (t.to(dev) for t in (inp.Q, inp.K, inp.V, inp.dO))
    O = torch.empty_like(Q)
    LSE = torch.empty(Q.shape[:3], dtype=torch.float32, device=dev)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    ws = torch.empty(fa.flexattn_backward_workspace_bytes(Q, K), dtype=torch.uint8, device=dev)
    fwd = lambda: fa.flexattn_forward(Q, K, V, score_id, mask_id, params, bm, inp.scale, O, LSE)
    bwd = lambda: fa.flexattn_backward_stages(Q, K, V, O, dO, LSE, score_id, mask_id, params, bm, inp.scale, dQ, dK,
                                              dV, ws, fa.BWD_ALL)
    t_f, t_b = event_ms(fwd, iters), event_ms(bwd, iters)
    t_s = stored_backward_ms(fa, (Q, K, V, O, dO, LSE, score_id, mask_id, params, bm, inp.scale, dQ, dK, dV),
                            int(stats[0] + stats[1]), iters)
    blocks = (wl.S // wl.Bq) * (wl.S // wl.Bk) * Bm
    print(json.dumps({
        "part": tag, "mask": wl.mask, "score": wl.score, "B": wl.B, "Hq": wl.Hq, "Hkv": wl.Hkv, "S": wl.S, "D": wl.D,
        "block": f"{wl.Bq}x{wl.Bk}", "all_partial": force_partial, "pairs": pairs,
        "density": round(pairs / (wl.B * wl.Hq * wl.S * wl.S), 4),
        "blocks_partial_full_total": [stats[0], stats[1], blocks],
        "fwd_ms": round(t_f, 4), "bwd_ms": round(t_b, 4), "bwd_stored_ms": round(t_s, 4),
        "fwd_tflops": round(4 * wl.D * pairs / (t_f * 1e-3) / 1e12, 1),
        "bwd_tflops": round(10 * wl.D * pairs / (t_b * 1e-3) / 1e12, 1),
        "bwd_stored_tflops": round(10 * wl.D * pairs / (t_s * 1e-3) / 1e12, 1)}), flush=True)


def decode_point(fa, wlm, wl, iters, tag, dev, identity_table=False):
    import torch
    ctx = [wl.ctx_max] * wl.B
    inp = wlm.make_decode_inputs(wl, ctx_lens=ctx)
    pt = inp.page_table
    Kp, Vp = inp.K_pool, inp.V_pool
    if identity_table:      # contiguous cache: page i of sequence b is pool page b * pages + i
        pages = (wl.ctx_max + wl.page_size - 1) // wl.page_size
        pt = torch.zeros_like(pt)
        pt[:, :pages] = (torch.arange(wl.B).view(-1, 1) * pages + torch.arange(pages).view(1, -1)).to(torch.int32)
    Q, Kp, Vp, pt, cl = inp.Q.to(dev), Kp.to(dev), Vp.to(dev), pt.to(dev), inp.ctx_lens.to(dev)
    O = torch.empty(wl.B, wl.Hq, wl.D, dtype=torch.bfloat16, device=dev)
    L = torch.empty(wl.B, wl.Hq, dtype=torch.float32, device=dev)
    ws = torch.empty(fa.flexattn_paged_decode_workspace_bytes(Q, Kp, pt), dtype=torch.uint8, device=dev)
    params = fa.ModParams()
    dec = lambda: fa.flexattn_paged_decode(Q, Kp, Vp, pt, cl, fa.SCORE_IDENTITY, fa.MASK_CTX_LEN, params, inp.scale, O, L,
                                           ws)
    ms = event_ms(dec, iters)
    nbytes = sum(ctx) * wl.Hkv * wl.D * 2 * 2
    print(json.dumps({"part": tag, "nseq": wl.B, "ctx_len": wl.ctx_max, "Hq": wl.Hq, "Hkv": wl.Hkv, "D": wl.D,
                      "page_size": wl.page_size, "contiguous_pages": identity_table, "ms": round(ms, 4),
                      "kv_bytes": nbytes, "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1)}), flush=True)


def prefill_point(fa, wlm, wl, kv_len, q_len, iters, dev):
    """Causal chunk of q_len tokens at the end of kv_len-token sequences: paged pool, then the same
    keys gathered into a contiguous [B, Hkv, kv_len, D] cache (same BlockMask, same offsets)."""
    import torch
    inp = wlm.make_prefill_inputs(wl, [kv_len] * wl.B, q_len)
    page, n_pool = wl.page_size, inp.K_pool.shape[0]
    params = fa.ModParams(q_offsets=inp.q_offsets.to(dev))
    bm = fa.alloc_blockmask(wl.B, 1, q_len, kv_len, wl.Bq, page, device=dev)
    fa.flexattn_blockmask_build(fa.MASK_CAUSAL, params, bm)
    pt = inp.page_table.to(dev)
    phys_kv, phys_full = torch.zeros_like(bm.kv_indices), torch.zeros_like(bm.full_kv_indices)
    fa.flexattn_paged_convert_blockmask(bm.kv_num_blocks, bm.kv_indices, pt, phys_kv)
    fa.flexattn_paged_convert_blockmask(bm.full_kv_num_blocks, bm.full_kv_indices, pt, phys_full)
    torch.cuda.synchronize()
    pairs = bm.stats.cpu().tolist()[3] * wl.Hq
    Q, Kp, Vp = inp.Q.to(dev), inp.K_pool.to(dev), inp.V_pool.to(dev)
    O = torch.empty_like(Q)
    LSE = torch.empty(Q.shape[:3], dtype=torch.float32, device=dev)
    t_paged = event_ms(lambda: fa.flexattn_paged_forward(Q, Kp, Vp, fa.SCORE_IDENTITY, fa.MASK_CAUSAL, params, bm, phys_kv,
                                                         phys_full, inp.scale, O, LSE), iters)
    O_paged = O.clone()
    pages = kv_len // page
    gather = lambda pool: (pool[pt[:, :pages].long()]                      # [B, pages, Hkv, page, D]
                           .permute(0, 2, 1, 3, 4).reshape(wl.B, wl.Hkv, kv_len, wl.D).contiguous())
    Kc, Vc = gather(Kp), gather(Vp)
    t_contig = event_ms(lambda: fa.flexattn_forward(Q, Kc, Vc, fa.SCORE_IDENTITY, fa.MASK_CAUSAL, params, bm, inp.scale,
                                                    O, LSE), iters)
    print(json.dumps({"part": "prefill", "nseq": wl.B, "kv_len": kv_len, "q_len": q_len, "Hq": wl.Hq, "Hkv": wl.Hkv,
                      "D": wl.D, "page_size": page, "pairs": pairs, "paged_ms": round(t_paged, 4),
                      "contiguous_ms": round(t_contig, 4),
                      "paged_tflops": round(4 * wl.D * pairs / (t_paged * 1e-3) / 1e12, 1),
                      "contiguous_tflops": round(4 * wl.D * pairs / (t_contig * 1e-3) / 1e12, 1),
                      "same_output": bool(torch.equal(O_paged, O))}), flush=True)


def na_point(fa, wlm, canvas, kernel, layout, tile, iters, dev):
    """Neighborhood attention on a canvas x canvas image, 4 x 16 heads of 64: block density, forward, backward."""
    import torch
    S = canvas * canvas
    wl = wlm.Workload(f"sweep_na_{canvas}_{kernel}_{layout}", B=4, Hq=16, Hkv=16, S=S, D=64, Bq=128, Bk=64, mask="none",
                      score="identity", seed=2600 + canvas + kernel)
    inp = wlm.make_train_inputs(wl, with_dO=True)
    params = fa.ModParams(na_width=canvas, na_height=canvas, na_kernel=kernel,
                          na_layout={"row_major": fa.NA_ROW_MAJOR, "tiled": fa.NA_TILED, "morton": fa.NA_MORTON}[layout],
                          na_tile=tile)
    bm = fa.alloc_blockmask(1, 1, S, S, wl.Bq, wl.Bk, device=dev)
    fa.flexattn_blockmask_build(fa.MASK_NEIGHBORHOOD, params, bm)
    torch.cuda.synchronize()
    stats = bm.stats.cpu().tolist()
    pairs = stats[3] * wl.B * wl.Hq
    Q, K, V, dO = (t.to(dev) for t in (inp.Q, inp.K, inp.V, inp.dO))
    O = torch.empty_like(Q)
    LSE = torch.empty(Q.shape[:3], dtype=torch.float32, device=dev)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    ws = torch.empty(fa.flexattn_backward_workspace_bytes(Q, K), dtype=torch.uint8, device=dev)
    fwd = lambda: fa.flexattn_forward(Q, K, V, fa.SCORE_IDENTITY, fa.MASK_NEIGHBORHOOD, params, bm, inp.scale, O, LSE)
    bwd = lambda: fa.flexattn_backward_stages(Q, K, V, O, dO, LSE, fa.SCORE_IDENTITY, fa.MASK_NEIGHBORHOOD, params, bm,
                                              inp.scale, dQ, dK, dV, ws, fa.BWD_ALL)
    t_f, t_b = event_ms(fwd, iters), event_ms(bwd, iters)
    t_s = stored_backward_ms(fa, (Q, K, V, O, dO, LSE, fa.SCORE_IDENTITY, fa.MASK_NEIGHBORHOOD, params, bm, inp.scale,
                                  dQ, dK, dV), int(stats[0] + stats[1]), iters)
    print(json.dumps({
        "part": "na", "canvas": canvas, "kernel": kernel, "layout": layout, "tile": tile, "tokens": S,
        "mask_density": round(stats[3] / (S * S), 5),
        "block_density": round((stats[0] + stats[1]) / stats[2], 5),
        "blocks_partial_full_total": stats[:3], "fwd_ms": round(t_f, 4), "bwd_ms": round(t_b, 4),
        "bwd_stored_ms": round(t_s, 4),
        "fwd_tflops": round(4 * wl.D * pairs / (t_f * 1e-3) / 1e12, 1),
        "bwd_tflops": round(10 * wl.D * pairs / (t_b * 1e-3) / 1e12, 1)}), flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--part", default="all", choices=["train", "variants", "split", "decode", "batch", "pages", "prefill", "na", "all"])
    ap.add_argument("--iters", type=int, default=10)
    args = ap.parse_args()

    import torch
    import flex_workloads as wlm
    import paper_2412_05496_amd as fa
    assert torch.cuda.is_available(), "bench_sweep.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    W = wlm.Workload
    parts = [args.part] if args.part != "all" else ["train", "variants", "split", "decode", "batch", "pages", "prefill", "na"]

    if "train" in parts:        # causal, D = 64, H = 16, B * S = 65536 (K + V = 256 MiB)
        for S in (1024, 2048, 4096, 8192, 16384, 32768, 65536):
            wl = W(f"sweep_causal_s{S}", B=65536 // S, Hq=16, Hkv=16, S=S, D=64, Bq=128, Bk=64, mask="causal",
                   score="identity", seed=2000 + S // 1024)
            train_point(fa, wlm, wl, args.iters, "train", dev)
    if "variants" in parts:     # seven variants at 16k tokens, with and without GQA
        variants = [("none", "identity", {}), ("causal", "identity", {}), ("causal", "alibi", {}),
                    ("swa_causal", "identity", {"window": 1024}), ("prefix_lm", "identity", {"prefix_len": 4096}),
                    ("causal", "softcap", {"softcap": 30.0}),
                    ("doc_causal", "identity", {"doc_len_min": 256, "doc_len_max": 4096})]
        for hkv in (16, 2):
            for i, (mask, score, kw) in enumerate(variants):
                wl = W(f"sweep_{mask}_{score}", B=4, Hq=16, Hkv=hkv, S=16384, D=64, Bq=128, Bk=64, mask=mask, score=score,
                       seed=2100 + i, **kw)
                train_point(fa, wlm, wl, args.iters, "variants", dev)
    if "split" in parts:        # full / partial split on, then off (every block evaluates mask_mod)
        wl = W("sweep_split_causal", B=4, Hq=16, Hkv=16, S=16384, D=64, Bq=128, Bk=64, mask="causal", score="identity",
               seed=2200)
        train_point(fa, wlm, wl, args.iters, "split", dev, force_partial=False)
        train_point(fa, wlm, wl, args.iters, "split", dev, force_partial=True)
    if "decode" in parts:       # about one million tokens of KV per point, 16-token pages
        for ctx in (1024, 4096, 16384, 32768, 65536, 131072):
            nseq = max(8, (1 << 20) // ctx)
            wl = W(f"sweep_decode_{ctx}", B=nseq, Hq=32, Hkv=8, S=1, D=128, Bq=1, Bk=16, mask="ctx_len", score="identity",
                   seed=2300 + ctx // 1024, backward=False, page_size=16, ctx_min=ctx, ctx_max=ctx,
                   max_pages=ctx // 16)
            decode_point(fa, wlm, wl, args.iters, "decode", dev)
    if "batch" in parts:        # few sequences: the split length follows the batch so that the chip stays full
        for nseq, ctx in ((1, 8192), (1, 32768), (1, 131072), (4, 8192), (4, 32768), (16, 8192), (16, 32768)):
            wl = W(f"sweep_batch_{nseq}x{ctx}", B=nseq, Hq=32, Hkv=8, S=1, D=128, Bq=1, Bk=16, mask="ctx_len",
                   score="identity", seed=2350 + nseq + ctx // 1024, backward=False, page_size=16, ctx_min=ctx,
                   ctx_max=ctx, max_pages=ctx // 16)
            decode_point(fa, wlm, wl, args.iters, "batch", dev)
    if "pages" in parts:        # page size 16 .. 256, scattered pages against a contiguous cache
        for page in (16, 32, 64, 128, 256):
            for ident in (False, True):
                wl = W(f"sweep_pages_{page}", B=64, Hq=32, Hkv=8, S=1, D=128, Bq=1, Bk=page, mask="ctx_len",
                       score="identity", seed=2400 + page, backward=False, page_size=page, ctx_min=16384,
                       ctx_max=16384, max_pages=16384 // page)
                decode_point(fa, wlm, wl, args.iters, "pages", dev, identity_table=ident)
    if "prefill" in parts:     # chunked prefill: 2048 new tokens on top of 16k / 64k cached, pages of 64 / 128
        for page in (64, 128):
            for nseq, kv_len in ((16, 16384), (4, 65536)):
                wl = W(f"sweep_prefill_{page}_{kv_len}", B=nseq, Hq=32, Hkv=8, S=2048, D=128, Bq=128, Bk=page,
                       mask="causal", score="identity", seed=2500 + page + kv_len // 1024, backward=False,
                       page_size=page, ctx_min=kv_len, ctx_max=kv_len, max_pages=kv_len // page)
                prefill_point(fa, wlm, wl, kv_len, 2048, args.iters, dev)
    if "na" in parts:          # canvas 64 / 128, kernels 7 / 13 / 27, three token orders (8 x 8 tiles)
        for canvas in (64, 128):
            for kernel in (7, 13, 27):
                for layout, tile in (("row_major", 0), ("tiled", 8), ("morton", 0)):
                    na_point(fa, wlm, canvas, kernel, layout, tile, args.iters, dev)
    return 0


if __name__ == "__main__":
    sys.exit(main())
