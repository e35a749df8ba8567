"""Benchmark of the FlexAttention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One step = BlockMask build + forward + backward (all three through the C ABI) on the dense
causal + tanh-softcap training shape B=4, H=16, S=8192, D=128 (bf16, synthetic N(0,1) inputs
resident in HBM).  `value` is TFLOP/s over UNMASKED FLOPs only: 4*D per unmasked (q, kv) pair for
the forward, 10*D for the backward (five GEMMs; recomputation is not credited).  The step's
backward is flexattn_backward_stored -- dS written to HBM by the dK/dV kernel and read back by a lean
dQ kernel, 4.4 GB of workspace -- which is the faster of the library's two on this shape; the
recomputing flexattn_backward is timed in the same run (`bwd_recompute`).

The JSON line also carries
  roofline      the longest kernel of the step against the dense bf16 MFMA peak, timed with
                events on the launch stream (`traffic` is the HBM byte count of that kernel from the
                rocprofv3 --pmc runs recorded under profiles/, not a measurement of this run);
  bwd_dq_roofline  the dQ kernel of the step's backward (a block-sparse GEMM over the stored dS) against the HBM peak;
  measured_peaks  what this chip sustains in this very run: an MFMA-only kernel and a plain
                streaming read, so that every fraction can also be read against achievable rates;
  cfg3, cfg4    forward and backward of the document-mask + ALiBi and the sliding-window/prefix +
                relative-bias GQA workloads (outside the timed step), with the BlockMask density;
  decode        the paged split-KV decode workload (64 sequences, 16-token pages) in HBM GB/s of
                algorithmic K+V bytes, with its own roofline object;
  cpu_baseline  the fp64 oracle timed on this host's cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def measured_traffic(kernel: str):
    """HBM bytes per launch of `kernel` from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
    same command (scaled by the copy-kernel calibration); the figures and the commands that produced
    them are in profiles/.  None if no figure is recorded."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        return json.load(f).get(kernel, {}).get("bytes")


def event_time_ms(fn, iters: int) -> float:
    """Average duration of fn() in ms, bracketed by events on the current (launch) stream."""
    import torch
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / iters


def train_leg(fa, wlm, wl, dev, iters: int, mfma_tflops: float, stored: bool = True, time_other: bool = True) -> dict:
    """Forward and backward of one of the other training workloads: ms, TFLOP/s over unmasked FLOPs,
    fractions of the datasheet and of the measured MFMA rate, BlockMask density.  `stored`: the backward
    is flexattn_backward_stored (dS kept in memory) rather than flexattn_backward; `time_other`: the
    other one is timed beside it."""
    import torch
    inp = wlm.make_train_inputs(wl, with_dO=True)
    Q, Kt, V, dO = (t.to(dev) for t in (inp.Q, inp.K, inp.V, inp.dO))
    note = None
    if wl.mask == "doc_causal":
        mask_id, score_id, Bm = fa.MASK_DOCUMENT_CAUSAL, fa.SCORE_ALIBI, wl.B
        params = fa.ModParams(doc_ids=inp.doc_ids.to(dev), alibi_bias=(-inp.slopes).to(dev))
        note = ("ALiBi slopes 2^(-8(h+1)/H), h = 0..H-1 (the usual 1-based reading of 2^(-8h/H)); documents: "
                + ", ".join(str(n) for n in inp.doc_lengths[0]) + " tokens")
    else:
        mask_id, score_id, Bm = fa.MASK_SWA_CAUSAL_OR_PREFIX, fa.SCORE_REL_BIAS, 1
        params = fa.ModParams(window=wl.window, prefix_len=wl.prefix_len, rel_bias=inp.rel_bias.to(dev))
    bm = fa.alloc_blockmask(Bm, 1, wl.S, wl.S, wl.Bq, wl.Bk, device=dev)
    fa.flexattn_blockmask_build(mask_id, params, bm)
    partial, full, total, unmasked = bm.stats.cpu().tolist()
    pairs = unmasked * (wl.B // Bm) * wl.Hq
    O = torch.empty_like(Q)
    LSE = torch.empty(Q.shape[:3], dtype=torch.float32, device=dev)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(Kt), torch.empty_like(V)
    ws = torch.empty(fa.flexattn_backward_workspace_bytes(Q, Kt), dtype=torch.uint8, device=dev)
    fwd = lambda: fa.flexattn_forward(Q, Kt, V, score_id, mask_id, params, bm, inp.scale, O, LSE)
    bwd_rc = lambda st=fa.BWD_ALL: fa.flexattn_backward_stages(Q, Kt, V, O, dO, LSE, score_id, mask_id, params, bm,
                                                               inp.scale, dQ, dK, dV, ws, st)
    st_ws = None
    if stored or time_other:
        st_ws = torch.empty(fa.flexattn_backward_stored_workspace_bytes(Q, Kt, bm, partial + full), dtype=torch.uint8,
                            device=dev)
    bwd_st = lambda st=fa.BWD_ALL: fa.flexattn_backward_stored(Q, Kt, V, O, dO, LSE, score_id, mask_id, params, bm,
                                                               inp.scale, dQ, dK, dV, partial + full, st_ws, st)
    bwd, bwd_other = (bwd_st, bwd_rc) if stored else (bwd_rc, bwd_st)
    fwd(), bwd()
    torch.cuda.synchronize()
    t_f, t_b = event_time_ms(fwd, iters), event_time_ms(bwd, iters)
    t_dkdv = event_time_ms(lambda: bwd(fa.BWD_DKDV), iters)
    t_dq = event_time_ms(lambda: bwd(fa.BWD_DQ), iters)
    f_f, f_b = 4 * wl.D * pairs / (t_f * 1e-3) / 1e12, 10 * wl.D * pairs / (t_b * 1e-3) / 1e12
    leg = {
        "workload": wl.name, "pairs": pairs, "fwd_ms": round(t_f, 4),
        "bwd": "flexattn_backward_stored (dS kept in memory)" if stored else "flexattn_backward (dQ recomputes S, dP)",
        "bwd_ms": round(t_b, 4), "bwd_dkdv_ms": round(t_dkdv, 4), "bwd_dq_ms": round(t_dq, 4),
        "bwd_workspace_gb": round((st_ws if stored else ws).numel() / 1e9, 3),
        "fwd_tflops": round(f_f, 1), "bwd_tflops": round(f_b, 1),
        "fwd_frac_of_bf16_peak": round(f_f / PEAK_BF16_TFLOPS, 4),
        "bwd_frac_of_bf16_peak": round(f_b / PEAK_BF16_TFLOPS, 4),
        "fwd_frac_of_measured_mfma": round(f_f / mfma_tflops, 4),
        "bwd_frac_of_measured_mfma": round(f_b / mfma_tflops, 4),
        "blockmask": {"partial": partial, "full": full, "total": total,
                      "block_density": round((partial + full) / total, 4),
                      "element_density": round(unmasked / (Bm * wl.S * wl.S), 4),
                      "executed_over_unmasked_pairs": round((partial + full) * wl.Bq * wl.Bk / unmasked, 4)},
    }
    if time_other:
        bwd_other()
        leg["bwd_recompute_ms" if stored else "bwd_stored_ms"] = round(event_time_ms(bwd_other, iters), 4)
    if note:
        leg["note"] = note
    return leg


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the cfg3 / cfg4 legs")
    ap.add_argument("--bwd-path", choices=("stored", "recompute"), default="stored",
                    help="the backward of the timed step: flexattn_backward_stored (dS kept in memory, default) or "
                         "flexattn_backward (S and dP recomputed for dQ)")
    ap.add_argument("--one-bwd-path", action="store_true",
                    help="do not time the other backward beside the step's (for profiler runs: both use the same dK/dV kernel)")
    ap.add_argument("--cpu-heads", type=int, default=12, help="(b, h) slices the oracle is timed on")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    import flex_workloads as wlm
    import paper_2412_05496_amd as fa

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, W = args.steps, args.warmup

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": 1 << 30, "launches": 3}))
        return 0

    # ------------------------------------------------------------------ training shape
    wl = wlm.CFG2
    inp = wlm.make_train_inputs(wl)
    Q, Kt, V, dO = (t.to(dev) for t in (inp.Q, inp.K, inp.V, inp.dO))
    params = fa.ModParams(softcap=wl.softcap)
    mask_id, score_id = fa.MASK_CAUSAL, fa.SCORE_SOFTCAP
    bm = fa.alloc_blockmask(1, 1, wl.S, wl.S, wl.Bq, wl.Bk, device=dev)
    bm_ws = torch.empty(fa.flexattn_blockmask_workspace_bytes(1, 1, wl.S, wl.S, wl.Bq, wl.Bk), dtype=torch.uint8,
                        device=dev)
    O = torch.empty_like(Q)
    LSE = torch.empty(Q.shape[:3], dtype=torch.float32, device=dev)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(Kt), torch.empty_like(V)
    bwd_ws = torch.empty(fa.flexattn_backward_workspace_bytes(Q, Kt), dtype=torch.uint8, device=dev)
    # The step's backward keeps dS in memory (flexattn_backward_stored: 5 GEMMs and 2 bytes of HBM
    # traffic each way per unmasked score); the recomputing one (7 GEMMs) is timed beside it.
    n_blocks = sum((r + 1) * wl.Bq // wl.Bk for r in range(wl.S // wl.Bq))   # causal, closed form; checked against stats below
    st_ws = torch.empty(fa.flexattn_backward_stored_workspace_bytes(Q, Kt, bm, n_blocks), dtype=torch.uint8, device=dev)

    def build():
        fa.flexattn_blockmask_build(mask_id, params, bm, bm_ws)

    def fwd():
        fa.flexattn_forward(Q, Kt, V, score_id, mask_id, params, bm, inp.scale, O, LSE)

    def bwd_recompute(stages=fa.BWD_ALL):
        fa.flexattn_backward_stages(Q, Kt, V, O, dO, LSE, score_id, mask_id, params, bm, inp.scale, dQ, dK, dV,
                                    bwd_ws, stages)

    def bwd_stored(stages=fa.BWD_ALL):
        fa.flexattn_backward_stored(Q, Kt, V, O, dO, LSE, score_id, mask_id, params, bm, inp.scale, dQ, dK, dV,
                                    n_blocks, st_ws, stages)

    stored = args.bwd_path == "stored"
    bwd, bwd_other = (bwd_stored, bwd_recompute) if stored else (bwd_recompute, bwd_stored)

    def step():
        build()
        fwd()
        bwd()

    for _ in range(W):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / K

    pairs = wl.B * wl.Hq * wl.S * (wl.S + 1) // 2
    stats = bm.stats.cpu().tolist()
    assert stats[3] * wl.B * wl.Hq == pairs, "BlockMask unmasked-pair count disagrees with the closed form"
    assert stats[0] + stats[1] == n_blocks, "BlockMask block count disagrees with the closed form"
    flops_fwd, flops_bwd = 4 * wl.D * pairs, 10 * wl.D * pairs
    value = (flops_fwd + flops_bwd) / (ms_per_step * 1e-3) / 1e12

    # per-kernel durations (events on the launch stream)
    kt = {
        "blockmask_build": event_time_ms(build, K),
        "fwd": event_time_ms(fwd, K),
        "bwd_delta": event_time_ms(lambda: bwd(fa.BWD_DELTA), K),
        "bwd_dkdv": event_time_ms(lambda: bwd(fa.BWD_DKDV), K),
        "bwd_dq": event_time_ms(lambda: bwd(fa.BWD_DQ), K),
    }
    # algorithmic FLOPs per launch: forward 4*D*pairs; of the backward's 10*D*pairs (five GEMMs) the
    # dK/dV kernel executes four GEMMs and, with dS in memory, the dQ kernel one -- nothing is computed
    # twice; the recomputing dQ kernel executes three, and the 10*D*pairs are then split 4 : 3
    # (recomputation earns nothing)
    share = (4 / 5, 1 / 5) if stored else (4 / 7, 3 / 7)
    alg = {"fwd": flops_fwd, "bwd_dkdv": flops_bwd * share[0], "bwd_dq": flops_bwd * share[1]}
    dom = max(alg, key=lambda k: kt[k])
    achieved = alg[dom] / (kt[dom] * 1e-3) / 1e12
    roofline = {"kernel": dom, "bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "traffic": measured_traffic(dom + ("_stored" if stored and dom != "fwd" else "")),
                "avg_ms": round(kt[dom], 4)}
    bwd_ms = kt["bwd_delta"] + kt["bwd_dkdv"] + kt["bwd_dq"]
    out = {
        "metric": "flex_attention fwd+bwd TFLOP/s (unmasked FLOPs), dense causal + softcap",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "B": wl.B, "H": wl.Hq, "S": wl.S, "D": wl.D, "mask": "causal",
                   "score_mod": "tanh softcap 30", "block": f"{wl.Bq}x{wl.Bk}",
                   "step": "blockmask_build + forward + backward "
                           + ("(flexattn_backward_stored: dS kept in memory)" if stored else "(flexattn_backward: dQ recomputes S, dP)")},
        "fwd_tflops": round(flops_fwd / (kt["fwd"] * 1e-3) / 1e12, 2),
        "fwd_frac_of_bf16_peak": round(flops_fwd / (kt["fwd"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "bwd_tflops": round(flops_bwd / (bwd_ms * 1e-3) / 1e12, 2),
        "bwd_frac_of_bf16_peak": round(flops_bwd / (bwd_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "kernel_ms": {k: round(v, 4) for k, v in kt.items()},
        "bwd_workspace_gb": round((st_ws if stored else bwd_ws).numel() / 1e9, 3),
        "blockmask": {"partial": stats[0], "full": stats[1], "total": stats[2]},
        "roofline": roofline,
    }

    if stored:
        # the dQ kernel of this path is a block-sparse GEMM bound by HBM: every dS block read once (2 bytes per
        # score of a non-empty block), K once per head, dQ written once
        dq_bytes = n_blocks * wl.Bq * wl.Bk * 2 * wl.B * wl.Hq + Kt.numel() * 2 + dQ.numel() * 2
        dq_gbs = dq_bytes / (kt["bwd_dq"] * 1e-3) / 1e9
        out["bwd_dq_roofline"] = {"kernel": "bwd_dq_stored", "bound": "hbm", "achieved": round(dq_gbs, 1),
                                  "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(dq_gbs / PEAK_HBM_GBS, 4),
                                  "traffic": measured_traffic("bwd_dq_stored"), "avg_ms": round(kt["bwd_dq"], 4),
                                  "algorithmic_bytes": dq_bytes}
    if not args.one_bwd_path:
        # the library's other backward on the same inputs
        bwd_other()
        ko = {"bwd_delta": event_time_ms(lambda: bwd_other(fa.BWD_DELTA), K),
              "bwd_dkdv": event_time_ms(lambda: bwd_other(fa.BWD_DKDV), K),
              "bwd_dq": event_time_ms(lambda: bwd_other(fa.BWD_DQ), K)}
        other_ms = sum(ko.values())
        out["bwd_recompute" if stored else "bwd_stored"] = {
            "what": ("flexattn_backward: dQ recomputes S and dP (7 GEMMs for the 5 credited), 4 MB workspace" if stored
                     else "flexattn_backward_stored: dS written by dK/dV and read by dQ (5 GEMMs), 4.4 GB workspace"),
            "kernel_ms": {k: round(v, 4) for k, v in ko.items()}, "bwd_ms": round(other_ms, 4),
            "bwd_tflops": round(flops_bwd / (other_ms * 1e-3) / 1e12, 2),
            "bwd_frac_of_bf16_peak": round(flops_bwd / (other_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)}

    # ------------------------------------------------------------------ what the chip sustains
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    probe_iters = 20000
    clocks = torch.zeros(fa.flexattn_probe_mfma_waves(), 2, dtype=torch.int64, device=dev)

    def mfma_probe(valu_mix: int, random_operands: bool):
        """(TFLOP/s of the MFMAs, sustained core clock in GHz)"""
        run = lambda n: fa.flexattn_probe_mfma(n, sink, valu_mix, random_operands, clocks)
        run(2000)
        ms = event_time_ms(lambda: run(probe_iters), 3)
        ck = clocks.cpu().double()
        return (fa.flexattn_probe_mfma_flops(probe_iters) / (ms * 1e-3) / 1e12,
                float(ck[:, 0].sum() / (ck[:, 1].sum() * 10.0)))

    mfma_const, ghz_const = mfma_probe(0, False)
    mfma_tflops, ghz_random = mfma_probe(0, True)            # the rate every fraction below refers to
    mix_const, _ = mfma_probe(1, False)
    mix_random, ghz_mix = mfma_probe(1, True)
    bwd_mix_random, ghz_bwd_mix = mfma_probe(2, True)
    stream_src = torch.empty(4 << 30, dtype=torch.uint8, device=dev).fill_(1)
    fa.flexattn_probe_stream_read(stream_src, sink)
    read_ms = event_time_ms(lambda: fa.flexattn_probe_stream_read(stream_src, sink), 5)
    read_gbs = stream_src.numel() / (read_ms * 1e-3) / 1e9
    del stream_src
    out["measured_peaks"] = {
        "mfma_bf16_tflops": round(mfma_tflops, 1), "mfma_core_ghz": round(ghz_random, 3),
        "mfma_bf16_tflops_constant_operands": round(mfma_const, 1), "mfma_core_ghz_constant_operands": round(ghz_const, 3),
        "mfma_with_softcap_valu_mix_tflops": round(mix_random, 1), "mfma_with_softcap_valu_mix_core_ghz": round(ghz_mix, 3),
        "mfma_with_softcap_valu_mix_tflops_constant_operands": round(mix_const, 1),
        "mfma_with_softcap_bwd_valu_mix_tflops": round(bwd_mix_random, 1),
        "mfma_with_softcap_bwd_valu_mix_core_ghz": round(ghz_bwd_mix, 3),
        # the two MFMA kernels against the stall-free instruction streams of their hot loops
        "fwd_frac_of_stall_free_mix": round(out["fwd_tflops"] / mix_random, 4),
        "bwd_dkdv_frac_of_stall_free_mix": round(8 * wl.D * pairs / (kt["bwd_dkdv"] * 1e-3) / 1e12 / bwd_mix_random, 4),   # the four GEMMs it executes
        "stream_read_gbs": round(read_gbs, 1),
        "how": "flexattn_probe_mfma: nothing but 32x32x16 bf16 MFMAs on register operands, 2 waves per SIMD, "
               "operands of random sign / exponent / mantissa (the chip clocks lower the more the operands toggle: "
               "compare the constant-operand figures); the valu_mix variant adds, independent of the MFMAs, the "
               "vector instructions the soft-capped forward spends per MFMA, i.e. the hot loop's instruction mix "
               "with nothing to wait for; flexattn_probe_stream_read: 4 GiB, 16-byte loads; events on the launch "
               "stream, core clock from the waves' cycle and real-time counters",
        "fwd_frac_of_measured_mfma": round(out["fwd_tflops"] / mfma_tflops, 4),
        "bwd_frac_of_measured_mfma": round(out["bwd_tflops"] / mfma_tflops, 4),
        "roofline_frac_of_measured_mfma": round(achieved / mfma_tflops, 4),
    }
    if "bwd_dq_roofline" in out:
        out["bwd_dq_roofline"]["frac_of_measured_stream_read"] = round(out["bwd_dq_roofline"]["achieved"] / read_gbs, 4)
    out["roofline"]["traffic_source"] = ("profiles/hbm_traffic.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of "
                                         "this command, scaled by the copy calibration; not measured in this run")

    # The same three launches on all-zero inputs: nothing in the instruction stream depends on the data, so
    # whatever they gain is the clock the chip gives up on N(0,1) operands (its power limit).
    saved = [t.clone() for t in (Q, Kt, V, dO)]
    for t in (Q, Kt, V, dO):
        t.zero_()
    fwd(), bwd()
    torch.cuda.synchronize()
    kz = {"fwd": event_time_ms(fwd, K), "bwd_dkdv": event_time_ms(lambda: bwd(fa.BWD_DKDV), K),
          "bwd_dq": event_time_ms(lambda: bwd(fa.BWD_DQ), K)}
    for t, keep in zip((Q, Kt, V, dO), saved):
        t.copy_(keep)
    del saved
    out["measured_peaks"]["kernel_ms_on_all_zero_inputs"] = {k: round(v, 4) for k, v in kz.items()}
    out["measured_peaks"]["speedup_on_all_zero_inputs"] = {k: round(kt[k] / v, 3) for k, v in kz.items()}

    # ------------------------------------------------------------------ the other training workloads
    if not args.no_other_configs:
        del Q, Kt, V, dO, O, LSE, dQ, dK, dV
        for key, owl in (("cfg3", wlm.CFG3), ("cfg4", wlm.CFG4)):
            out[key] = train_leg(fa, wlm, owl, dev, max(3, K // 4), mfma_tflops, stored, not args.one_bwd_path)

    # ------------------------------------------------------------------ paged decode
    if not args.no_decode:
        dwl = wlm.CFG5
        dinp = wlm.make_decode_inputs(dwl)
        dQ_, Kp, Vp = dinp.Q.to(dev), dinp.K_pool.to(dev), dinp.V_pool.to(dev)
        pt, ctx = dinp.page_table.to(dev), dinp.ctx_lens.to(dev)
        dO_ = torch.empty(dwl.B, dwl.Hq, dwl.D, dtype=torch.bfloat16, device=dev)
        dL = torch.empty(dwl.B, dwl.Hq, dtype=torch.float32, device=dev)
        dws = torch.empty(fa.flexattn_paged_decode_workspace_bytes(dQ_, Kp, pt), dtype=torch.uint8, device=dev)
        dparams = fa.ModParams()

        def dec():
            fa.flexattn_paged_decode(dQ_, Kp, Vp, pt, ctx, fa.SCORE_IDENTITY, fa.MASK_CTX_LEN, dparams, dinp.scale,
                                     dO_, dL, dws)

        for _ in range(W):
            dec()
        torch.cuda.synchronize()
        dms = event_time_ms(dec, K)
        tokens = int(dinp.ctx_lens.sum())
        alg_bytes = tokens * dwl.Hkv * dwl.D * 2 * 2          # K and V, bf16
        gbs = alg_bytes / (dms * 1e-3) / 1e9
        out["decode"] = {
            "workload": dwl.name, "ms": round(dms, 4), "tokens": tokens, "algorithmic_bytes": alg_bytes,
            "value": round(gbs, 1), "unit": "GB/s",
            "roofline": {"kernel": "decode_split+combine", "bound": "hbm", "achieved": round(gbs, 1),
                         "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4),
                         "traffic": measured_traffic("decode_split"),
                         "traffic_source": out["roofline"]["traffic_source"],
                         "frac_of_measured_stream_read": round(gbs / read_gbs, 4)},
        }
        del Kp, Vp

    # ------------------------------------------------------------------ oracle on the host cores
    if not args.no_cpu_baseline:
        from oracle import flex_oracle as fo
        heads = [(b, h) for b in range(wl.B) for h in range(wl.Hq)][:: max(1, wl.B * wl.Hq // args.cpu_heads)]
        heads = heads[:args.cpu_heads]
        score_mod, mask_mod = fo.Softcap(wl.softcap), fo.causal_mask
        t0 = time.perf_counter()
        for b, h in heads:
            fo.attention_head(inp.Q[b, h], inp.K[b, h], inp.V[b, h], score_mod, mask_mod, inp.scale, b, h)
            fo.attention_head_backward(inp.Q[b, h], inp.K[b, h], inp.V[b, h], inp.dO[b, h], score_mod, mask_mod,
                                       inp.scale, b, h)
        cpu_s = time.perf_counter() - t0
        head_flops = 14 * wl.D * (wl.S * (wl.S + 1) // 2)
        out["cpu_baseline"] = {
            "value": round(len(heads) * head_flops / cpu_s / 1e12, 5), "unit": "TFLOP/s",
            "cores": torch.get_num_threads(), "kind": "oracle",
            "sample": f"fp64 oracle forward+backward of {len(heads)} of {wl.B * wl.Hq} (b, h) slices of {wl.name} "
                      f"in {cpu_s:.1f} s (same unmasked-FLOP convention)",
        }

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
