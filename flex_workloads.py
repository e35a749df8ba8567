"""Seeded synthetic inputs for the FlexAttention hot path.

This module only draws random tensors and integer tables; it holds none of the
method's arithmetic (no masks, no score modifications, no softmax).  Both the
CPU oracle's tests and the HIP path's tests/bench take their inputs from here,
so the two sides see identical bit patterns.

All floating-point tensors are drawn as fp32 N(0,1) from a seeded CPU
``torch.Generator`` and rounded once to bf16; the oracle widens those bf16
values exactly to fp64.

The five named workloads mirror the shapes of the paper's evaluation
(section 6.2: bf16, causal / alibi / sliding-window / prefix-LM / soft-cap /
document variants, with and without GQA; section 6.4: paged decode with
16-token pages) at the sizes this repository is benchmarked on.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Optional

import torch


@dataclass(frozen=True)
class Workload:
    """Shape and modifier description of one synthetic workload."""

    name: str
    B: int
    Hq: int
    Hkv: int
    S: int                # Q_LEN == KV_LEN for the training shapes
    D: int
    Bq: int               # BlockMask block size along Q_LEN
    Bk: int               # BlockMask block size along KV_LEN
    mask: str             # "causal" | "doc_causal" | "swa_causal_or_prefix" | "ctx_len"
    score: str            # "identity" | "softcap" | "alibi" | "rel_bias" | "alibi_softcap" | "rel_bias_softcap"
    seed: int
    backward: bool = True
    softcap: float = 0.0
    window: int = 0
    prefix_len: int = 0
    rel_len: int = 0
    doc_len_min: int = 0
    doc_len_max: int = 0
    # decode only
    page_size: int = 0
    ctx_min: int = 0
    ctx_max: int = 0
    max_pages: int = 0

    def scaled(self, **kw) -> "Workload":
        """Same recipe at other sizes (used for parity cases the oracle can finish)."""
        return replace(self, **kw)


CFG1 = Workload("cfg1_causal_s256", B=1, Hq=2, Hkv=2, S=256, D=64, Bq=64, Bk=64,
                mask="causal", score="identity", seed=1001, backward=False)
CFG2 = Workload("cfg2_causal_softcap_s8192", B=4, Hq=16, Hkv=16, S=8192, D=128, Bq=128, Bk=64,
                mask="causal", score="softcap", softcap=30.0, seed=1002)
CFG3 = Workload("cfg3_document_alibi_s16384", B=1, Hq=16, Hkv=16, S=16384, D=64, Bq=128, Bk=64,
                mask="doc_causal", score="alibi", seed=1003, doc_len_min=256, doc_len_max=4096)
CFG4 = Workload("cfg4_swa_prefix_relbias_gqa_s32768", B=2, Hq=32, Hkv=8, S=32768, D=128,
                Bq=128, Bk=64, mask="swa_causal_or_prefix", score="rel_bias", seed=1004,
                window=4096, prefix_len=1024, rel_len=256)
CFG5 = Workload("cfg5_paged_decode", B=64, Hq=32, Hkv=8, S=1, D=128, Bq=1, Bk=16,
                mask="ctx_len", score="identity", seed=1005, backward=False,
                page_size=16, ctx_min=1024, ctx_max=32768, max_pages=2048)

CONFIGS = [CFG1, CFG2, CFG3, CFG4, CFG5]


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


def randn_bf16(gen: torch.Generator, *shape: int, std: float = 1.0) -> torch.Tensor:
    """fp32 N(0, std) rounded once to bf16 (CPU tensor)."""
    x = torch.randn(*shape, generator=gen, dtype=torch.float32)
    if std != 1.0:
        x = x * std
    return x.to(torch.bfloat16)


def document_lengths(gen: torch.Generator, S: int, lo: int, hi: int) -> list[int]:
    """Draw lengths uniformly in [lo, hi] until they fill S; the last one is cut to fit."""
    out, total = [], 0
    while total < S:
        L = int(torch.randint(lo, hi + 1, (1,), generator=gen).item())
        L = min(L, S - total)
        out.append(L)
        total += L
    return out


def document_ids(lengths: list[int]) -> torch.Tensor:
    """Token -> document index map (int32, nondecreasing) for packed documents."""
    ids = torch.empty(sum(lengths), dtype=torch.int32)
    pos = 0
    for i, L in enumerate(lengths):
        ids[pos:pos + L] = i
        pos += L
    return ids


def alibi_slopes(H: int) -> torch.Tensor:
    """Per-head slopes 2^(-8 (h+1) / H), h = 0..H-1 (fp32)."""
    return torch.tensor([2.0 ** (-8.0 * (h + 1) / H) for h in range(H)], dtype=torch.float32)


@dataclass
class TrainInputs:
    wl: Workload
    Q: torch.Tensor        # [B, Hq, S, D] bf16
    K: torch.Tensor        # [B, Hkv, S, D] bf16
    V: torch.Tensor        # [B, Hkv, S, D] bf16
    dO: Optional[torch.Tensor]          # [B, Hq, S, D] bf16
    scale: float
    doc_ids: Optional[torch.Tensor] = None      # [B, S] int32
    doc_lengths: Optional[list] = None
    slopes: Optional[torch.Tensor] = None       # [Hq] fp32
    rel_bias: Optional[torch.Tensor] = None     # [Hq, rel_len] fp32


def make_train_inputs(wl: Workload, with_dO: Optional[bool] = None) -> TrainInputs:
    """Q, K, V (and dO) plus whatever side tables the workload's mods capture."""
    gen = _gen(wl.seed)
    Q = randn_bf16(gen, wl.B, wl.Hq, wl.S, wl.D)
    K = randn_bf16(gen, wl.B, wl.Hkv, wl.S, wl.D)
    V = randn_bf16(gen, wl.B, wl.Hkv, wl.S, wl.D)
    want_dO = wl.backward if with_dO is None else with_dO
    dO = randn_bf16(gen, wl.B, wl.Hq, wl.S, wl.D) if want_dO else None
    inp = TrainInputs(wl, Q, K, V, dO, 1.0 / math.sqrt(wl.D))
    if wl.mask == "doc_causal":
        rows, lens = [], []
        for _ in range(wl.B):
            L = document_lengths(gen, wl.S, wl.doc_len_min, wl.doc_len_max)
            lens.append(L)
            rows.append(document_ids(L))
        inp.doc_ids = torch.stack(rows).contiguous()
        inp.doc_lengths = lens
    if "alibi" in wl.score:
        inp.slopes = alibi_slopes(wl.Hq)
    if "rel_bias" in wl.score:
        inp.rel_bias = (torch.randn(wl.Hq, wl.rel_len, generator=gen, dtype=torch.float32) * 0.1).contiguous()
    return inp


@dataclass
class DecodeInputs:
    wl: Workload
    Q: torch.Tensor            # [nseq, Hq, 1, D] bf16
    K_pool: torch.Tensor       # [n_pool_pages, Hkv, page_size, D] bf16
    V_pool: torch.Tensor       # [n_pool_pages, Hkv, page_size, D] bf16
    page_table: torch.Tensor   # [nseq, max_pages] int32 (unused entries = 0)
    ctx_lens: torch.Tensor     # [nseq] int32
    scale: float


def make_decode_inputs(wl: Workload, ctx_lens: Optional[list[int]] = None,
                       slack_pages: int = 0) -> DecodeInputs:
    """Paged KV cache: pages of every sequence scattered over one pool by a seeded permutation."""
    gen = _gen(wl.seed)
    nseq, P = wl.B, wl.page_size
    if ctx_lens is None:
        ctx = torch.randint(wl.ctx_min, wl.ctx_max + 1, (nseq,), generator=gen, dtype=torch.int64)
    else:
        assert len(ctx_lens) == nseq
        ctx = torch.tensor(ctx_lens, dtype=torch.int64)
    n_pages_seq = (ctx + P - 1) // P
    assert int(n_pages_seq.max().item()) <= wl.max_pages
    n_pool = int(n_pages_seq.sum().item()) + slack_pages
    n_pool = max(n_pool, 1)
    perm = torch.randperm(n_pool, generator=gen).to(torch.int32)
    page_table = torch.zeros(nseq, wl.max_pages, dtype=torch.int32)
    pos = 0
    for b in range(nseq):
        n = int(n_pages_seq[b].item())
        page_table[b, :n] = perm[pos:pos + n]
        pos += n
    Q = randn_bf16(gen, nseq, wl.Hq, 1, wl.D)
    K_pool = randn_bf16(gen, n_pool, wl.Hkv, P, wl.D)
    V_pool = randn_bf16(gen, n_pool, wl.Hkv, P, wl.D)
    return DecodeInputs(wl, Q, K_pool, V_pool, page_table.contiguous(),
                        ctx.to(torch.int32).contiguous(), 1.0 / math.sqrt(wl.D))


@dataclass
class PrefillInputs:
    wl: Workload
    Q: torch.Tensor            # [nseq, Hq, q_len, D] bf16: the chunk's queries
    K_pool: torch.Tensor
    V_pool: torch.Tensor
    page_table: torch.Tensor
    kv_lens: torch.Tensor      # [nseq] int32: tokens in the cache, the chunk's own included
    q_offsets: torch.Tensor    # [nseq] int32: position of the chunk's first query = kv_lens - q_len
    scale: float


def make_prefill_inputs(wl: Workload, kv_lens: list[int], q_len: int, slack_pages: int = 0) -> PrefillInputs:
    """A chunk of q_len new tokens per sequence on top of a paged cache (chunked prefill): the cache
    already holds the chunk's own keys, so sequence b has kv_lens[b] >= q_len tokens."""
    assert all(n >= q_len for n in kv_lens)
    d = make_decode_inputs(wl, ctx_lens=kv_lens, slack_pages=slack_pages)
    gen = _gen(wl.seed + 7919)
    Q = randn_bf16(gen, wl.B, wl.Hq, q_len, wl.D)
    return PrefillInputs(wl, Q, d.K_pool, d.V_pool, d.page_table, d.ctx_lens,
                         (d.ctx_lens - q_len).to(torch.int32).contiguous(), d.scale)


def blockmask_all_partial(alloc_blockmask, bm):
    """The same BlockMask with every FULL block listed as PARTIAL, i.e. the full-block optimisation
    switched off (index-list surgery only; `alloc_blockmask` allocates the eight arrays)."""
    out = alloc_blockmask(bm.Bm, bm.Hm, bm.q_len, bm.kv_len, bm.Bq, bm.Bk, device=bm.kv_num_blocks.device)
    for num, idx, fnum, fidx, onum, oidx, ofnum, ofidx in (
            (bm.kv_num_blocks, bm.kv_indices, bm.full_kv_num_blocks, bm.full_kv_indices,
             out.kv_num_blocks, out.kv_indices, out.full_kv_num_blocks, out.full_kv_indices),
            (bm.q_num_blocks, bm.q_indices, bm.full_q_num_blocks, bm.full_q_indices,
             out.q_num_blocks, out.q_indices, out.full_q_num_blocks, out.full_q_indices)):
        n = idx.shape[-1]
        pos = torch.arange(n, device=idx.device)
        big = torch.iinfo(torch.int32).max
        a = torch.where(pos < num.unsqueeze(-1), idx, big)
        b = torch.where(pos < fnum.unsqueeze(-1), fidx, big)
        merged = torch.sort(torch.cat([a, b], dim=-1), dim=-1).values[..., :n]
        total = num + fnum
        oidx.copy_(torch.where(pos < total.unsqueeze(-1), merged, 0).to(torch.int32))
        onum.copy_(total)
        ofnum.zero_()
        ofidx.zero_()
    if bm.stats is not None and out.stats is not None:
        out.stats.copy_(bm.stats)
    for name in ("kv_order", "q_order"):      # listed blocks per line are unchanged, so is the work order
        if getattr(bm, name, None) is not None and getattr(out, name, None) is not None:
            getattr(out, name).copy_(getattr(bm, name))
    return out
