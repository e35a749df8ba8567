"""fp64 CPU oracle for the FlexAttention hot path.  TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline``
leg may import this module; the product path (``paper_2412_05496_amd``) never
does, and this module imports nothing from it.

Everything here is the plain definition written out with PyTorch CPU ops in
float64: the full row of scores is materialised, modified, masked and
soft-maxed; there is no tiling over KV, no online softmax, no block skipping.

What follows what (paper = arXiv 2412.05496):

* ``flex_attention``            Eq. 1: softmax(mod(Q K^T / sqrt(d_k))) V, with the
                                tensor shapes of section 2.1 and the mod order of
                                section 3.1 (score_mod on the scaled score, then
                                mask_mod -> -inf).
* mask_mods / score_mods        section 3.1 ("Mapping to concrete examples") and
                                section 3.2 (and_mask / or_mask, prefix-LM).
* ``create_block_mask``         section 4.2: a block is skipped iff every scalar in it
                                is masked; "full" iff none is; "partial" otherwise.
* ``convert_block_mask_paged``  section 5.1 ("Fused indirect memory access",
                                "mask_mod and score_mod Conversion").
* ``paged_decode``              section 5.1: the physical cache is addressed through
                                the page table; the result must equal attention
                                over the logical (un-paged) cache.
* ``with_q_offset`` / ``QOffset``  section 5.2: at inference the mods are called with q_idx + offset,
                                the number of tokens already processed.
* ``paged_attention``           sections 5.1 + 5.2 for a chunk of several query tokens per sequence
                                (chunked prefill): un-page, then Eq. 1 with the mods shifted
                                by each sequence's offset.
* ``neighborhood_mask``         appendix (Neighborhood Attention): every pixel of a 2-D canvas attends
                                to its K x K nearest pixels; the tokens are laid out row by row,
                                in 2-D tiles, or along the Morton curve.
* ``flex_attention_backward_captured``  gradients of the tensors a score_mod captures (the bias of
                                the ALiBi example, the table of the relative-bias example,
                                section 3.1): chain rule through the mods, pinned by finite
                                differences and library autograd in the tests.
* ``flex_attention_backward``   the paper only states that a backward template
                                exists (section 4.1); this is ordinary calculus on
                                Eq. 1, pinned by finite differences in the tests.

Conventions taken where the paper is silent: natural-log LSE of the modified,
masked, scaled scores; a row with every key masked gives O = 0, LSE = -inf and
zero gradients; consecutive query heads share a KV head (hkv = hq // G).
"""
from __future__ import annotations

import math
from typing import Callable, Optional, Sequence

import torch

F64 = torch.float64
NEG_INF = float("-inf")

# --------------------------------------------------------------------------
# mask_mod(b, h, q_idx, kv_idx) -> bool            (section 3.1)
# b, h are Python ints; q_idx is an int64 column [nq, 1]; kv_idx an int64 row [1, nkv].
# --------------------------------------------------------------------------
MaskMod = Callable[[int, int, torch.Tensor, torch.Tensor], torch.Tensor]


def no_mask(b, h, q_idx, kv_idx):
    return torch.ones(q_idx.shape[0], kv_idx.shape[1], dtype=torch.bool)


def causal_mask(b, h, q_idx, kv_idx):
    return q_idx >= kv_idx


def sliding_window_mask(window: int) -> MaskMod:
    """q_idx - kv_idx <= window (one-sided, as the paper writes it)."""
    def mod(b, h, q_idx, kv_idx):
        return (q_idx - kv_idx) <= window
    return mod


def document_mask(document_id: torch.Tensor) -> MaskMod:
    """document_id[b, q_idx] == document_id[b, kv_idx]; document_id is [B, S] (or [1, S])."""
    doc = document_id.to(torch.int64)

    def mod(b, h, q_idx, kv_idx):
        row = doc[b if doc.shape[0] > 1 else 0]
        return row[q_idx] == row[kv_idx]
    return mod


def prefix_mask(prefix_len: int) -> MaskMod:
    """Keys inside the prefix are visible to every query."""
    def mod(b, h, q_idx, kv_idx):
        return (kv_idx < prefix_len) & (q_idx >= 0)
    return mod


def ctx_len_mask(ctx_lens: torch.Tensor) -> MaskMod:
    """kv_idx < ctx_len[b] (decode: only the filled part of a sequence's cache is visible)."""
    ctx = ctx_lens.to(torch.int64)

    def mod(b, h, q_idx, kv_idx):
        return (kv_idx < int(ctx[b])) & (q_idx >= 0)
    return mod


def and_mask(*mods: MaskMod) -> MaskMod:
    def mod(b, h, q_idx, kv_idx):
        out = mods[0](b, h, q_idx, kv_idx)
        for m in mods[1:]:
            out = out & m(b, h, q_idx, kv_idx)
        return out
    return mod


def or_mask(*mods: MaskMod) -> MaskMod:
    def mod(b, h, q_idx, kv_idx):
        out = mods[0](b, h, q_idx, kv_idx)
        for m in mods[1:]:
            out = out | m(b, h, q_idx, kv_idx)
        return out
    return mod


# --------------------------------------------------------------------------
# score_mod(score, b, h, q_idx, kv_idx) -> score'   (section 3.1)
# Each carries d score' / d score for the backward pass.
# --------------------------------------------------------------------------
class ScoreMod:
    def __call__(self, score, b, h, q_idx, kv_idx):
        raise NotImplementedError

    def grad(self, score, b, h, q_idx, kv_idx):
        """d score_mod / d score evaluated at `score` (same shape)."""
        raise NotImplementedError

    def captured_grad(self, score, b, h, q_idx, kv_idx, g_out, out: dict):
        """Adds to out[name] the gradient of the tensors this mod captures, given g_out = dL / d(this
        mod's output) (same shape as score).  Mods that capture no tensor add nothing."""


class Identity(ScoreMod):
    def __call__(self, score, b, h, q_idx, kv_idx):
        return score

    def grad(self, score, b, h, q_idx, kv_idx):
        return torch.ones_like(score)


class Alibi(ScoreMod):
    """score + alibi_bias[h] * (q_idx - kv_idx)."""

    def __init__(self, alibi_bias: torch.Tensor):
        self.bias = alibi_bias.to(F64)

    def __call__(self, score, b, h, q_idx, kv_idx):
        return score + self.bias[h] * (q_idx - kv_idx).to(F64)

    def grad(self, score, b, h, q_idx, kv_idx):
        return torch.ones_like(score)

    def captured_grad(self, score, b, h, q_idx, kv_idx, g_out, out):
        d = out.setdefault("alibi_bias", torch.zeros_like(self.bias))
        d[h] += (g_out * (q_idx - kv_idx).to(F64)).sum()


class Softcap(ScoreMod):
    """cap * tanh(score / cap)."""

    def __init__(self, cap: float):
        self.cap = float(cap)

    def __call__(self, score, b, h, q_idx, kv_idx):
        return self.cap * torch.tanh(score / self.cap)

    def grad(self, score, b, h, q_idx, kv_idx):
        t = torch.tanh(score / self.cap)
        return 1.0 - t * t


class RelBias(ScoreMod):
    """score + table[h, clamp(q_idx - kv_idx, 0, rel_len - 1)]."""

    def __init__(self, table: torch.Tensor):
        self.table = table.to(F64)

    def __call__(self, score, b, h, q_idx, kv_idx):
        rel = (q_idx - kv_idx).clamp(0, self.table.shape[1] - 1)
        return score + self.table[h][rel]

    def grad(self, score, b, h, q_idx, kv_idx):
        return torch.ones_like(score)

    def captured_grad(self, score, b, h, q_idx, kv_idx, g_out, out):
        d = out.setdefault("rel_bias", torch.zeros_like(self.table))
        rel = (q_idx - kv_idx).clamp(0, self.table.shape[1] - 1).expand_as(g_out)
        d[h].index_add_(0, rel.reshape(-1), g_out.reshape(-1))


class Compose(ScoreMod):
    """Nested score_mods: outer(inner(score))."""

    def __init__(self, inner: ScoreMod, outer: ScoreMod):
        self.inner, self.outer = inner, outer

    def __call__(self, score, b, h, q_idx, kv_idx):
        return self.outer(self.inner(score, b, h, q_idx, kv_idx), b, h, q_idx, kv_idx)

    def grad(self, score, b, h, q_idx, kv_idx):
        mid = self.inner(score, b, h, q_idx, kv_idx)
        return self.outer.grad(mid, b, h, q_idx, kv_idx) * self.inner.grad(score, b, h, q_idx, kv_idx)

    def captured_grad(self, score, b, h, q_idx, kv_idx, g_out, out):
        mid = self.inner(score, b, h, q_idx, kv_idx)
        self.outer.captured_grad(mid, b, h, q_idx, kv_idx, g_out, out)
        self.inner.captured_grad(score, b, h, q_idx, kv_idx, g_out * self.outer.grad(mid, b, h, q_idx, kv_idx), out)


# --------------------------------------------------------------------------
# Forward (Eq. 1)
# --------------------------------------------------------------------------
def _idx(lo: int, hi: int) -> torch.Tensor:
    return torch.arange(lo, hi, dtype=torch.int64)


def _modified_scores(Qh, Kh, score_mod, mask_mod, scale, b, h, q_idx):
    """Rows `q_idx` of mod(Q K^T * scale) for one head: (s_mod, keep)."""
    kv_idx = _idx(0, Kh.shape[0]).view(1, -1)
    qi = q_idx.view(-1, 1)
    s = (Qh[q_idx] @ Kh.T) * scale
    s_mod = score_mod(s, b, h, qi, kv_idx)
    keep = mask_mod(b, h, qi, kv_idx)
    return s, s_mod, keep


def _softmax_rows(s_mod, keep):
    """Safe softmax over the last axis of masked scores: (P, LSE).  All-masked rows: P = 0, LSE = -inf."""
    s_m = torch.where(keep, s_mod, torch.full_like(s_mod, NEG_INF))
    m = s_m.max(dim=1).values
    dead = torch.isinf(m) & (m < 0)
    m_safe = torch.where(dead, torch.zeros_like(m), m)
    e = torch.exp(s_m - m_safe[:, None])          # masked entries: exp(-inf) = 0
    l = e.sum(dim=1)
    l_safe = torch.where(dead, torch.ones_like(l), l)
    P = e / l_safe[:, None]
    lse = torch.where(dead, torch.full_like(m, NEG_INF), m_safe + torch.log(l_safe))
    return P, lse


def attention_head(Qh, Kh, Vh, score_mod: ScoreMod, mask_mod: MaskMod, scale: float,
                   b: int, h: int, q_rows: Optional[torch.Tensor] = None, stripe: int = 1024):
    """One (b, h): O[rows, D], LSE[rows] in fp64.  Qh [Sq, D]; Kh, Vh [Skv, D] (any float dtype)."""
    Qh, Kh, Vh = Qh.to(F64), Kh.to(F64), Vh.to(F64)
    rows = _idx(0, Qh.shape[0]) if q_rows is None else q_rows.to(torch.int64)
    O = torch.empty(rows.numel(), Vh.shape[1], dtype=F64)
    LSE = torch.empty(rows.numel(), dtype=F64)
    for r0 in range(0, rows.numel(), stripe):
        q_idx = rows[r0:r0 + stripe]
        _, s_mod, keep = _modified_scores(Qh, Kh, score_mod, mask_mod, scale, b, h, q_idx)
        P, lse = _softmax_rows(s_mod, keep)
        O[r0:r0 + stripe] = P @ Vh
        LSE[r0:r0 + stripe] = lse
    return O, LSE


def flex_attention(Q, K, V, score_mod: ScoreMod, mask_mod: MaskMod, scale: Optional[float] = None):
    """Q [B,Hq,Sq,D]; K,V [B,Hkv,Skv,D] -> O [B,Hq,Sq,D] fp64, LSE [B,Hq,Sq] fp64."""
    B, Hq, Sq, D = Q.shape
    Hkv = K.shape[1]
    assert Hq % Hkv == 0
    G = Hq // Hkv
    scale = 1.0 / math.sqrt(D) if scale is None else scale
    O = torch.empty(B, Hq, Sq, V.shape[3], dtype=F64)
    LSE = torch.empty(B, Hq, Sq, dtype=F64)
    for b in range(B):
        for h in range(Hq):
            O[b, h], LSE[b, h] = attention_head(Q[b, h], K[b, h // G], V[b, h // G],
                                                score_mod, mask_mod, scale, b, h)
    return O, LSE


# --------------------------------------------------------------------------
# Backward
# --------------------------------------------------------------------------
def attention_head_backward(Qh, Kh, Vh, dOh, score_mod: ScoreMod, mask_mod: MaskMod, scale: float,
                            b: int, h: int, q_rows: Optional[torch.Tensor] = None, stripe: int = 1024):
    """One query head: dQ [rows, D] and this head's contributions dK, dV [Skv, D] (fp64).

    With P the softmax of the modified masked scores:
      dV = P^T dO;  dP = dO V^T;  delta = rowsum(P * dP);  dS' = P * (dP - delta);
      dS = dS' * (d score_mod / d s);  dQ = scale * dS K;  dK = scale * dS^T Q.
    Masked entries have P = 0 and so contribute nothing.  With `q_rows`, only those query rows
    are evaluated: dQ holds exactly their rows, dK / dV only their contributions.
    """
    Qh, Kh, Vh, dOh = Qh.to(F64), Kh.to(F64), Vh.to(F64), dOh.to(F64)
    rows = _idx(0, Qh.shape[0]) if q_rows is None else q_rows.to(torch.int64)
    dQ = torch.empty(rows.numel(), Qh.shape[1], dtype=F64)
    dK = torch.zeros_like(Kh)
    dV = torch.zeros_like(Vh)
    kv_idx = _idx(0, Kh.shape[0]).view(1, -1)
    for r0 in range(0, rows.numel(), stripe):
        q_idx = rows[r0:r0 + stripe]
        s, s_mod, keep = _modified_scores(Qh, Kh, score_mod, mask_mod, scale, b, h, q_idx)
        P, _ = _softmax_rows(s_mod, keep)
        dO_r = dOh[q_idx]
        dV += P.T @ dO_r
        dP = dO_r @ Vh.T
        delta = (P * dP).sum(dim=1, keepdim=True)
        dS_mod = P * (dP - delta)
        g = score_mod.grad(s, b, h, q_idx.view(-1, 1), kv_idx)
        dS = torch.where(keep, dS_mod * g, torch.zeros_like(dS_mod))
        dQ[r0:r0 + stripe] = scale * (dS @ Kh)
        dK += scale * (dS.T @ Qh[q_idx])
    return dQ, dK, dV


def flex_attention_backward(Q, K, V, dO, score_mod: ScoreMod, mask_mod: MaskMod,
                            scale: Optional[float] = None):
    """dQ [B,Hq,Sq,D], dK, dV [B,Hkv,Skv,D] in fp64; dK/dV sum over the G query heads of a group."""
    B, Hq, Sq, D = Q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    scale = 1.0 / math.sqrt(D) if scale is None else scale
    dQ = torch.empty(B, Hq, Sq, D, dtype=F64)
    dK = torch.zeros(B, Hkv, K.shape[2], D, dtype=F64)
    dV = torch.zeros(B, Hkv, V.shape[2], V.shape[3], dtype=F64)
    for b in range(B):
        for h in range(Hq):
            dq, dk, dv = attention_head_backward(Q[b, h], K[b, h // G], V[b, h // G], dO[b, h],
                                                 score_mod, mask_mod, scale, b, h)
            dQ[b, h] = dq
            dK[b, h // G] += dk
            dV[b, h // G] += dv
    return dQ, dK, dV


def flex_attention_backward_captured(Q, K, V, dO, score_mod: ScoreMod, mask_mod: MaskMod,
                                     scale: Optional[float] = None, stripe: int = 1024) -> dict:
    """Gradients of the tensors the score_mod captures (ALiBi bias per head, relative-bias table;
    section 3.1 examples), summed over batch and positions: {name: tensor like the captured one}.
    With dS' = P * (dP - delta) the gradient flowing into the score_mod's output (zero where masked),
    every mod passes it on to what it captures (chain rule through the mods applied after it)."""
    B, Hq, Sq, D = Q.shape
    G = Hq // K.shape[1]
    scale = 1.0 / math.sqrt(D) if scale is None else scale
    out: dict = {}
    kv_idx = _idx(0, K.shape[2]).view(1, -1)
    for b in range(B):
        for h in range(Hq):
            Qh, Kh, Vh, dOh = (t.to(F64) for t in (Q[b, h], K[b, h // G], V[b, h // G], dO[b, h]))
            for r0 in range(0, Sq, stripe):
                q_idx = _idx(r0, min(r0 + stripe, Sq))
                s, s_mod, keep = _modified_scores(Qh, Kh, score_mod, mask_mod, scale, b, h, q_idx)
                P, _ = _softmax_rows(s_mod, keep)
                dP = dOh[q_idx] @ Vh.T
                delta = (P * dP).sum(dim=1, keepdim=True)
                g_out = torch.where(keep, P * (dP - delta), torch.zeros_like(P))
                score_mod.captured_grad(s, b, h, q_idx.view(-1, 1), kv_idx, g_out, out)
    return out


# --------------------------------------------------------------------------
# BlockMask (section 4.2)
# --------------------------------------------------------------------------
def block_kinds(mask_mod: MaskMod, Bm: int, Hm: int, q_len: int, kv_len: int, Bq: int, Bk: int):
    """Brute force: per block, count unmasked scalars.  Returns int8 [Bm,Hm,NR,NC]:
    0 = skipped (all masked), 1 = partial, 2 = full (none masked); plus the total unmasked count.
    Lengths that are no multiple of the block size: NR and NC round up, and the part of a last
    block that lies outside the score matrix counts as masked (such a block is never full)."""
    NR, NC = -(-q_len // Bq), -(-kv_len // Bk)
    kinds = torch.zeros(Bm, Hm, NR, NC, dtype=torch.int8)
    pairs = 0
    kv_idx = _idx(0, kv_len).view(1, -1)
    for b in range(Bm):
        for h in range(Hm):
            for i in range(NR):
                rows = min(Bq, q_len - i * Bq)
                q_idx = _idx(i * Bq, i * Bq + rows).view(-1, 1)
                keep = torch.zeros(Bq, NC * Bk, dtype=torch.bool)
                keep[:rows, :kv_len] = mask_mod(b, h, q_idx, kv_idx).expand(rows, kv_len)
                cnt = keep.reshape(Bq, NC, Bk).sum(dim=(0, 2))
                pairs += int(cnt.sum())
                kinds[b, h, i] = (cnt > 0).to(torch.int8) + (cnt == Bq * Bk).to(torch.int8)
    return kinds, pairs


def _compact(flags: torch.Tensor):
    """flags bool [..., R, C] -> (num [..., R] int32, indices [..., R, C] int32 ascending, tail 0)."""
    C = flags.shape[-1]
    num = flags.sum(dim=-1).to(torch.int32)
    col = _idx(0, C).expand(flags.shape)
    key = torch.where(flags, col, col + C)                  # set entries first, ascending
    order = torch.argsort(key, dim=-1, stable=True)
    pos = _idx(0, C).expand(flags.shape)
    idx = torch.where(pos < num[..., None].to(torch.int64), order, torch.zeros_like(order))
    return num, idx.to(torch.int32)


def create_block_mask(mask_mod: MaskMod, Bm: int, Hm: int, q_len: int, kv_len: int, Bq: int, Bk: int):
    """The eight int32 arrays of a BlockMask plus statistics.

    kv_num_blocks / kv_indices list the PARTIAL blocks of each row of blocks,
    full_kv_* the FULL ones; q_* / full_q_* are the same sets listed per column of
    blocks (the transpose the backward pass walks).  Indices ascend; entries past the
    count are 0.
    """
    kinds, pairs = block_kinds(mask_mod, Bm, Hm, q_len, kv_len, Bq, Bk)
    partial, full = kinds == 1, kinds == 2
    out = {}
    out["kv_num_blocks"], out["kv_indices"] = _compact(partial)
    out["full_kv_num_blocks"], out["full_kv_indices"] = _compact(full)
    out["q_num_blocks"], out["q_indices"] = _compact(partial.transpose(-1, -2))
    out["full_q_num_blocks"], out["full_q_indices"] = _compact(full.transpose(-1, -2))
    out["stats"] = {"partial": int(partial.sum()), "full": int(full.sum()),
                    "total": kinds.numel(), "unmasked_pairs": pairs}
    out["kv_order"] = work_order(out["kv_num_blocks"] + out["full_kv_num_blocks"], reversed_when_long=True)
    out["q_order"] = work_order(out["q_num_blocks"] + out["full_q_num_blocks"], reversed_when_long=False)
    return out


WORK_ORDER_MAX_LINES = 8192


def work_order(counts: torch.Tensor, reversed_when_long: bool) -> torch.Tensor:
    """Not in the paper: the order in which a launch should take the rows (columns) of blocks so that
    its longest ones start first -- the lines of each plane by descending number of listed blocks,
    ties by ascending index.  counts [Bm, Hm, n] -> int32 [Bm, Hm, n], a permutation per plane.
    More than WORK_ORDER_MAX_LINES lines are not sorted: n-1 .. 0 (rows) resp. 0 .. n-1 (columns)."""
    n = counts.shape[-1]
    if n > WORK_ORDER_MAX_LINES:
        line = torch.arange(n - 1, -1, -1) if reversed_when_long else torch.arange(n)
        return line.expand(counts.shape).to(torch.int32).contiguous()
    return torch.argsort(counts.to(torch.int64), dim=-1, descending=True, stable=True).to(torch.int32)


def convert_block_mask_paged(num_blocks: torch.Tensor, indices: torch.Tensor, page_table: torch.Tensor,
                             n_pool_pages: int):
    """Logical -> physical KV block lists (section 5.1).  num_blocks [B,Hm,NR], indices [B,Hm,NR,NC]
    (Bk == page size), page_table [B, max_pages].  Counts are unchanged; each of the first `num`
    entries j becomes page_table[b, j]; the tail stays 0.  Also returns the physical -> logical
    vector for the pages the lists touch (-1 elsewhere)."""
    B, Hm, NR, NC = indices.shape
    phys = torch.zeros_like(indices)
    phys2log = torch.full((n_pool_pages,), -1, dtype=torch.int32)
    for b in range(B):
        for h in range(Hm):
            for i in range(NR):
                n = int(num_blocks[b, h, i])
                logical = indices[b, h, i, :n].to(torch.int64)
                p = page_table[b][logical]
                phys[b, h, i, :n] = p
                phys2log[p.to(torch.int64)] = logical.to(torch.int32)
    return phys, phys2log


# --------------------------------------------------------------------------
# Paged decode (section 5.1): un-page, then Eq. 1 with Q_LEN = 1
# --------------------------------------------------------------------------
def unpage(pool: torch.Tensor, page_table_row: torch.Tensor, n_tokens: int) -> torch.Tensor:
    """pool [n_pages, Hkv, P, D] -> logical [Hkv, n_tokens, D] for one sequence."""
    P = pool.shape[2]
    n_pages = (n_tokens + P - 1) // P
    pages = pool[page_table_row[:n_pages].to(torch.int64)]           # [n_pages, Hkv, P, D]
    logical = pages.permute(1, 0, 2, 3).reshape(pool.shape[1], n_pages * P, pool.shape[3])
    return logical[:, :n_tokens]


def paged_decode(Q, K_pool, V_pool, page_table, ctx_lens, score_mod: ScoreMod, scale: Optional[float] = None,
                 mask_mod: Optional[MaskMod] = None):
    """Q [nseq,Hq,1,D]; pools [n_pages,Hkv,P,D]; page_table [nseq,max_pages]; ctx_lens [nseq].
    Returns O [nseq,Hq,1,D], LSE [nseq,Hq,1] (fp64).  The query's position is ctx_len - 1."""
    nseq, Hq, _, D = Q.shape
    Hkv = K_pool.shape[1]
    G = Hq // Hkv
    scale = 1.0 / math.sqrt(D) if scale is None else scale
    mask = ctx_len_mask(ctx_lens) if mask_mod is None else mask_mod
    O = torch.zeros(nseq, Hq, 1, D, dtype=F64)
    LSE = torch.full((nseq, Hq, 1), NEG_INF, dtype=F64)
    P = K_pool.shape[2]
    for b in range(nseq):
        n = int(ctx_lens[b])
        n_padded = ((n + P - 1) // P) * P          # the mask, not the slicing, hides the ragged tail
        if n_padded == 0:
            continue
        Kl = unpage(K_pool, page_table[b], n_padded)
        Vl = unpage(V_pool, page_table[b], n_padded)
        q_pos = torch.tensor([max(n - 1, 0)], dtype=torch.int64)
        for h in range(Hq):
            Qh = Q[b, h].to(F64)
            kv_idx = _idx(0, n_padded).view(1, -1)
            s = (Qh @ Kl[h // G].to(F64).T) * scale
            s_mod = score_mod(s, b, h, q_pos.view(-1, 1), kv_idx)
            keep = mask(b, h, q_pos.view(-1, 1), kv_idx).expand(1, n_padded)
            Pm, lse = _softmax_rows(s_mod, keep)
            O[b, h] = Pm @ Vl[h // G].to(F64)
            LSE[b, h] = lse
    return O, LSE


# --------------------------------------------------------------------------
# Offset conversion (section 5.2) and paged attention with several query tokens
# --------------------------------------------------------------------------
def with_q_offset(mask_mod: MaskMod, q_offsets: torch.Tensor) -> MaskMod:
    """The inference counterpart of a mask_mod: it sees q_idx + q_offsets[b]."""
    off = q_offsets.to(torch.int64)

    def mod(b, h, q_idx, kv_idx):
        return mask_mod(b, h, q_idx + off[b], kv_idx)
    return mod


class QOffset(ScoreMod):
    """The inference counterpart of a score_mod: it sees q_idx + q_offsets[b]."""

    def __init__(self, inner: ScoreMod, q_offsets: torch.Tensor):
        self.inner, self.off = inner, q_offsets.to(torch.int64)

    def __call__(self, score, b, h, q_idx, kv_idx):
        return self.inner(score, b, h, q_idx + self.off[b], kv_idx)

    def grad(self, score, b, h, q_idx, kv_idx):
        return self.inner.grad(score, b, h, q_idx + self.off[b], kv_idx)

    def captured_grad(self, score, b, h, q_idx, kv_idx, g_out, out):
        self.inner.captured_grad(score, b, h, q_idx + self.off[b], kv_idx, g_out, out)


def paged_attention(Q, K_pool, V_pool, page_table, kv_lens, q_offsets, score_mod: ScoreMod, mask_mod: MaskMod,
                    scale: Optional[float] = None):
    """Q [nseq,Hq,Lq,D] (query i of sequence b sits at position q_offsets[b] + i); pools
    [n_pages,Hkv,P,D]; page_table [nseq,max_pages]; kv_lens [nseq] tokens held by the cache of each
    sequence.  `score_mod` / `mask_mod` are the user's (training-time) mods: they are shifted here.
    Keys run over whole pages; as in paged_decode the mask, not the slicing, hides what lies past
    kv_lens[b].  Returns O [nseq,Hq,Lq,D], LSE [nseq,Hq,Lq] (fp64)."""
    nseq, Hq, Lq, D = Q.shape
    Hkv, P = K_pool.shape[1], K_pool.shape[2]
    G = Hq // Hkv
    scale = 1.0 / math.sqrt(D) if scale is None else scale
    score_inf, mask_inf = QOffset(score_mod, q_offsets), with_q_offset(mask_mod, q_offsets)
    O = torch.zeros(nseq, Hq, Lq, D, dtype=F64)
    LSE = torch.full((nseq, Hq, Lq), NEG_INF, dtype=F64)
    for b in range(nseq):
        n_padded = ((int(kv_lens[b]) + P - 1) // P) * P
        if n_padded == 0:
            continue
        Kl = unpage(K_pool, page_table[b], n_padded)
        Vl = unpage(V_pool, page_table[b], n_padded)
        for h in range(Hq):
            O[b, h], LSE[b, h] = attention_head(Q[b, h], Kl[h // G], Vl[h // G], score_inf, mask_inf, scale, b, h)
    return O, LSE


# --------------------------------------------------------------------------
# Neighborhood attention on a 2-D canvas (appendix, "Neighborhood Attention (NA)")
# --------------------------------------------------------------------------
def _spread_bits(v: int) -> int:
    """Bit i of v moves to bit 2 i."""
    out, i = 0, 0
    while v >> i:
        out |= ((v >> i) & 1) << (2 * i)
        i += 1
    return out


def na_token_index(x: int, y: int, width: int, height: int, layout: str, tile: int = 0) -> int:
    """Where pixel (x, y) of a width x height canvas sits in the token sequence.
    row_major: row after row.  tiled: tile x tile squares, the squares row after row, the pixels of
    a square row after row.  morton: bits of x and y interleaved, x in the even positions."""
    if layout == "row_major":
        return y * width + x
    if layout == "tiled":
        assert width % tile == 0 and height % tile == 0
        return ((y // tile) * (width // tile) + x // tile) * tile * tile + (y % tile) * tile + x % tile
    if layout == "morton":
        assert width == height and width & (width - 1) == 0
        return _spread_bits(x) | (_spread_bits(y) << 1)
    raise ValueError(layout)


def na_token_xy(width: int, height: int, layout: str, tile: int = 0):
    """(xs, ys): pixel of every token, by enumerating the canvas through na_token_index."""
    xs = torch.empty(width * height, dtype=torch.int64)
    ys = torch.empty(width * height, dtype=torch.int64)
    for y in range(height):
        for x in range(width):
            i = na_token_index(x, y, width, height, layout, tile)
            xs[i], ys[i] = x, y
    return xs, ys


def neighborhood_mask(width: int, height: int, kernel: int, layout: str = "row_major", tile: int = 0) -> MaskMod:
    """A query pixel attends to the kernel x kernel pixels nearest to it: the window centred on the
    pixel, moved inside the canvas where it would stick out (every query sees exactly kernel^2 keys)."""
    assert kernel % 2 == 1 and kernel <= width and kernel <= height
    xs, ys = na_token_xy(width, height, layout, tile)
    r = kernel // 2

    def mod(b, h, q_idx, kv_idx):
        cx = xs[q_idx].clamp(r, width - 1 - r)
        cy = ys[q_idx].clamp(r, height - 1 - r)
        return ((cx - xs[kv_idx]).abs() <= r) & ((cy - ys[kv_idx]).abs() <= r)
    return mod
