"""ctypes binding of libflexattn.so: argument marshalling only.

Every function here has the name of the C entry point it wraps (see include/flexattn.h), takes
torch CUDA tensors for device memory, launches on torch's current stream and raises
FlexAttnError on a non-zero status.  No step of the computation runs in Python.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libflexattn.so")

# ---- ids (mirrors of the #defines in flexattn.h) -----------------------------------------
M_CAUSAL, M_SLIDING_WINDOW, M_DOCUMENT, M_PREFIX, M_CTX_LEN, M_NEIGHBORHOOD = 1, 2, 4, 8, 16, 32


def mask_or(term0: int, term1: int) -> int:
    return term0 | (term1 << 8)


MASK_NONE = 0
MASK_CAUSAL = M_CAUSAL
MASK_SLIDING_WINDOW = M_SLIDING_WINDOW
MASK_SWA_CAUSAL = M_CAUSAL | M_SLIDING_WINDOW
MASK_DOCUMENT = M_DOCUMENT
MASK_DOCUMENT_CAUSAL = M_DOCUMENT | M_CAUSAL
MASK_PREFIX_LM = mask_or(M_CAUSAL, M_PREFIX)
MASK_SWA_CAUSAL_OR_PREFIX = mask_or(MASK_SWA_CAUSAL, M_PREFIX)
MASK_CTX_LEN = M_CTX_LEN
MASK_CTX_LEN_WINDOW = M_CTX_LEN | M_SLIDING_WINDOW
MASK_NEIGHBORHOOD = M_NEIGHBORHOOD
NA_ROW_MAJOR, NA_TILED, NA_MORTON = 0, 1, 2

SCORE_IDENTITY, SCORE_ALIBI, SCORE_REL_BIAS, SCORE_SOFTCAP = 0, 1, 2, 4

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = 0, -1, -2, -3, -4


class FlexAttnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib().flexattn_strerror(status).decode()
        if status == ERR_HIP:
            msg += f" (hipError {_lib().flexattn_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{status}]")


class _ModParams(C.Structure):
    _fields_ = [("window", C.c_int32), ("prefix_len", C.c_int32), ("softcap", C.c_float), ("rel_len", C.c_int32),
                ("doc_ids", C.c_void_p), ("doc_stride_b", C.c_int64), ("alibi_bias", C.c_void_p),
                ("rel_bias", C.c_void_p), ("ctx_lens", C.c_void_p), ("q_offsets", C.c_void_p),
                ("na_width", C.c_int32), ("na_height", C.c_int32), ("na_kernel", C.c_int32),
                ("na_layout", C.c_int32), ("na_tile", C.c_int32)]


class _Tensor(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("stride_b", C.c_int64), ("stride_h", C.c_int64), ("stride_s", C.c_int64)]


class _BlockMask(C.Structure):
    _fields_ = [("Bm", C.c_int32), ("Hm", C.c_int32), ("q_len", C.c_int32), ("kv_len", C.c_int32),
                ("Bq", C.c_int32), ("Bk", C.c_int32),
                ("kv_num_blocks", C.c_void_p), ("kv_indices", C.c_void_p),
                ("full_kv_num_blocks", C.c_void_p), ("full_kv_indices", C.c_void_p),
                ("q_num_blocks", C.c_void_p), ("q_indices", C.c_void_p),
                ("full_q_num_blocks", C.c_void_p), ("full_q_indices", C.c_void_p),
                ("kv_order", C.c_void_p), ("q_order", C.c_void_p)]


class _BlockMaskSizes(C.Structure):
    _fields_ = [("NR", C.c_int32), ("NC", C.c_int32)] + [(n, C.c_int64) for n in (
        "kv_num_blocks", "kv_indices", "full_kv_num_blocks", "full_kv_indices",
        "q_num_blocks", "q_indices", "full_q_num_blocks", "full_q_indices", "kv_order", "q_order")]


class _Dims(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("q_len", C.c_int32),
                ("kv_len", C.c_int32), ("D", C.c_int32)]


class _DecodeDims(C.Structure):
    _fields_ = [("nseq", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
                ("page_size", C.c_int32), ("max_pages", C.c_int32), ("n_pool_pages", C.c_int32)]


_handle = None


def _lib():
    """Loads the HIP library; there is no fallback path."""
    global _handle
    if _handle is not None:
        return _handle
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2412_05496_amd.build` "
                          "(the HIP library is the only implementation; there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    P = C.POINTER
    lib.flexattn_strerror.restype = C.c_char_p
    lib.flexattn_strerror.argtypes = [C.c_int]
    lib.flexattn_last_hip_error.restype = C.c_int
    lib.flexattn_version.restype = C.c_int
    lib.flexattn_is_supported.restype = C.c_int
    lib.flexattn_is_supported.argtypes = [C.c_uint32, C.c_uint32, C.c_int32]
    lib.flexattn_blockmask_sizes.restype = C.c_int
    lib.flexattn_blockmask_sizes.argtypes = [C.c_int32] * 6 + [P(_BlockMaskSizes)]
    lib.flexattn_blockmask_workspace_bytes.restype = C.c_size_t
    lib.flexattn_blockmask_workspace_bytes.argtypes = [C.c_int32] * 6
    lib.flexattn_blockmask_build.restype = C.c_int
    lib.flexattn_blockmask_build.argtypes = [C.c_uint32, P(_ModParams), P(_BlockMask), C.c_void_p, C.c_void_p,
                                             C.c_size_t, C.c_void_p]
    lib.flexattn_forward.restype = C.c_int
    lib.flexattn_forward.argtypes = [P(_Dims), P(_Tensor), P(_Tensor), P(_Tensor), C.c_uint32, C.c_uint32,
                                     P(_ModParams), P(_BlockMask), C.c_float, P(_Tensor), C.c_void_p, C.c_void_p]
    lib.flexattn_paged_forward.restype = C.c_int
    lib.flexattn_paged_forward.argtypes = [P(_Dims), P(_Tensor), C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                           C.c_uint32, C.c_uint32, P(_ModParams), P(_BlockMask), C.c_void_p,
                                           C.c_void_p, C.c_float, P(_Tensor), C.c_void_p, C.c_void_p]
    lib.flexattn_backward_workspace_bytes.restype = C.c_size_t
    lib.flexattn_backward_workspace_bytes.argtypes = [P(_Dims)]
    lib.flexattn_backward.restype = C.c_int
    lib.flexattn_backward.argtypes = [P(_Dims), P(_Tensor), P(_Tensor), P(_Tensor), P(_Tensor), P(_Tensor),
                                      C.c_void_p, C.c_uint32, C.c_uint32, P(_ModParams), P(_BlockMask), C.c_float,
                                      P(_Tensor), P(_Tensor), P(_Tensor), C.c_void_p, C.c_size_t, C.c_void_p]
    lib.flexattn_backward_stages.restype = C.c_int
    lib.flexattn_backward_stages.argtypes = lib.flexattn_backward.argtypes + [C.c_uint32]
    lib.flexattn_backward_stored_workspace_bytes.restype = C.c_size_t
    lib.flexattn_backward_stored_workspace_bytes.argtypes = [P(_Dims), P(_BlockMask), C.c_int64]
    lib.flexattn_backward_stored.restype = C.c_int
    lib.flexattn_backward_stored.argtypes = (lib.flexattn_backward.argtypes[:15] +
                                             [C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p, C.c_uint32])
    lib.flexattn_backward_captured_workspace_bytes.restype = C.c_size_t
    lib.flexattn_backward_captured_workspace_bytes.argtypes = [P(_Dims), P(_BlockMask), C.c_uint32, P(_ModParams)]
    lib.flexattn_backward_captured.restype = C.c_int
    lib.flexattn_backward_captured.argtypes = [P(_Dims), P(_Tensor), P(_Tensor), P(_Tensor), P(_Tensor), P(_Tensor),
                                               C.c_void_p, C.c_uint32, C.c_uint32, P(_ModParams), P(_BlockMask),
                                               C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.flexattn_paged_convert_blockmask.restype = C.c_int
    lib.flexattn_paged_convert_blockmask.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                                     C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                                     C.c_int32, C.c_void_p]
    lib.flexattn_paged_decode_workspace_bytes.restype = C.c_size_t
    lib.flexattn_paged_decode_workspace_bytes.argtypes = [P(_DecodeDims)]
    lib.flexattn_paged_decode.restype = C.c_int
    lib.flexattn_paged_decode.argtypes = [P(_DecodeDims), C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p,
                                          C.c_void_p, C.c_int64, C.c_void_p, C.c_uint32, C.c_uint32,
                                          P(_ModParams), C.c_float, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_size_t, C.c_void_p]
    lib.flexattn_probe_mfma_flops.restype = C.c_double
    lib.flexattn_probe_mfma_flops.argtypes = [C.c_int64]
    lib.flexattn_probe_mfma.restype = C.c_int
    lib.flexattn_probe_mfma.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.flexattn_probe_mfma_waves.restype = C.c_int32
    lib.flexattn_probe_stream_read.restype = C.c_int
    lib.flexattn_probe_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.flexattn_paged_decode_static_capacity.restype = C.c_size_t
    lib.flexattn_paged_decode_static_capacity.argtypes = []
    lib.flexattn_paged_decode_static.restype = C.c_int
    lib.flexattn_paged_decode_static.argtypes = lib.flexattn_paged_decode.argtypes[:14] + [C.c_void_p]
    _handle = lib
    return lib


def library_path() -> str:
    return _LIB_PATH


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _check(status: int, where: str):
    if status != OK:
        raise FlexAttnError(status, where)


@dataclass
class ModParams:
    """Values captured by the mods (device tensors).  Mirrors flexattn_mod_params."""
    window: int = 0
    prefix_len: int = 0
    softcap: float = 0.0
    doc_ids: Optional[torch.Tensor] = None       # int32 [B, S] or [S]
    alibi_bias: Optional[torch.Tensor] = None    # fp32 [Hq]
    rel_bias: Optional[torch.Tensor] = None      # fp32 [Hq, rel_len]
    ctx_lens: Optional[torch.Tensor] = None      # int32 [B]
    q_offsets: Optional[torch.Tensor] = None     # int32 [B]: the mods see q_idx + q_offsets[b]
    na_width: int = 0                            # neighborhood attention: canvas, kernel, token order
    na_height: int = 0
    na_kernel: int = 0
    na_layout: int = 0
    na_tile: int = 0

    def _c(self) -> _ModParams:
        p = _ModParams()
        p.window, p.prefix_len, p.softcap = int(self.window), int(self.prefix_len), float(self.softcap)
        p.na_width, p.na_height, p.na_kernel = int(self.na_width), int(self.na_height), int(self.na_kernel)
        p.na_layout, p.na_tile = int(self.na_layout), int(self.na_tile)
        if self.doc_ids is not None:
            assert self.doc_ids.dtype == torch.int32 and self.doc_ids.is_cuda and self.doc_ids.stride(-1) == 1
            p.doc_ids = self.doc_ids.data_ptr()
            p.doc_stride_b = self.doc_ids.stride(0) if self.doc_ids.dim() == 2 and self.doc_ids.shape[0] > 1 else 0
        if self.alibi_bias is not None:
            assert self.alibi_bias.dtype == torch.float32 and self.alibi_bias.is_cuda and self.alibi_bias.is_contiguous()
            p.alibi_bias = self.alibi_bias.data_ptr()
        if self.rel_bias is not None:
            assert self.rel_bias.dtype == torch.float32 and self.rel_bias.is_cuda and self.rel_bias.is_contiguous()
            p.rel_bias = self.rel_bias.data_ptr()
            p.rel_len = self.rel_bias.shape[-1]
        if self.ctx_lens is not None:
            assert self.ctx_lens.dtype == torch.int32 and self.ctx_lens.is_cuda and self.ctx_lens.is_contiguous()
            p.ctx_lens = self.ctx_lens.data_ptr()
        if self.q_offsets is not None:
            assert self.q_offsets.dtype == torch.int32 and self.q_offsets.is_cuda and self.q_offsets.is_contiguous()
            p.q_offsets = self.q_offsets.data_ptr()
        return p


@dataclass
class BlockMask:
    """Device arrays of a BlockMask (flexattn_blockmask) plus its geometry."""
    Bm: int
    Hm: int
    q_len: int
    kv_len: int
    Bq: int
    Bk: int
    kv_num_blocks: torch.Tensor
    kv_indices: torch.Tensor
    full_kv_num_blocks: torch.Tensor
    full_kv_indices: torch.Tensor
    q_num_blocks: torch.Tensor
    q_indices: torch.Tensor
    full_q_num_blocks: torch.Tensor
    full_q_indices: torch.Tensor
    stats: Optional[torch.Tensor] = None     # int64[4]: partial, full, total blocks, unmasked scalars
    kv_order: Optional[torch.Tensor] = None  # [Bm, Hm, NR] rows of blocks, longest first (optional)
    q_order: Optional[torch.Tensor] = None   # [Bm, Hm, NC] columns of blocks, longest first (optional)

    def _c(self) -> _BlockMask:
        return _BlockMask(self.Bm, self.Hm, self.q_len, self.kv_len, self.Bq, self.Bk,
                          self.kv_num_blocks.data_ptr(), self.kv_indices.data_ptr(),
                          self.full_kv_num_blocks.data_ptr(), self.full_kv_indices.data_ptr(),
                          self.q_num_blocks.data_ptr(), self.q_indices.data_ptr(),
                          self.full_q_num_blocks.data_ptr(), self.full_q_indices.data_ptr(),
                          _ptr(self.kv_order), _ptr(self.q_order))


def _tensor(t: torch.Tensor) -> _Tensor:
    assert t.is_cuda and t.dtype == torch.bfloat16 and t.dim() == 4 and t.stride(3) == 1
    return _Tensor(t.data_ptr(), t.stride(0), t.stride(1), t.stride(2))


def _dims(Q: torch.Tensor, K: torch.Tensor) -> _Dims:
    return _Dims(Q.shape[0], Q.shape[1], K.shape[1], Q.shape[2], K.shape[2], Q.shape[3])


def flexattn_blockmask_sizes(Bm: int, Hm: int, q_len: int, kv_len: int, Bq: int, Bk: int) -> _BlockMaskSizes:
    sizes = _BlockMaskSizes()
    _check(_lib().flexattn_blockmask_sizes(Bm, Hm, q_len, kv_len, Bq, Bk, C.byref(sizes)),
           "flexattn_blockmask_sizes")
    return sizes


def alloc_blockmask(Bm: int, Hm: int, q_len: int, kv_len: int, Bq: int, Bk: int, device="cuda",
                    work_order: bool = True) -> BlockMask:
    """Caller-side allocation of the eight int32 arrays and (work_order) the two order arrays (the
    library allocates nothing), sized by flexattn_blockmask_sizes and viewed as
    [Bm, Hm, NR(, NC)] / [Bm, Hm, NC(, NR)]."""
    sz = flexattn_blockmask_sizes(Bm, Hm, q_len, kv_len, Bq, Bk)
    i32 = dict(dtype=torch.int32, device=device)

    def arr(count, *shape):
        return torch.empty(count, **i32).view(Bm, Hm, *shape)

    return BlockMask(Bm, Hm, q_len, kv_len, Bq, Bk,
                     arr(sz.kv_num_blocks, sz.NR), arr(sz.kv_indices, sz.NR, sz.NC),
                     arr(sz.full_kv_num_blocks, sz.NR), arr(sz.full_kv_indices, sz.NR, sz.NC),
                     arr(sz.q_num_blocks, sz.NC), arr(sz.q_indices, sz.NC, sz.NR),
                     arr(sz.full_q_num_blocks, sz.NC), arr(sz.full_q_indices, sz.NC, sz.NR),
                     torch.empty(4, dtype=torch.int64, device=device),
                     arr(sz.kv_order, sz.NR) if work_order else None,
                     arr(sz.q_order, sz.NC) if work_order else None)


def flexattn_is_supported(mask_id: int, score_id: int, D: int) -> bool:
    return bool(_lib().flexattn_is_supported(mask_id, score_id, D))


def flexattn_blockmask_workspace_bytes(Bm, Hm, q_len, kv_len, Bq, Bk) -> int:
    return _lib().flexattn_blockmask_workspace_bytes(Bm, Hm, q_len, kv_len, Bq, Bk)


def flexattn_blockmask_build(mask_id: int, params: ModParams, bm: BlockMask, ws: Optional[torch.Tensor] = None):
    if ws is None:
        n = flexattn_blockmask_workspace_bytes(bm.Bm, bm.Hm, bm.q_len, bm.kv_len, bm.Bq, bm.Bk)
        ws = torch.empty(max(n, 1), dtype=torch.uint8, device=bm.kv_indices.device)
    p, c = params._c(), bm._c()
    _check(_lib().flexattn_blockmask_build(mask_id, C.byref(p), C.byref(c), _ptr(bm.stats), ws.data_ptr(),
                                           ws.numel(), _stream()), "flexattn_blockmask_build")
    return bm


def flexattn_forward(Q, K, V, score_id: int, mask_id: int, params: ModParams, bm: BlockMask, scale: float,
                     O: torch.Tensor, LSE: torch.Tensor):
    assert LSE.dtype == torch.float32 and LSE.is_contiguous() and LSE.shape == Q.shape[:3]
    d, p, c = _dims(Q, K), params._c(), bm._c()
    tq, tk, tv, to = _tensor(Q), _tensor(K), _tensor(V), _tensor(O)
    _check(_lib().flexattn_forward(C.byref(d), C.byref(tq), C.byref(tk), C.byref(tv), score_id, mask_id,
                                   C.byref(p), C.byref(c), scale, C.byref(to), LSE.data_ptr(), _stream()),
           "flexattn_forward")
    return O, LSE


def flexattn_paged_forward(Q, K_pool, V_pool, score_id: int, mask_id: int, params: ModParams, bm: BlockMask,
                           phys_kv_indices: torch.Tensor, phys_full_kv_indices: torch.Tensor, scale: float,
                           O: torch.Tensor, LSE: torch.Tensor):
    """Q [nseq, Hq, q_len, D]; pools [n_pages, Hkv, page, D] contiguous; `bm` is the logical BlockMask
    (Bm == nseq, Bk == page), the phys_* tensors its converted kv lists."""
    assert K_pool.is_contiguous() and V_pool.is_contiguous() and K_pool.shape == V_pool.shape
    assert LSE.dtype == torch.float32 and LSE.is_contiguous() and LSE.shape == Q.shape[:3]
    for phys, logical in ((phys_kv_indices, bm.kv_indices), (phys_full_kv_indices, bm.full_kv_indices)):
        assert phys.dtype == torch.int32 and phys.is_contiguous() and phys.shape == logical.shape
    n_pool, Hkv, page, D = K_pool.shape
    d = _Dims(Q.shape[0], Q.shape[1], Hkv, Q.shape[2], bm.kv_len, D)
    p, c, tq, to = params._c(), bm._c(), _tensor(Q), _tensor(O)
    _check(_lib().flexattn_paged_forward(C.byref(d), C.byref(tq), K_pool.data_ptr(), V_pool.data_ptr(), page, n_pool,
                                         score_id, mask_id, C.byref(p), C.byref(c), phys_kv_indices.data_ptr(),
                                         phys_full_kv_indices.data_ptr(), scale, C.byref(to), LSE.data_ptr(),
                                         _stream()),
           "flexattn_paged_forward")
    return O, LSE


def flexattn_backward_workspace_bytes(Q, K) -> int:
    d = _dims(Q, K)
    return _lib().flexattn_backward_workspace_bytes(C.byref(d))


def flexattn_backward(Q, K, V, O, dO, LSE, score_id: int, mask_id: int, params: ModParams, bm: BlockMask,
                      scale: float, dQ, dK, dV, ws: Optional[torch.Tensor] = None):
    if ws is None:
        ws = torch.empty(max(flexattn_backward_workspace_bytes(Q, K), 1), dtype=torch.uint8, device=Q.device)
    d, p, c = _dims(Q, K), params._c(), bm._c()
    ts = [_tensor(t) for t in (Q, K, V, O, dO, dQ, dK, dV)]
    _check(_lib().flexattn_backward(C.byref(d), *(C.byref(t) for t in ts[:5]), LSE.data_ptr(), score_id, mask_id,
                                    C.byref(p), C.byref(c), scale, *(C.byref(t) for t in ts[5:]),
                                    ws.data_ptr(), ws.numel(), _stream()), "flexattn_backward")
    return dQ, dK, dV


def flexattn_backward_stored_workspace_bytes(Q, K, bm: BlockMask, n_blocks: int) -> int:
    d, c = _dims(Q, K), bm._c()
    return _lib().flexattn_backward_stored_workspace_bytes(C.byref(d), C.byref(c), n_blocks)


def flexattn_backward_stored(Q, K, V, O, dO, LSE, score_id: int, mask_id: int, params: ModParams, bm: BlockMask,
                             scale: float, dQ, dK, dV, n_blocks: int, ws: Optional[torch.Tensor] = None,
                             stages: int = 7):
    """The backward that keeps dS in memory; n_blocks = stats[0] + stats[1] of the BlockMask build.
    dQ / dK / dV may be None for stages that are not selected; `ws` must persist between stages."""
    if ws is None:
        n = flexattn_backward_stored_workspace_bytes(Q, K, bm, n_blocks)
        ws = torch.empty(max(n, 1), dtype=torch.uint8, device=Q.device)
    d, p, c = _dims(Q, K), params._c(), bm._c()
    ins = [_tensor(t) for t in (Q, K, V, O, dO)]
    outs = [None if t is None else _tensor(t) for t in (dQ, dK, dV)]
    _check(_lib().flexattn_backward_stored(C.byref(d), *(C.byref(t) for t in ins), LSE.data_ptr(), score_id,
                                           mask_id, C.byref(p), C.byref(c), scale,
                                           *(None if t is None else C.byref(t) for t in outs),
                                           n_blocks, ws.data_ptr(), ws.numel(), _stream(), stages),
           "flexattn_backward_stored")
    return dQ, dK, dV


BWD_DELTA, BWD_DKDV, BWD_DQ, BWD_ALL = 1, 2, 4, 7


def flexattn_backward_stages(Q, K, V, O, dO, LSE, score_id: int, mask_id: int, params: ModParams, bm: BlockMask,
                             scale: float, dQ, dK, dV, ws: torch.Tensor, stages: int):
    """dQ / dK / dV may be None for stages that are not selected; `ws` must persist between stages."""
    d, p, c = _dims(Q, K), params._c(), bm._c()
    ins = [_tensor(t) for t in (Q, K, V, O, dO)]
    outs = [None if t is None else _tensor(t) for t in (dQ, dK, dV)]
    _check(_lib().flexattn_backward_stages(C.byref(d), *(C.byref(t) for t in ins), LSE.data_ptr(), score_id, mask_id,
                                           C.byref(p), C.byref(c), scale,
                                           *(None if t is None else C.byref(t) for t in outs),
                                           ws.data_ptr(), ws.numel(), _stream(), stages), "flexattn_backward_stages")
    return dQ, dK, dV


def flexattn_backward_captured(Q, K, V, O, dO, LSE, score_id: int, mask_id: int, params: ModParams, bm: BlockMask,
                               scale: float, d_alibi_bias: Optional[torch.Tensor] = None,
                               d_rel_bias: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """Gradients of the captured alibi_bias [Hq] / rel_bias [Hq, rel_len] (fp32, written)."""
    for t in (d_alibi_bias, d_rel_bias):
        assert t is None or (t.dtype == torch.float32 and t.is_cuda and t.is_contiguous())
    d, p, c = _dims(Q, K), params._c(), bm._c()
    if ws is None:
        n = _lib().flexattn_backward_captured_workspace_bytes(C.byref(d), C.byref(c), score_id, C.byref(p))
        ws = torch.empty(max(n, 1), dtype=torch.uint8, device=Q.device)
    ts = [_tensor(t) for t in (Q, K, V, O, dO)]
    _check(_lib().flexattn_backward_captured(C.byref(d), *(C.byref(t) for t in ts), LSE.data_ptr(), score_id, mask_id,
                                             C.byref(p), C.byref(c), scale, _ptr(d_alibi_bias), _ptr(d_rel_bias),
                                             ws.data_ptr(), ws.numel(), _stream()),
           "flexattn_backward_captured")
    return d_alibi_bias, d_rel_bias


def flexattn_paged_convert_blockmask(num_blocks, indices, page_table, phys_indices, phys2log=None):
    Bm, Hm, NR, NC = indices.shape
    n_pool = phys2log.numel() if phys2log is not None else 2 ** 31 - 1
    _check(_lib().flexattn_paged_convert_blockmask(num_blocks.data_ptr(), indices.data_ptr(), Bm, Hm, NR, NC,
                                                   page_table.data_ptr(), page_table.stride(0),
                                                   phys_indices.data_ptr(), _ptr(phys2log), n_pool, _stream()),
           "flexattn_paged_convert_blockmask")
    return phys_indices, phys2log


def _decode_dims(Q, K_pool, page_table) -> _DecodeDims:
    nseq, Hq, D = Q.shape[0], Q.shape[1], Q.shape[-1]
    n_pool, Hkv, page = K_pool.shape[0], K_pool.shape[1], K_pool.shape[2]
    return _DecodeDims(nseq, Hq, Hkv, D, page, page_table.shape[1], n_pool)


def flexattn_paged_decode_workspace_bytes(Q, K_pool, page_table) -> int:
    d = _decode_dims(Q, K_pool, page_table)
    return _lib().flexattn_paged_decode_workspace_bytes(C.byref(d))


def flexattn_paged_decode(Q, K_pool, V_pool, page_table, ctx_lens, score_id: int, mask_id: int, params: ModParams,
                          scale: float, O, LSE=None, ws: Optional[torch.Tensor] = None):
    """Q [nseq, Hq, 1, D] or [nseq, Hq, D]; pools [n_pages, Hkv, page, D] contiguous."""
    assert K_pool.is_contiguous() and V_pool.is_contiguous() and O.is_contiguous()
    assert Q.stride(-1) == 1 and Q.stride(1) == Q.shape[-1]
    if ws is None:
        ws = torch.empty(max(flexattn_paged_decode_workspace_bytes(Q, K_pool, page_table), 1), dtype=torch.uint8,
                         device=Q.device)
    d, p = _decode_dims(Q, K_pool, page_table), params._c()
    _check(_lib().flexattn_paged_decode(C.byref(d), Q.data_ptr(), Q.stride(0), K_pool.data_ptr(), V_pool.data_ptr(),
                                        page_table.data_ptr(), page_table.stride(0), ctx_lens.data_ptr(), score_id,
                                        mask_id, C.byref(p), scale, O.data_ptr(), _ptr(LSE), ws.data_ptr(),
                                        ws.numel(), _stream()), "flexattn_paged_decode")
    return O, LSE


def flexattn_paged_decode_static_capacity() -> int:
    return _lib().flexattn_paged_decode_static_capacity()


def flexattn_paged_decode_static(Q, K_pool, V_pool, page_table, ctx_lens, score_id: int, mask_id: int,
                                 params: ModParams, scale: float, O, LSE=None):
    """flexattn_paged_decode on the library's own static workspace (nothing is allocated)."""
    assert K_pool.is_contiguous() and V_pool.is_contiguous() and O.is_contiguous()
    assert Q.stride(-1) == 1 and Q.stride(1) == Q.shape[-1]
    d, p = _decode_dims(Q, K_pool, page_table), params._c()
    _check(_lib().flexattn_paged_decode_static(C.byref(d), Q.data_ptr(), Q.stride(0), K_pool.data_ptr(),
                                               V_pool.data_ptr(), page_table.data_ptr(), page_table.stride(0),
                                               ctx_lens.data_ptr(), score_id, mask_id, C.byref(p), scale,
                                               O.data_ptr(), _ptr(LSE), _stream()), "flexattn_paged_decode_static")
    return O, LSE


def flexattn_probe_mfma_flops(iters: int) -> float:
    return _lib().flexattn_probe_mfma_flops(iters)


def flexattn_probe_mfma_waves() -> int:
    return _lib().flexattn_probe_mfma_waves()


def flexattn_probe_mfma(iters: int, sink: torch.Tensor, valu_mix: int = 0, random_operands: bool = False,
                        clocks: Optional[torch.Tensor] = None):
    """clocks: optional int64 [flexattn_probe_mfma_waves(), 2] (core cycles, 100 MHz ticks) per wave."""
    assert clocks is None or (clocks.dtype == torch.int64 and clocks.numel() >= 2 * flexattn_probe_mfma_waves())
    _check(_lib().flexattn_probe_mfma(iters, valu_mix, int(random_operands), sink.data_ptr(), _ptr(clocks),
                                      _stream()), "flexattn_probe_mfma")


def flexattn_probe_stream_read(src: torch.Tensor, sink: torch.Tensor):
    _check(_lib().flexattn_probe_stream_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(),
                                             _stream()), "flexattn_probe_stream_read")
