"""The C-ABI library loads, exports every symbol include/flexattn.h declares, and rejects bad
arguments on the host before anything touches a GPU (CPU only; no compute calls)."""
import ctypes as C
import os
import re

import pytest

import paper_2412_05496_amd as fa
from paper_2412_05496_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "flexattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(flexattn_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding._lib()
    names = declared_symbols()
    assert {"flexattn_blockmask_build", "flexattn_forward", "flexattn_backward", "flexattn_paged_decode",
            "flexattn_paged_convert_blockmask", "flexattn_paged_forward"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_strerror_and_version():
    lib = binding._lib()
    assert lib.flexattn_version() >= 100
    assert lib.flexattn_strerror(0) == b"ok"
    for st in (-1, -2, -3, -4):
        assert lib.flexattn_strerror(st) not in (b"ok", b"unknown status")


def test_supported_variants():
    assert fa.flexattn_is_supported(fa.MASK_CAUSAL, fa.SCORE_SOFTCAP, 128)
    assert fa.flexattn_is_supported(fa.MASK_DOCUMENT_CAUSAL, fa.SCORE_ALIBI, 64)
    assert fa.flexattn_is_supported(fa.MASK_SWA_CAUSAL_OR_PREFIX, fa.SCORE_REL_BIAS, 128)
    assert fa.flexattn_is_supported(fa.MASK_SWA_CAUSAL, fa.SCORE_SOFTCAP, 128)
    assert fa.flexattn_is_supported(fa.MASK_CAUSAL, fa.SCORE_ALIBI | fa.SCORE_SOFTCAP, 64)
    assert not fa.flexattn_is_supported(fa.MASK_CAUSAL, fa.SCORE_SOFTCAP, 96)
    assert not fa.flexattn_is_supported(fa.MASK_CTX_LEN, fa.SCORE_REL_BIAS | fa.SCORE_SOFTCAP, 128)


def test_null_and_bad_arguments_are_rejected_on_the_host():
    lib = binding._lib()
    assert lib.flexattn_forward(None, None, None, None, 0, 0, None, None, 1.0, None, None, None) == fa.ERR_INVALID_ARG
    assert lib.flexattn_blockmask_build(0, None, None, None, None, 0, None) == fa.ERR_INVALID_ARG
    assert lib.flexattn_paged_decode(None, None, 0, None, None, None, 0, None, 0, 0, None, 1.0, None, None, None, 0,
                                     None) == fa.ERR_INVALID_ARG
    d = binding._Dims(1, 3, 2, 128, 128, 128)           # Hq not a multiple of Hkv
    bm = binding._BlockMask(1, 1, 128, 128, 64, 64, 1, 1, 1, 1, 1, 1, 1, 1)
    assert lib.flexattn_forward(C.byref(d), None, None, None, 0, 0, None, C.byref(bm), 1.0, None, None,
                                None) == fa.ERR_INVALID_ARG
    d = binding._Dims(1, 2, 2, 128, 128, 96)            # head dimension not compiled in
    assert lib.flexattn_forward(C.byref(d), None, None, None, 0, 0, None, C.byref(bm), 1.0, None, None,
                                None) == fa.ERR_UNSUPPORTED
    d = binding._Dims(1, 2, 2, 128, 128, 128)
    bm = binding._BlockMask(1, 1, 128, 128, 32, 64, 1, 1, 1, 1, 1, 1, 1, 1)   # Bq = 32 unsupported
    assert lib.flexattn_forward(C.byref(d), None, None, None, 0, 0, None, C.byref(bm), 1.0, None, None,
                                None) == fa.ERR_UNSUPPORTED
    # paged forward: a page must be a BlockMask block, and every sequence needs its own lists
    t = binding._Tensor(16, 0, 0, 128)
    bm = binding._BlockMask(2, 1, 128, 256, 128, 64, 1, 1, 1, 1, 1, 1, 1, 1)
    d = binding._Dims(2, 2, 2, 128, 256, 128)
    args = (0, 0, None, C.byref(bm), 16, 16, 1.0, C.byref(t), 16, None)
    assert lib.flexattn_paged_forward(C.byref(d), C.byref(t), 16, 16, 128, 8, *args) == fa.ERR_UNSUPPORTED
    assert lib.flexattn_paged_forward(C.byref(d), C.byref(t), 16, 16, 64, 0, *args) == fa.ERR_INVALID_ARG
    assert lib.flexattn_paged_forward(C.byref(d), C.byref(t), 16, 24, 64, 8, *args) == fa.ERR_INVALID_ARG
    bm1 = binding._BlockMask(1, 1, 128, 256, 128, 64, 1, 1, 1, 1, 1, 1, 1, 1)
    args1 = (0, 0, None, C.byref(bm1), 16, 16, 1.0, C.byref(t), 16, None)
    assert lib.flexattn_paged_forward(C.byref(d), C.byref(t), 16, 16, 64, 8, *args1) == fa.ERR_INVALID_ARG
    # a mask without its parameters is refused; lengths need not be multiples of the block size
    bm = binding._BlockMask(1, 1, 100, 128, 64, 64, 1, 1, 1, 1, 1, 1, 1, 1)
    assert lib.flexattn_blockmask_build(fa.MASK_CAUSAL, None, C.byref(bm), None, 1, 1 << 20, None) == fa.ERR_INVALID_ARG
    p = binding._ModParams()
    assert lib.flexattn_blockmask_build(fa.MASK_CAUSAL, C.byref(p), C.byref(bm), None, 1, 1, None) == fa.ERR_WORKSPACE
    assert fa.flexattn_blockmask_workspace_bytes(1, 1, 100, 129, 64, 64) >= 2 * 3
    # document mask without doc_ids
    bm = binding._BlockMask(1, 1, 128, 128, 64, 64, 1, 1, 1, 1, 1, 1, 1, 1)
    assert lib.flexattn_blockmask_build(fa.MASK_DOCUMENT, C.byref(p), C.byref(bm), None, 1, 1 << 20,
                                        None) == fa.ERR_INVALID_ARG
    # workspace too small
    assert lib.flexattn_blockmask_build(fa.MASK_CAUSAL, C.byref(p), C.byref(bm), None, 1, 1, None) == fa.ERR_WORKSPACE


def test_workspace_queries():
    assert fa.flexattn_blockmask_workspace_bytes(1, 1, 8192, 8192, 128, 64) >= 64 * 128
    dd = binding._DecodeDims(64, 32, 8, 128, 16, 2048, 1000)
    n = binding._lib().flexattn_paged_decode_workspace_bytes(C.byref(dd))
    assert n >= 64 * 32 * 130 * 4 and n % 4 == 0
    d = binding._Dims(4, 16, 16, 8192, 8192, 128)
    assert binding._lib().flexattn_backward_workspace_bytes(C.byref(d)) == 2 * 4 * 16 * 8192 * 4


def test_product_does_not_import_oracle():
    pkg = os.path.join(ROOT, "paper_2412_05496_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("no CPU fallback", ""), f


def test_blockmask_sizes_is_host_arithmetic():
    lib = binding._lib()
    sz = binding._BlockMaskSizes()
    assert lib.flexattn_blockmask_sizes(2, 3, 1000, 517, 128, 64, C.byref(sz)) == fa.OK
    NR, NC = 8, 9                                     # ceil(1000 / 128), ceil(517 / 64)
    assert (sz.NR, sz.NC) == (NR, NC)
    assert sz.kv_num_blocks == sz.full_kv_num_blocks == 6 * NR
    assert sz.kv_indices == sz.full_kv_indices == 6 * NR * NC
    assert sz.q_num_blocks == sz.full_q_num_blocks == 6 * NC
    assert sz.q_indices == sz.full_q_indices == 6 * NC * NR
    assert sz.kv_order == 6 * NR and sz.q_order == 6 * NC
    assert lib.flexattn_blockmask_sizes(1, 1, 0, 64, 64, 64, C.byref(sz)) == fa.ERR_INVALID_ARG
    assert lib.flexattn_blockmask_sizes(1, 1, 64, 64, 64, 64, None) == fa.ERR_INVALID_ARG
    assert lib.flexattn_blockmask_sizes(64, 64, 1 << 20, 1 << 20, 64, 64, C.byref(sz)) == fa.ERR_UNSUPPORTED
    # the workspace of the builder is one byte per block, rounded up to 256
    assert lib.flexattn_blockmask_workspace_bytes(2, 3, 1000, 517, 128, 64) == (6 * NR * NC + 255) // 256 * 256


def test_decode_workspace_follows_the_split_length():
    """Splits are 1024 keys when nseq * Hkv * (addressable context) fills the chip that way, and
    shorter (down to 128) for small batches; the workspace holds D + 2 floats per (seq, head, split)."""
    lib = binding._lib()

    def ws(nseq, Hq, Hkv, D, page, max_pages):
        d = binding._DecodeDims(nseq, Hq, Hkv, D, page, max_pages, 1)
        return lib.flexattn_paged_decode_workspace_bytes(C.byref(d))

    assert ws(64, 32, 8, 128, 16, 2048) == 64 * 32 * 32 * 130 * 4          # config 5: 32 splits of 1024
    assert ws(1, 32, 8, 128, 16, 512) == 1 * 32 * 64 * 130 * 4             # 8192 tokens, 8 heads: 128-key splits
    assert ws(1, 32, 8, 128, 16, 2048) == 1 * 32 * 128 * 130 * 4           # 32768 tokens, 8 heads: 256-key splits
    assert ws(4, 8, 8, 64, 256, 128) == 4 * 8 * 32 * 66 * 4                # 32768 tokens x 32 units: 1024-key splits
    assert ws(2, 4, 2, 64, 16, 4) == 2 * 4 * 1 * 66 * 4                    # shorter than one split
    assert ws(2, 4, 2, 64, 24, 4) == 0 and ws(2, 4, 2, 64, 2048, 4) == 0   # page sizes that are refused
    assert ws(2, 4, 2, 64, 8, 4) == 0


def test_stored_backward_workspace_is_host_arithmetic():
    """Row scalars (256-byte aligned), one int32 per column of blocks + 1, one per block position, then
    2 * Bq * Bk bytes per block and per head that shares no BlockMask plane with an equal (b, hq)."""
    lib = binding._lib()
    al = lambda n: (n + 255) // 256 * 256
    d = binding._Dims(4, 16, 16, 8192, 8192, 128)
    bm = binding._BlockMask(1, 1, 8192, 8192, 128, 64)
    NR, NC, n_blocks = 64, 128, 4160
    want = al(2 * 4 * 16 * 8192 * 4) + al((NC + 1) * 4) + al(NR * NC * 4) + 4 * 16 * n_blocks * 128 * 64 * 2
    assert lib.flexattn_backward_stored_workspace_bytes(C.byref(d), C.byref(bm), n_blocks) == want
    # one plane per (b, hq): the planes' blocks are numbered through, nothing is stored twice
    bm2 = binding._BlockMask(4, 16, 8192, 8192, 128, 64)
    want2 = al(2 * 4 * 16 * 8192 * 4) + al((64 * NC + 1) * 4) + al(64 * NR * NC * 4) + 64 * n_blocks * 128 * 64 * 2
    assert lib.flexattn_backward_stored_workspace_bytes(C.byref(d), C.byref(bm2), 64 * n_blocks) == want2
    # no block at all still leaves room for one (slots are clamped into the capacity)
    assert (lib.flexattn_backward_stored_workspace_bytes(C.byref(d), C.byref(bm), 0)
            == lib.flexattn_backward_stored_workspace_bytes(C.byref(d), C.byref(bm), 1))
    assert lib.flexattn_backward_stored_workspace_bytes(C.byref(d), C.byref(bm), -1) == 0
    assert lib.flexattn_backward_stored_workspace_bytes(C.byref(d), C.byref(bm), 1 << 29) == 0
    assert lib.flexattn_backward_stored_workspace_bytes(None, C.byref(bm), 1) == 0
    assert lib.flexattn_backward_stored(C.byref(d), None, None, None, None, None, None, 0, 0, None, C.byref(bm), 1.0,
                                        None, None, None, -1, None, 0, None, 7) == fa.ERR_INVALID_ARG
