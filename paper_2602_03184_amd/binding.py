"""ctypes binding of libdsk.so: argument marshalling only.

`dsk_compress`, `dsk_select_topk` and `dsk_sparse_decode_attn` take the same argument
structs as the C ABI (include/dsk.h) and a HIP stream handle; every step of the path runs in
the HIP kernels.  The helpers below them only allocate device buffers with torch and fill
the structs.  There is no CPU fallback: importing this module without a built libdsk.so
raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libdsk.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libdsk.so is not built (%s). Run `python paper_2602_03184_amd/build.py` first; "
        "the DynSplit-KV path has no fallback implementation." % LIB_PATH)
_lib = C.CDLL(LIB_PATH)

# ---- status codes / stages (mirror include/dsk.h) ------------------------------------------
DSK_OK = 0
DSK_ERR_NULL, DSK_ERR_SHAPE, DSK_ERR_PARAM, DSK_ERR_ALIGN = -1, -2, -3, -4
DSK_ERR_WORKSPACE, DSK_ERR_CAPACITY, DSK_ERR_ORDER, DSK_ERR_LAUNCH, DSK_ERR_VERSION = -5, -6, -7, -8, -9
DSK_STAGE_CANDIDATES, DSK_STAGE_IMPORTANCE, DSK_STAGE_SEGMENT, DSK_STAGE_SUMMARIES = 1, 2, 4, 8
DSK_STAGE_ALL = 15
DSK_HEAD_DIM = 128
DSK_MAX_CLASSES = 64
DSK_ATTN_PARTIALS_ONLY = 1
DSK_ATTN_SHARED_SELECTION = 2
DSK_SELECT_SHARED_BY_KV_GROUP = 1
DSK_REUSE_PLAN_ONLY = 1
DSK_REUSE_MAX_K = 2048
DSK_SUMMARY_MINMAX, DSK_SUMMARY_MEAN = 0, 1

_p = C.c_void_p


class dsk_compress_args(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32), ("stages", C.c_uint32),
        ("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
        ("total_tokens", C.c_int32), ("max_seqlen", C.c_int32),
        ("cu_seqlens", _p),
        ("K", _p), ("V", _p),
        ("k_stride_tok", C.c_int64), ("k_stride_head", C.c_int64),
        ("v_stride_tok", C.c_int64), ("v_stride_head", C.c_int64),
        ("token_ids", _p), ("delim_ids", _p),
        ("n_class", C.c_int32), ("max_cand_total", C.c_int32),
        ("cand_pos", _p), ("cand_class", _p), ("cand_cu", _p),
        ("M", C.c_int32), ("W", C.c_int32), ("R", C.c_int32),
        ("alpha_imp", C.c_float), ("imp_scale", C.c_float),
        ("samp_pos", _p), ("qwin", _p), ("class_weight_q", _p), ("class_mean", _p), ("samp_score", _p),
        ("samp_score_sum", _p), ("imp_layers", C.c_int32),
        ("C", C.c_int32), ("delta", C.c_int32),
        ("C_per_seq", _p), ("delta_per_seq", _p),
        ("alpha_num", C.c_int32), ("alpha_den", C.c_int32),
        ("b", C.c_int32), ("max_blocks_total", C.c_int32),
        ("block_start", _p), ("cu_blocks", _p), ("slot_base", _p), ("cu_slots", _p),
        ("ksum", _p), ("vsum", _p),
        ("summary_mode", C.c_int32), ("sum_stride_blocks", C.c_int32),
        ("dev_status", _p),
        ("workspace", _p), ("workspace_bytes", C.c_size_t),
    ]


class dsk_select_args(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32),
        ("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
        ("max_blocks_total", C.c_int32), ("max_blocks_used", C.c_int32), ("max_blocks_per_seq", C.c_int32),
        ("cu_blocks", _p), ("block_start", _p), ("slot_base", _p),
        ("ksum", _p), ("q", _p),
        ("b", C.c_int32), ("budget", C.c_int32), ("budget_per_seq", _p), ("flags", C.c_uint32),
        ("sel_slot", _p), ("sel_start", _p), ("sel_len", _p), ("sel_count", _p),
        ("scores", _p),
        ("blocks_used", _p), ("seq_row0", _p),
        ("workspace", _p), ("workspace_bytes", C.c_size_t),
    ]


class dsk_attn_args(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32),
        ("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
        ("q", _p), ("K", _p), ("V", _p),
        ("k_stride_tok", C.c_int64), ("k_stride_head", C.c_int64),
        ("v_stride_tok", C.c_int64), ("v_stride_head", C.c_int64),
        ("total_tokens", C.c_int32), ("k", C.c_int32), ("b", C.c_int32),
        ("sel_start", _p), ("sel_len", _p), ("sel_count", _p),
        ("scale", C.c_float), ("flags", C.c_uint32),
        ("out", _p), ("out_bf16", _p), ("lse", _p),
        ("workspace", _p), ("workspace_bytes", C.c_size_t),
    ]


class dsk_dense_attn_args(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32),
        ("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
        ("q", _p), ("K", _p), ("V", _p),
        ("k_stride_tok", C.c_int64), ("k_stride_head", C.c_int64),
        ("v_stride_tok", C.c_int64), ("v_stride_head", C.c_int64),
        ("total_tokens", C.c_int32), ("max_seqlen", C.c_int32),
        ("cu_seqlens", _p),
        ("scale", C.c_float), ("flags", C.c_uint32),
        ("out", _p), ("out_bf16", _p), ("lse", _p),
        ("workspace", _p), ("workspace_bytes", C.c_size_t),
    ]


class dsk_append_args(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32),
        ("Hkv", C.c_int32), ("D", C.c_int32),
        ("len_old", C.c_int32), ("len_new", C.c_int32),
        ("K", _p), ("V", _p),
        ("k_stride_tok", C.c_int64), ("k_stride_head", C.c_int64),
        ("v_stride_tok", C.c_int64), ("v_stride_head", C.c_int64),
        ("token_ids", _p), ("delim_ids", _p), ("n_class", C.c_int32),
        ("class_weight_q", _p),
        ("C", C.c_int32), ("delta", C.c_int32), ("alpha_num", C.c_int32), ("alpha_den", C.c_int32),
        ("b", C.c_int32),
        ("max_blocks_total", C.c_int32),
        ("block_start", _p), ("cu_blocks", _p), ("slot_base", _p),
        ("ksum", _p), ("vsum", _p),
        ("summary_mode", C.c_int32),
        ("first_recomputed", _p), ("first_stale_slot", _p), ("dev_status", _p),
        ("workspace", _p), ("workspace_bytes", C.c_size_t),
    ]


class dsk_append_batch_args(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32),
        ("B", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
        ("total_rows", C.c_int32), ("max_new_tokens", C.c_int32),
        ("seq_row0", _p), ("seq_len", _p), ("len_new", _p),
        ("K", _p), ("V", _p),
        ("k_stride_tok", C.c_int64), ("k_stride_head", C.c_int64),
        ("v_stride_tok", C.c_int64), ("v_stride_head", C.c_int64),
        ("token_ids", _p), ("delim_ids", _p), ("n_class", C.c_int32),
        ("class_weight_q", _p),
        ("C", C.c_int32), ("delta", C.c_int32), ("alpha_num", C.c_int32), ("alpha_den", C.c_int32),
        ("b", C.c_int32),
        ("C_per_seq", _p), ("delta_per_seq", _p),
        ("max_blocks_total", C.c_int32),
        ("cu_blocks", _p), ("blocks_used", _p), ("block_start", _p), ("slot_base", _p),
        ("ksum", _p), ("vsum", _p),
        ("summary_mode", C.c_int32),
        ("first_recomputed", _p), ("first_stale_slot", _p), ("dev_status", _p),
        ("workspace", _p), ("workspace_bytes", C.c_size_t),
    ]


class dsk_reuse_args(C.Structure):
    _fields_ = [
        ("struct_size", C.c_uint32),
        ("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32),
        ("k", C.c_int32), ("b", C.c_int32), ("flags", C.c_uint32),
        ("sel_slot", _p), ("sel_start", _p), ("sel_len", _p), ("sel_count", _p),
        ("stale_from", _p),
        ("res_slot", _p), ("res_len", _p), ("res_start", _p), ("res_count", _p),
        ("load_pos", _p), ("load_slot", _p), ("load_start", _p), ("load_len", _p), ("load_count", _p),
        ("reuse_count", _p),
        ("K", _p), ("V", _p),
        ("k_stride_tok", C.c_int64), ("k_stride_head", C.c_int64),
        ("v_stride_tok", C.c_int64), ("v_stride_head", C.c_int64),
        ("total_tokens", C.c_int32),
        ("Kres", _p), ("Vres", _p),
        ("workspace", _p), ("workspace_bytes", C.c_size_t),
    ]


class dsk_attn_partials(C.Structure):
    _fields_ = [
        ("ml_offset", C.c_size_t), ("acc_offset", C.c_size_t),
        ("nchunks", C.c_int32), ("slots_per_chunk", C.c_int32),
    ]


_lib.dsk_version.restype = C.c_uint32
_lib.dsk_version.argtypes = []
_lib.dsk_strerror.restype = C.c_char_p
_lib.dsk_strerror.argtypes = [C.c_int32]
_lib.dsk_block_capacity.restype = C.c_int64
_lib.dsk_block_capacity.argtypes = [C.c_int32, C.c_int32, C.c_int32]
for _name, _cls in (("compress", dsk_compress_args), ("select", dsk_select_args), ("attn", dsk_attn_args),
                    ("dense_attn", dsk_dense_attn_args), ("append", dsk_append_args),
                    ("append_batch", dsk_append_batch_args), ("reuse", dsk_reuse_args)):
    _f = getattr(_lib, "dsk_%s_workspace_bytes" % _name)
    _f.restype = C.c_size_t
    _f.argtypes = [C.POINTER(_cls)]
_lib.dsk_attn_partials_layout.restype = C.c_int32
_lib.dsk_attn_partials_layout.argtypes = [C.POINTER(dsk_attn_args), C.POINTER(dsk_attn_partials)]
_lib.dsk_dense_decode_attn.restype = C.c_int32
_lib.dsk_dense_decode_attn.argtypes = [C.POINTER(dsk_dense_attn_args), _p]
_lib.dsk_append_tokens.restype = C.c_int32
_lib.dsk_append_tokens.argtypes = [C.POINTER(dsk_append_args), _p]
_lib.dsk_append_tokens_batch.restype = C.c_int32
_lib.dsk_append_tokens_batch.argtypes = [C.POINTER(dsk_append_batch_args), _p]
_lib.dsk_reuse_update.restype = C.c_int32
_lib.dsk_reuse_update.argtypes = [C.POINTER(dsk_reuse_args), _p]
_lib.dsk_compress.restype = C.c_int32
_lib.dsk_compress.argtypes = [C.POINTER(dsk_compress_args), _p]
_lib.dsk_select_topk.restype = C.c_int32
_lib.dsk_select_topk.argtypes = [C.POINTER(dsk_select_args), _p]
_lib.dsk_sparse_decode_attn.restype = C.c_int32
_lib.dsk_sparse_decode_attn.argtypes = [C.POINTER(dsk_attn_args), _p]
_lib.dsk_sparse_decode_attn_static.restype = C.c_int32
_lib.dsk_sparse_decode_attn_static.argtypes = [C.POINTER(dsk_attn_args), _p]
DSK_STATIC_SCRATCH_BYTES = 2112 * 1024


class DskError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (what, dsk_strerror(status), status))


# ---- the C ABI, same names -------------------------------------------------------------------
def dsk_version() -> int:
    return int(_lib.dsk_version())


def dsk_strerror(status: int) -> str:
    return _lib.dsk_strerror(int(status)).decode()


def dsk_block_capacity(total_tokens: int, B: int, min_chunk: int) -> int:
    return int(_lib.dsk_block_capacity(total_tokens, B, min_chunk))


def dsk_compress_workspace_bytes(args: dsk_compress_args) -> int:
    return int(_lib.dsk_compress_workspace_bytes(C.byref(args)))


def dsk_select_workspace_bytes(args: dsk_select_args) -> int:
    return int(_lib.dsk_select_workspace_bytes(C.byref(args)))


def dsk_attn_workspace_bytes(args: dsk_attn_args) -> int:
    return int(_lib.dsk_attn_workspace_bytes(C.byref(args)))


def dsk_dense_attn_workspace_bytes(args: dsk_dense_attn_args) -> int:
    return int(_lib.dsk_dense_attn_workspace_bytes(C.byref(args)))


def dsk_dense_decode_attn(args: dsk_dense_attn_args, stream=None, check: bool = True) -> int:
    st = int(_lib.dsk_dense_decode_attn(C.byref(args), _stream_handle(stream)))
    if check and st != DSK_OK:
        raise DskError(st, "dsk_dense_decode_attn")
    return st


def dsk_append_workspace_bytes(args: dsk_append_args) -> int:
    return int(_lib.dsk_append_workspace_bytes(C.byref(args)))


def dsk_append_tokens(args: dsk_append_args, stream=None, check: bool = True) -> int:
    st = int(_lib.dsk_append_tokens(C.byref(args), _stream_handle(stream)))
    if check and st != DSK_OK:
        raise DskError(st, "dsk_append_tokens")
    return st


def dsk_append_batch_workspace_bytes(args: dsk_append_batch_args) -> int:
    return int(_lib.dsk_append_batch_workspace_bytes(C.byref(args)))


def dsk_append_tokens_batch(args: dsk_append_batch_args, stream=None, check: bool = True) -> int:
    st = int(_lib.dsk_append_tokens_batch(C.byref(args), _stream_handle(stream)))
    if check and st != DSK_OK:
        raise DskError(st, "dsk_append_tokens_batch")
    return st


def dsk_reuse_workspace_bytes(args: dsk_reuse_args) -> int:
    return int(_lib.dsk_reuse_workspace_bytes(C.byref(args)))


def dsk_reuse_update(args: dsk_reuse_args, stream=None, check: bool = True) -> int:
    st = int(_lib.dsk_reuse_update(C.byref(args), _stream_handle(stream)))
    if check and st != DSK_OK:
        raise DskError(st, "dsk_reuse_update")
    return st


def dsk_attn_partials_layout(args: dsk_attn_args) -> dsk_attn_partials:
    lay = dsk_attn_partials()
    status = int(_lib.dsk_attn_partials_layout(C.byref(args), C.byref(lay)))
    if status != DSK_OK:
        raise DskError(status, "dsk_attn_partials_layout")
    return lay


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def dsk_compress(args: dsk_compress_args, stream=None, check: bool = True) -> int:
    st = int(_lib.dsk_compress(C.byref(args), _stream_handle(stream)))
    if check and st != DSK_OK:
        raise DskError(st, "dsk_compress")
    return st


def dsk_select_topk(args: dsk_select_args, stream=None, check: bool = True) -> int:
    st = int(_lib.dsk_select_topk(C.byref(args), _stream_handle(stream)))
    if check and st != DSK_OK:
        raise DskError(st, "dsk_select_topk")
    return st


def dsk_sparse_decode_attn(args: dsk_attn_args, stream=None, check: bool = True) -> int:
    st = int(_lib.dsk_sparse_decode_attn(C.byref(args), _stream_handle(stream)))
    if check and st != DSK_OK:
        raise DskError(st, "dsk_sparse_decode_attn")
    return st


def dsk_sparse_decode_attn_static(args: dsk_attn_args, stream=None, check: bool = True) -> int:
    """dsk_sparse_decode_attn with the partials in the library's static scratch array (no workspace)."""
    st = int(_lib.dsk_sparse_decode_attn_static(C.byref(args), _stream_handle(stream)))
    if check and st != DSK_OK:
        raise DskError(st, "dsk_sparse_decode_attn_static")
    return st


# ---- marshalling helpers ---------------------------------------------------------------------
def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _ws(nbytes: int, device) -> torch.Tensor:
    # torch's caching allocator hands out 512-byte aligned blocks
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _kv_strides(X: torch.Tensor):
    """X: bf16 [Hkv, tokens, D] view (any head/token strides, unit channel stride)."""
    assert X.dim() == 3 and X.dtype == torch.bfloat16
    if X.numel() == 0:                       # no token: nothing is read, any valid strides do
        return DSK_HEAD_DIM, DSK_HEAD_DIM
    assert X.stride(2) == 1
    return X.stride(1), X.stride(0)


@dataclass
class Compressed:
    """Device buffers written by dsk_compress plus the geometry they were sized for."""
    B: int
    Hq: int
    Hkv: int
    b: int
    total_tokens: int
    max_blocks_total: int
    cu_seqlens: torch.Tensor
    block_start: torch.Tensor
    cu_blocks: torch.Tensor
    slot_base: torch.Tensor
    cu_slots: Optional[torch.Tensor]
    ksum: Optional[torch.Tensor]
    vsum: Optional[torch.Tensor]
    cand_pos: Optional[torch.Tensor]
    cand_class: Optional[torch.Tensor]
    cand_cu: Optional[torch.Tensor]
    samp_pos: Optional[torch.Tensor]
    class_weight_q: Optional[torch.Tensor]
    class_mean: Optional[torch.Tensor]
    samp_score: Optional[torch.Tensor]
    dev_status: torch.Tensor
    args: dsk_compress_args
    keep: tuple


def compress(*, cu_seqlens: torch.Tensor, max_seqlen: int, Hq: int, K: Optional[torch.Tensor],
             V: Optional[torch.Tensor] = None, stages: int = DSK_STAGE_SEGMENT | DSK_STAGE_SUMMARIES,
             token_ids: Optional[torch.Tensor] = None, delim_ids: Optional[torch.Tensor] = None,
             n_class: int = 16, cand_pos: Optional[torch.Tensor] = None,
             cand_class: Optional[torch.Tensor] = None, cand_cu: Optional[torch.Tensor] = None,
             max_cand_total: Optional[int] = None,
             M: int = 0, W: int = 8, R: int = 128, alpha_imp: float = 1.0, imp_scale: float = 0.0,
             samp_pos: Optional[torch.Tensor] = None, qwin: Optional[torch.Tensor] = None,
             class_weight_q: Optional[torch.Tensor] = None,
             C_: int = 32, delta: int = 16, C_per_seq: Optional[torch.Tensor] = None,
             delta_per_seq: Optional[torch.Tensor] = None, min_chunk: Optional[int] = None,
             alpha_num: int = 5, alpha_den: int = 10, b: int = 16,
             max_blocks_total: Optional[int] = None, block_start: Optional[torch.Tensor] = None,
             cu_blocks: Optional[torch.Tensor] = None, slot_base: Optional[torch.Tensor] = None,
             cu_slots: Optional[torch.Tensor] = None, want_vsum: bool = False, Hkv: Optional[int] = None, total_tokens: Optional[int] = None,
             summary_mode: int = DSK_SUMMARY_MINMAX, want_candidates: bool = True,
             samp_score_sum: Optional[torch.Tensor] = None, imp_layers: int = 0, stream=None,
             check: bool = True) -> Compressed:
    """Allocate outputs / workspace with torch, fill dsk_compress_args and call dsk_compress.

    `want_candidates=False` (stages CANDIDATES + SEGMENT, no sampling): the candidate lists are
    not produced; the per-token classes go straight to the segmentation.

    `total_tokens` defaults to the token extent of K (or of token_ids).  Buffers a skipped
    stage would have produced must be passed in."""
    dev = cu_seqlens.device
    B = cu_seqlens.numel() - 1
    if Hkv is None:
        Hkv = K.shape[0]
    if total_tokens is None:
        total_tokens = K.shape[1] if K is not None else token_ids.numel()
    a = dsk_compress_args()
    a.struct_size = C.sizeof(dsk_compress_args)
    a.stages = stages
    a.B, a.Hq, a.Hkv, a.D = B, Hq, Hkv, DSK_HEAD_DIM
    a.total_tokens, a.max_seqlen = total_tokens, max_seqlen
    a.cu_seqlens = _ptr(cu_seqlens)
    if K is not None:
        a.K = _ptr(K)
        a.k_stride_tok, a.k_stride_head = _kv_strides(K)
    if V is not None:
        a.V = _ptr(V)
        a.v_stride_tok, a.v_stride_head = _kv_strides(V)
    a.token_ids, a.delim_ids = _ptr(token_ids), _ptr(delim_ids)
    a.n_class = n_class
    i32 = dict(dtype=torch.int32, device=dev)
    if max_cand_total is None:
        max_cand_total = cand_pos.numel() if cand_pos is not None else total_tokens
    if stages & DSK_STAGE_CANDIDATES and not want_candidates:
        assert stages & DSK_STAGE_SEGMENT and M == 0
        cand_pos = cand_class = cand_cu = None
        max_cand_total = 0
    elif stages & DSK_STAGE_CANDIDATES:
        cand_pos = torch.empty(max(max_cand_total, 1), **i32)
        cand_class = torch.empty(max(max_cand_total, 1), dtype=torch.uint8, device=dev)
        cand_cu = torch.empty(B + 1, **i32)
        if M > 0:
            samp_pos = torch.empty(B, n_class, M, **i32)
    a.max_cand_total = max_cand_total
    a.cand_pos, a.cand_class, a.cand_cu = _ptr(cand_pos), _ptr(cand_class), _ptr(cand_cu)
    a.M, a.W, a.R, a.alpha_imp, a.imp_scale = M, W, R, alpha_imp, imp_scale
    class_mean = samp_score = None
    if stages & DSK_STAGE_IMPORTANCE:
        class_mean = torch.empty(B, n_class, dtype=torch.float32, device=dev)
        samp_score = torch.empty(B, n_class, M, dtype=torch.float32, device=dev)
    a.samp_pos, a.qwin = _ptr(samp_pos), _ptr(qwin)
    a.class_weight_q = _ptr(class_weight_q)
    a.class_mean, a.samp_score = _ptr(class_mean), _ptr(samp_score)
    a.samp_score_sum, a.imp_layers = _ptr(samp_score_sum), imp_layers
    a.C, a.delta = C_, delta
    a.C_per_seq, a.delta_per_seq = _ptr(C_per_seq), _ptr(delta_per_seq)
    a.alpha_num, a.alpha_den, a.b = alpha_num, alpha_den, b
    if max_blocks_total is None:
        if block_start is not None:
            max_blocks_total = block_start.numel() - 1
        else:
            mc = min_chunk if min_chunk is not None else C_ - delta
            max_blocks_total = dsk_block_capacity(total_tokens, B, mc)
    if stages & DSK_STAGE_SEGMENT:
        block_start = torch.zeros(max_blocks_total + 4, **i32)  # both tables are read in 16-byte vectors
        slot_base = torch.zeros(max_blocks_total + 4, **i32)   # read in 16-byte vectors by dsk_select_topk
        cu_blocks = torch.empty(B + 1, **i32)
        cu_slots = torch.empty(B + 1, **i32)
    a.max_blocks_total = max_blocks_total
    a.block_start, a.cu_blocks, a.slot_base = _ptr(block_start), _ptr(cu_blocks), _ptr(slot_base)
    a.cu_slots = _ptr(cu_slots)
    ksum = vsum = None
    if stages & DSK_STAGE_SUMMARIES:
        ksum = torch.empty(Hkv, max_blocks_total, 2, DSK_HEAD_DIM, dtype=torch.bfloat16, device=dev)
        if want_vsum:
            vsum = torch.empty_like(ksum)
    a.ksum, a.vsum = _ptr(ksum), _ptr(vsum)
    a.summary_mode = summary_mode
    dev_status = torch.zeros(1, **i32)
    a.dev_status = _ptr(dev_status)
    ws = _ws(dsk_compress_workspace_bytes(a), dev)
    a.workspace, a.workspace_bytes = _ptr(ws), ws.numel()
    keep = (cu_seqlens, K, V, token_ids, delim_ids, qwin, C_per_seq, delta_per_seq, ws)
    dsk_compress(a, stream, check=check)
    return Compressed(B=B, Hq=Hq, Hkv=Hkv, b=b, total_tokens=total_tokens, max_blocks_total=max_blocks_total,
                      cu_seqlens=cu_seqlens, block_start=block_start, cu_blocks=cu_blocks, slot_base=slot_base,
                      cu_slots=cu_slots, ksum=ksum, vsum=vsum, cand_pos=cand_pos, cand_class=cand_class, cand_cu=cand_cu,
                      samp_pos=samp_pos, class_weight_q=class_weight_q, class_mean=class_mean,
                      samp_score=samp_score, dev_status=dev_status, args=a, keep=keep)


@dataclass
class Selection:
    k: int
    b: int
    sel_slot: torch.Tensor     # int32 [B, Hq, k]
    sel_start: torch.Tensor
    sel_len: torch.Tensor
    sel_count: torch.Tensor    # int32 [B, Hq]
    scores: Optional[torch.Tensor]
    args: dsk_select_args
    keep: tuple
    shared: bool = False       # one selection per KV head (the arrays are [B, Hkv, ...])


def make_select_args(comp: Compressed, q: torch.Tensor, budget: int, *, want_scores: bool = False,
                     out: Optional[Selection] = None, max_blocks_used: int = 0,
                     max_blocks_per_seq: int = 0, shared: bool = False,
                     budget_per_seq: Optional[torch.Tensor] = None) -> Selection:
    """Fill dsk_select_args for query q (bf16 [B, Hq, D]); buffers are reused from `out`.
    `max_blocks_used`: optional host-known bound on the total block count (0 = capacity);
    `max_blocks_per_seq`: optional bound on the blocks of any one sequence;
    `shared`: one selection per KV head instead of per query head (DSK_SELECT_SHARED_BY_KV_GROUP)."""
    dev = q.device
    B, Hq = comp.B, comp.Hq
    assert q.shape == (B, Hq, DSK_HEAD_DIM) and q.dtype == torch.bfloat16 and q.is_contiguous()
    k = budget // comp.b
    i32 = dict(dtype=torch.int32, device=dev)
    a = dsk_select_args()
    a.struct_size = C.sizeof(dsk_select_args)
    a.B, a.Hq, a.Hkv, a.D = B, Hq, comp.Hkv, DSK_HEAD_DIM
    a.max_blocks_total = comp.max_blocks_total
    a.max_blocks_used = max_blocks_used
    a.max_blocks_per_seq = max_blocks_per_seq
    a.cu_blocks, a.block_start, a.slot_base = _ptr(comp.cu_blocks), _ptr(comp.block_start), _ptr(comp.slot_base)
    a.ksum, a.q = _ptr(comp.ksum), _ptr(q)
    a.b, a.budget = comp.b, budget
    a.flags = DSK_SELECT_SHARED_BY_KV_GROUP if shared else 0
    a.budget_per_seq = _ptr(budget_per_seq)
    # tables with a region per sequence (RegionBatch): blocks in use and first K/V row of each sequence
    a.blocks_used, a.seq_row0 = _ptr(getattr(comp, "blocks_used", None)), _ptr(getattr(comp, "seq_row0", None))
    Hsel = comp.Hkv if shared else Hq
    if out is None:
        sel_slot = torch.empty(B, Hsel, max(k, 1), **i32)
        sel_start = torch.empty(B, Hsel, max(k, 1), **i32)
        sel_len = torch.empty(B, Hsel, max(k, 1), **i32)
        sel_count = torch.empty(B, Hsel, **i32)
        scores = torch.empty(Hsel, comp.max_blocks_total, dtype=torch.float32, device=dev) if want_scores else None
    else:
        assert out.shared == shared
        sel_slot, sel_start, sel_len, sel_count, scores = out.sel_slot, out.sel_start, out.sel_len, out.sel_count, out.scores
    a.sel_slot, a.sel_start, a.sel_len, a.sel_count = _ptr(sel_slot), _ptr(sel_start), _ptr(sel_len), _ptr(sel_count)
    a.scores = _ptr(scores)
    ws = _ws(dsk_select_workspace_bytes(a), dev) if out is None else out.keep[-1]
    a.workspace, a.workspace_bytes = _ptr(ws), ws.numel()
    return Selection(k=k, b=comp.b, sel_slot=sel_slot, sel_start=sel_start, sel_len=sel_len, sel_count=sel_count,
                     scores=scores, args=a, keep=(comp, q, budget_per_seq, ws), shared=shared)


def select_topk(comp: Compressed, q: torch.Tensor, budget: int, *, want_scores: bool = False, stream=None,
                check: bool = True, max_blocks_used: int = 0, max_blocks_per_seq: int = 0,
                shared: bool = False, budget_per_seq: Optional[torch.Tensor] = None) -> Selection:
    sel = make_select_args(comp, q, budget, want_scores=want_scores, max_blocks_used=max_blocks_used,
                           max_blocks_per_seq=max_blocks_per_seq, shared=shared, budget_per_seq=budget_per_seq)
    dsk_select_topk(sel.args, stream, check=check)
    return sel


@dataclass
class AttnOut:
    out: torch.Tensor   # f32 [B, Hq, D]
    lse: torch.Tensor   # f32 [B, Hq]
    args: dsk_attn_args
    keep: tuple
    out_bf16: Optional[torch.Tensor] = None   # bf16 [B, Hq, D] when asked for


def make_attn_args(q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, sel_start: torch.Tensor,
                   sel_len: torch.Tensor, sel_count: torch.Tensor, b: int, *, scale: float = 0.0,
                   out: Optional[AttnOut] = None, flags: int = 0, want_bf16: bool = False) -> AttnOut:
    dev = q.device
    B, Hq, D = q.shape
    assert D == DSK_HEAD_DIM and q.dtype == torch.bfloat16 and q.is_contiguous()
    k = sel_start.shape[2]
    a = dsk_attn_args()
    a.struct_size = C.sizeof(dsk_attn_args)
    a.B, a.Hq, a.Hkv, a.D = B, Hq, K.shape[0], D
    a.q, a.K, a.V = _ptr(q), _ptr(K), _ptr(V)
    a.k_stride_tok, a.k_stride_head = _kv_strides(K)
    a.v_stride_tok, a.v_stride_head = _kv_strides(V)
    a.total_tokens, a.k, a.b = K.shape[1], k, b
    a.sel_start, a.sel_len, a.sel_count = _ptr(sel_start), _ptr(sel_len), _ptr(sel_count)
    a.scale = scale
    a.flags = flags
    if out is None:
        o = torch.empty(B, Hq, D, dtype=torch.float32, device=dev)
        lse = torch.empty(B, Hq, dtype=torch.float32, device=dev)
        ws = _ws(dsk_attn_workspace_bytes(a), dev)
    else:
        o, lse, ws = out.out, out.lse, out.keep[-1]
    a.out, a.lse = _ptr(o), _ptr(lse)
    ob = out.out_bf16 if out is not None else None
    if want_bf16 and ob is None:
        ob = torch.empty(B, Hq, D, dtype=torch.bfloat16, device=dev)
    a.out_bf16 = _ptr(ob)
    a.workspace, a.workspace_bytes = _ptr(ws), ws.numel()
    return AttnOut(out=o, lse=lse, args=a, keep=(q, K, V, sel_start, sel_len, sel_count, ws), out_bf16=ob)


def sparse_decode_attn(q, K, V, sel_start, sel_len, sel_count, b, *, scale: float = 0.0, stream=None,
                       check: bool = True, want_bf16: bool = False, flags: int = 0) -> AttnOut:
    r = make_attn_args(q, K, V, sel_start, sel_len, sel_count, b, scale=scale, want_bf16=want_bf16, flags=flags)
    dsk_sparse_decode_attn(r.args, stream, check=check)
    return r


def make_dense_attn_args(q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, cu_seqlens: torch.Tensor,
                         max_seqlen: int, *, scale: float = 0.0, out: Optional[AttnOut] = None,
                         want_bf16: bool = False) -> AttnOut:
    dev = q.device
    B, Hq, D = q.shape
    assert D == DSK_HEAD_DIM and q.dtype == torch.bfloat16 and q.is_contiguous()
    assert cu_seqlens.dtype == torch.int32 and cu_seqlens.numel() == B + 1
    a = dsk_dense_attn_args()
    a.struct_size = C.sizeof(dsk_dense_attn_args)
    a.B, a.Hq, a.Hkv, a.D = B, Hq, K.shape[0], D
    a.q, a.K, a.V = _ptr(q), _ptr(K), _ptr(V)
    a.k_stride_tok, a.k_stride_head = _kv_strides(K)
    a.v_stride_tok, a.v_stride_head = _kv_strides(V)
    a.total_tokens, a.max_seqlen = K.shape[1], max_seqlen
    a.cu_seqlens = _ptr(cu_seqlens)
    a.scale = scale
    a.flags = 0
    if out is None:
        o = torch.empty(B, Hq, D, dtype=torch.float32, device=dev)
        lse = torch.empty(B, Hq, dtype=torch.float32, device=dev)
        ws = _ws(dsk_dense_attn_workspace_bytes(a), dev)
    else:
        o, lse, ws = out.out, out.lse, out.keep[-1]
    a.out, a.lse = _ptr(o), _ptr(lse)
    ob = out.out_bf16 if out is not None else None
    if want_bf16 and ob is None:
        ob = torch.empty(B, Hq, D, dtype=torch.bfloat16, device=dev)
    a.out_bf16 = _ptr(ob)
    a.workspace, a.workspace_bytes = _ptr(ws), ws.numel()
    return AttnOut(out=o, lse=lse, args=a, keep=(q, K, V, cu_seqlens, ws), out_bf16=ob)


def dense_decode_attn(q, K, V, cu_seqlens, max_seqlen, *, scale: float = 0.0, stream=None,
                      check: bool = True, want_bf16: bool = False) -> AttnOut:
    att = make_dense_attn_args(q, K, V, cu_seqlens, max_seqlen, scale=scale, want_bf16=want_bf16)
    dsk_dense_decode_attn(att.args, stream, check=check)
    return att


@dataclass
class Appender:
    """Argument struct of dsk_append_tokens bound to the tables of one single-sequence
    Compressed; set len_old / len_new and call step()."""
    args: dsk_append_args
    first_recomputed: torch.Tensor
    first_stale_slot: torch.Tensor      # int32 [1]: usable as stale_from of dsk_reuse_update
    keep: tuple

    def step(self, len_old: int, len_new: int, stream=None, check: bool = True) -> int:
        self.args.len_old, self.args.len_new = len_old, len_new
        return dsk_append_tokens(self.args, stream, check=check)


def make_appender(comp: Compressed, K: torch.Tensor, V: Optional[torch.Tensor], token_ids: torch.Tensor,
                  delim_ids: torch.Tensor, class_weight_q: torch.Tensor, *, C_: int, delta: int,
                  alpha_num: int, alpha_den: int, b: int) -> Appender:
    """comp must come from a B = 1 compress; its block_start / slot_base / cu_blocks / ksum (and
    vsum) are updated in place by every step()."""
    dev = K.device
    assert comp.cu_blocks.numel() == 2, "one sequence per appender"
    a = dsk_append_args()
    a.struct_size = C.sizeof(dsk_append_args)
    a.Hkv, a.D = K.shape[0], DSK_HEAD_DIM
    a.K = _ptr(K)
    a.k_stride_tok, a.k_stride_head = _kv_strides(K)
    if comp.vsum is not None:
        a.V = _ptr(V)
        a.v_stride_tok, a.v_stride_head = _kv_strides(V)
    a.token_ids, a.delim_ids, a.n_class = _ptr(token_ids), _ptr(delim_ids), delim_ids.numel()
    a.class_weight_q = _ptr(class_weight_q)
    a.C, a.delta, a.alpha_num, a.alpha_den, a.b = C_, delta, alpha_num, alpha_den, b
    a.max_blocks_total = comp.args.max_blocks_total
    a.block_start, a.cu_blocks, a.slot_base = _ptr(comp.block_start), _ptr(comp.cu_blocks), _ptr(comp.slot_base)
    a.ksum, a.vsum = _ptr(comp.ksum), _ptr(comp.vsum)
    a.summary_mode = comp.args.summary_mode
    first = torch.zeros(1, dtype=torch.int32, device=dev)
    a.first_recomputed = _ptr(first)
    stale = torch.zeros(1, dtype=torch.int32, device=dev)
    a.first_stale_slot = _ptr(stale)
    a.dev_status = _ptr(comp.dev_status)
    ws = _ws(dsk_append_workspace_bytes(a), dev)
    a.workspace, a.workspace_bytes = _ptr(ws), ws.numel()
    return Appender(args=a, first_recomputed=first, first_stale_slot=stale, keep=(comp, K, V, token_ids, delim_ids, class_weight_q, ws))


@dataclass
class RegionBatch:
    """Block tables and summaries of a batch in which every sequence owns a region with room to
    grow (the layout of dsk_append_tokens_batch).  Usable wherever make_select_args takes a
    Compressed."""
    B: int
    Hq: int
    Hkv: int
    b: int
    total_rows: int
    max_blocks_total: int
    seq_row0: torch.Tensor      # int32 [B]
    seq_len: torch.Tensor       # int32 [B], kept by the caller / the appender
    cu_blocks: torch.Tensor     # int32 [B+1] region starts
    blocks_used: torch.Tensor   # int32 [B]
    block_start: torch.Tensor   # int32 [max_blocks_total + 4], positions count from each sequence's first token
    slot_base: torch.Tensor
    ksum: torch.Tensor          # bf16 [Hkv, max_blocks_total, 2, D]
    vsum: Optional[torch.Tensor]
    dev_status: torch.Tensor
    summary_mode: int
    keep: tuple = ()


def compress_regions(*, seq_row0, seq_len, region_entries, Hq: int, K: torch.Tensor, V: Optional[torch.Tensor],
                     token_ids: torch.Tensor, delim_ids: torch.Tensor, class_weight_q: torch.Tensor,
                     C_per_seq, delta_per_seq, alpha_num: int, alpha_den: int, b: int,
                     summary_mode: int = DSK_SUMMARY_MINMAX, want_vsum: bool = False, stream=None) -> RegionBatch:
    """Fill the region of every sequence with one dsk_compress call (B = 1, stages CANDIDATES +
    SEGMENT + SUMMARIES, no candidate lists) on that sequence's rows.  seq_row0 / seq_len /
    region_entries / C_per_seq / delta_per_seq: Python ints per sequence; class_weight_q uint8
    [B, n_class]."""
    dev = K.device
    B = len(seq_row0)
    Hkv, total_rows = K.shape[0], K.shape[1]
    n_class = delim_ids.numel()
    i32 = dict(dtype=torch.int32, device=dev)
    blk0 = [0]
    for n in region_entries:
        blk0.append(blk0[-1] + int(n))
    cap = blk0[-1]
    block_start = torch.zeros(cap + 4, **i32)
    slot_base = torch.zeros(cap + 4, **i32)
    ksum = torch.zeros(Hkv, cap, 2, DSK_HEAD_DIM, dtype=torch.bfloat16, device=dev)
    vsum = torch.zeros_like(ksum) if want_vsum else None
    blocks_used = torch.zeros(B, **i32)
    dev_status = torch.zeros(1, **i32)
    kst, ksh = _kv_strides(K)
    keep = []
    for s in range(B):
        row0, L, n_ent = int(seq_row0[s]), int(seq_len[s]), int(region_entries[s])
        assert n_ent >= 2 and row0 + L <= total_rows
        a = dsk_compress_args()
        a.struct_size = C.sizeof(dsk_compress_args)
        a.stages = DSK_STAGE_CANDIDATES | DSK_STAGE_SEGMENT | DSK_STAGE_SUMMARIES
        a.B, a.Hq, a.Hkv, a.D = 1, Hq, Hkv, DSK_HEAD_DIM
        a.total_tokens, a.max_seqlen = L, L
        cu = torch.tensor([0, L], **i32)
        a.cu_seqlens = _ptr(cu)
        a.K = K.data_ptr() + row0 * kst * 2
        a.k_stride_tok, a.k_stride_head = kst, ksh
        if want_vsum:
            vst, vsh = _kv_strides(V)
            a.V = V.data_ptr() + row0 * vst * 2
            a.v_stride_tok, a.v_stride_head = vst, vsh
        a.token_ids, a.delim_ids, a.n_class = token_ids.data_ptr() + 4 * row0, _ptr(delim_ids), n_class
        a.class_weight_q = class_weight_q.data_ptr() + s * n_class
        a.C, a.delta = int(C_per_seq[s]), int(delta_per_seq[s])
        a.alpha_num, a.alpha_den, a.b = alpha_num, alpha_den, b
        a.max_blocks_total = n_ent - 1
        a.sum_stride_blocks = cap
        cub = torch.zeros(2, **i32)
        a.block_start, a.slot_base = block_start.data_ptr() + 4 * blk0[s], slot_base.data_ptr() + 4 * blk0[s]
        a.cu_blocks = _ptr(cub)
        a.ksum = ksum.data_ptr() + blk0[s] * 2 * DSK_HEAD_DIM * 2
        a.vsum = vsum.data_ptr() + blk0[s] * 2 * DSK_HEAD_DIM * 2 if want_vsum else None
        a.summary_mode = summary_mode
        a.dev_status = _ptr(dev_status)
        ws = _ws(dsk_compress_workspace_bytes(a), dev)
        a.workspace, a.workspace_bytes = _ptr(ws), ws.numel()
        dsk_compress(a, stream)
        blocks_used[s:s + 1].copy_(cub[1:2])
        keep.append((cu, cub, ws))
    return RegionBatch(B=B, Hq=Hq, Hkv=Hkv, b=b, total_rows=total_rows, max_blocks_total=cap,
                       seq_row0=torch.tensor([int(x) for x in seq_row0], **i32),
                       seq_len=torch.tensor([int(x) for x in seq_len], **i32),
                       cu_blocks=torch.tensor(blk0, **i32), blocks_used=blocks_used, block_start=block_start,
                       slot_base=slot_base, ksum=ksum, vsum=vsum, dev_status=dev_status, summary_mode=summary_mode,
                       keep=tuple(keep) + (K, V, token_ids, delim_ids, class_weight_q))


@dataclass
class BatchAppender:
    """Argument struct of dsk_append_tokens_batch bound to a RegionBatch.  With `len_new` (int32 [B]
    on the device, filled by the caller before step()) every sequence grows to its entry; without,
    every sequence grows by max_new_tokens per step.  The call advances the RegionBatch's seq_len
    itself, so a loop of steps can be captured in a HIP graph."""
    args: dsk_append_batch_args
    rb: RegionBatch
    len_new: Optional[torch.Tensor]
    first_recomputed: torch.Tensor
    first_stale_slot: torch.Tensor
    keep: tuple

    def step(self, stream=None, check: bool = True) -> int:
        return dsk_append_tokens_batch(self.args, stream, check=check)


def make_batch_appender(rb: RegionBatch, K: torch.Tensor, V: Optional[torch.Tensor], token_ids: torch.Tensor,
                        delim_ids: torch.Tensor, class_weight_q: torch.Tensor, *, C_: int, delta: int,
                        C_per_seq: Optional[torch.Tensor], delta_per_seq: Optional[torch.Tensor],
                        alpha_num: int, alpha_den: int, max_new_tokens: int = 1,
                        lockstep: bool = False) -> BatchAppender:
    dev = K.device
    i32 = dict(dtype=torch.int32, device=dev)
    a = dsk_append_batch_args()
    a.struct_size = C.sizeof(dsk_append_batch_args)
    a.B, a.Hkv, a.D = rb.B, rb.Hkv, DSK_HEAD_DIM
    a.total_rows, a.max_new_tokens = rb.total_rows, max_new_tokens
    len_new = None if lockstep else rb.seq_len.clone()
    a.seq_row0, a.seq_len, a.len_new = _ptr(rb.seq_row0), _ptr(rb.seq_len), _ptr(len_new)
    a.K = _ptr(K)
    a.k_stride_tok, a.k_stride_head = _kv_strides(K)
    if rb.vsum is not None:
        a.V = _ptr(V)
        a.v_stride_tok, a.v_stride_head = _kv_strides(V)
    a.token_ids, a.delim_ids, a.n_class = _ptr(token_ids), _ptr(delim_ids), delim_ids.numel()
    a.class_weight_q = _ptr(class_weight_q)
    a.C, a.delta, a.alpha_num, a.alpha_den, a.b = C_, delta, alpha_num, alpha_den, rb.b
    a.C_per_seq, a.delta_per_seq = _ptr(C_per_seq), _ptr(delta_per_seq)
    a.max_blocks_total = rb.max_blocks_total
    a.cu_blocks, a.blocks_used = _ptr(rb.cu_blocks), _ptr(rb.blocks_used)
    a.block_start, a.slot_base = _ptr(rb.block_start), _ptr(rb.slot_base)
    a.ksum, a.vsum = _ptr(rb.ksum), _ptr(rb.vsum)
    a.summary_mode = rb.summary_mode
    first = torch.zeros(rb.B, **i32)
    stale = torch.zeros(rb.B, **i32)
    a.first_recomputed, a.first_stale_slot = _ptr(first), _ptr(stale)
    a.dev_status = _ptr(rb.dev_status)
    ws = _ws(dsk_append_batch_workspace_bytes(a), dev)
    a.workspace, a.workspace_bytes = _ptr(ws), ws.numel()
    return BatchAppender(args=a, rb=rb, len_new=len_new, first_recomputed=first, first_stale_slot=stale,
                         keep=(K, V, token_ids, delim_ids, class_weight_q, C_per_seq, delta_per_seq, ws))


@dataclass
class Reuser:
    """Resident K/V buffers of one batch and the state dsk_reuse_update carries from step to step."""
    k: int
    b: int
    res_slot: torch.Tensor     # int32 [B, Hq, k], -1 = empty
    res_len: torch.Tensor
    res_start: torch.Tensor
    res_count: torch.Tensor    # int32 [B, Hq]
    load_pos: torch.Tensor     # int32 [B, Hq, k]
    load_slot: torch.Tensor
    load_start: torch.Tensor
    load_len: torch.Tensor
    load_count: torch.Tensor   # int32 [B, Hq]
    reuse_count: torch.Tensor  # int32 [B]
    Kres: Optional[torch.Tensor]   # bf16 [Hq, B*k*b, D]
    Vres: Optional[torch.Tensor]
    args: dsk_reuse_args
    keep: tuple

    def step(self, stream=None, check: bool = True) -> int:
        return dsk_reuse_update(self.args, stream, check=check)

    def attn_args(self, q: torch.Tensor, *, scale: float = 0.0, out: Optional[AttnOut] = None) -> AttnOut:
        """Arguments of dsk_sparse_decode_attn over the resident buffers: every query head its own
        K/V, or -- when the reuser was built on a selection shared per KV head -- one buffer per KV
        head read by all its query heads."""
        shared = self.res_start.shape[1] != q.shape[1]
        return make_attn_args(q, self.Kres, self.Vres, self.res_start, self.res_len, self.res_count, self.b,
                              scale=scale, out=out, flags=DSK_ATTN_SHARED_SELECTION if shared else 0)


def make_reuser(sel: Selection, K: Optional[torch.Tensor], V: Optional[torch.Tensor], Hkv: int, *,
                stale_from: Optional[torch.Tensor] = None, plan_only: bool = False) -> Reuser:
    """sel: the Selection whose buffers every step's dsk_select_topk writes.  K / V: bf16
    [Hkv, tokens, D] views the device can read (HBM, or pinned host memory)."""
    dev = sel.sel_slot.device
    B, Hq, k = sel.sel_slot.shape
    b = sel.b
    i32 = dict(dtype=torch.int32, device=dev)
    a = dsk_reuse_args()
    a.struct_size = C.sizeof(dsk_reuse_args)
    a.B, a.Hq, a.Hkv, a.D = B, Hq, Hkv, DSK_HEAD_DIM
    a.k, a.b, a.flags = k, b, DSK_REUSE_PLAN_ONLY if plan_only else 0
    a.sel_slot, a.sel_start, a.sel_len, a.sel_count = (_ptr(sel.sel_slot), _ptr(sel.sel_start), _ptr(sel.sel_len),
                                                       _ptr(sel.sel_count))
    a.stale_from = _ptr(stale_from)
    res_slot = torch.full((B, Hq, k), -1, **i32)
    res_len = torch.zeros(B, Hq, k, **i32)
    res_start = torch.zeros(B, Hq, k, **i32)
    res_count = torch.zeros(B, Hq, **i32)
    load_pos, load_slot = torch.empty(B, Hq, k, **i32), torch.empty(B, Hq, k, **i32)
    load_start, load_len = torch.empty(B, Hq, k, **i32), torch.empty(B, Hq, k, **i32)
    load_count = torch.zeros(B, Hq, **i32)
    reuse_count = torch.zeros(B, **i32)
    a.res_slot, a.res_len, a.res_start, a.res_count = _ptr(res_slot), _ptr(res_len), _ptr(res_start), _ptr(res_count)
    a.load_pos, a.load_slot, a.load_start, a.load_len = _ptr(load_pos), _ptr(load_slot), _ptr(load_start), _ptr(load_len)
    a.load_count, a.reuse_count = _ptr(load_count), _ptr(reuse_count)
    Kres = Vres = None
    if not plan_only:
        a.K, a.V = _ptr(K), _ptr(V)
        a.k_stride_tok, a.k_stride_head = _kv_strides(K)
        a.v_stride_tok, a.v_stride_head = _kv_strides(V)
        a.total_tokens = K.shape[1]
        Kres = torch.zeros(Hq, B * k * b, DSK_HEAD_DIM, dtype=torch.bfloat16, device=dev)
        Vres = torch.zeros(Hq, B * k * b, DSK_HEAD_DIM, dtype=torch.bfloat16, device=dev)
        a.Kres, a.Vres = _ptr(Kres), _ptr(Vres)
    ws = _ws(dsk_reuse_workspace_bytes(a), dev)
    a.workspace, a.workspace_bytes = _ptr(ws), ws.numel()
    return Reuser(k=k, b=b, res_slot=res_slot, res_len=res_len, res_start=res_start, res_count=res_count,
                  load_pos=load_pos, load_slot=load_slot, load_start=load_start, load_len=load_len,
                  load_count=load_count, reuse_count=reuse_count, Kres=Kres, Vres=Vres, args=a,
                  keep=(sel, K, V, stale_from, ws))
