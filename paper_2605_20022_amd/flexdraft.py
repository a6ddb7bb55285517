"""ctypes binding of libflexdraft.so: argument marshalling only.

Every function here has the name of the C entry point it forwards to
(include/flexdraft.h).  Torch is used for device memory and the current stream;
no arithmetic of the method happens in Python.  If the shared library has not
been built, loading raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# FLEXDRAFT_LIB names another build of the same library (same C ABI), e.g. one compiled with other tuning macros
LIB_PATH = os.environ.get("FLEXDRAFT_LIB") or os.path.join(_HERE, "libflexdraft.so")

FD_F32, FD_BF16 = 0, 1
FD_ATTN_FORCE_GENERIC = 1
FD_ATTN_PLANNED = 2
FD_OK = 0
STATUS_NAMES = {0: "FD_OK", 1: "FD_ERR_INVALID_ARG", 2: "FD_ERR_UNSUPPORTED",
                3: "FD_ERR_WORKSPACE_TOO_SMALL", 4: "FD_ERR_HIP"}


class fd_attn_args(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("page_size", C.c_int32), ("dtype", C.c_int32), ("sm_scale", C.c_float), ("flags", C.c_int32),
        ("total_rows", C.c_int32), ("max_kv_len", C.c_int32), ("max_new_rows", C.c_int32), ("num_pages", C.c_int32),
        ("kv_chunk", C.c_int32), ("page_indices_len", C.c_int32),
        ("k_cache", C.c_void_p), ("v_cache", C.c_void_p),
        ("cache_stride_page", C.c_int64), ("cache_stride_head", C.c_int64), ("cache_stride_token", C.c_int64),
        ("page_indptr", C.c_void_p), ("page_indices", C.c_void_p), ("kv_len", C.c_void_p),
        ("row_indptr", C.c_void_p), ("verify_len", C.c_void_p), ("mask_vis", C.c_void_p),
        ("mask_blocks", C.c_void_p),
        ("q", C.c_void_p), ("k_new", C.c_void_p), ("v_new", C.c_void_p),
        ("out", C.c_void_p), ("lse", C.c_void_p),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
        ("status", C.c_void_p),
    ]


class FlexDraftError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{STATUS_NAMES.get(code, code)}: {msg}")
        self.code = code


_lib = None

EXPORTS = ["fd_verify_draft_attn_workspace", "fd_verify_draft_attn", "fd_accept_greedy", "fd_accept_sample",
           "fd_accept_workspace", "fd_draft_select", "fd_draft_select_workspace", "fd_append_kv", "fd_select_branch", "fd_last_error", "fd_version", "fd_verify_draft_attn_static",
           "fd_verify_draft_plan"]


def load() -> C.CDLL:
    """Load the HIP library; raises if it has not been built (python -m paper_2605_20022_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python paper_2605_20022_amd/build.py` "
                           "(hipcc, gfx950). There is no CPU fallback.")
    lib = C.CDLL(LIB_PATH)
    lib.fd_verify_draft_attn_workspace.restype = C.c_size_t
    lib.fd_verify_draft_attn_workspace.argtypes = [C.POINTER(fd_attn_args)]
    lib.fd_verify_draft_attn.restype = C.c_int
    lib.fd_verify_draft_attn.argtypes = [C.POINTER(fd_attn_args), C.c_void_p]
    lib.fd_accept_greedy.restype = C.c_int
    lib.fd_accept_greedy.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p,
                                     C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_size_t, C.c_void_p]
    lib.fd_accept_sample.restype = C.c_int
    lib.fd_accept_sample.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int32, C.c_float,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_size_t, C.c_void_p]
    lib.fd_accept_workspace.restype = C.c_size_t
    lib.fd_accept_workspace.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    lib.fd_draft_select.restype = C.c_int
    lib.fd_draft_select.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int32, C.c_float, C.c_float, C.c_void_p,
                                    C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_void_p, C.c_size_t, C.c_void_p]
    lib.fd_draft_select_workspace.restype = C.c_size_t
    lib.fd_draft_select_workspace.argtypes = [C.c_int32, C.c_int32]
    lib.fd_append_kv.restype = C.c_int
    lib.fd_append_kv.argtypes = [C.POINTER(fd_attn_args), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.fd_verify_draft_plan.restype = C.c_int
    lib.fd_verify_draft_plan.argtypes = [C.POINTER(fd_attn_args), C.c_void_p]
    lib.fd_verify_draft_attn_static.restype = C.c_int
    lib.fd_verify_draft_attn_static.argtypes = [C.POINTER(fd_attn_args), C.c_void_p]
    lib.fd_select_branch.restype = C.c_int
    lib.fd_select_branch.argtypes = [C.c_void_p] * 6 + [C.c_int32] * 3 + [C.c_void_p] * 3
    lib.fd_last_error.restype = C.c_char_p
    lib.fd_version.restype = C.c_char_p
    _lib = lib
    return lib


def _check(code: int):
    if code != FD_OK:
        raise FlexDraftError(code, load().fd_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return FD_BF16
    if t.dtype == torch.float32:
        return FD_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _i32(t: torch.Tensor, name: str) -> torch.Tensor:
    if t.dtype != torch.int32 or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous int32 tensor")
    return t


def make_attn_args(q, k_new, v_new, k_cache, v_cache, page_indptr, page_indices, kv_len, row_indptr,
                   verify_len, mask_vis=None, mask_blocks=None, *, out, lse=None, max_kv_len: int, max_new_rows: int,
                   sm_scale: float = 0.0, flags: int = 0, kv_chunk: int = 0, workspace=None, status=None):
    """Fill an fd_attn_args from tensors.  k_cache / v_cache: [pages, Hkv, page_size, D] views
    (any strides with a contiguous last dimension)."""
    R, Hq, D = q.shape
    Hkv = k_new.shape[1]
    for name, t in (("q", q), ("k_new", k_new), ("v_new", v_new), ("out", out)):
        if not t.is_contiguous():
            raise TypeError(f"{name} must be contiguous")
    if k_cache.stride(3) != 1 or v_cache.stride() != k_cache.stride():
        raise TypeError("k_cache / v_cache need a contiguous last dimension and identical strides")
    a = fd_attn_args()
    a.batch = kv_len.shape[0]; a.num_q_heads = Hq; a.num_kv_heads = Hkv; a.head_dim = D
    a.page_size = k_cache.shape[2]; a.dtype = _dtype_code(q); a.sm_scale = sm_scale; a.flags = flags
    a.total_rows = R; a.max_kv_len = int(max_kv_len); a.max_new_rows = int(max_new_rows)
    a.num_pages = k_cache.shape[0]; a.kv_chunk = kv_chunk; a.page_indices_len = page_indices.numel()
    a.k_cache = k_cache.data_ptr(); a.v_cache = v_cache.data_ptr()
    a.cache_stride_page = k_cache.stride(0); a.cache_stride_head = k_cache.stride(1)
    a.cache_stride_token = k_cache.stride(2)
    a.page_indptr = _i32(page_indptr, "page_indptr").data_ptr()
    a.page_indices = _i32(page_indices, "page_indices").data_ptr()
    a.kv_len = _i32(kv_len, "kv_len").data_ptr()
    a.row_indptr = _i32(row_indptr, "row_indptr").data_ptr()
    a.verify_len = _i32(verify_len, "verify_len").data_ptr()
    a.mask_vis = None if mask_vis is None else _i32(mask_vis, "mask_vis").data_ptr()
    a.mask_blocks = None if mask_blocks is None else _i32(mask_blocks, "mask_blocks").data_ptr()
    a.q = q.data_ptr(); a.k_new = k_new.data_ptr(); a.v_new = v_new.data_ptr()
    a.out = out.data_ptr(); a.lse = None if lse is None else lse.data_ptr()
    if workspace is not None:
        a.workspace = workspace.data_ptr(); a.workspace_bytes = workspace.numel() * workspace.element_size()
    a.status = None if status is None else status.data_ptr()
    return a


def fd_verify_draft_attn_workspace(args: fd_attn_args) -> int:
    return int(load().fd_verify_draft_attn_workspace(C.byref(args)))


def fd_verify_draft_attn(args: fd_attn_args, stream=None) -> None:
    """Enqueue the attention call described by `args` on `stream` (default: torch's current stream)."""
    _check(load().fd_verify_draft_attn(C.byref(args), _stream(stream)))


def fd_verify_draft_plan(args: fd_attn_args, stream=None) -> None:
    """Write the plan for `args` into args.workspace; attention calls with FD_ATTN_PLANNED start from it."""
    _check(load().fd_verify_draft_plan(C.byref(args), _stream(stream)))


def fd_verify_draft_attn_static(args: fd_attn_args, stream=None) -> None:
    """The same call on the library's own static scratch buffer: args.workspace is ignored."""
    _check(load().fd_verify_draft_attn_static(C.byref(args), _stream(stream)))


FD_STATIC_SCRATCH_BYTES = 44 << 20


def fd_accept_workspace(batch: int, total_rows: int, vocab: int, sampling: bool) -> int:
    return int(load().fd_accept_workspace(batch, total_rows, vocab, 1 if sampling else 0))


def fd_accept_greedy(target_logits, row_indptr, input_tokens, accept_len, bonus_token, *, vocab=None,
                     max_rows_per_seq: int, row_argmax=None, workspace, stream=None) -> None:
    Rv = target_logits.shape[0]
    vocab = target_logits.shape[1] if vocab is None else vocab
    if target_logits.stride(1) != 1:
        raise TypeError("logits rows must be contiguous")
    _check(load().fd_accept_greedy(
        _ptr(target_logits), _dtype_code(target_logits), target_logits.stride(0), vocab,
        _ptr(_i32(row_indptr, "row_indptr")), _ptr(_i32(input_tokens, "input_tokens")),
        accept_len.shape[0], Rv, max_rows_per_seq,
        _ptr(_i32(accept_len, "accept_len")), _ptr(_i32(bonus_token, "bonus_token")),
        None if row_argmax is None else _ptr(_i32(row_argmax, "row_argmax")),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def fd_accept_sample(target_logits, draft_logits, row_indptr, input_tokens, u_accept, u_resample,
                     accept_len, bonus_token, *, temperature: float, vocab=None, max_rows_per_seq: int,
                     workspace, stream=None) -> None:
    Rv = target_logits.shape[0]
    vocab = target_logits.shape[1] if vocab is None else vocab
    if target_logits.stride(1) != 1 or draft_logits.stride() != target_logits.stride() or \
            draft_logits.dtype != target_logits.dtype:
        raise TypeError("target / draft logits must share dtype and strides, rows contiguous")
    for name, t in (("u_accept", u_accept), ("u_resample", u_resample)):
        if t.dtype != torch.float32 or not t.is_contiguous():
            raise TypeError(f"{name} must be contiguous float32")
    _check(load().fd_accept_sample(
        _ptr(target_logits), _ptr(draft_logits), _dtype_code(target_logits), target_logits.stride(0), vocab,
        float(temperature), _ptr(_i32(row_indptr, "row_indptr")), _ptr(_i32(input_tokens, "input_tokens")),
        _ptr(u_accept), _ptr(u_resample), accept_len.shape[0], Rv, max_rows_per_seq,
        _ptr(_i32(accept_len, "accept_len")), _ptr(_i32(bonus_token, "bonus_token")),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def fd_draft_select_workspace(total_rows: int, vocab: int) -> int:
    return int(load().fd_draft_select_workspace(total_rows, vocab))


def fd_draft_select(draft_logits, row_indptr, draft_tokens, keep_len, *, temperature: float, threshold: float,
                    max_rows_per_seq: int, confidence=None, vocab=None, workspace, stream=None) -> None:
    R = draft_logits.shape[0]
    vocab = draft_logits.shape[1] if vocab is None else vocab
    if R and draft_logits.stride(1) != 1:
        raise TypeError("logits rows must be contiguous")
    _check(load().fd_draft_select(
        _ptr(draft_logits), _dtype_code(draft_logits), draft_logits.stride(0) if R else vocab, vocab,
        float(temperature), float(threshold), _ptr(_i32(row_indptr, "row_indptr")), keep_len.shape[0], R,
        int(max_rows_per_seq), _ptr(_i32(draft_tokens, "draft_tokens")),
        None if confidence is None else _ptr(confidence), _ptr(_i32(keep_len, "keep_len")),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def fd_append_kv(args: fd_attn_args, k_cache, v_cache, accept_len, kv_len_out, stream=None) -> None:
    """Commit new rows 0 .. accept_len[i] of the call described by `args` to the paged cache
    k_cache / v_cache (written; laid out as args' strides say)."""
    _check(load().fd_append_kv(C.byref(args), _ptr(k_cache), _ptr(v_cache), _ptr(_i32(accept_len, "accept_len")),
                               _ptr(_i32(kv_len_out, "kv_len_out")), _stream(stream)))


def fd_select_branch(block_tokens, block_indptr, mask_blocks, accept_len, out_tokens, *, first_vis=None,
                     verify_len=None, out_block=None, stream=None) -> None:
    B = accept_len.shape[0]
    _check(load().fd_select_branch(
        _ptr(_i32(block_tokens, "block_tokens")), _ptr(_i32(block_indptr, "block_indptr")),
        _ptr(_i32(mask_blocks, "mask_blocks")), _ptr(_i32(accept_len, "accept_len")),
        None if first_vis is None else _ptr(_i32(first_vis, "first_vis")),
        None if verify_len is None else _ptr(_i32(verify_len, "verify_len")), B, block_tokens.numel(),
        out_tokens.shape[1], _ptr(_i32(out_tokens, "out_tokens")),
        None if out_block is None else _ptr(_i32(out_block, "out_block")), _stream(stream)))


def fd_version() -> str:
    return load().fd_version().decode()


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """256-byte aligned device buffer of at least nbytes (torch allocations are 256-byte aligned)."""
    return torch.empty(max(256, (nbytes + 255) // 256 * 256), dtype=torch.uint8, device=device)
