"""ctypes binding of libsparsed.so: argument marshalling only.

Every function has the name of the C entry point it wraps (minus the ``sparsed_`` prefix) and
passes torch device tensors' pointers, shapes and strides straight through; all arithmetic of
the method runs in the HIP kernels behind the C ABI (include/sparsed.h). There is no CPU or
PyTorch fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch  # imported before the library so that it resolves HIP from the runtime torch loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsparsed.so")

SPARSED_BF16, SPARSED_F32 = 0, 1

EXPORTS = [
    "sparsed_attn_dense", "sparsed_select_pattern", "sparsed_attn_sparse", "sparsed_select_pattern_isolated",
    "sparsed_kept_blocks", "sparsed_n_dense_steps", "sparsed_select_workspace_bytes", "sparsed_index_validate",
    "sparsed_status_string", "sparsed_last_error", "sparsed_version",
    "sparsed_index_fill_window", "sparsed_index_window_entries", "sparsed_probe_mfma_bf16", "sparsed_probe_valu_f32", "sparsed_probe_mix_bf16",
    "sparsed_select_pattern_isolated_tokens", "sparsed_select_tokens_workspace_bytes",
    "sparsed_select_pattern_static", "sparsed_select_workspace_min_bytes",
]


class SparsedError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"sparsed status {status}: {message}")
        self.status = status


class _Tensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("dtype", ctypes.c_int32),
                ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("L", ctypes.c_int32), ("D", ctypes.c_int32),
                ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_l", ctypes.c_int64)]


class _BlockIndex(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("nqb", ctypes.c_int32), ("nkb", ctypes.c_int32),
                ("block_q", ctypes.c_int32), ("block_k", ctypes.c_int32), ("cap_per_head", ctypes.c_int32),
                ("row_ptr", ctypes.c_void_p), ("col_idx", ctypes.c_void_p)]


class _Exec(ctypes.Structure):
    _fields_ = [("stream", ctypes.c_void_p), ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("lse_out", ctypes.c_void_p), ("lse_in", ctypes.c_void_p), ("pooled_out", ctypes.c_void_p),
                ("seq_lens", ctypes.c_void_p)]


_lib = None


def load_library(build_if_missing: bool = True) -> ctypes.CDLL:
    """Load libsparsed.so (building it first only if it does not exist) and declare signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        if not build_if_missing:
            raise FileNotFoundError(_LIB_PATH)
        from . import build as _build

        _build.build(force=True)
    lib = ctypes.CDLL(_LIB_PATH)
    T, I, E = ctypes.POINTER(_Tensor), ctypes.POINTER(_BlockIndex), ctypes.POINTER(_Exec)
    lib.sparsed_attn_dense.argtypes = [T, T, T, T, E]
    lib.sparsed_attn_dense.restype = ctypes.c_int
    lib.sparsed_select_pattern.argtypes = [T, T, ctypes.c_int32, ctypes.c_int32, ctypes.c_double, I, E]
    lib.sparsed_select_pattern.restype = ctypes.c_int
    lib.sparsed_select_pattern_static.argtypes = [T, T, ctypes.c_int32, ctypes.c_int32, ctypes.c_double, I, E]
    lib.sparsed_select_pattern_static.restype = ctypes.c_int
    lib.sparsed_select_pattern_isolated.argtypes = [T, T, ctypes.c_int32, ctypes.c_int32, ctypes.c_double, ctypes.c_int32, I, E]
    lib.sparsed_select_pattern_isolated.restype = ctypes.c_int
    lib.sparsed_select_pattern_isolated_tokens.argtypes = [T, T, ctypes.c_int32, ctypes.c_int32, ctypes.c_double, ctypes.c_int32, I, E]
    lib.sparsed_select_pattern_isolated_tokens.restype = ctypes.c_int
    lib.sparsed_select_tokens_workspace_bytes.argtypes = [T, ctypes.c_int32, ctypes.c_int32]
    lib.sparsed_select_tokens_workspace_bytes.restype = ctypes.c_size_t
    lib.sparsed_attn_sparse.argtypes = [T, T, T, I, T, E]
    lib.sparsed_attn_sparse.restype = ctypes.c_int
    lib.sparsed_kept_blocks.argtypes = [ctypes.c_double, ctypes.c_int32]
    lib.sparsed_kept_blocks.restype = ctypes.c_int32
    lib.sparsed_n_dense_steps.argtypes = [ctypes.c_int32, ctypes.c_double]
    lib.sparsed_n_dense_steps.restype = ctypes.c_int32
    lib.sparsed_select_workspace_bytes.argtypes = [T, ctypes.c_int32, ctypes.c_int32]
    lib.sparsed_select_workspace_bytes.restype = ctypes.c_size_t
    lib.sparsed_select_workspace_min_bytes.argtypes = [T, ctypes.c_int32, ctypes.c_int32]
    lib.sparsed_select_workspace_min_bytes.restype = ctypes.c_size_t
    lib.sparsed_index_validate.argtypes = [I, E]
    lib.sparsed_index_validate.restype = ctypes.c_int
    lib.sparsed_index_fill_window.argtypes = [I, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, E]
    lib.sparsed_index_fill_window.restype = ctypes.c_int
    lib.sparsed_index_window_entries.argtypes = [ctypes.c_int32] * 5
    lib.sparsed_index_window_entries.restype = ctypes.c_int64
    lib.sparsed_probe_mfma_bf16.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_double), E]
    lib.sparsed_probe_mfma_bf16.restype = ctypes.c_int
    lib.sparsed_probe_valu_f32.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_double), E]
    lib.sparsed_probe_valu_f32.restype = ctypes.c_int
    lib.sparsed_probe_mix_bf16.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_double), E]
    lib.sparsed_probe_mix_bf16.restype = ctypes.c_int
    lib.sparsed_status_string.argtypes = [ctypes.c_int]
    lib.sparsed_status_string.restype = ctypes.c_char_p
    lib.sparsed_last_error.argtypes = []
    lib.sparsed_last_error.restype = ctypes.c_char_p
    lib.sparsed_version.argtypes = []
    lib.sparsed_version.restype = ctypes.c_int32
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != 0:
        lib = load_library()
        msg = lib.sparsed_last_error().decode() or lib.sparsed_status_string(status).decode()
        raise SparsedError(status, msg)


def _tensor(t: torch.Tensor, name: str) -> _Tensor:
    if t.dim() != 4:
        raise ValueError(f"{name} must be [B, H, L, D]")
    if t.dtype == torch.bfloat16:
        dt = SPARSED_BF16
    elif t.dtype == torch.float32:
        dt = SPARSED_F32
    else:
        raise ValueError(f"{name}: dtype {t.dtype} is not bf16 or fp32")
    if t.stride(3) != 1:
        raise ValueError(f"{name}: last dimension must be contiguous")
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    B, H, L, D = t.shape
    return _Tensor(t.data_ptr(), dt, B, H, L, D, t.stride(0), t.stride(1), t.stride(2))


def _stream_ptr(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


@dataclass
class BlockIndex:
    """Per-head CSR over key blocks (the sparse pattern of Eq. 4) in device memory."""

    row_ptr: torch.Tensor   # int32 [B, H, nqb + 1]
    col_idx: torch.Tensor   # int32 [B, H, cap_per_head]
    block_q: int
    block_k: int
    nkb: int

    @property
    def nqb(self) -> int:
        return self.row_ptr.shape[2] - 1

    def _c(self) -> _BlockIndex:
        B, H, _ = self.row_ptr.shape
        if self.row_ptr.dtype != torch.int32 or self.col_idx.dtype != torch.int32:
            raise ValueError("block index tensors must be int32")
        if not (self.row_ptr.is_contiguous() and self.col_idx.is_contiguous()):
            raise ValueError("block index tensors must be contiguous")
        return _BlockIndex(B, H, self.nqb, self.nkb, self.block_q, self.block_k, self.col_idx.shape[2],
                           self.row_ptr.data_ptr(), self.col_idx.data_ptr())


def version() -> int:
    return int(load_library().sparsed_version())


def kept_blocks(rho: float, n: int) -> int:
    return int(load_library().sparsed_kept_blocks(float(rho), int(n)))


def n_dense_steps(T: int, skip: float) -> int:
    return int(load_library().sparsed_n_dense_steps(int(T), float(skip)))


def select_workspace_bytes(q: torch.Tensor, block_q: int, block_k: int) -> int:
    """sparsed_select_workspace_bytes: the workspace that lets selection pool in one pass when no lse is handed over."""
    B, H, L, D = q.shape
    t = _Tensor(None, SPARSED_BF16 if q.dtype == torch.bfloat16 else SPARSED_F32, B, H, L, D, 0, 0, 0)
    return int(load_library().sparsed_select_workspace_bytes(ctypes.byref(t), block_q, block_k))


def select_workspace_min_bytes(q: torch.Tensor, block_q: int, block_k: int) -> int:
    """sparsed_select_workspace_min_bytes: the least the selection calls accept (statistics + pooled scores)."""
    B, H, L, D = q.shape
    t = _Tensor(None, SPARSED_BF16 if q.dtype == torch.bfloat16 else SPARSED_F32, B, H, L, D, 0, 0, 0)
    return int(load_library().sparsed_select_workspace_min_bytes(ctypes.byref(t), block_q, block_k))


def _seq_lens_ptr(seq_lens, B):
    if seq_lens is None:
        return None
    if seq_lens.dtype != torch.int32 or not seq_lens.is_cuda or not seq_lens.is_contiguous() or seq_lens.numel() != B:
        raise ValueError("seq_lens must be a contiguous int32 device tensor [B]")
    return seq_lens.data_ptr()


def attn_dense(q, k, v, out: Optional[torch.Tensor] = None, lse_out: Optional[torch.Tensor] = None, stream=None,
               seq_lens: Optional[torch.Tensor] = None):
    """sparsed_attn_dense: full bidirectional attention (Eq. 1). Returns ``out``."""
    lib = load_library()
    if out is None:
        out = torch.empty_like(q)
    ex = _Exec(_stream_ptr(stream), None, 0, lse_out.data_ptr() if lse_out is not None else None, None, None,
               _seq_lens_ptr(seq_lens, q.shape[0]))
    if lse_out is not None and (lse_out.dtype != torch.float32 or not lse_out.is_contiguous()
                                or lse_out.numel() != q.shape[0] * q.shape[1] * q.shape[2]):
        raise ValueError("lse_out must be contiguous fp32 [B, Hq, L]")
    tq, tk, tv, to = _tensor(q, "q"), _tensor(k, "k"), _tensor(v, "v"), _tensor(out, "out")
    _check(lib.sparsed_attn_dense(ctypes.byref(tq), ctypes.byref(tk), ctypes.byref(tv), ctypes.byref(to), ctypes.byref(ex)))
    return out


def _select(q, k, block_q, block_k, rho, prefill_blocks, lse_in, workspace, pooled_out, index, stream, prefill_tokens=None,
            seq_lens=None):
    lib = load_library()
    B, H, L, D = q.shape
    nqb, nkb = -(-L // block_q), -(-L // block_k)
    if prefill_tokens is not None:
        keep = kept_blocks(rho, -(-prefill_tokens // block_k)) + kept_blocks(rho, nkb - prefill_tokens // block_k)
    elif prefill_blocks is None:
        keep = kept_blocks(rho, nkb)
    else:
        keep = kept_blocks(rho, prefill_blocks) + kept_blocks(rho, nkb - prefill_blocks)
    if index is None:
        index = BlockIndex(torch.empty(B, H, nqb + 1, dtype=torch.int32, device=q.device),
                           torch.empty(B, H, max(nqb * keep, 1), dtype=torch.int32, device=q.device), block_q, block_k, nkb)
    if workspace is None:
        tq0 = _tensor(q, "q")
        if prefill_tokens is not None:
            need = int(lib.sparsed_select_tokens_workspace_bytes(ctypes.byref(tq0), block_q, block_k))
        elif lse_in is not None:
            need = select_workspace_min_bytes(q, block_q, block_k)   # the slabs of the one-pass kernel would go unused
        else:
            need = select_workspace_bytes(q, block_q, block_k)
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    if pooled_out is not None and (pooled_out.dtype != torch.float32 or not pooled_out.is_contiguous()
                                   or pooled_out.numel() != B * H * nqb * nkb):
        raise ValueError("pooled_out must be contiguous fp32 [B, Hq, nqb, nkb]")
    if lse_in is not None and (lse_in.dtype != torch.float32 or not lse_in.is_contiguous() or lse_in.numel() != B * H * L):
        raise ValueError("lse_in must be contiguous fp32 [B, Hq, L]")
    if stream is not None and int(stream.cuda_stream) != int(torch.cuda.current_stream(q.device).cuda_stream):
        # the kernels run on `stream`; keep the allocator from handing these blocks to later work on the current stream
        for t in (workspace, index.row_ptr, index.col_idx):
            t.record_stream(stream)
    ex = _Exec(_stream_ptr(stream), workspace.data_ptr(), workspace.numel() * workspace.element_size(), None,
               lse_in.data_ptr() if lse_in is not None else None, pooled_out.data_ptr() if pooled_out is not None else None,
               _seq_lens_ptr(seq_lens, B))
    tq, tk, ci = _tensor(q, "q"), _tensor(k, "k"), index._c()
    if prefill_tokens is not None:
        st = lib.sparsed_select_pattern_isolated_tokens(ctypes.byref(tq), ctypes.byref(tk), block_q, block_k, float(rho),
                                                        int(prefill_tokens), ctypes.byref(ci), ctypes.byref(ex))
    elif prefill_blocks is None:
        st = lib.sparsed_select_pattern(ctypes.byref(tq), ctypes.byref(tk), block_q, block_k, float(rho), ctypes.byref(ci),
                                        ctypes.byref(ex))
    else:
        st = lib.sparsed_select_pattern_isolated(ctypes.byref(tq), ctypes.byref(tk), block_q, block_k, float(rho),
                                                 int(prefill_blocks), ctypes.byref(ci), ctypes.byref(ex))
    _check(st)
    return index


def select_pattern(q, k, block_q: int, block_k: int, rho: float, lse_in=None, workspace=None, pooled_out=None,
                   index: Optional[BlockIndex] = None, stream=None, seq_lens: Optional[torch.Tensor] = None) -> BlockIndex:
    """sparsed_select_pattern: pooled post-softmax scores + per-row top-k -> CSR block index."""
    return _select(q, k, block_q, block_k, rho, None, lse_in, workspace, pooled_out, index, stream, seq_lens=seq_lens)


STATIC_SCRATCH_BYTES = 32 << 20


def select_pattern_static(q, k, block_q: int, block_k: int, rho: float, index: BlockIndex, lse_in=None, pooled_out=None,
                          stream=None, seq_lens: Optional[torch.Tensor] = None) -> BlockIndex:
    """sparsed_select_pattern_static: selection with the library's built-in scratch; allocates nothing (the caller
    brings the index to fill)."""
    lib = load_library()
    ex = _Exec(_stream_ptr(stream), None, 0, None, lse_in.data_ptr() if lse_in is not None else None,
               pooled_out.data_ptr() if pooled_out is not None else None, _seq_lens_ptr(seq_lens, q.shape[0]))
    tq, tk, ci = _tensor(q, "q"), _tensor(k, "k"), index._c()
    _check(lib.sparsed_select_pattern_static(ctypes.byref(tq), ctypes.byref(tk), block_q, block_k, float(rho), ctypes.byref(ci),
                                             ctypes.byref(ex)))
    return index


def select_pattern_isolated(q, k, block_q: int, block_k: int, rho: float, prefill_blocks: int, lse_in=None, workspace=None,
                            pooled_out=None, index: Optional[BlockIndex] = None, stream=None,
                            seq_lens: Optional[torch.Tensor] = None) -> BlockIndex:
    """sparsed_select_pattern_isolated: separate top-rho% over prefill and generation key blocks."""
    return _select(q, k, block_q, block_k, rho, int(prefill_blocks), lse_in, workspace, pooled_out, index, stream, seq_lens=seq_lens)


def select_pattern_isolated_tokens(q, k, block_q: int, block_k: int, rho: float, prefill_tokens: int, lse_in=None,
                                   workspace=None, pooled_out=None, index: Optional[BlockIndex] = None, stream=None,
                                   seq_lens: Optional[torch.Tensor] = None) -> BlockIndex:
    """sparsed_select_pattern_isolated_tokens: isolated selection with the boundary at a key token."""
    return _select(q, k, block_q, block_k, rho, None, lse_in, workspace, pooled_out, index, stream, prefill_tokens=int(prefill_tokens),
                   seq_lens=seq_lens)


def attn_sparse(q, k, v, index: BlockIndex, out: Optional[torch.Tensor] = None, stream=None,
                seq_lens: Optional[torch.Tensor] = None):
    """sparsed_attn_sparse: block-sparse attention with a stored pattern (Eq. 3, Eq. 4). Returns ``out``."""
    lib = load_library()
    if out is None:
        out = torch.empty_like(q)
    ex = _Exec(_stream_ptr(stream), None, 0, None, None, None, _seq_lens_ptr(seq_lens, q.shape[0]))
    tq, tk, tv, to, ci = _tensor(q, "q"), _tensor(k, "k"), _tensor(v, "v"), _tensor(out, "out"), index._c()
    _check(lib.sparsed_attn_sparse(ctypes.byref(tq), ctypes.byref(tk), ctypes.byref(tv), ctypes.byref(ci), ctypes.byref(to),
                                   ctypes.byref(ex)))
    return out


def probe_mfma_bf16(random_operands: bool, iters: int = 20000) -> float:
    """sparsed_probe_mfma_bf16: sustained TFLOP/s of bf16 matrix instructions alone (diagnostic, synchronises)."""
    out = ctypes.c_double(0.0)
    ws = torch.empty(512 * 1024, dtype=torch.uint8, device="cuda")
    ex = _Exec(_stream_ptr(None), ws.data_ptr(), ws.numel(), None, None, None, None)
    _check(load_library().sparsed_probe_mfma_bf16(1 if random_operands else 0, iters, ctypes.byref(out), ctypes.byref(ex)))
    return out.value


def probe_valu_f32(op: str, iters: int = 20000) -> float:
    """sparsed_probe_valu_f32: sustained 1e9 lane-operations/s of fp32 "fma" or "exp2" alone (diagnostic, synchronises)."""
    out = ctypes.c_double(0.0)
    ws = torch.empty(512 * 1024, dtype=torch.uint8, device="cuda")
    ex = _Exec(_stream_ptr(None), ws.data_ptr(), ws.numel(), None, None, None, None)
    _check(load_library().sparsed_probe_valu_f32({"fma": 0, "exp2": 1}[op], iters, ctypes.byref(out), ctypes.byref(ex)))
    return out.value


def probe_mix_bf16(vector_per_mfma: int, lds_operands: bool, iters: int = 20000) -> float:
    """sparsed_probe_mix_bf16: TFLOP/s of matrix instructions issued together with vector instructions (a quarter of them
    exp2) and, optionally, LDS operand reads: the ceiling for an attention-like inner loop (diagnostic, synchronises)."""
    out = ctypes.c_double(0.0)
    ws = torch.empty(512 * 1024, dtype=torch.uint8, device="cuda")
    ex = _Exec(_stream_ptr(None), ws.data_ptr(), ws.numel(), None, None, None, None)
    _check(load_library().sparsed_probe_mix_bf16(int(vector_per_mfma), 1 if lds_operands else 0, iters, ctypes.byref(out), ctypes.byref(ex)))
    return out.value


def index_window_entries(seq_len: int, block_q: int, block_k: int, window_tokens: int, sink_tokens: int) -> int:
    return int(load_library().sparsed_index_window_entries(seq_len, block_q, block_k, window_tokens, sink_tokens))


def index_fill_window(B: int, H: int, seq_len: int, block_q: int, block_k: int, window_tokens: int, sink_tokens: int,
                      device, stream=None) -> BlockIndex:
    """sparsed_index_fill_window: sliding-window (+ sink) pattern as a block index for attn_sparse."""
    lib = load_library()
    cap = index_window_entries(seq_len, block_q, block_k, window_tokens, sink_tokens)
    if cap < 0:
        raise SparsedError(5, "bad window pattern arguments")
    index = BlockIndex(torch.empty(B, H, -(-seq_len // block_q) + 1, dtype=torch.int32, device=device),
                       torch.empty(B, H, max(cap, 1), dtype=torch.int32, device=device), block_q, block_k, -(-seq_len // block_k))
    ex = _Exec(_stream_ptr(stream), None, 0, None, None, None)
    ci = index._c()
    _check(lib.sparsed_index_fill_window(ctypes.byref(ci), seq_len, window_tokens, sink_tokens, ctypes.byref(ex)))
    return index


def index_validate(index: BlockIndex, stream=None) -> None:
    """sparsed_index_validate: raises SparsedError if any row is malformed (synchronises)."""
    lib = load_library()
    flag = torch.empty(256, dtype=torch.uint8, device=index.row_ptr.device)   # the call synchronises before it returns
    ex = _Exec(_stream_ptr(stream), flag.data_ptr(), flag.numel(), None, None, None, None)
    ci = index._c()
    _check(lib.sparsed_index_validate(ctypes.byref(ci), ctypes.byref(ex)))
