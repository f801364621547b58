"""Thin ctypes binding of libsalad (the C ABI declared in include/salad.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.
PyTorch is used for device memory and streams.  There is no CPU fallback: if the shared
library has not been built, loading fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
_CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libsalad.so")
SOURCES = ["salad_api.hip", "mask_gate_finalize.hip", "linear_state.hip", "sparse_attn.hip",
           "sparse_attn_v2.hip", "sparse_attn_v5.hip", "linear_apply.hip", "proj.hip", "topk.hip"]

SALAD_OK, SALAD_EINVAL, SALAD_ENOTSUP, SALAD_ENOSPC, SALAD_EHIP = range(5)
SALAD_F32, SALAD_BF16 = 0, 1
SALAD_HEAD_SPATIAL, SALAD_HEAD_TEMPORAL = 0, 1
SALAD_PHI_RELU = 0
SALAD_FLAG_UNFUSED_EPILOGUE = 1

EXPORTS = ["salad_last_error", "salad_kept_from_sparsity", "salad_block_mask_nnz", "salad_block_mask",
           "salad_block_mask_nnz_mode", "salad_block_mask_mode",
           "salad_tile_lists_bytes", "salad_tile_lists", "salad_proj_pack_bytes", "salad_proj_pack", "salad_fwd_workspace_bytes", "salad_sparse_linear_attn_fwd", "salad_linear_state_fwd",
           "salad_gate_fwd", "salad_gate_fwd_static", "salad_timing_enable", "salad_timing_read", "salad_tune"]


class SaladError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"libsalad status {status}: {text}")
        self.status = status


class FwdParams(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("H", C.c_int32), ("N", C.c_int32), ("d", C.c_int32),
        ("dtype", C.c_int32),
        ("T", C.c_int32), ("Hh", C.c_int32), ("W", C.c_int32), ("block", C.c_int32),
        ("q", C.c_void_p), ("k", C.c_void_p), ("v", C.c_void_p),
        ("out", C.c_void_p),
        ("row_ptr", C.c_void_p), ("col_idx", C.c_void_p),
        ("head_kind_host", C.c_void_p),
        ("softmax_scale", C.c_float),
        ("phi", C.c_int32),
        ("eps", C.c_float),
        ("lam", C.c_float),
        ("head_scale", C.c_void_p),
        ("s_dev", C.c_void_p),
        ("x_t", C.c_void_p),
        ("w_gate", C.c_void_p),
        ("b_gate", C.c_float),
        ("s_out", C.c_void_p),
        ("o_sparse_dbg", C.c_void_p),
        ("o_linear_dbg", C.c_void_p),
        ("workspace", C.c_void_p),
        ("workspace_bytes", C.c_size_t),
        ("flags", C.c_int32),
        ("hip_stream", C.c_void_p),
        ("drop_threshold", C.c_float),
        ("dropped_out", C.c_void_p),
        ("w_proj", C.c_void_p),
        ("topk", C.c_int32),
        ("topk_key_block", C.c_int32),
        ("topk_mask_out", C.c_void_p),
        ("rope_cos", C.c_void_p),
        ("rope_sin", C.c_void_p),
        ("tile_lists", C.c_void_p),
        ("w_proj_packed", C.c_void_p),
    ]


class KernelTimes(C.Structure):
    _fields_ = [("gate_ms", C.c_float), ("state_ms", C.c_float), ("finalize_ms", C.c_float),
                ("attn_ms", C.c_float), ("epilogue_ms", C.c_float), ("calls", C.c_int32), ("proj_ms", C.c_float), ("topk_ms", C.c_float)]


def build_library(verbose: bool = False) -> str:
    """Compile csrc/*.hip for gfx950 into libsalad.so next to this file (hipcc cross-compiles
    without a GPU).  One hipcc process per source file, side by side, then one link."""
    import shutil
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
    tmp = tempfile.mkdtemp(prefix="salad_build_")
    try:
        def compile_one(src):
            obj = os.path.join(tmp, src.replace(".hip", ".o"))
            r = subprocess.run(["hipcc", "-c"] + flags + ["-o", obj, os.path.join(_CSRC, src)],
                               capture_output=True, text=True)
            return src, obj, r
        with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
            results = list(ex.map(compile_one, SOURCES))
        for src, _, r in results:
            if verbose or r.returncode != 0:
                print(src, r.stdout, r.stderr)
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed compiling {src}")
        r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + [o for _, o, _ in results],
                           capture_output=True, text=True)
        if verbose or r.returncode != 0:
            print(r.stdout, r.stderr)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed linking libsalad.so")
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return LIB_PATH


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(or paper_2601_16515_amd.binding.build_library()) first; there is no fallback path")
        L = C.CDLL(LIB_PATH)
        L.salad_last_error.restype = C.c_char_p
        L.salad_kept_from_sparsity.restype = C.c_int32
        L.salad_kept_from_sparsity.argtypes = [C.c_int32, C.c_double]
        L.salad_block_mask_nnz.restype = C.c_int64
        L.salad_block_mask_nnz.argtypes = [C.c_int32] * 5 + [C.c_void_p]
        L.salad_block_mask.restype = C.c_int
        L.salad_block_mask.argtypes = [C.c_int32] * 5 + [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.salad_block_mask_nnz_mode.restype = C.c_int64
        L.salad_block_mask_nnz_mode.argtypes = [C.c_int32] * 5 + [C.c_void_p, C.c_int32]
        L.salad_block_mask_mode.restype = C.c_int
        L.salad_block_mask_mode.argtypes = [C.c_int32] * 5 + [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
        L.salad_tile_lists_bytes.restype = C.c_size_t
        L.salad_tile_lists_bytes.argtypes = [C.c_int32, C.c_int32]
        L.salad_tile_lists.restype = C.c_int
        L.salad_tile_lists.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
        L.salad_proj_pack_bytes.restype = C.c_size_t
        L.salad_proj_pack_bytes.argtypes = [C.c_int32, C.c_int32]
        L.salad_proj_pack.restype = C.c_int
        L.salad_proj_pack.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
        L.salad_fwd_workspace_bytes.restype = C.c_size_t
        L.salad_fwd_workspace_bytes.argtypes = [C.POINTER(FwdParams)]
        L.salad_sparse_linear_attn_fwd.restype = C.c_int
        L.salad_sparse_linear_attn_fwd.argtypes = [C.POINTER(FwdParams)]
        L.salad_linear_state_fwd.restype = C.c_int
        L.salad_linear_state_fwd.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                             C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.salad_gate_fwd.restype = C.c_int
        L.salad_gate_fwd.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                     C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.salad_gate_fwd_static.restype = C.c_int
        L.salad_gate_fwd_static.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                            C.c_void_p, C.c_void_p]
        L.salad_timing_enable.restype = C.c_int
        L.salad_timing_enable.argtypes = [C.c_int32]
        L.salad_timing_read.restype = C.c_int
        L.salad_timing_read.argtypes = [C.POINTER(KernelTimes), C.c_int32]
        L.salad_tune.restype = C.c_int
        L.salad_tune.argtypes = [C.c_char_p, C.c_int32]
        _lib = L
    return _lib


def _check(st: int) -> None:
    if st != SALAD_OK:
        raise SaladError(st, lib().salad_last_error().decode())


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.bfloat16:
        return SALAD_BF16
    if t.dtype == torch.float32:
        return SALAD_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


# ---------------------------------------------------------------------------------------------
# same names as the C entry points
# ---------------------------------------------------------------------------------------------

def salad_kept_from_sparsity(nb: int, sparsity: float) -> int:
    return int(lib().salad_kept_from_sparsity(nb, sparsity))


SALAD_WINDOW_SHIFTED, SALAD_WINDOW_TRUNCATED = 0, 1


def salad_block_mask_nnz(T: int, Hh: int, W: int, block: int, kept: Sequence[int]) -> int:
    arr = (C.c_int32 * len(kept))(*kept)
    return int(lib().salad_block_mask_nnz(T, Hh, W, block, len(kept), arr))


def salad_block_mask_nnz_mode(T: int, Hh: int, W: int, block: int, kept: Sequence[int], window_mode: int) -> int:
    arr = (C.c_int32 * len(kept))(*kept)
    return int(lib().salad_block_mask_nnz_mode(T, Hh, W, block, len(kept), arr, window_mode))


def salad_block_mask(T: int, Hh: int, W: int, block: int, kept: Sequence[int], device="cuda"):
    """Returns (row_ptr, col_idx) int32 device tensors."""
    import torch
    H = len(kept)
    arr = (C.c_int32 * H)(*kept)
    nnz = lib().salad_block_mask_nnz(T, Hh, W, block, H, arr)
    if nnz < 0:
        raise SaladError(SALAD_EINVAL, "salad_block_mask_nnz rejected the arguments")
    nb = (T * Hh * W + block - 1) // block
    row_ptr = torch.empty(H * nb + 1, dtype=torch.int32, device=device)
    col_idx = torch.empty(max(nnz, 1), dtype=torch.int32, device=device)
    _check(lib().salad_block_mask(T, Hh, W, block, H, arr, row_ptr.data_ptr(), col_idx.data_ptr(), nnz, _stream()))
    return row_ptr, col_idx[:nnz]


def salad_block_mask_mode(T: int, Hh: int, W: int, block: int, kept: Sequence[int], window_mode: int, device="cuda"):
    """Returns (row_ptr, col_idx) int32 device tensors for the given window shape at the sequence ends."""
    import torch
    H = len(kept)
    arr = (C.c_int32 * H)(*kept)
    nnz = lib().salad_block_mask_nnz_mode(T, Hh, W, block, H, arr, window_mode)
    if nnz < 0:
        raise SaladError(SALAD_EINVAL, "salad_block_mask_nnz_mode rejected the arguments")
    nb = (T * Hh * W + block - 1) // block
    row_ptr = torch.empty(H * nb + 1, dtype=torch.int32, device=device)
    col_idx = torch.empty(max(nnz, 1), dtype=torch.int32, device=device)
    _check(lib().salad_block_mask_mode(T, Hh, W, block, H, arr, window_mode, row_ptr.data_ptr(), col_idx.data_ptr(), nnz, _stream()))
    return row_ptr, col_idx[:nnz]


def salad_proj_pack(w_proj, H: int, d: int):
    """W_p [H*d, H*d] (bf16 device tensor) rearranged once for the projection GEMM; returns a 256-byte aligned uint8
    device tensor to pass as w_proj_packed."""
    import torch
    need = int(lib().salad_proj_pack_bytes(H, d))
    if need == 0:
        raise SaladError(SALAD_ENOTSUP, "salad_proj_pack_bytes: shape outside the projection's envelope")
    buf = torch.empty(need + 256, dtype=torch.uint8, device=w_proj.device)
    off = (-buf.data_ptr()) % 256
    view = buf[off:off + need]
    _check(lib().salad_proj_pack(w_proj.data_ptr(), H, d, view.data_ptr(), need, _stream()))
    return view


def salad_tile_lists(row_ptr, col_idx, H: int, nb: int):
    """Visit lists of the large-tile kernel for a CSR, built once; returns a 256-byte aligned uint8 device tensor to pass
    as tile_lists (None when the shape does not use them)."""
    import torch
    need = int(lib().salad_tile_lists_bytes(H, nb))
    if need == 0:
        return None
    buf = torch.empty(need + 256, dtype=torch.uint8, device=row_ptr.device)
    off = (-buf.data_ptr()) % 256
    view = buf[off:off + need]
    _check(lib().salad_tile_lists(row_ptr.data_ptr(), col_idx.data_ptr(), H, nb, view.data_ptr(), need, _stream()))
    return view


def salad_fwd_workspace_bytes(B: int, H: int, N: int, d: int, dtype: int, full_proj: bool = False,
                              topk: int = 0, rope: bool = False) -> int:
    p = FwdParams()
    p.B, p.H, p.N, p.d, p.dtype = B, H, N, d, dtype
    p.w_proj = 1 if full_proj else None          # the query only looks at whether the pointer is NULL
    p.topk = int(topk)                           # ... and at topk (slots per query of the regrouped Top-K path)
    p.rope_cos = 1 if rope else None             # ... and at whether the rotary tables are given
    return int(lib().salad_fwd_workspace_bytes(C.byref(p)))


class Workspace:
    """Caller-owned scratch for the layer call, sized by the library's query."""

    def __init__(self, B: int, H: int, N: int, d: int, dtype: int, device="cuda", full_proj: bool = False,
                 topk: int = 0, rope: bool = False):
        import torch
        self.bytes = salad_fwd_workspace_bytes(B, H, N, d, dtype, full_proj, topk, rope)
        self.buf = torch.empty(max(self.bytes, 256) + 256, dtype=torch.uint8, device=device)
        self.ptr = (self.buf.data_ptr() + 255) & ~255


def make_fwd_params(q, k, v, out, grid: Tuple[int, int, int], row_ptr, col_idx, head_kind=None, *,
                    lam: float = 1.0, head_scale=None, s=None, x_t=None, w_gate=None, b_gate: float = 0.0,
                    eps: float = 1e-6, softmax_scale: float = 0.0, s_out=None, o_sparse_dbg=None,
                    o_linear_dbg=None, workspace: Optional[Workspace] = None, flags: int = 0, block: int = 64,
                    drop_threshold: float = 0.0, dropped_out=None, w_proj=None, topk: int = 0,
                    topk_key_block: int = 0, topk_mask_out=None, rope_cos=None, rope_sin=None, tile_lists=None, w_proj_packed=None):
    """Fill a salad_fwd_params from torch tensors.  Returns (params, keepalive)."""
    B, H, N, d = q.shape
    p = FwdParams()
    p.B, p.H, p.N, p.d = B, H, N, d
    p.dtype = _dtype_code(q)
    p.T, p.Hh, p.W = grid
    p.block = block
    p.q, p.k, p.v, p.out = q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr()
    p.row_ptr, p.col_idx = _ptr(row_ptr), _ptr(col_idx)
    hk = None
    if head_kind is not None:
        hk = (C.c_uint8 * H)(*[int(x) for x in head_kind])
        p.head_kind_host = C.cast(hk, C.c_void_p)
    p.softmax_scale = softmax_scale
    p.phi = SALAD_PHI_RELU
    p.eps = eps
    p.lam = lam
    p.head_scale = _ptr(head_scale)
    p.s_dev = _ptr(s)
    p.x_t = _ptr(x_t)
    p.w_gate = _ptr(w_gate)
    p.b_gate = b_gate
    p.s_out = _ptr(s_out)
    p.o_sparse_dbg = _ptr(o_sparse_dbg)
    p.o_linear_dbg = _ptr(o_linear_dbg)
    if workspace is not None:
        p.workspace = workspace.ptr
        p.workspace_bytes = workspace.bytes
    p.flags = flags
    p.hip_stream = _stream()
    p.drop_threshold = drop_threshold
    p.dropped_out = _ptr(dropped_out)
    p.w_proj = _ptr(w_proj)
    p.topk, p.topk_key_block, p.topk_mask_out = int(topk), int(topk_key_block), _ptr(topk_mask_out)
    p.rope_cos, p.rope_sin = _ptr(rope_cos), _ptr(rope_sin)
    p.tile_lists = _ptr(tile_lists)
    p.w_proj_packed = _ptr(w_proj_packed)
    return p, (hk, workspace, tile_lists, w_proj_packed)


def salad_sparse_linear_attn_fwd(q, k, v, grid, row_ptr, col_idx, head_kind=None, *, out=None, **kw):
    """Whole layer.  Allocates `out` (and a workspace unless one is passed) with torch, then makes
    exactly one library call."""
    import torch
    B, H, N, d = q.shape
    for t in (q, k, v):
        assert t.is_cuda and t.is_contiguous() and t.shape == q.shape and t.dtype == q.dtype
    if out is None:
        out = torch.empty_like(q)
    if kw.get("workspace") is None:
        kw["workspace"] = Workspace(B, H, N, d, _dtype_code(q), q.device, full_proj=kw.get("w_proj") is not None or kw.get("w_proj_packed") is not None,
                                    topk=kw.get("topk", 0), rope=kw.get("rope_cos") is not None)
    p, keep = make_fwd_params(q, k, v, out, grid, row_ptr, col_idx, head_kind, **kw)
    _check(lib().salad_sparse_linear_attn_fwd(C.byref(p)))
    return out


def salad_fwd_call(p: FwdParams) -> None:
    """Re-issue a prepared call (benchmark loop: no allocation, no marshalling)."""
    _check(lib().salad_sparse_linear_attn_fwd(C.byref(p)))


def salad_linear_state_fwd(k, v, workspace: Optional[Workspace] = None):
    import torch
    B, H, N, d = k.shape
    assert k.is_cuda and k.is_contiguous() and v.is_contiguous() and v.shape == k.shape
    code = _dtype_code(k)
    ws = workspace or Workspace(B, H, N, d, code, k.device)
    Hs = torch.empty(B, H, d, d, dtype=torch.float32, device=k.device)
    Z = torch.empty(B, H, d, dtype=torch.float32, device=k.device)
    _check(lib().salad_linear_state_fwd(k.data_ptr(), v.data_ptr(), B, H, N, d, code, Hs.data_ptr(), Z.data_ptr(),
                                        ws.ptr, ws.bytes, _stream()))
    return Hs, Z


def salad_gate_fwd(x_t, w_gate, b_gate: float = 0.0):
    import torch
    B, N, D = x_t.shape
    assert x_t.is_cuda and x_t.is_contiguous() and w_gate.dtype == torch.float32 and w_gate.numel() == D
    s = torch.empty(B, dtype=torch.float32, device=x_t.device)
    ws = torch.empty(4 * B * 2048 + 1024, dtype=torch.uint8, device=x_t.device)
    ptr = (ws.data_ptr() + 255) & ~255
    _check(lib().salad_gate_fwd(x_t.data_ptr(), w_gate.data_ptr(), b_gate, B, N, D, _dtype_code(x_t), s.data_ptr(),
                                ptr, ws.numel() - 256, _stream()))
    return s


def salad_gate_fwd_static(x_t, w_gate, s_out, b_gate: float = 0.0) -> None:
    """The gate through the library's static scratch buffer: the caller passes the output, nothing is allocated."""
    import torch
    B, N, D = x_t.shape
    assert x_t.is_cuda and x_t.is_contiguous() and w_gate.dtype == torch.float32 and w_gate.numel() == D
    assert s_out.is_cuda and s_out.dtype == torch.float32 and s_out.numel() == B and s_out.is_contiguous()
    _check(lib().salad_gate_fwd_static(x_t.data_ptr(), w_gate.data_ptr(), b_gate, B, N, D, _dtype_code(x_t),
                                       s_out.data_ptr(), _stream()))


def salad_timing_enable(on) -> None:
    """False/0 off, True/1 events around every stage, 2 around the attention stage only."""
    _check(lib().salad_timing_enable(int(on)))


def salad_timing_read(reset: bool = True) -> KernelTimes:
    kt = KernelTimes()
    _check(lib().salad_timing_read(C.byref(kt), 1 if reset else 0))
    return kt


def salad_tune(key: str, value: int) -> None:
    _check(lib().salad_tune(key.encode(), value))
