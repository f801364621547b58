"""ctypes front end of the CPU oracle (oracle/salad_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg.  It imports nothing from the GPU package and the GPU package imports
nothing from here.  All arithmetic lives in the C file; this module marshals numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "salad_oracle.c")
# SALAD_ORACLE_SANITIZE=1 selects a second build of the same source with the host AddressSanitizer and
# UndefinedBehaviorSanitizer (CPU only; the process must have libasan preloaded, see tests/test_oracle_sanitized.py)
_SANITIZE = os.environ.get("SALAD_ORACLE_SANITIZE", "") == "1"
_LIB = os.path.join(_HERE, "libsalad_oracle_asan.so" if _SANITIZE else "libsalad_oracle.so")
_lib: Optional[C.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C + OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        opt = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"] \
            if _SANITIZE else ["-O2", "-march=native"]
        cmd = ["gcc"] + opt + ["-fopenmp", "-fPIC", "-shared", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.salad_oracle_block_mask.restype = C.c_int64
        _lib.salad_oracle_block_mask_truncated.restype = C.c_int64
        _lib.salad_oracle_row_of_position.restype = C.c_int64
        _lib.salad_oracle_kept_from_sparsity.restype = C.c_int32
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def threads() -> int:
    return int(_load().salad_oracle_threads())


def kept_from_sparsity(nb: int, sparsity: float) -> int:
    return int(_load().salad_oracle_kept_from_sparsity(C.c_int32(nb), C.c_double(sparsity)))


def row_of_position(kind: int, p: int, T: int, Hh: int, W: int) -> int:
    return int(_load().salad_oracle_row_of_position(C.c_int(kind), C.c_int64(p), C.c_int(T),
                                                    C.c_int(Hh), C.c_int(W)))


def block_mask(T: int, Hh: int, W: int, block: int, kept: Sequence[int], truncated: bool = False
               ) -> Tuple[np.ndarray, np.ndarray]:
    """CSR (row_ptr [H*nb+1], col_idx [nnz]) of kept KV blocks per (head, query block).  truncated: the window is
    cut at the sequence ends instead of shifted inward."""
    kept = np.ascontiguousarray(kept, dtype=np.int32)
    H = kept.shape[0]
    N = T * Hh * W
    nb = (N + block - 1) // block
    row_ptr = np.zeros(H * nb + 1, dtype=np.int32)
    col_idx = np.zeros(int(nb * np.clip(kept, 0, nb).astype(np.int64).sum()) + 1, dtype=np.int32)
    fn = _load().salad_oracle_block_mask_truncated if truncated else _load().salad_oracle_block_mask
    nnz = fn(C.c_int(T), C.c_int(Hh), C.c_int(W), C.c_int(block),
             C.c_int(H), _p(kept), _p(row_ptr), _p(col_idx))
    if nnz < 0:
        raise ValueError("invalid mask arguments")
    return row_ptr, col_idx[:nnz].copy()


def sparse_attn(q, k, v, grid: Tuple[int, int, int], block: int, head_kind, row_ptr, col_idx,
                scale: Optional[float] = None, sel: Optional[Sequence[int]] = None
                ) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. (2) on the selected query blocks.  Returns (out [B,H,nsel*block,d] float64,
    rows [B,H,nsel*block] int64 stored row index or -1)."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    B, H, N, d = q.shape
    T, Hh, W = grid
    nb = (N + block - 1) // block
    sel = np.arange(nb, dtype=np.int32) if sel is None else np.ascontiguousarray(sel, dtype=np.int32)
    nsel = sel.shape[0]
    head_kind = np.ascontiguousarray(head_kind, dtype=np.uint8)
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    out = np.zeros((B, H, nsel * block, d), dtype=np.float64)
    rows = np.zeros((B, H, nsel * block), dtype=np.int64)
    sc = (1.0 / np.sqrt(d)) if scale is None else float(scale)
    rc = _load().salad_oracle_sparse_attn(_p(q), _p(k), _p(v), C.c_int(B), C.c_int(H), C.c_int64(N),
                                          C.c_int(d), C.c_int(T), C.c_int(Hh), C.c_int(W),
                                          C.c_int(block), _p(head_kind), _p(row_ptr), _p(col_idx),
                                          C.c_double(sc), _p(sel), C.c_int(nsel), _p(out), _p(rows))
    if rc != 0:
        raise ValueError("salad_oracle_sparse_attn: invalid arguments")
    return out, rows


def linear_state(k, v) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. (3) sums: Hs [B,H,d,d] = sum_j relu(K_j)^T V_j and Z [B,H,d] = sum_j relu(K_j)."""
    k, v = _f32(k), _f32(v)
    B, H, N, d = k.shape
    Hs = np.zeros((B, H, d, d), dtype=np.float64)
    Z = np.zeros((B, H, d), dtype=np.float64)
    _load().salad_oracle_linear_state(_p(k), _p(v), C.c_int(B), C.c_int(H), C.c_int64(N), C.c_int(d),
                                      _p(Hs), _p(Z))
    return Hs, Z


def linear_apply(q, Hs, Z, eps: float, rows: Optional[np.ndarray] = None) -> np.ndarray:
    """Eq. (3) quotient for stored rows `rows` [B,H,nrows] (default: every row, in stored order)."""
    q = _f32(q)
    B, H, N, d = q.shape
    if rows is None:
        rows = np.broadcast_to(np.arange(N, dtype=np.int64), (B, H, N))
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    nrows = rows.shape[-1]
    Hs = np.ascontiguousarray(Hs, dtype=np.float64)
    Z = np.ascontiguousarray(Z, dtype=np.float64)
    out = np.zeros((B, H, nrows, d), dtype=np.float64)
    _load().salad_oracle_linear_apply(_p(q), _p(Hs), _p(Z), C.c_int(B), C.c_int(H), C.c_int64(N),
                                      C.c_int(d), C.c_double(eps), _p(rows), C.c_int64(nrows), _p(out))
    return out


def linear_state_rope(k, v, cos, sin) -> np.ndarray:
    """Rotated linear state Hr [B,H,d,d] = sum_j (R_j relu(K_j))^T V_j; cos, sin: float32 [N, d/2] (pair (2p, 2p+1))."""
    k, v = _f32(k), _f32(v)
    cos, sin = _f32(cos), _f32(sin)
    B, H, N, d = k.shape
    assert cos.shape == (N, d // 2) and sin.shape == (N, d // 2)
    Hr = np.zeros((B, H, d, d), dtype=np.float64)
    rc = _load().salad_oracle_linear_state_rope(_p(k), _p(v), _p(cos), _p(sin), C.c_int(B), C.c_int(H), C.c_int64(N),
                                                C.c_int(d), _p(Hr))
    if rc != 0:
        raise ValueError("salad_oracle_linear_state_rope: invalid arguments")
    return Hr


def linear_apply_rope(q, Hr, Z, eps: float, cos, sin, rows: Optional[np.ndarray] = None) -> np.ndarray:
    """(R_n relu(Q_n)) Hr / (relu(Q_n).Z + eps) for stored rows `rows` [B,H,nrows] (default: every row)."""
    q = _f32(q)
    cos, sin = _f32(cos), _f32(sin)
    B, H, N, d = q.shape
    if rows is None:
        rows = np.broadcast_to(np.arange(N, dtype=np.int64), (B, H, N))
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    nrows = rows.shape[-1]
    Hr = np.ascontiguousarray(Hr, dtype=np.float64)
    Z = np.ascontiguousarray(Z, dtype=np.float64)
    out = np.zeros((B, H, nrows, d), dtype=np.float64)
    rc = _load().salad_oracle_linear_apply_rope(_p(q), _p(Hr), _p(Z), _p(cos), _p(sin), C.c_int(B), C.c_int(H),
                                                C.c_int64(N), C.c_int(d), C.c_double(eps), _p(rows),
                                                C.c_int64(nrows), _p(out))
    if rc != 0:
        raise ValueError("salad_oracle_linear_apply_rope: invalid arguments")
    return out


def linear_attn_quadratic(q, k, v, eps: float) -> np.ndarray:
    """Un-reassociated linear attention of one head, [N,d] inputs; O(N^2 d)."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    N, d = q.shape
    out = np.zeros((N, d), dtype=np.float64)
    _load().salad_oracle_linear_attn_quadratic(_p(q), _p(k), _p(v), C.c_int64(N), C.c_int(d),
                                               C.c_double(eps), _p(out))
    return out


def gate(x_t, w_gate, bias: float = 0.0) -> np.ndarray:
    """Alg. 1 Level 2: s[b] = mean_n sigmoid(x_t[b,n,:] . w + bias)."""
    x_t, w_gate = _f32(x_t), _f32(w_gate)
    B, N, D = x_t.shape
    s = np.zeros(B, dtype=np.float64)
    rc = _load().salad_oracle_gate(_p(x_t), _p(w_gate), C.c_double(bias), C.c_int(B), C.c_int64(N),
                                   C.c_int(D), _p(s))
    if rc != 0:
        raise MemoryError("salad_oracle_gate")
    return s


def combine(o_s, o_l, lam: float, head_scale, s) -> np.ndarray:
    """Alg. 1 residual integration with Proj = lambda * a_h * I: O_s + lambda a_h s_b O_l."""
    o_s = np.ascontiguousarray(o_s, dtype=np.float64)
    o_l = np.ascontiguousarray(o_l, dtype=np.float64)
    B, H, nrows, d = o_s.shape
    hs = None if head_scale is None else _f32(head_scale)
    s = np.ascontiguousarray(s, dtype=np.float64)
    out = np.zeros_like(o_s)
    _load().salad_oracle_combine(_p(o_s), _p(o_l), C.c_int(B), C.c_int(H), C.c_int64(nrows), C.c_int(d),
                                 C.c_double(lam), _p(hs), _p(s), _p(out))
    return out


def combine_proj(q, Hs, Z, eps: float, o_s, rows, w_proj, lam: float, s, rope=None) -> np.ndarray:
    """Alg. 1 residual integration with the full projection: O_s + lambda s_b (O_l W_p), W_p [D,D] over the
    concatenated heads; evaluated on the compact rows of each (b, h) (`rows`: their stored row indices).
    rope = (cos, sin) [N, d/2]: the linear branch carries the rotary embedding of Sec. 4.1 (Hs is then the rotated state)."""
    q = _f32(q)
    B, H, N, d = q.shape
    o_s = np.ascontiguousarray(o_s, dtype=np.float64)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    nrows = rows.shape[-1]
    Hs = np.ascontiguousarray(Hs, dtype=np.float64)
    Z = np.ascontiguousarray(Z, dtype=np.float64)
    wp = np.ascontiguousarray(w_proj, dtype=np.float64)
    assert wp.shape == (H * d, H * d)
    s = np.ascontiguousarray(s, dtype=np.float64)
    out = np.zeros_like(o_s)
    if rope is not None:
        cs, sn = _f32(rope[0]), _f32(rope[1])
        assert cs.shape == (N, d // 2) and sn.shape == (N, d // 2)
        rc = _load().salad_oracle_combine_proj_rope(_p(q), _p(Hs), _p(Z), _p(cs), _p(sn), C.c_int(B), C.c_int(H), C.c_int64(N),
                                                    C.c_int(d), C.c_double(eps), _p(o_s), _p(rows), C.c_int64(nrows), _p(wp),
                                                    C.c_double(lam), _p(s), _p(out))
        if rc != 0:
            raise ValueError("salad_oracle_combine_proj_rope: invalid arguments")
        return out
    _load().salad_oracle_combine_proj(_p(q), _p(Hs), _p(Z), C.c_int(B), C.c_int(H), C.c_int64(N), C.c_int(d),
                                      C.c_double(eps), _p(o_s), _p(rows), C.c_int64(nrows), _p(wp),
                                      C.c_double(lam), _p(s), _p(out))
    return out


def _kind_args(head_kind, grid, H):
    """(head_kind pointer or None, T, Hh, W) for the Top-K entry points: None = every head in the stored order."""
    if head_kind is None:
        return None, None, 1, 1, 1
    hk = np.ascontiguousarray(head_kind, dtype=np.uint8)
    assert hk.shape == (H,) and grid is not None
    return hk, _p(hk), int(grid[0]), int(grid[1]), int(grid[2])


def topk_select(q, k, key_block: int, topk: int, head_kind=None, grid=None) -> np.ndarray:
    """App. A.1.2 steps 1-2: per query token the `topk` key blocks (runs of `key_block` tokens of the head's own order:
    stored order, or grouped by location for a temporal head, App. A.1.1) whose mean key has the largest dot product
    with the query, as a uint64 bit mask [B,H,N] indexed by the query's stored row (bit J = block J kept)."""
    q, k = _f32(q), _f32(k)
    B, H, N, d = q.shape
    mask = np.zeros((B, H, N), dtype=np.uint64)
    keep, hkp, T, Hh, W = _kind_args(head_kind, grid, H)
    rc = _load().salad_oracle_topk_select(_p(q), _p(k), C.c_int(B), C.c_int(H), C.c_int64(N), C.c_int(d),
                                          C.c_int(key_block), C.c_int(topk), hkp, C.c_int(T), C.c_int(Hh), C.c_int(W), _p(mask))
    if rc != 0:
        raise ValueError("salad_oracle_topk_select: invalid arguments (more than 64 key blocks?)")
    return mask


def topk_attn(q, k, v, key_block: int, mask, scale: Optional[float] = None,
              rows: Optional[np.ndarray] = None, head_kind=None, grid=None) -> np.ndarray:
    """App. A.1.2 step 3: Eq. (2) with the token-level mask of `topk_select`, on stored rows `rows` [B,H,nrows]
    (default: every row).  Returns [B,H,nrows,d] float64."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    B, H, N, d = q.shape
    if rows is None:
        rows = np.broadcast_to(np.arange(N, dtype=np.int64), (B, H, N))
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    mask = np.ascontiguousarray(mask, dtype=np.uint64)
    out = np.zeros((B, H, rows.shape[-1], d), dtype=np.float64)
    sc = (1.0 / np.sqrt(d)) if scale is None else float(scale)
    keep, hkp, T, Hh, W = _kind_args(head_kind, grid, H)
    rc = _load().salad_oracle_topk_attn(_p(q), _p(k), _p(v), C.c_int(B), C.c_int(H), C.c_int64(N), C.c_int(d),
                                        C.c_int(key_block), _p(mask), C.c_double(sc), hkp, C.c_int(T), C.c_int(Hh), C.c_int(W),
                                        _p(rows), C.c_int64(rows.shape[-1]), _p(out))
    if rc != 0:
        raise ValueError("salad_oracle_topk_attn: invalid arguments")
    return out


def branch_drop(s, tau: float) -> np.ndarray:
    """Sec. 4.3: which samples' linear branches are pruned (dynamic scale below the threshold)."""
    s = np.ascontiguousarray(s, dtype=np.float64)
    dropped = np.zeros(s.shape[0], dtype=np.int32)
    _load().salad_oracle_branch_drop(_p(s), C.c_int(s.shape[0]), C.c_double(tau), _p(dropped))
    return dropped


def salad_forward(q, k, v, x_t, w_gate, head_scale, grid, block, head_kind, kept, lam=1.0, eps=1e-6,
                  b_gate=0.0, scale=None, sel=None, s_override=None, drop_threshold=0.0,
                  w_proj=None, topk: int = 0, key_block: int = 0, rope=None, truncated: bool = False) -> Dict[str, np.ndarray]:
    """Whole layer (Alg. 1 from SparseAttn to the residual sum) on the selected query blocks.

    Returns compact row sets [B,H,nsel*block,d] for o_sparse, o_linear and out, the stored row
    index of each compact row (`rows`, -1 = beyond N), the full state (Hs, Z) and s [B]."""
    T, Hh, W = grid
    row_ptr, col_idx = block_mask(T, Hh, W, block, kept, truncated=truncated)
    topk_mask = None
    if topk > 0:   # Top-K dynamic mask (App. A.1.2) instead of the sliding window; key blocks in each head's own order
        N = q.shape[2]
        nb = (N + block - 1) // block
        sel_b = np.arange(nb) if sel is None else np.asarray(sel)
        pos = (sel_b[:, None] * block + np.arange(block)[None, :]).reshape(-1)
        rows = np.broadcast_to(np.where(pos < N, pos, -1).astype(np.int64), q.shape[:2] + (pos.size,)).copy()
        topk_mask = topk_select(q, k, key_block, topk, head_kind, grid)
        o_s = topk_attn(q, k, v, key_block, topk_mask, scale, rows, head_kind, grid)
    else:
        o_s, rows = sparse_attn(q, k, v, grid, block, head_kind, row_ptr, col_idx, scale, sel)
    Hs, Z = linear_state(k, v)
    if rope is not None:         # (cos, sin) tables [N, d/2]: rotary embedding inside the linear branch
        Hs = linear_state_rope(k, v, rope[0], rope[1])
        o_l = linear_apply_rope(q, Hs, Z, eps, rope[0], rope[1], rows)
    else:
        o_l = linear_apply(q, Hs, Z, eps, rows)
    s = gate(x_t, w_gate, b_gate) if s_override is None else np.asarray(s_override, dtype=np.float64)
    dropped = branch_drop(s, drop_threshold)
    # a pruned branch contributes exactly nothing: its samples are combined with a zero dynamic scale
    s_eff = np.where(dropped != 0, 0.0, s)
    if w_proj is not None:       # full Level-1 projection across heads instead of the per-head scalars
        out = combine_proj(q, Hs, Z, eps, o_s, rows, w_proj, lam, s_eff, rope=rope)
    else:
        out = combine(o_s, o_l, lam, head_scale, s_eff)
    return {"o_sparse": o_s, "o_linear": o_l, "out": out, "rows": rows, "Hs": Hs, "Z": Z, "s": s,
            "row_ptr": row_ptr, "col_idx": col_idx, "dropped": dropped, "topk_mask": topk_mask}
