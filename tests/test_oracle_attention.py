"""Pins for the oracle's sparse branch, linear branch, gate and combination (no GPU).

Each pin compares the oracle with something that is not the oracle: a library routine
(torch's scaled_dot_product_attention in float64, scipy's expit), a different formulation of the
same quantity (the quadratic form of linear attention), or a closed form that the definitions
force (uniform weights for Q = 0, constant V, zero static scale).
"""
import numpy as np
import pytest
import torch
from scipy.special import expit

from paper_2601_16515_amd import workloads as wl


def _qkv(seed, B, H, N, d, scale=1.0):
    q = wl.normal(seed, "q", (B, H, N, d)) * scale
    k = wl.normal(seed, "k", (B, H, N, d)) * scale
    v = wl.normal(seed, "v", (B, H, N, d))
    return q, k, v


def _scatter(compact, rows, N):
    """compact [B,H,R,d] + rows [B,H,R] -> stored layout [B,H,N,d]."""
    B, H, R, d = compact.shape
    out = np.full((B, H, N, d), np.nan)
    for b in range(B):
        for h in range(H):
            ok = rows[b, h] >= 0
            out[b, h, rows[b, h][ok]] = compact[b, h][ok]
    assert not np.isnan(out).any()
    return out


def _token_mask(oracle, grid, block, kind, row_ptr, col_idx, h, nb):
    T, Hh, W = grid
    N = T * Hh * W
    M = np.zeros((N, N), dtype=bool)
    order = np.array([oracle.row_of_position(kind, p, T, Hh, W) for p in range(N)])
    for i in range(nb):
        qrows = order[i * block:min((i + 1) * block, N)]
        for j in col_idx[row_ptr[h * nb + i]:row_ptr[h * nb + i + 1]]:
            M[np.ix_(qrows, order[j * block:min((j + 1) * block, N)])] = True
    return M


# ---------------------------------------------------------------- sparse branch, Eq. (1)/(2)

@pytest.mark.parametrize("grid,block,d", [((3, 5, 7), 16, 32), ((2, 8, 9), 64, 64)])
def test_dense_window_equals_library_softmax_attention(oracle, grid, block, d):
    """kept = nb (zero sparsity): Eq. (2) reduces to Eq. (1); compare with torch SDPA in float64.
    Both head orders must give the same result (dense attention is permutation-equivariant)."""
    T, Hh, W = grid
    N = T * Hh * W
    nb = (N + block - 1) // block
    q, k, v = _qkv(11, 1, 2, N, d)
    row_ptr, col_idx = oracle.block_mask(T, Hh, W, block, [nb, nb])
    out, rows = oracle.sparse_attn(q, k, v, grid, block, [0, 1], row_ptr, col_idx)
    got = _scatter(out, rows, N)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).double(), torch.from_numpy(k).double(), torch.from_numpy(v).double()).numpy()
    assert np.abs(got - ref).max() < 1e-12


@pytest.mark.parametrize("truncated", [False, True], ids=["shifted", "truncated"])
@pytest.mark.parametrize("grid,block,kept", [((3, 5, 7), 16, [2, 3]), ((4, 6, 5), 16, [1, 4]),
                                              ((2, 9, 9), 64, [2, 1])])
def test_sparse_equals_library_attention_with_token_mask(oracle, grid, block, kept, truncated):
    """Eq. (2): masked softmax.  The token-level boolean mask is expanded from the CSR and handed
    to torch SDPA (float64); ragged last block, both head orders and both window shapes at the sequence ends."""
    T, Hh, W = grid
    N = T * Hh * W
    nb = (N + block - 1) // block
    d = 32
    q, k, v = _qkv(12, 1, 2, N, d, scale=1.5)
    row_ptr, col_idx = oracle.block_mask(T, Hh, W, block, kept, truncated=truncated)
    out, rows = oracle.sparse_attn(q, k, v, grid, block, [0, 1], row_ptr, col_idx)
    got = _scatter(out, rows, N)
    for h, kind in enumerate([0, 1]):
        M = _token_mask(oracle, grid, block, kind, row_ptr, col_idx, h, nb)
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(q[:, h]).double(), torch.from_numpy(k[:, h]).double(),
            torch.from_numpy(v[:, h]).double(), attn_mask=torch.from_numpy(M)[None]).numpy()
        assert np.abs(got[:, h] - ref).max() < 1e-12


def test_zero_queries_give_mean_of_kept_values(oracle):
    """Q = 0 makes every kept weight equal, so O_s[p] is the arithmetic mean of V over exactly the
    kept, existing tokens.  Pins the mask wiring, the tail and the permutation end to end."""
    grid, block = (3, 7, 5), 16
    T, Hh, W = grid
    N = T * Hh * W
    nb = (N + block - 1) // block
    _, _, v = _qkv(13, 1, 2, N, 8)
    q = np.zeros_like(v)
    k = wl.normal(13, "k", v.shape)
    kept = [3, 2]
    row_ptr, col_idx = oracle.block_mask(T, Hh, W, block, kept)
    out, rows = oracle.sparse_attn(q, k, v, grid, block, [0, 1], row_ptr, col_idx)
    got = _scatter(out, rows, N)
    for h, kind in enumerate([0, 1]):
        M = _token_mask(oracle, grid, block, kind, row_ptr, col_idx, h, nb)
        ref = (M.astype(np.float64) @ v[0, h].astype(np.float64)) / M.sum(1, keepdims=True)
        assert np.abs(got[0, h] - ref).max() < 1e-13


def test_constant_values_and_convexity(oracle):
    grid, block = (2, 6, 7), 16
    N = 2 * 6 * 7
    q, k, v = _qkv(14, 1, 2, N, 16, scale=2.0)
    row_ptr, col_idx = oracle.block_mask(*grid, block, [2, 3])
    c = wl.normal(14, "const", (16,))
    vc = np.broadcast_to(c, v.shape).copy()
    out, rows = oracle.sparse_attn(q, k, vc, grid, block, [1, 0], row_ptr, col_idx)
    ok = rows >= 0
    assert np.abs(out[ok] - c).max() < 1e-14                 # softmax weights sum to one
    out, rows = oracle.sparse_attn(q, k, v, grid, block, [1, 0], row_ptr, col_idx)
    lo, hi = v.min(axis=2, keepdims=True), v.max(axis=2, keepdims=True)
    assert np.all(out[ok] >= np.broadcast_to(lo, out.shape)[ok] - 1e-12)
    assert np.all(out[ok] <= np.broadcast_to(hi, out.shape)[ok] + 1e-12)


def test_selected_blocks_match_full_evaluation(oracle):
    grid, block = (4, 5, 6), 16
    N = 120
    q, k, v = _qkv(15, 2, 2, N, 16)
    row_ptr, col_idx = oracle.block_mask(*grid, block, [3, 3])
    full, rows_full = oracle.sparse_attn(q, k, v, grid, block, [0, 1], row_ptr, col_idx)
    sel = [0, 3, 7]
    part, rows = oracle.sparse_attn(q, k, v, grid, block, [0, 1], row_ptr, col_idx, sel=sel)
    for s, i in enumerate(sel):
        assert np.array_equal(part[:, :, s * block:(s + 1) * block], full[:, :, i * block:(i + 1) * block])
        assert np.array_equal(rows[:, :, s * block:(s + 1) * block], rows_full[:, :, i * block:(i + 1) * block])
    assert (rows_full[:, :, -8:] == -1).all() and (rows_full[:, :, :-8] >= 0).all()   # 120 = 7*16 + 8


def test_softmax_scale_argument(oracle):
    grid, block = (1, 4, 8), 16
    q, k, v = _qkv(16, 1, 1, 32, 16)
    row_ptr, col_idx = oracle.block_mask(*grid, block, [2])
    a, _ = oracle.sparse_attn(q, k, v, grid, block, [0], row_ptr, col_idx, scale=0.5)
    b, _ = oracle.sparse_attn(2.0 * q, k, v, grid, block, [0], row_ptr, col_idx, scale=0.25)
    assert np.abs(a - b).max() < 1e-13
    dflt, _ = oracle.sparse_attn(q, k, v, grid, block, [0], row_ptr, col_idx)
    c, _ = oracle.sparse_attn(q, k, v, grid, block, [0], row_ptr, col_idx, scale=0.25)   # 1/sqrt(16)
    assert np.array_equal(dflt, c)


# ---------------------------------------------------------------- linear branch, Eq. (3)

def test_linear_state_form_equals_quadratic_form(oracle):
    """Associativity (Sec. 3, Linear Attention): phi(Q)(phi(K)^T V) == (phi(Q)phi(K)^T)V."""
    N, d, eps = 150, 24, 1e-6
    q, k, v = _qkv(21, 1, 3, N, d)
    Hs, Z = oracle.linear_state(k, v)
    fast = oracle.linear_apply(q, Hs, Z, eps)
    for h in range(3):
        slow = oracle.linear_attn_quadratic(q[0, h], k[0, h], v[0, h], eps)
        assert np.abs(fast[0, h] - slow).max() < 1e-11
        # and against the formula written with numpy matmuls
        A = np.maximum(q[0, h].astype(np.float64), 0) @ np.maximum(k[0, h].astype(np.float64), 0).T
        ref = (A @ v[0, h].astype(np.float64)) / (A.sum(1, keepdims=True) + eps)
        assert np.abs(slow - ref).max() < 1e-11


def test_linear_state_values(oracle):
    N, d = 70, 8
    _, k, v = _qkv(22, 2, 2, N, d)
    Hs, Z = oracle.linear_state(k, v)
    kp = np.maximum(k.astype(np.float64), 0)
    assert np.abs(Hs - np.einsum("bhna,bhnc->bhac", kp, v.astype(np.float64))).max() < 1e-11
    assert np.abs(Z - kp.sum(2)).max() < 1e-11


def test_linear_invariances(oracle):
    N, d = 90, 16
    q, k, v = _qkv(23, 1, 2, N, d)
    Hs, Z = oracle.linear_state(k, v)
    base = oracle.linear_apply(q, Hs, Z, 0.0)
    # constant V -> that constant (weights are a convex combination when eps = 0)
    c = wl.normal(23, "c", (d,))
    Hc, Zc = oracle.linear_state(k, np.broadcast_to(c, v.shape).copy())
    assert np.abs(oracle.linear_apply(q, Hc, Zc, 0.0) - c).max() < 1e-12
    # jointly shuffling (K, V) rows changes nothing: the branch ignores token order
    perm = np.argsort(wl.uniform(23, "perm", (N,)))
    Hp, Zp = oracle.linear_state(k[:, :, perm], v[:, :, perm])
    assert np.abs(oracle.linear_apply(q, Hp, Zp, 0.0) - base).max() < 1e-12
    # positive rescaling of K cancels between numerator and denominator
    Ha, Za = oracle.linear_state(4.0 * k, v)
    assert np.abs(oracle.linear_apply(q, Ha, Za, 0.0) - base).max() < 1e-12
    # a transposed state (H^T instead of H) must not pass
    assert np.abs(oracle.linear_apply(q, Hs.transpose(0, 1, 3, 2).copy(), Z, 0.0) - base).max() > 1e-3
    # rows argument picks stored rows
    rows = np.array([[[5, -1, 17], [0, 89, 3]]], dtype=np.int64)
    part = oracle.linear_apply(q, Hs, Z, 0.0, rows)
    assert np.array_equal(part[0, 0, 0], base[0, 0, 5]) and np.array_equal(part[0, 1, 1], base[0, 1, 89])
    assert np.all(part[0, 0, 1] == 0)


def test_linear_eps_guards_empty_denominator(oracle):
    N, d = 20, 8
    q, k, v = _qkv(24, 1, 1, N, d)
    q[0, 0, 3] = -np.abs(q[0, 0, 3])           # phi(Q_3) = 0
    Hs, Z = oracle.linear_state(k, v)
    out = oracle.linear_apply(q, Hs, Z, 1e-6)
    assert np.all(out[0, 0, 3] == 0.0) and np.isfinite(out).all()


# ---------------------------------------------------------------- gate, Alg. 1 Level 2

def test_gate_closed_forms(oracle):
    B, N, D = 2, 37, 24
    x = wl.normal(31, "x", (B, N, D))
    w = wl.normal(31, "w", (D,), std=0.5)
    assert np.array_equal(oracle.gate(x, np.zeros(D, np.float32)), np.full(B, 0.5))
    s = oracle.gate(x, w)
    assert np.all((s > 0) & (s < 1))
    ref = expit(x.astype(np.float64) @ w.astype(np.float64)).mean(axis=1)      # library sigmoid
    assert np.abs(s - ref).max() < 1e-14
    # identical tokens: the mean of equal sigmoids is that sigmoid
    xc = np.broadcast_to(x[:, :1], x.shape).copy()
    assert np.abs(oracle.gate(xc, w, 0.3) - expit(xc[:, 0].astype(np.float64) @ w.astype(np.float64) + 0.3)).max() < 1e-14
    assert np.all(oracle.gate(x, w, 40.0) > 1 - 1e-9) and np.all(oracle.gate(x, w, -40.0) < 1e-9)
    assert np.all(oracle.gate(x, w, 0.5) > oracle.gate(x, w, 0.0))
    # sigmoid-then-mean, not mean-then-sigmoid
    z = x.astype(np.float64) @ w.astype(np.float64)
    assert np.abs(s - expit(z.mean(axis=1))).max() > 1e-4


# ---------------------------------------------------------------- combination, Alg. 1 / Eq. (lambda)

def test_combination_closed_forms(oracle):
    w = wl.small("c", 2, 2, 16, 2, 6, 7, "f32", 0.5, seed=41, block=16)
    inp = wl.make_inputs(w)
    grid = (w.T, w.Hh, w.W)
    kw = dict(grid=grid, block=w.block, head_kind=[0, 1], kept=[3, 3], eps=0.0)
    r = oracle.salad_forward(inp["q"], inp["k"], inp["v"], inp["x_t"], inp["w_gate"], inp["head_scale"], lam=0.7, **kw)
    ok = r["rows"] >= 0
    # zero-initialised static scale: the layer is the sparse branch, bit for bit
    z = oracle.salad_forward(inp["q"], inp["k"], inp["v"], inp["x_t"], inp["w_gate"], np.zeros(2, np.float32), lam=0.7, **kw)
    assert np.array_equal(z["out"], z["o_sparse"])
    z = oracle.salad_forward(inp["q"], inp["k"], inp["v"], inp["x_t"], inp["w_gate"], inp["head_scale"], lam=0.0, **kw)
    assert np.array_equal(z["out"], z["o_sparse"])
    # linear in lambda
    r2 = oracle.salad_forward(inp["q"], inp["k"], inp["v"], inp["x_t"], inp["w_gate"], inp["head_scale"], lam=1.4, **kw)
    assert np.abs((r2["out"] - r["o_sparse"]) - 2.0 * (r["out"] - r["o_sparse"])).max() < 1e-13
    # constant V = c: both branches return c, so out = (1 + lambda a_h s_b) c
    c = wl.normal(41, "c", (w.d,))
    vc = np.broadcast_to(c, inp["v"].shape).copy()
    rc = oracle.salad_forward(inp["q"], inp["k"], vc, inp["x_t"], inp["w_gate"], inp["head_scale"], lam=0.7, **kw)
    for b in range(w.B):
        for h in range(w.H):
            coef = 1.0 + 0.7 * float(inp["head_scale"][h]) * rc["s"][b]
            m = ok[b, h]
            assert np.abs(rc["out"][b, h][m] - coef * c).max() < 1e-12
    assert abs(rc["s"][0] - rc["s"][1]) > 1e-6          # the dynamic scale differs per sample
    # the dynamic scale is the gate of x_t, one scalar per sample
    assert np.abs(r["s"] - oracle.gate(inp["x_t"], inp["w_gate"])).max() == 0.0


# ---------------------------------------------------------------- full Level-1 projection, Alg. 1 "Proj"

def test_full_projection(oracle):
    w = wl.small("proj", 2, 3, 16, 2, 6, 7, "f32", 0.5, seed=44, block=16)     # D = 48
    inp = wl.make_inputs(w)
    D = w.H * w.d
    kw = dict(grid=(w.T, w.Hh, w.W), block=w.block, head_kind=[0, 1, 0], kept=[3, 3, 2], eps=1e-6)
    args = (inp["q"], inp["k"], inp["v"], inp["x_t"], inp["w_gate"])
    a = inp["head_scale"].astype(np.float64)
    per_head = oracle.salad_forward(*args, inp["head_scale"], lam=0.8, **kw)
    ok = per_head["rows"] >= 0
    # the per-head form is the block-diagonal special case
    wp = np.kron(np.diag(a), np.eye(w.d))
    full = oracle.salad_forward(*args, None, lam=0.8, w_proj=wp, **kw)
    assert np.abs(full["out"] - per_head["out"])[ok].max() < 1e-12
    # zero-initialised projection (Sec. 4.2): the layer is the sparse branch, bit for bit
    z = oracle.salad_forward(*args, None, lam=0.8, w_proj=np.zeros((D, D)), **kw)
    assert np.array_equal(z["out"], z["o_sparse"])
    # linear in W_p
    w1 = wl.normal(44, "w1", (D, D)).astype(np.float64) * 0.1
    w2 = wl.normal(44, "w2", (D, D)).astype(np.float64) * 0.1
    o1 = oracle.salad_forward(*args, None, lam=0.8, w_proj=w1, **kw)["out"]
    o2 = oracle.salad_forward(*args, None, lam=0.8, w_proj=w2, **kw)["out"]
    o12 = oracle.salad_forward(*args, None, lam=0.8, w_proj=w1 + 2.0 * w2, **kw)["out"]
    os_ = per_head["o_sparse"]
    assert np.abs((o12 - os_) - ((o1 - os_) + 2.0 * (o2 - os_)))[ok].max() < 1e-12
    # one non-zero entry W_p[(h1, a), (h2, c)] moves exactly column c of head h2, by lambda s_b O_l[h1, n, a];
    # for a spatial head h2 and a spatial head h1 the compact rows of both are the same stored rows
    h1, aa, h2, cc = 2, 5, 0, 9
    e = np.zeros((D, D)); e[h1 * w.d + aa, h2 * w.d + cc] = 1.0
    oe = oracle.salad_forward(*args, None, lam=0.8, w_proj=e, **kw)
    delta = oe["out"] - oe["o_sparse"]
    assert np.array_equal(oe["rows"][:, h1], oe["rows"][:, h2])
    expect = 0.8 * oe["s"][:, None] * oe["o_linear"][:, h1, :, aa]
    assert np.abs(delta[:, h2, :, cc] - expect)[ok[:, h2]].max() < 1e-12
    delta[:, h2, :, cc] = 0.0
    assert np.abs(delta).max() == 0.0
    # a transposed projection is a different layer (index convention: row = input channel)
    ot = oracle.salad_forward(*args, None, lam=0.8, w_proj=w1.T, **kw)["out"]
    assert np.abs(ot - o1)[ok].max() > 1e-3
    # a temporal output head takes the other heads' linear outputs at its own stored rows
    assert not np.array_equal(oe["rows"][:, 1], oe["rows"][:, 0])
    et = np.zeros((D, D)); et[0 * w.d + 3, 1 * w.d + 4] = 1.0
    ot = oracle.salad_forward(*args, None, lam=0.8, w_proj=et, **kw)
    ol0_full = oracle.linear_apply(inp["q"], ot["Hs"], ot["Z"], 1e-6, ot["rows"][:, 1:2].repeat(w.H, axis=1))[:, 0]
    d1 = (ot["out"] - ot["o_sparse"])[:, 1, :, 4]
    assert np.abs(d1 - 0.8 * ot["s"][:, None] * ol0_full[:, :, 3])[ok[:, 1]].max() < 1e-12


# ---------------------------------------------------------------- branch dropping, Sec. 4.3

def test_branch_dropping(oracle):
    """A sample whose dynamic scale lies below the threshold loses its linear branch entirely; the others
    are untouched.  Strict inequality; a threshold of 0 never drops (the scale is a mean of sigmoids > 0)."""
    w = wl.small("drop", 3, 2, 16, 2, 6, 7, "f32", 0.5, seed=43, block=16)
    inp = wl.make_inputs(w)
    # per-sample offsets push the three gates apart
    x = inp["x_t"].copy()
    wg = inp["w_gate"]
    x[0] += 40.0 * wg / np.dot(wg, wg) * 0.05
    x[2] -= 40.0 * wg / np.dot(wg, wg) * 0.05
    kw = dict(grid=(w.T, w.Hh, w.W), block=w.block, head_kind=[0, 1], kept=[3, 3], lam=0.9)
    args = (inp["q"], inp["k"], inp["v"], x, wg, inp["head_scale"])
    base = oracle.salad_forward(*args, **kw)
    s = base["s"]
    assert s[2] < s[1] < s[0] and s[0] - s[2] > 0.05
    assert not base["dropped"].any() and np.array_equal(oracle.salad_forward(*args, drop_threshold=0.0, **kw)["out"], base["out"])
    # threshold between the two smallest scales: only sample 2 is pruned
    tau = 0.5 * (s[1] + s[2])
    r = oracle.salad_forward(*args, drop_threshold=tau, **kw)
    assert r["dropped"].tolist() == [0, 0, 1]
    assert np.array_equal(r["out"][2], r["o_sparse"][2])                    # exactly the sparse branch
    assert np.array_equal(r["out"][:2], base["out"][:2])                    # the others unchanged
    assert np.abs(base["out"][2] - base["o_sparse"][2]).max() > 1e-3        # and the branch did matter
    # above every scale: all pruned; the reported scale itself is not altered
    r = oracle.salad_forward(*args, drop_threshold=1.5, **kw)
    assert r["dropped"].all() and np.array_equal(r["out"], r["o_sparse"]) and np.array_equal(r["s"], s)
    # strict inequality, decided on the float32 value of the scale
    s32 = float(np.float32(s[1]))
    assert oracle.branch_drop(s, s32).tolist() == [0, 0, 1]
    assert oracle.branch_drop(s, float(np.nextafter(np.float32(s32), np.float32(2.0)))).tolist() == [0, 1, 1]
    # monotone in the threshold
    counts = [int(oracle.branch_drop(s, t).sum()) for t in np.linspace(0.0, 1.0, 21)]
    assert counts == sorted(counts) and counts[0] == 0 and counts[-1] == 3


def test_tiny_config_runs_in_seconds(oracle):
    """The smallest benchmark configuration end to end (B=1, H=2, d=64, grid 4x16x16)."""
    import time
    w = wl.TINY
    inp = wl.make_inputs(w)
    k = oracle.kept_from_sparsity(w.nb, w.sparsity)
    t0 = time.time()
    r = oracle.salad_forward(inp["q"], inp["k"], inp["v"], inp["x_t"], inp["w_gate"], inp["head_scale"],
                             grid=(w.T, w.Hh, w.W), block=w.block, head_kind=wl.head_kinds(w), kept=[k] * w.H)
    assert time.time() - t0 < 20
    assert r["out"].shape == (1, 2, 1024, 64) and np.isfinite(r["out"]).all()
    assert 0.45 < r["s"][0] < 0.55          # w_gate ~ N(0, 0.02^2): pre-activations are small
    # the linear branch is smaller than the sparse one on N(0,1) inputs
    assert np.abs(r["o_linear"]).mean() < 0.5 * np.abs(r["o_sparse"]).mean()


# ----------------------------------------------------------------------- Top-K block-sparse mask (App. A.1.2)

def _bits(mask):
    """uint64 [...] -> bool [..., 64]"""
    return ((mask[..., None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)).astype(bool)


def _scores64(q, k, key_block):
    """The plain definition in float64: q . mean of each key block (numpy, not the oracle)."""
    B, H, N, d = q.shape
    nbk = -(-N // key_block)
    means = np.stack([k[:, :, J * key_block:min(N, (J + 1) * key_block)].astype(np.float64).mean(axis=2)
                      for J in range(nbk)], axis=2)                                  # [B,H,nbk,d]
    return np.einsum("bhnd,bhjd->bhnj", q.astype(np.float64), means)


@pytest.mark.parametrize("B,H,N,d,key_block,topk", [(1, 2, 300, 16, 64, 2), (2, 1, 517, 32, 128, 3),
                                                    (1, 1, 1000, 128, 64, 4), (1, 2, 130, 8, 64, 1)])
def test_topk_select_against_float64_definition(oracle, B, H, N, d, key_block, topk):
    """The float32 fixed-order selection equals the top-k of the float64 scores wherever those leave a clear
    margin between the k-th and the (k+1)-th block, always keeps exactly k blocks, and never keeps a block whose
    float64 score is clearly below the k-th (ragged last block: its mean is over its own tokens)."""
    q, k, _ = _qkv(31, B, H, N, d)
    q, k = wl.round_to_bf16(q), wl.round_to_bf16(k)
    sel = _bits(oracle.topk_select(q, k, key_block, topk))
    sc = _scores64(q, k, key_block)
    nbk = sc.shape[-1]
    assert not sel[..., nbk:].any()
    kk = min(topk, nbk)
    assert (sel.sum(-1) == kk).all()
    srt = np.sort(sc, axis=-1)[..., ::-1]
    kth = srt[..., kk - 1]
    tol = 1e-4 * np.abs(sc).max()
    assert (np.where(sel[..., :nbk], sc, np.inf).min(-1) >= kth - tol).all()
    if kk < nbk:
        clear = (kth - srt[..., kk]) > tol
        assert clear.mean() > 0.9                      # the pin bites on almost every query
        want = sc >= kth[..., None]
        assert (sel[..., :nbk] == want)[clear].all()


def test_topk_select_exact_cases(oracle):
    """Integer-valued data, where float32 is exact: block J's keys all equal (J+1) e_J, so the score of block J is
    (J+1) q_J and the selection is the top-k of those integers; equal scores go to the lower block index."""
    d, key_block, nbk = 8, 64, 6
    N = key_block * nbk - 10                           # ragged last block (constant keys: the mean is unchanged)
    k = np.zeros((1, 1, N, d), dtype=np.float32)
    for J in range(nbk):
        k[0, 0, J * key_block:(J + 1) * key_block, J] = J + 1
    rng = np.random.default_rng(5)
    q = rng.integers(-4, 5, size=(1, 1, N, d)).astype(np.float32)
    sc = q[0, 0, :, :nbk] * np.arange(1, nbk + 1)
    for topk in (1, 2, 4):
        sel = _bits(oracle.topk_select(q, k, key_block, topk))[0, 0, :, :nbk]
        order = np.argsort(-sc, axis=-1, kind="stable")[:, :topk]     # stable: ties keep the lower index first
        want = np.zeros_like(sel)
        np.put_along_axis(want, order, True, axis=-1)
        assert (sel == want).all()
    # all keys identical: every score ties, the first k blocks win
    k1 = np.ones((1, 1, N, d), dtype=np.float32)
    sel = _bits(oracle.topk_select(q, k1, key_block, 3))[0, 0]
    assert sel[:, :3].all() and not sel[:, 3:].any()
    # k >= number of blocks keeps everything
    sel = _bits(oracle.topk_select(q, k, key_block, 99))[0, 0]
    assert sel[:, :nbk].all() and not sel[:, nbk:].any()


def test_topk_attention_against_masked_softmax(oracle):
    """Step 3: attention over the tokens of the kept blocks = a library softmax over a token mask built here;
    with every block kept it is dense attention."""
    B, H, N, d, key_block = 1, 2, 333, 16, 64
    q, k, v = _qkv(37, B, H, N, d)
    rng = np.random.default_rng(11)
    nbk = -(-N // key_block)
    mask = np.zeros((B, H, N), dtype=np.uint64)
    pick = rng.random((B, H, N, nbk)) < 0.4
    pick[..., 0] |= ~pick.any(-1)                      # at least one block each
    for J in range(nbk):
        mask |= pick[..., J].astype(np.uint64) << np.uint64(J)
    out = oracle.topk_attn(q, k, v, key_block, mask)
    tok = np.repeat(pick, key_block, axis=-1)[..., :N]                        # [B,H,N(query),N(key)]
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).double(), torch.from_numpy(k).double(), torch.from_numpy(v).double(),
        attn_mask=torch.from_numpy(tok)).numpy()
    assert np.abs(out - ref).max() < 1e-12
    full = np.full((B, H, N), (1 << nbk) - 1, dtype=np.uint64)
    dense = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).double(), torch.from_numpy(k).double(), torch.from_numpy(v).double()).numpy()
    assert np.abs(oracle.topk_attn(q, k, v, key_block, full) - dense).max() < 1e-12
    # rows argument: a subset in another order, negative entries skipped
    rows = np.broadcast_to(np.array([5, -1, 332, 64], dtype=np.int64), (B, H, 4)).copy()
    sub = oracle.topk_attn(q, k, v, key_block, mask, rows=rows)
    assert np.abs(sub[:, :, [0, 2, 3]] - ref[:, :, [5, 332, 64]]).max() < 1e-12 and (sub[:, :, 1] == 0).all()


def test_topk_layer(oracle):
    """The whole layer with the Top-K mask: the sparse branch is topk_attn on the selected mask, the rest of the
    layer is unchanged; keeping every block reproduces the dense layer."""
    w = wl.small("topk", 1, 2, 16, 3, 5, 9, "f32", 0.5, seed=41)              # N = 135
    inp = wl.make_inputs(w)
    kinds = np.zeros(w.H, dtype=np.uint8)
    common = dict(grid=(w.T, w.Hh, w.W), block=w.block, head_kind=kinds, lam=1.5)
    args = (inp["q"], inp["k"], inp["v"], inp["x_t"], inp["w_gate"], inp["head_scale"])
    r = oracle.salad_forward(*args, kept=[1] * w.H, topk=2, key_block=64, **common)
    m = oracle.topk_select(inp["q"], inp["k"], 64, 2)
    assert np.array_equal(r["topk_mask"], m)
    ok = r["rows"][0, 0] >= 0
    assert np.abs(r["o_sparse"][:, :, ok] - oracle.topk_attn(inp["q"], inp["k"], inp["v"], 64, m)).max() < 1e-14
    dense = oracle.salad_forward(*args, kept=[w.nb] * w.H, **common)
    allk = oracle.salad_forward(*args, kept=[1] * w.H, topk=64, key_block=64, **common)
    assert np.abs(dense["out"] - allk["out"]).max() < 1e-12


# ------------------------------------------------------------- rotary embedding inside the linear branch (Sec. 4.1)

def _rope_tables(N, d, seed=3, scale=1.0):
    """Angles theta[n, p] = position-like ramp times per-pair frequencies (any table serves the definition)."""
    rng = np.random.default_rng(seed)
    freq = 10000.0 ** (-np.arange(d // 2) / (d // 2)) * scale
    pos = np.arange(N, dtype=np.float64)[:, None] + rng.integers(0, 3, size=(N, 1))
    th = pos * freq[None, :]
    return np.cos(th).astype(np.float32), np.sin(th).astype(np.float32), th


def test_rope_linear_branch_against_complex_quadratic_form(oracle):
    """Channel pairs as complex numbers: (R_i phi q_i) . (R_j phi k_j) = Re(sum_p conj(a_ip) b_jp) with
    a = phi(q) e^{i theta}.  The reassociated oracle must equal that quadratic form (written here with numpy),
    numerator rotated, normaliser not."""
    B, H, N, d, eps = 1, 2, 70, 8, 1e-3
    q, k, v = _qkv(51, B, H, N, d)
    cs, sn, _ = _rope_tables(N, d)
    rot = cs.astype(np.float64) + 1j * sn.astype(np.float64)                        # [N, d/2] as stored (float32 values)
    fq, fk = np.maximum(q, 0).astype(np.float64), np.maximum(k, 0).astype(np.float64)
    a = (fq[..., 0::2] + 1j * fq[..., 1::2]) * rot
    b = (fk[..., 0::2] + 1j * fk[..., 1::2]) * rot
    A = np.real(np.einsum("bhip,bhjp->bhij", a, np.conj(b)))                        # rotated similarities
    num = np.einsum("bhij,bhjd->bhid", A, v.astype(np.float64))
    den = np.einsum("bhid,bhd->bhi", fq, fk.sum(axis=2)) + eps
    ref = num / den[..., None]
    Hr = oracle.linear_state_rope(k, v, cs, sn)
    _, Z = oracle.linear_state(k, v)
    got = oracle.linear_apply_rope(q, Hr, Z, eps, cs, sn)
    assert np.abs(got - ref).max() < 1e-12 * max(1.0, np.abs(ref).max())
    assert np.abs(A - np.einsum("bhid,bhjd->bhij", fq, fk)).max() > 0.1             # the rotation matters here


def test_rope_special_cases(oracle):
    """Zero angles give the plain linear branch; a common shift of all angles cancels (only differences of
    angles enter the numerator); a quarter turn of one pair is the closed form (a, b) -> (-b, a)."""
    B, H, N, d, eps = 1, 1, 40, 4, 1e-2
    q, k, v = _qkv(53, B, H, N, d)
    Hs, Z = oracle.linear_state(k, v)
    plain = oracle.linear_apply(q, Hs, Z, eps)
    one, zero = np.ones((N, d // 2), np.float32), np.zeros((N, d // 2), np.float32)
    assert np.abs(oracle.linear_apply_rope(q, oracle.linear_state_rope(k, v, one, zero), Z, eps, one, zero) - plain).max() < 1e-13
    assert np.abs(oracle.linear_state_rope(k, v, one, zero) - Hs).max() < 1e-13
    _, _, th = _rope_tables(N, d, scale=30.0)
    outs = []
    for shift in (0.0, 0.7):
        cs, sn = np.cos(th + shift), np.sin(th + shift)                             # float64 tables rounded alike
        cs, sn = cs.astype(np.float32), sn.astype(np.float32)
        outs.append(oracle.linear_apply_rope(q, oracle.linear_state_rope(k, v, cs, sn), Z, eps, cs, sn))
    assert np.abs(outs[0] - outs[1]).max() < 1e-5 * np.abs(outs[0]).max()           # float32 tables: ~1e-7 each
    assert np.abs(outs[0] - plain).max() > 1e-2
    # quarter turn on pair 0 of the keys only (queries unrotated): Hr rows 0, 1 = (-b, a) combinations
    k1 = np.abs(k)
    csq = np.ones((N, 2), np.float32); snq = np.zeros((N, 2), np.float32)
    csq[:, 0], snq[:, 0] = 0.0, 1.0
    Hr = oracle.linear_state_rope(k1, v, csq, snq)
    H0, _ = oracle.linear_state(k1, v)
    assert np.abs(Hr[0, 0, 0] + H0[0, 0, 1]).max() < 1e-12 and np.abs(Hr[0, 0, 1] - H0[0, 0, 0]).max() < 1e-12
    assert np.abs(Hr[0, 0, 2:] - H0[0, 0, 2:]).max() < 1e-12


def test_rope_layer(oracle):
    """The layer with the rotary linear branch: sparse branch, gate and normaliser unchanged, O_l the rotated form."""
    w = wl.small("rope", 1, 2, 16, 3, 5, 9, "f32", 0.5, seed=43)
    inp = wl.make_inputs(w)
    kinds = wl.head_kinds(w)
    cs, sn, _ = _rope_tables(w.N, w.d)
    common = dict(grid=(w.T, w.Hh, w.W), block=w.block, head_kind=kinds, kept=[2] * w.H, lam=1.5)
    args = (inp["q"], inp["k"], inp["v"], inp["x_t"], inp["w_gate"], inp["head_scale"])
    plain = oracle.salad_forward(*args, **common)
    r = oracle.salad_forward(*args, rope=(cs, sn), **common)
    assert np.array_equal(r["o_sparse"], plain["o_sparse"]) and np.array_equal(r["Z"], plain["Z"])
    want = oracle.linear_apply_rope(inp["q"], oracle.linear_state_rope(inp["k"], inp["v"], cs, sn), r["Z"], w.eps, cs, sn, r["rows"])
    assert np.array_equal(r["o_linear"], want)
    coef = 1.5 * inp["head_scale"].astype(np.float64)[None, :, None, None] * r["s"][:, None, None, None]
    assert np.abs(r["out"] - (r["o_sparse"] + coef * r["o_linear"])).max() < 1e-12


def test_full_projection_with_rotary_linear_branch(oracle):
    """Alg. 1 "Proj" across heads applied to the rotary linear branch of Sec. 4.1.  Pins: the block-diagonal projection
    diag(a_h) x I reproduces the per-head rotary layer; zero angles reproduce the plain full projection; one non-zero
    entry of W_p moves exactly one output column by lambda s_b times the named channel of the rotary O_l; a transposed
    W_p fails."""
    w = wl.small("proj-rope", 2, 3, 16, 2, 6, 7, "f32", 0.5, seed=45, block=16)     # D = 48
    inp = wl.make_inputs(w)
    D = w.H * w.d
    cs, sn, _ = _rope_tables(w.N, w.d)
    kw = dict(grid=(w.T, w.Hh, w.W), block=w.block, head_kind=[0, 1, 0], kept=[3, 3, 2], eps=1e-6)
    args = (inp["q"], inp["k"], inp["v"], inp["x_t"], inp["w_gate"])
    a = inp["head_scale"].astype(np.float64)
    per_head = oracle.salad_forward(*args, inp["head_scale"], lam=0.8, rope=(cs, sn), **kw)
    ok = per_head["rows"] >= 0
    wp = np.kron(np.diag(a), np.eye(w.d))
    full = oracle.salad_forward(*args, None, lam=0.8, w_proj=wp, rope=(cs, sn), **kw)
    assert np.abs(full["out"] - per_head["out"])[ok].max() < 1e-12
    plain_rope = oracle.salad_forward(*args, inp["head_scale"], lam=0.8, **kw)
    assert np.abs(per_head["out"] - plain_rope["out"])[ok].max() > 1e-3          # the rotation matters on these inputs
    # identity rotation: the plain full projection
    w1 = wl.normal(45, "w1", (D, D)).astype(np.float64) * 0.1
    one, zero = np.ones((w.N, w.d // 2), np.float32), np.zeros((w.N, w.d // 2), np.float32)
    r0 = oracle.salad_forward(*args, None, lam=0.8, w_proj=w1, rope=(one, zero), **kw)["out"]
    p0 = oracle.salad_forward(*args, None, lam=0.8, w_proj=w1, **kw)["out"]
    assert np.abs(r0 - p0)[ok].max() < 1e-12
    # a single entry W_p[(h1, aa), (h2, cc)] (two spatial heads: same compact rows)
    h1, aa, h2, cc = 2, 5, 0, 9
    e = np.zeros((D, D)); e[h1 * w.d + aa, h2 * w.d + cc] = 1.0
    oe = oracle.salad_forward(*args, None, lam=0.8, w_proj=e, rope=(cs, sn), **kw)
    delta = oe["out"] - oe["o_sparse"]
    assert np.array_equal(oe["rows"][:, h1], oe["rows"][:, h2])
    want = 0.8 * oe["s"][:, None] * per_head["o_linear"][:, h1, :, aa]
    okr = oe["rows"][:, h2] >= 0
    assert np.abs(delta[:, h2, :, cc] - want)[okr].max() < 1e-12
    mask = np.ones_like(delta, dtype=bool); mask[:, h2, :, cc] = False
    assert np.abs(delta[mask]).max() == 0.0
    et = oracle.salad_forward(*args, None, lam=0.8, w_proj=e.T.copy(), rope=(cs, sn), **kw)
    assert np.abs(et["out"] - oe["out"])[ok].max() > 1e-6


def test_topk_over_the_temporal_token_order(oracle):
    """Top-K key blocks of a temporal head are runs of its own order (App. A.1.1: tokens grouped by location).  Pin:
    selecting and attending over keys and values that were permuted into that order by hand, with the stored-order
    routine, gives the same mask and the same output (queries keep their stored rows); T = 1 makes both orders equal;
    a spatial head next to a temporal one is untouched."""
    T, Hh, W, d, kb, topk = 5, 4, 6, 8, 16, 3
    N = T * Hh * W
    B, H = 1, 2
    q, k, v = _qkv(61, B, H, N, d)
    kinds = np.array([0, 1], dtype=np.uint8)
    mask = oracle.topk_select(q, k, kb, topk, kinds, (T, Hh, W))
    out = oracle.topk_attn(q, k, v, kb, mask, head_kind=kinds, grid=(T, Hh, W))
    # position p of the temporal order holds stored row (p mod T) * Hh * W + p div T
    p = np.arange(N)
    perm = (p % T) * (Hh * W) + p // T
    assert sorted(perm.tolist()) == list(range(N))
    kp, vp = k.copy(), v.copy()
    kp[:, 1], vp[:, 1] = k[:, 1][:, perm], v[:, 1][:, perm]
    mask_p = oracle.topk_select(q, kp, kb, topk)
    out_p = oracle.topk_attn(q, kp, vp, kb, mask_p)
    assert np.array_equal(mask, mask_p)
    assert np.abs(out - out_p).max() < 1e-12
    # the spatial head is what the stored-order routine gives on the untouched tensors
    plain = oracle.topk_select(q, k, kb, topk)
    assert np.array_equal(mask[:, 0], plain[:, 0]) and not np.array_equal(mask[:, 1], plain[:, 1])
    # T = 1: the two orders coincide
    q1, k1, v1 = _qkv(62, 1, 2, 40, d)
    assert np.array_equal(oracle.topk_select(q1, k1, 8, 2, kinds, (1, 5, 8)), oracle.topk_select(q1, k1, 8, 2))
    # the layer: temporal Top-K head inside salad_forward
    w = wl.small("topk-temporal", 1, 2, 16, T, Hh, W, "f32", 0.5, seed=63)
    inp = wl.make_inputs(w)
    r = oracle.salad_forward(inp["q"], inp["k"], inp["v"], inp["x_t"], inp["w_gate"], inp["head_scale"], grid=(T, Hh, W),
                             block=w.block, head_kind=kinds, kept=[1, 1], topk=topk, key_block=64)
    want = oracle.topk_select(inp["q"], inp["k"], 64, topk, kinds, (T, Hh, W))
    assert np.array_equal(r["topk_mask"], want)
