"""Pins for the oracle's block mask and token orders (no GPU).

What fixes the mask other than the oracle itself: the kept counts and densities that follow
from the stated sparsities (tests/golden/mask_density.txt), the structure a sliding window must
have (Sec. 3: locality; App. A.1.1: the temporal order makes frames of one location
consecutive), and a token-level expansion compared with a check written in grid coordinates.
"""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "mask_density.txt")


def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            p = line.split()
            rows.append((p[0], int(p[1]), int(p[2]), int(p[3]), int(p[4]), float(p[5]), int(p[6]),
                         int(p[7]), int(p[8]), float(p[9])))
    return rows


@pytest.mark.parametrize("row", _golden_rows(), ids=lambda r: r[0])
def test_kept_count_and_density_match_stated_sparsity(oracle, row):
    name, T, Hh, W, H, rho, nb, kept, nnz, dens = row
    N = T * Hh * W
    assert (N + 63) // 64 == nb
    k = oracle.kept_from_sparsity(nb, rho)
    assert k == kept
    assert abs(100.0 * k / nb - dens) < 0.006
    if nnz <= 400000:  # build the CSR itself for the smaller ones
        row_ptr, col_idx = oracle.block_mask(T, Hh, W, 64, [k] * H)
        assert col_idx.shape[0] == nnz == H * nb * k
        assert row_ptr[-1] == nnz and row_ptr.shape[0] == H * nb + 1


def test_kept_from_sparsity_limits(oracle):
    assert oracle.kept_from_sparsity(512, 1.0) == 1      # never an empty row
    assert oracle.kept_from_sparsity(512, 0.0) == 512
    assert oracle.kept_from_sparsity(512, -0.5) == 512
    assert oracle.kept_from_sparsity(1, 0.9) == 1
    ks = [oracle.kept_from_sparsity(195, r) for r in np.linspace(0, 1, 41)]
    assert all(a >= b for a, b in zip(ks, ks[1:]))       # monotone in sparsity


@pytest.mark.parametrize("grid,kept", [((4, 16, 16), [4, 4]), ((3, 5, 7), [1, 2]), ((5, 9, 11), [3, 8]),
                                        ((2, 8, 8), [2, 2]), ((7, 6, 10), [7, 6])])
def test_window_structure(oracle, grid, kept):
    T, Hh, W = grid
    block = 64 if T * Hh * W >= 512 else 16
    nb = (T * Hh * W + block - 1) // block
    kept = [min(k, nb) for k in kept]
    row_ptr, col_idx = oracle.block_mask(T, Hh, W, block, kept)
    starts = []
    for h, k in enumerate(kept):
        for i in range(nb):
            cols = col_idx[row_ptr[h * nb + i]:row_ptr[h * nb + i + 1]]
            assert len(cols) == k                              # constant count per query block
            assert np.all(np.diff(cols) == 1)                  # one contiguous window
            assert cols[0] >= 0 and cols[-1] < nb
            assert cols[0] <= i <= cols[-1]                    # a block always sees itself
            interior = (i - k // 2 >= 0) and (i - k // 2 + k <= nb)
            if interior:                                       # centred, extra block on the left
                assert cols[0] == i - k // 2
                assert (i - cols[0]) - (cols[-1] - i) in (0, 1)
            starts.append(cols[0])
        s = np.array(starts[-nb:])
        assert np.all((np.diff(s) == 0) | (np.diff(s) == 1))   # the window slides, never jumps
        assert s[0] == 0 and s[-1] == nb - k


@pytest.mark.parametrize("grid,kept", [((4, 16, 16), [4, 5]), ((3, 5, 7), [1, 2]), ((5, 9, 11), [3, 8]),
                                        ((2, 8, 8), [2, 2]), ((7, 6, 10), [7, 6])])
def test_truncated_window(oracle, grid, kept):
    """The window cut at the sequence ends instead of shifted inward: written here as a set intersection; interior
    rows are those of the constant-count window; the end rows lose exactly the blocks that do not exist; the number
    of kept pairs has a closed form; and the mask is symmetric for odd window sizes (block j in the window of i exactly
    when i is in the window of j)."""
    T, Hh, W = grid
    block = 64 if T * Hh * W >= 512 else 16
    nb = (T * Hh * W + block - 1) // block
    kept = [min(k, nb) for k in kept]
    row_ptr, col_idx = oracle.block_mask(T, Hh, W, block, kept, truncated=True)
    rp_c, ci_c = oracle.block_mask(T, Hh, W, block, kept)
    assert row_ptr[0] == 0 and row_ptr[-1] == len(col_idx)
    nnz = 0
    for h, k in enumerate(kept):
        member = np.zeros((nb, nb), dtype=bool)
        for i in range(nb):
            cols = list(col_idx[row_ptr[h * nb + i]:row_ptr[h * nb + i + 1]])
            want = sorted(set(range(i - k // 2, i - k // 2 + k)) & set(range(nb)))
            assert cols == want
            assert i in cols                                   # a block always sees itself
            member[i, cols] = True
            if i - k // 2 >= 0 and i - k // 2 + k <= nb:       # interior: the two readings agree
                assert cols == list(ci_c[rp_c[h * nb + i]:rp_c[h * nb + i + 1]])
            else:
                assert len(cols) < k
            nnz += len(cols)
        left, right = k // 2, k - 1 - k // 2                   # blocks on either side of the query block
        lost = sum(range(1, left + 1)) + sum(range(1, right + 1))    # 1 + 2 + ... missing at each end
        assert member.sum() == nb * k - lost                         # closed form: 1 + 2 + ... blocks missing at each end
        if k % 2 == 1:
            assert np.array_equal(member, member.T)
    assert nnz == len(col_idx)


def test_truncated_full_window_and_bad_arguments(oracle):
    # kept = nb does not make the truncated window dense (its left part sticks out at the start); kept = 1 is the diagonal
    nb = 12
    row_ptr, col_idx = oracle.block_mask(3, 8, 8, 16, [nb], truncated=True)
    assert list(col_idx[row_ptr[0]:row_ptr[1]]) == list(range(0, nb - nb // 2))
    assert list(col_idx[row_ptr[nb - 1]:row_ptr[nb]]) == list(range(nb - 1 - nb // 2, nb))
    row_ptr, col_idx = oracle.block_mask(3, 8, 8, 16, [1], truncated=True)
    assert list(col_idx) == list(range(nb)) and list(row_ptr) == list(range(nb + 1))
    with pytest.raises(ValueError):
        oracle.block_mask(2, 4, 4, 16, [0], truncated=True)
    with pytest.raises(ValueError):
        oracle.block_mask(2, 4, 4, 16, [3], truncated=True)   # nb = 2


def test_full_window_is_dense(oracle):
    row_ptr, col_idx = oracle.block_mask(3, 8, 8, 16, [12, 12])
    nb = 12
    for r in range(2 * nb):
        assert list(col_idx[row_ptr[r]:row_ptr[r + 1]]) == list(range(nb))


def test_invalid_kept_rejected(oracle):
    with pytest.raises(ValueError):
        oracle.block_mask(2, 4, 4, 16, [0])
    with pytest.raises(ValueError):
        oracle.block_mask(2, 4, 4, 16, [3])   # nb = 2


@pytest.mark.parametrize("grid", [(4, 16, 16), (3, 5, 7), (1, 6, 6), (9, 1, 1), (21, 3, 4)])
def test_token_orders(oracle, grid):
    T, Hh, W = grid
    N, HW = T * Hh * W, Hh * W
    spatial = np.array([oracle.row_of_position(0, p, T, Hh, W) for p in range(N)])
    temporal = np.array([oracle.row_of_position(1, p, T, Hh, W) for p in range(N)])
    assert np.array_equal(spatial, np.arange(N))                     # default order is the stored one
    assert np.array_equal(np.sort(temporal), np.arange(N))           # a permutation
    if T == 1 or HW == 1:
        assert np.array_equal(temporal, np.arange(N))                # nothing to regroup
    # stored index n = t*HW + loc (time slowest).  In the temporal order the T frames of one
    # location are consecutive (neighbouring positions are HW apart in storage) and the
    # locations follow one another in raster order.
    t_of, loc_of = temporal // HW, temporal % HW
    for p in range(N - 1):
        if (p + 1) % T != 0:
            assert temporal[p + 1] - temporal[p] == HW and loc_of[p + 1] == loc_of[p]
        else:
            assert loc_of[p + 1] == loc_of[p] + 1 and t_of[p + 1] == 0 and t_of[p] == T - 1


def test_token_level_mask_against_grid_coordinates(oracle):
    """Expand the CSR to a token-level boolean in stored order and compare with a direct rule on
    (t, y, x): two tokens interact iff the block of the key (in the head's order) lies in the
    query block's window, computed here from coordinates without the oracle's order helper."""
    T, Hh, W, block = 3, 4, 6, 8
    N, HW = T * Hh * W, Hh * W
    nb = (N + block - 1) // block
    kept = [3, 4]
    row_ptr, col_idx = oracle.block_mask(T, Hh, W, block, kept)
    for h, kind in enumerate([0, 1]):
        M = np.zeros((N, N), dtype=bool)
        for i in range(nb):
            qpos = [p for p in range(i * block, (i + 1) * block) if p < N]
            qrows = [oracle.row_of_position(kind, p, T, Hh, W) for p in qpos]
            for j in col_idx[row_ptr[h * nb + i]:row_ptr[h * nb + i + 1]]:
                kpos = [p for p in range(j * block, (j + 1) * block) if p < N]
                krows = [oracle.row_of_position(kind, p, T, Hh, W) for p in kpos]
                M[np.ix_(qrows, krows)] = True
        k = kept[h]
        D = np.zeros((N, N), dtype=bool)
        for tq in range(T):
            for yq in range(Hh):
                for xq in range(W):
                    nq = (tq * Hh + yq) * W + xq
                    pq = nq if kind == 0 else (yq * W + xq) * T + tq
                    bi = pq // block
                    lo = min(max(bi - k // 2, 0), nb - k)
                    for tk in range(T):
                        for yk in range(Hh):
                            for xk in range(W):
                                nk = (tk * Hh + yk) * W + xk
                                pk = nk if kind == 0 else (yk * W + xk) * T + tk
                                D[nq, nk] = lo <= pk // block < lo + k
        assert np.array_equal(M, D)
        assert M.sum(axis=1).min() > 0
    # temporal head: a query reaches all frames of its own location (T=3 < block)
