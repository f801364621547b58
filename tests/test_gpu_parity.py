"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Integer work (the mask) must match bit for bit; floating point within max-abs 2e-2 and
relative L2 5e-3 (bf16 inputs, fp32 accumulation), per branch and combined."""
import numpy as np
import pytest
import torch

from paper_2601_16515_amd import binding as sb
from paper_2601_16515_amd import workloads as wl
from tests.gpu_util import MAX_ABS, REL_L2, compare_layer, errors, gather_rows, run_layer, say, to_dev, upload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    sb.lib()   # fails loudly if libsalad.so is missing


# --------------------------------------------------------------------------------------------- mask

@pytest.mark.parametrize("grid,kept", [
    ((4, 16, 16), [4, 4]), ((5, 6, 9), [1, 5, 3]), ((8, 30, 52), [49] * 12), ((21, 30, 52), [51] * 12),
    ((21, 30, 52), [512, 1, 26, 256]), ((1, 1, 1), [1]), ((21, 45, 80), [118] * 40),
])
def test_block_mask_bit_exact(oracle, grid, kept):
    say(f"mask grid={grid} kept[0]={kept[0]} H={len(kept)}")
    row_ptr, col_idx = sb.salad_block_mask(*grid, 64, kept)
    torch.cuda.synchronize()
    rp, ci = oracle.block_mask(*grid, 64, kept)
    assert np.array_equal(row_ptr.cpu().numpy(), rp)
    assert np.array_equal(col_idx.cpu().numpy(), ci)


@pytest.mark.parametrize("grid,kept", [
    ((4, 16, 16), [4, 5]), ((5, 6, 9), [1, 5, 3]), ((21, 30, 52), [51] * 12), ((21, 30, 52), [512, 1, 26, 255]),
    ((1, 1, 1), [1]), ((21, 45, 80), [118] * 40),
])
def test_block_mask_truncated_bit_exact(oracle, grid, kept):
    """The window cut at the sequence ends (rows of different lengths, first entries in closed form) against the oracle."""
    say(f"truncated mask grid={grid} kept[0]={kept[0]} H={len(kept)}")
    row_ptr, col_idx = sb.salad_block_mask_mode(*grid, 64, kept, sb.SALAD_WINDOW_TRUNCATED)
    torch.cuda.synchronize()
    rp, ci = oracle.block_mask(*grid, 64, kept, truncated=True)
    assert np.array_equal(row_ptr.cpu().numpy(), rp)
    assert np.array_equal(col_idx.cpu().numpy(), ci)
    assert sb.salad_block_mask_nnz_mode(*grid, 64, kept, sb.SALAD_WINDOW_TRUNCATED) == len(ci)
    same = sb.salad_block_mask_mode(*grid, 64, kept, sb.SALAD_WINDOW_SHIFTED)
    ref = sb.salad_block_mask(*grid, 64, kept)
    assert torch.equal(same[0], ref[0]) and torch.equal(same[1], ref[1])


def test_layer_with_truncated_window(oracle):
    """The layer on the truncated-window mask built on the device (short rows at both ends of every head, both head
    orders, prebuilt visit lists) against the oracle on its own truncated mask."""
    w = SMALL[7]                                      # N = 1170: 19 blocks, 3 heads
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [4, 7, 5]
    row_ptr, col_idx = sb.salad_block_mask_mode(w.T, w.Hh, w.W, 64, kept, sb.SALAD_WINDOW_TRUNCATED)
    csr = (row_ptr.cpu().numpy(), col_idx.cpu().numpy())
    ref = _oracle_layer(oracle, w, inp, kept, kinds, truncated=True)
    assert np.array_equal(csr[0], ref["row_ptr"]) and np.array_equal(csr[1], ref["col_idx"])
    res = run_layer(w, inp, dev, kept, kinds, csr=csr)
    compare_layer(res, ref, label="truncated window")
    fast = run_layer(w, inp, dev, kept, kinds, csr=csr, dbg=False, prebuilt_lists=True)
    assert np.array_equal(fast["out"], res["out"])


# --------------------------------------------------------------------------------------------- gate

@pytest.mark.parametrize("B,N,D,dtype", [(1, 1024, 128, "f32"), (2, 270, 1536, "bf16"), (1, 4099, 5120, "bf16"),
                                         (3, 7, 64, "bf16"), (1, 1, 8, "f32"), (1, 12480, 1536, "bf16"),
                                         (2, 1031, 8192, "bf16"), (1, 300, 6152, "bf16"), (1, 77, 8192, "f32")])
def test_gate_parity(oracle, B, N, D, dtype):
    say(f"gate B={B} N={N} D={D} {dtype}")
    x = wl.normal(50, "x", (B, N, D))
    if dtype == "bf16":
        x = wl.round_to_bf16(x)
    wg = wl.normal(50, "w", (D,), std=0.05)
    for bias in (0.0, 0.7):
        s = sb.salad_gate_fwd(to_dev(x, dtype), torch.from_numpy(wg).cuda(), bias)
        torch.cuda.synchronize()
        ref = oracle.gate(x, wg, bias)
        assert np.abs(s.cpu().numpy().astype(np.float64) - ref).max() < 2e-6


# ------------------------------------------------------------------------------------- linear state

@pytest.mark.parametrize("B,H,N,d,dtype", [(1, 2, 270, 128, "bf16"), (2, 3, 1000, 128, "bf16"), (1, 2, 777, 64, "bf16"),
                                           (1, 1, 64, 128, "bf16"), (1, 1, 5, 64, "bf16"), (1, 2, 300, 64, "f32"),
                                           (1, 12, 12480, 128, "bf16")])
def test_linear_state_parity(oracle, B, H, N, d, dtype):
    say(f"state B={B} H={H} N={N} d={d} {dtype}")
    k = wl.normal(60, "k", (B, H, N, d))
    v = wl.normal(60, "v", (B, H, N, d))
    if dtype == "bf16":
        k, v = wl.round_to_bf16(k), wl.round_to_bf16(v)
    Hs, Z = sb.salad_linear_state_fwd(to_dev(k, dtype), to_dev(v, dtype))
    torch.cuda.synchronize()
    rH, rZ = oracle.linear_state(k, v)
    aH, eH = errors(Hs.cpu().numpy().astype(np.float64), rH)
    aZ, eZ = errors(Z.cpu().numpy().astype(np.float64), rZ)
    say(f"  Hs rel_l2={eH:.3e} Z rel_l2={eZ:.3e}")
    assert eH < 2e-6 and eZ < 2e-6          # exact bf16 products, fp32 accumulation


def test_linear_state_chunking_does_not_change_result(oracle):
    """Different numbers of token chunks (workgroups) only change the fp32 summation order."""
    k = wl.round_to_bf16(wl.normal(61, "k", (1, 2, 2000, 128)))
    v = wl.round_to_bf16(wl.normal(61, "v", (1, 2, 2000, 128)))
    rH, rZ = oracle.linear_state(k, v)
    try:
        for wgs in (2, 7, 64, 4096):
            sb.salad_tune("state_wgs", wgs)
            Hs, Z = sb.salad_linear_state_fwd(to_dev(k, "bf16"), to_dev(v, "bf16"))
            torch.cuda.synchronize()
            assert errors(Hs.cpu().numpy().astype(np.float64), rH)[1] < 2e-6
            assert errors(Z.cpu().numpy().astype(np.float64), rZ)[1] < 2e-6
    finally:
        sb.salad_tune("state_wgs", 256)


# -------------------------------------------------------------------------------------- whole layer

def _oracle_layer(oracle, w, inp, kept, kinds, sel=None, **kw):
    return oracle.salad_forward(inp["q"], inp["k"], inp["v"], inp["x_t"], inp["w_gate"], inp["head_scale"],
                                grid=(w.T, w.Hh, w.W), block=w.block, head_kind=kinds, kept=kept,
                                lam=kw.pop("lam", w.lam), eps=kw.pop("eps", w.eps), sel=sel, **kw)


SMALL = [
    wl.small("tail14-d128", 1, 2, 128, 5, 6, 9, "bf16", 0.5, seed=101),      # N=270: 5 blocks, 14-token tail
    wl.small("odd-blocks-d128", 2, 3, 128, 7, 9, 11, "bf16", 0.6, seed=102),  # N=693: 11 blocks, tail 53, B=2
    wl.small("d64", 1, 4, 64, 6, 10, 10, "bf16", 0.7, seed=103),              # N=600: 10 blocks, tail 24
    wl.small("one-block", 1, 2, 128, 2, 3, 5, "bf16", 0.0, seed=104),         # N=30 < one block
    wl.small("exact-blocks", 1, 2, 128, 4, 8, 16, "bf16", 0.75, seed=105),    # N=512, no tail
    wl.small("T-gt-block", 1, 2, 128, 70, 3, 2, "bf16", 0.5, seed=106),       # T=70 > 64: a location spans blocks
    wl.small("single-token", 1, 1, 128, 1, 1, 1, "bf16", 0.0, seed=109),      # N=1
    wl.small("five-tiles-d128", 1, 3, 128, 9, 10, 13, "bf16", 0.8, seed=110), # N=1170: 19 blocks = 5 tiles of 4, tail 18
    wl.small("d64-ragged", 2, 2, 64, 3, 11, 13, "bf16", 0.5, seed=111),       # N=429, d=64, B=2
    wl.small("d64-one-block", 1, 3, 64, 2, 3, 5, "bf16", 0.0, seed=114),      # N=30 < one block, d=64
    wl.small("d64-single-token", 2, 1, 64, 1, 1, 1, "bf16", 0.0, seed=115),   # N=1, d=64, B=2
    wl.small("d64-T-gt-block", 1, 2, 64, 70, 3, 3, "bf16", 0.5, seed=116),    # d=64, T=70 > 64: temporal rows far apart
]


@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
def test_layer_parity_small_bf16(oracle, w):
    say(f"layer {w.name} N={w.N} nb={w.nb}")
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    k = sb.salad_kept_from_sparsity(w.nb, w.sparsity)
    kept = [max(1, min(w.nb, k + (h % 2))) for h in range(w.H)]      # heads differ in window size
    res = run_layer(w, inp, dev, kept, kinds)
    ref = _oracle_layer(oracle, w, inp, kept, kinds)
    assert np.array_equal(res["row_ptr"], ref["row_ptr"]) and np.array_equal(res["col_idx"], ref["col_idx"])
    assert np.abs(res["s"] - ref["s"]).max() < 2e-6
    compare_layer(res, ref, label=w.name)


def test_layer_parity_tiny_config_fp32(oracle):
    w = wl.TINY
    say(f"layer {w.name} (fp32) N={w.N}")
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [sb.salad_kept_from_sparsity(w.nb, w.sparsity)] * w.H
    assert kept == [4, 4]
    res = run_layer(w, inp, dev, kept, kinds)
    ref = _oracle_layer(oracle, w, inp, kept, kinds)
    assert np.array_equal(res["col_idx"], ref["col_idx"])
    compare_layer(res, ref, tol_abs=1e-4, tol_rel=1e-5, label="tiny-f32")


def test_fp32_path_ragged_d128(oracle):
    w = wl.small("f32-d128", 1, 2, 128, 3, 7, 9, "f32", 0.4, seed=107)       # N=189
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [2, 3]
    res = run_layer(w, inp, dev, kept, kinds)
    compare_layer(res, _oracle_layer(oracle, w, inp, kept, kinds), tol_abs=1e-4, tol_rel=1e-5, label="f32-d128")


@pytest.mark.parametrize("d", [64, 128])
def test_sixty_four_heads(oracle, d):
    """The largest head count the boundary takes (64: the head-order mask is a 64-bit word, the last head temporal),
    every head with its own window size.  The gate runs over D = 4096 (d = 64) and D = 8192 (d = 128, the widest row the
    layer can have: gate weights in LDS)."""
    w = wl.small(f"heads64-d{d}", 1, 64, d, 3, 5, 21, "bf16", 0.5, seed=140 + d)      # N = 315: 5 blocks, tail 59
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    assert kinds[63] == 1
    kept = [1 + (h * 7) % 5 for h in range(w.H)]
    res = run_layer(w, inp, dev, kept, kinds)
    ref = _oracle_layer(oracle, w, inp, kept, kinds)
    assert np.abs(res["s"] - ref["s"]).max() < 2e-6
    assert np.array_equal(res["row_ptr"], ref["row_ptr"]) and np.array_equal(res["col_idx"], ref["col_idx"])
    compare_layer(res, ref, label=w.name)


def test_zero_static_scale_gives_sparse_branch_exactly(oracle):
    """Zero-initialised static scale (Sec. 4.2): the layer output is the sparse branch alone; the
    three ways of switching the linear branch off agree bit for bit."""
    w = SMALL[1]
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [4] * w.H
    r0 = run_layer(w, inp, dev, kept, kinds, lam=0.0, dbg=False)
    r1 = run_layer(w, inp, dev, kept, kinds, head_scale=torch.zeros(w.H, device="cuda"), dbg=False)
    r2 = run_layer(w, inp, dev, kept, kinds, s=torch.zeros(w.B, device="cuda"), dbg=False)
    assert torch.equal(r0["out_t"], r1["out_t"]) and torch.equal(r0["out_t"], r2["out_t"])
    ref = _oracle_layer(oracle, w, inp, kept, kinds, lam=0.0)
    assert np.array_equal(ref["out"], ref["o_sparse"])
    compare_layer(r0, ref, label="lambda=0")


def test_linear_dominant_case(oracle):
    """On N(0,1) inputs the linear term is below the bf16 spacing of O_s, so a large static scale
    makes the combined output sensitive to the linear branch."""
    w = SMALL[0]
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [3, 2]
    res = run_layer(w, inp, dev, kept, kinds, lam=100.0)
    ref = _oracle_layer(oracle, w, inp, kept, kinds, lam=100.0)
    got, ok = gather_rows(res["out"], ref["rows"])
    lin_share = np.abs(ref["out"] - ref["o_sparse"])[ok].mean() / np.abs(ref["out"])[ok].mean()
    assert lin_share > 0.5
    a, r = errors(got[ok], ref["out"][ok])
    say(f"  linear-dominant: share={lin_share:.2f} max_abs={a:.3e} rel_l2={r:.3e}")
    assert r <= REL_L2


@pytest.mark.parametrize("kept_n", [19, 6], ids=["all-blocks", "window-6"])
@pytest.mark.parametrize("profile", ["rising", "falling", "mixed"])
def test_softmax_reference_moves_across_blocks(oracle, profile, kept_n):
    """Key magnitudes that change by large factors from one 64-token block to the next, so that the largest
    logit a query has seen so far jumps by tens of binades between blocks (rising), never again reaches the
    first block's (falling), or both (mixed): the running reference of the online softmax has to move, and
    what was accumulated before has to be rescaled, many times per row."""
    w = SMALL[7]                                   # N = 1170: 19 blocks, 3 heads (one temporal)
    inp = wl.make_inputs(w)
    blk = np.arange(w.N) // 64
    if profile == "rising":
        g = 1.0 + 3.0 * blk
    elif profile == "falling":
        g = 1.0 + 3.0 * (blk.max() - blk)
    else:
        g = np.array([1.0, 30.0, 2.0, 55.0, 8.0])[(blk * 7 + 3) % 5]
    inp["k"] = wl.round_to_bf16(inp["k"] * g[None, None, :, None].astype(np.float32))
    # With such keys the softmax is close to one-hot and the output is a single V row: values up to 4.5, where one
    # bf16 rounding alone is 1.6e-2 and the two roundings of the regrouped Top-K path (partial results are stored in
    # bf16) 3.1e-2.  A quarter of the magnitude keeps the absolute bar meaningful for every path; exact in bf16.
    inp["v"] = inp["v"] * np.float32(0.25)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [kept_n] * w.H
    res = run_layer(w, inp, dev, kept, kinds)
    ref = _oracle_layer(oracle, w, inp, kept, kinds)
    compare_layer(res, ref, label=f"{profile}/{kept_n}: ")
    if profile == "mixed":
        # the other attention kernels keep their own running maximum
        for variant in (1, 2):
            sb.salad_tune("attn_variant", variant)
            try:
                res = run_layer(w, inp, dev, kept, kinds)
            finally:
                sb.salad_tune("attn_variant", 0)
            compare_layer(res, ref, label=f"{profile}/{kept_n}/variant{variant}: ")
        # Top-K modes (stored order, all heads spatial): gathered queries and token mask
        kinds0 = np.zeros(w.H, dtype=np.uint8)
        ref_t = _oracle_layer(oracle, w, inp, [1] * w.H, kinds0, topk=3, key_block=128)
        for tv in (0, 1):
            sb.salad_tune("topk_variant", tv)
            try:
                res_t = run_layer(w, inp, dev, [1] * w.H, kinds0, topk=3, topk_key_block=128)
            finally:
                sb.salad_tune("topk_variant", 0)
            assert np.array_equal(res_t["topk_mask"], ref_t["topk_mask"])
            compare_layer(res_t, ref_t, label=f"{profile}/topk-variant{tv}: ")


def test_precomputed_s_and_bias_and_scale_arguments(oracle):
    w = SMALL[2]
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [3] * w.H
    s = torch.tensor([0.31], device="cuda")
    res = run_layer(w, inp, dev, kept, kinds, s=s, softmax_scale=0.2, eps=1e-3)
    ref = _oracle_layer(oracle, w, inp, kept, kinds, s_override=[0.31], scale=0.2, eps=1e-3)
    assert abs(res["s"][0] - 0.31) < 1e-7
    compare_layer(res, ref, label="s_dev")
    res = run_layer(w, inp, dev, kept, kinds, b_gate=-1.5)
    ref = _oracle_layer(oracle, w, inp, kept, kinds, b_gate=-1.5)
    assert np.abs(res["s"] - ref["s"]).max() < 2e-6 and ref["s"][0] < 0.25
    compare_layer(res, ref, label="b_gate")


def test_zero_queries_average_the_kept_values(oracle):
    """Q = 0: O_s is the plain mean of V over the kept, existing tokens (pins mask wiring, tail and
    token orders on the GPU without the oracle's softmax)."""
    w = SMALL[1]
    inp = wl.make_inputs(w)
    inp["q"] = np.zeros_like(inp["q"])
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [3, 4, 2]
    res = run_layer(w, inp, dev, kept, kinds, lam=0.0)
    rp, ci = oracle.block_mask(w.T, w.Hh, w.W, 64, kept)
    for h in range(w.H):
        order = np.array([oracle.row_of_position(int(kinds[h]), p, w.T, w.Hh, w.W) for p in range(w.N)])
        for i in range(w.nb):
            cols = ci[rp[h * w.nb + i]:rp[h * w.nb + i + 1]]
            krows = np.concatenate([order[j * 64:min((j + 1) * 64, w.N)] for j in cols])
            mean = inp["v"][:, h][:, krows].astype(np.float64).mean(axis=1)          # [B, d]
            qrows = order[i * 64:min((i + 1) * 64, w.N)]
            got = res["o_sparse"][:, h][:, qrows]                                      # [B, rows, d]
            assert np.abs(got - mean[:, None, :]).max() < 3e-3


def test_arbitrary_csr(oracle):
    """Any CSR with ascending unique block ids per row is accepted (e.g. a Top-K selection): rows
    of different lengths, non-contiguous ids, neighbouring query blocks with disjoint lists."""
    w = wl.small("csr", 1, 2, 128, 4, 10, 16, "bf16", 0.5, seed=108)    # N=640, nb=10
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    u = wl.uniform(108, "pick", (w.H * w.nb, w.nb))
    row_ptr, col_idx = [0], []
    for r in range(w.H * w.nb):
        cnt = (1 + (r * 7) % 5) if r != 3 else 0          # one empty row: its sparse output is defined as zero
        cols = sorted(np.argsort(u[r])[:cnt].tolist())
        col_idx += cols
        row_ptr.append(len(col_idx))
    csr = (np.array(row_ptr, np.int32), np.array(col_idx, np.int32))
    res = run_layer(w, inp, dev, None, kinds, csr=csr)
    o_s, rows = oracle.sparse_attn(inp["q"], inp["k"], inp["v"], (w.T, w.Hh, w.W), 64, kinds, *csr)
    got, ok = gather_rows(res["o_sparse"], rows)
    a, r = errors(got[ok], o_s[ok])
    say(f"  arbitrary CSR: o_sparse max_abs={a:.3e} rel_l2={r:.3e}")
    assert r <= REL_L2


def test_unfused_epilogue_matches(oracle):
    w = SMALL[1]
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [4] * w.H
    ref = _oracle_layer(oracle, w, inp, kept, kinds, lam=30.0)
    res = run_layer(w, inp, dev, kept, kinds, lam=30.0, flags=sb.SALAD_FLAG_UNFUSED_EPILOGUE)
    compare_layer(res, ref, label="unfused")


@pytest.mark.parametrize("grid,kept,truncated", [((9, 10, 13), [4, 7, 5], False), ((9, 10, 13), [4, 7, 5], True),
                                                 ((21, 30, 52), [51] * 3, False), ((5, 6, 9), [1, 5], True)])
def test_tile_lists_layout(oracle, grid, kept, truncated):
    """salad_tile_lists against the documented layout, rebuilt here from the oracle's CSR: per (head, tile of 4 query
    blocks) the ascending union of the rows' kept blocks, each entry block | (kept-by-row bits << 24), rotated to start at
    the entry whose block id is smallest modulo the list length; counts after the lists at the next 256-byte boundary."""
    T, Hh, W = grid
    H, nb = len(kept), (T * Hh * W + 63) // 64
    rp, ci = oracle.block_mask(T, Hh, W, 64, kept, truncated=truncated)
    row_ptr, col_idx = torch.from_numpy(rp).cuda(), torch.from_numpy(ci).cuda()
    buf = sb.salad_tile_lists(row_ptr, col_idx, H, nb)
    torch.cuda.synchronize()
    raw = buf.cpu().numpy()
    ntiles, cap = (nb + 3) // 4, (nb + 63) // 64 * 64
    nlist = H * ntiles * cap * 4
    lists = raw[:nlist].view(np.uint32).reshape(H, ntiles, cap)
    counts = raw[(nlist + 255) // 256 * 256:][:H * ntiles * 4].view(np.int32).reshape(H, ntiles)
    for h in range(H):
        for t in range(ntiles):
            bits = {}
            for i in range(4):
                r = 4 * t + i
                if r < nb:
                    for c in ci[rp[h * nb + r]:rp[h * nb + r + 1]]:
                        bits[int(c)] = bits.get(int(c), 0) | (1 << (24 + i))
            asc = [b | m for b, m in sorted(bits.items())]
            n = len(asc)
            assert counts[h, t] == n
            rot = min(range(n), key=lambda i: ((asc[i] & 0xffffff) % n, i)) if n else 0
            assert lists[h, t, :n].tolist() == asc[rot:] + asc[:rot]


def test_prebuilt_tile_lists_give_the_same_bits(oracle):
    """salad_tile_lists builds the large-tile kernel's visit lists once per CSR; a layer call that is handed them skips
    its own pre-pass and must produce the bits of a call that builds them itself (window mask and an arbitrary CSR)."""
    w = SMALL[7]
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [4, 5, 4]
    a = run_layer(w, inp, dev, kept, kinds, dbg=False)
    b = run_layer(w, inp, dev, kept, kinds, dbg=False, prebuilt_lists=True)
    assert np.array_equal(a["out"], b["out"])
    ref = _oracle_layer(oracle, w, inp, kept, kinds)
    compare_layer(b, ref, label="prebuilt lists")
    rng = np.random.default_rng(5)
    rows = [np.sort(rng.choice(w.nb, size=int(rng.integers(1, 7)), replace=False)) for _ in range(w.H * w.nb)]
    row_ptr = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int32)
    col_idx = np.concatenate(rows).astype(np.int32)
    a = run_layer(w, inp, dev, kept, kinds, dbg=False, csr=(row_ptr, col_idx))
    b = run_layer(w, inp, dev, kept, kinds, dbg=False, csr=(row_ptr, col_idx), prebuilt_lists=True)
    assert np.array_equal(a["out"], b["out"])


@pytest.mark.parametrize("variant", [1, 2], ids=["128-row-fallback", "first-generation"])
def test_fallback_attention_kernels(oracle, variant):
    """The d=128 kernels that serve as fallbacks (block list too long for LDS, huge N, inexact division)
    produce the same layer within the same tolerances; selected here through the tuning knob."""
    w = SMALL[7]                                      # five tiles of 4 query blocks, ragged tail, 3 heads
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [4, 5, 4]
    ref = _oracle_layer(oracle, w, inp, kept, kinds)
    sb.salad_tune("attn_variant", variant)
    try:
        res = run_layer(w, inp, dev, kept, kinds)
    finally:
        sb.salad_tune("attn_variant", 0)
    compare_layer(res, ref, label=f"variant{variant}")


def test_run_to_run_bit_reproducible():
    w = SMALL[1]
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    outs = [run_layer(w, inp, dev, [4] * w.H, kinds, dbg=False)["out_t"] for _ in range(3)]
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


@pytest.mark.parametrize("flags", [0, sb.SALAD_FLAG_UNFUSED_EPILOGUE], ids=["fused", "unfused"])
def test_branch_dropping(oracle, flags):
    """Sec. 4.3: with a threshold between the two samples' dynamic scales only the lower one loses its linear
    branch; its output is then the sparse branch alone, bit for bit what lambda = 0 gives."""
    w = SMALL[1]                                      # B = 2, 3 heads, 11 blocks
    inp = wl.make_inputs(w)
    wg = inp["w_gate"]
    inp["x_t"] = inp["x_t"].copy()
    inp["x_t"][1] = wl.round_to_bf16(inp["x_t"][1] + (2.0 * wg / float(np.dot(wg, wg))).astype(np.float32))   # pre-activations of sample 1 up by ~2
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [4] * w.H
    base = _oracle_layer(oracle, w, inp, kept, kinds, lam=20.0)
    s = base["s"]
    assert s[1] - s[0] > 0.2
    tau = float(0.5 * (s[0] + s[1]))
    ref = _oracle_layer(oracle, w, inp, kept, kinds, lam=20.0, drop_threshold=tau)
    assert ref["dropped"].tolist() == [1, 0]
    res = run_layer(w, inp, dev, kept, kinds, lam=20.0, flags=flags, drop_threshold=tau)
    assert res["dropped"].tolist() == [1, 0]
    assert np.abs(res["s"] - s).max() < 2e-6          # the reported scale is the gate's, pruned or not
    compare_layer(res, ref, check_linear=False, label="drop")
    sparse_only = run_layer(w, inp, dev, kept, kinds, lam=0.0, flags=0)["out_t"]
    assert torch.equal(res["out_t"][0], sparse_only[0])            # pruned sample: exactly the sparse branch
    assert not torch.equal(res["out_t"][1], sparse_only[1])        # the other one kept its linear branch
    # thresholds outside the range: nobody / everybody
    none = run_layer(w, inp, dev, kept, kinds, lam=20.0, flags=flags, drop_threshold=1e-6)
    full = run_layer(w, inp, dev, kept, kinds, lam=20.0, flags=flags)
    assert none["dropped"].tolist() == [0, 0] and torch.equal(none["out_t"], full["out_t"])
    assert full["dropped"].tolist() == [-1, -1]       # not written when dropping is off
    every = run_layer(w, inp, dev, kept, kinds, lam=20.0, flags=flags, drop_threshold=2.0)
    assert every["dropped"].tolist() == [1, 1] and torch.equal(every["out_t"], sparse_only)


def _random_shapes(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        T, Hh, W = int(rng.integers(1, 9)), int(rng.integers(1, 13)), int(rng.integers(1, 13))
        H, B, d = int(rng.integers(1, 5)), int(rng.integers(1, 3)), int(rng.choice([64, 128]))
        out.append(wl.small(f"rand{i}-T{T}x{Hh}x{W}-H{H}-B{B}-d{d}", B, H, d, T, Hh, W, "bf16", 0.5, seed=1000 + seed * 100 + i))
    return out


@pytest.mark.parametrize("w", _random_shapes(16, 1), ids=lambda w: w.name)
def test_layer_parity_random_shapes(oracle, w):
    """Seeded random small grids (1 to 1152 tokens), head counts, batch sizes, both head widths, random window sizes and
    head orders: the whole layer against the oracle, and the benchmark launch bit-equal to the call with per-branch outputs."""
    rng = np.random.default_rng(w.seed)
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = rng.integers(0, 2, size=w.H).astype(np.uint8)
    kept = [int(rng.integers(1, w.nb + 1)) for _ in range(w.H)]
    res = run_layer(w, inp, dev, kept, kinds)
    ref = _oracle_layer(oracle, w, inp, kept, kinds)
    assert np.array_equal(res["row_ptr"], ref["row_ptr"]) and np.array_equal(res["col_idx"], ref["col_idx"])
    assert np.abs(res["s"] - ref["s"]).max() < 2e-6
    compare_layer(res, ref, label=w.name)
    fast = run_layer(w, inp, dev, kept, kinds, dbg=False, prebuilt_lists=True)
    assert np.array_equal(fast["out"], res["out"])


def _random_shapes_d128(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        T, Hh, W = int(rng.integers(1, 9)), int(rng.integers(2, 13)), int(rng.integers(2, 13))
        H, B = int(rng.integers(1, 5)), int(rng.integers(1, 3))
        out.append(wl.small(f"randw{i}-T{T}x{Hh}x{W}-H{H}-B{B}", B, H, 128, T, Hh, W, "bf16", 0.5, seed=2000 + seed * 100 + i))
    return out


@pytest.mark.parametrize("w", _random_shapes_d128(12, 2), ids=lambda w: w.name)
def test_widened_rows_random_shapes(oracle, w):
    """Seeded random small shapes through the widened rows and their combinations: rotary linear branch (fused and with
    the separate apply pass), full projection with and without the rotation, Top-K masks (mixed head orders; mask bit for
    bit), each against the oracle."""
    rng = np.random.default_rng(w.seed)
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = rng.integers(0, 2, size=w.H).astype(np.uint8)
    kept = [int(rng.integers(1, w.nb + 1)) for _ in range(w.H)]
    cs, sn = wl.rope_tables(w.T, w.Hh, w.W, w.d)
    rope_dev = (torch.from_numpy(cs).cuda(), torch.from_numpy(sn).cuda())
    flags = sb.SALAD_FLAG_UNFUSED_EPILOGUE if rng.integers(0, 2) else 0
    ref = _oracle_layer(oracle, w, inp, kept, kinds, lam=10.0, rope=(cs, sn))
    res = run_layer(w, inp, dev, kept, kinds, lam=10.0, rope=rope_dev, flags=flags)
    compare_layer(res, ref, label=f"{w.name} rope flags={flags}")
    D = w.H * w.d
    wp = wl.round_to_bf16((wl.normal(w.seed, "w_proj", (D, D)) / np.sqrt(D) * 4.0).astype(np.float32))
    wp_dev = torch.from_numpy(wp).cuda().to(torch.bfloat16)
    with_rope = bool(rng.integers(0, 2))
    ref = _oracle_layer(oracle, w, inp, kept, kinds, w_proj=wp.astype(np.float64), rope=(cs, sn) if with_rope else None)
    res = run_layer(w, inp, dev, kept, kinds, head_scale=None, w_proj=wp_dev, rope=rope_dev if with_rope else None, dbg=False)
    compare_layer(res, ref, check_linear=False, label=f"{w.name} proj rope={with_rope}")
    key_block = int(rng.choice([64, 128]))
    nbk = -(-w.N // key_block)
    topk = int(rng.integers(1, min(8, nbk) + 1))
    ref = _oracle_layer(oracle, w, inp, kept, kinds, lam=5.0, topk=topk, key_block=key_block)
    res = run_layer(w, inp, dev, kept, kinds, lam=5.0, topk=topk, topk_key_block=key_block)
    assert np.array_equal(res["topk_mask"], ref["topk_mask"])
    compare_layer(res, ref, label=f"{w.name} topk={topk}/{key_block}")
    # without the debug outputs (topk <= 4: the partial results are merged inside the linear-apply pass)
    fast = run_layer(w, inp, dev, kept, kinds, lam=5.0, topk=topk, topk_key_block=key_block, dbg=False)
    assert np.array_equal(fast["topk_mask"], ref["topk_mask"])
    compare_layer(fast, ref, check_linear=False, label=f"{w.name} topk={topk}/{key_block} fast")


def test_d64_large_tile_modes(oracle):
    """bf16 d = 64 on the large-tile kernel through the modes of the layer call: lambda = 0 (sparse branch alone, bit
    equal to what a pruned sample gets), branch dropping with B = 2, the unfused epilogue, a precomputed s, and an
    arbitrary CSR with an empty row."""
    w = SMALL[8]                                      # d64-ragged: N = 429, B = 2, 2 heads
    inp = wl.make_inputs(w)
    wg = inp["w_gate"]
    inp["x_t"] = inp["x_t"].copy()
    inp["x_t"][1] = wl.round_to_bf16(inp["x_t"][1] + (2.0 * wg / float(np.dot(wg, wg))).astype(np.float32))
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [3, 4]
    base = _oracle_layer(oracle, w, inp, kept, kinds, lam=20.0)
    tau = float(0.5 * (base["s"][0] + base["s"][1]))
    ref = _oracle_layer(oracle, w, inp, kept, kinds, lam=20.0, drop_threshold=tau)
    assert ref["dropped"].tolist() == [1, 0]
    sparse_only = run_layer(w, inp, dev, kept, kinds, lam=0.0)
    compare_layer(sparse_only, _oracle_layer(oracle, w, inp, kept, kinds, lam=0.0), check_linear=False, label="d64 lambda=0")
    for flags in (0, sb.SALAD_FLAG_UNFUSED_EPILOGUE):
        res = run_layer(w, inp, dev, kept, kinds, lam=20.0, flags=flags, drop_threshold=tau)
        assert res["dropped"].tolist() == [1, 0]
        compare_layer(res, ref, check_linear=False, label=f"d64 drop flags={flags}")
        assert torch.equal(res["out_t"][0], sparse_only["out_t"][0])
        full = run_layer(w, inp, dev, kept, kinds, lam=20.0, flags=flags)
        compare_layer(full, base, label=f"d64 flags={flags}")
    s_fixed = np.array([0.25, 0.75], dtype=np.float32)
    res_s = run_layer(w, inp, dev, kept, kinds, lam=3.0, s=torch.from_numpy(s_fixed).cuda())
    compare_layer(res_s, _oracle_layer(oracle, w, inp, kept, kinds, lam=3.0, s_override=s_fixed.astype(np.float64)), label="d64 s_dev")
    rng = np.random.default_rng(9)
    rows = [np.sort(rng.choice(w.nb, size=int(rng.integers(0 if r == 2 else 1, 5)), replace=False)) for r in range(w.H * w.nb)]
    csr = (np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int32), np.concatenate(rows).astype(np.int32))
    res_c = run_layer(w, inp, dev, None, kinds, csr=csr)
    o_s, rws = oracle.sparse_attn(inp["q"], inp["k"], inp["v"], (w.T, w.Hh, w.W), 64, kinds, *csr)
    got, ok = gather_rows(res_c["o_sparse"], rws)
    assert errors(got[ok], o_s[ok])[1] <= REL_L2


def test_branch_dropping_fp32(oracle):
    w = wl.small("drop-f32", 2, 2, 64, 3, 6, 8, "f32", 0.5, seed=112)       # N = 144
    inp = wl.make_inputs(w)
    wg = inp["w_gate"]
    inp["x_t"] = inp["x_t"].copy()
    inp["x_t"][0] += (2.0 * wg / float(np.dot(wg, wg))).astype(np.float32)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [2, 2]
    base = _oracle_layer(oracle, w, inp, kept, kinds, lam=5.0)
    tau = float(0.5 * (base["s"][0] + base["s"][1]))
    ref = _oracle_layer(oracle, w, inp, kept, kinds, lam=5.0, drop_threshold=tau)
    res = run_layer(w, inp, dev, kept, kinds, lam=5.0, drop_threshold=tau)
    assert ref["dropped"].tolist() == [0, 1] and res["dropped"].tolist() == [0, 1]
    compare_layer(res, ref, check_linear=False, tol_abs=1e-4, tol_rel=1e-5, label="drop-f32")


PROJ_SHAPES = [
    SMALL[1],                                                                    # B = 2, H = 3 (odd: one output head per workgroup), N = 693
    wl.small("proj-even-heads", 2, 4, 128, 7, 9, 11, "bf16", 0.6, seed=112),     # H = 4: two output heads per workgroup, 3 row tiles, tail
]


@pytest.mark.parametrize("w", PROJ_SHAPES, ids=lambda w: w.name)
def test_full_projection(oracle, w):
    """Alg. 1 "Proj" as a full D x D matrix across heads: O_s + lambda s_b (O_l W_p), against the oracle; the
    block-diagonal W_p reproduces the per-head form; pruned samples stay the sparse branch."""
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [4] * w.H
    D = w.H * w.d
    wp = wl.round_to_bf16((wl.normal(113, "w_proj", (D, D)) / np.sqrt(D)).astype(np.float32))
    wp_dev = torch.from_numpy(wp).cuda().to(torch.bfloat16)
    ref = _oracle_layer(oracle, w, inp, kept, kinds, lam=25.0, w_proj=wp.astype(np.float64))
    ref_ps = _oracle_layer(oracle, w, inp, kept, kinds, lam=25.0)
    assert errors(ref["out"], ref_ps["out"])[1] > 0.05                 # the projection is not a small effect here
    res = run_layer(w, inp, dev, kept, kinds, lam=25.0, head_scale=None, w_proj=wp_dev)
    compare_layer(res, ref, check_linear=False, label="full-proj")
    # W_p rearranged once for the layer (salad_proj_pack) and handed in instead of w_proj: the same bits
    packed = sb.salad_proj_pack(wp_dev, w.H, w.d)
    res_p = run_layer(w, inp, dev, kept, kinds, lam=25.0, head_scale=None, w_proj_packed=packed)
    assert np.array_equal(res_p["out"], res["out"])
    # block-diagonal projection = per-head scalars (a_h representable in bf16)
    a = wl.round_to_bf16(inp["head_scale"])
    wd = torch.from_numpy(np.kron(np.diag(a), np.eye(w.d, dtype=np.float32)).astype(np.float32)).cuda().to(torch.bfloat16)
    res_d = run_layer(w, inp, dev, kept, kinds, lam=25.0, head_scale=None, w_proj=wd)
    res_h = run_layer(w, inp, dev, kept, kinds, lam=25.0, head_scale=torch.from_numpy(a).cuda())
    assert errors(res_d["out"], res_h["out"])[1] < 3e-3
    # with branch dropping: the pruned sample is the sparse branch alone
    tau = 2.0
    res_dr = run_layer(w, inp, dev, kept, kinds, lam=25.0, head_scale=None, w_proj=wp_dev, drop_threshold=tau)
    sparse_only = run_layer(w, inp, dev, kept, kinds, lam=0.0)["out_t"]
    assert res_dr["dropped"].tolist() == [1, 1] and torch.equal(res_dr["out_t"], sparse_only)


@pytest.mark.parametrize("variant", [0, 1], ids=["regrouped", "token-mask"])
@pytest.mark.parametrize("wi,key_block,topk", [(1, 64, 4), (7, 128, 2), (0, 64, 8), (6, 64, 1), (4, 64, 3)],
                         ids=["N693-B2-kb64-k4", "N1170-kb128-k2", "N270-all-blocks", "single-token", "N512-k3"])
def test_topk_mask_layer(oracle, topk_variant, wi, key_block, topk, variant):
    """Top-K dynamic mask (App. A.1.2): the per-query block selection matches the oracle bit for bit (both sides
    take the decision in the same fixed float32 order), and the layer output on that mask meets the bf16 bar, for
    both attention paths (queries regrouped by key block and merged; token mask on ordinary query tiles)."""
    topk_variant(variant)
    w = SMALL[wi]
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = np.zeros(w.H, dtype=np.uint8)               # Top-K works on the stored order
    kept = [1] * w.H                                    # unused by the Top-K path
    ref = _oracle_layer(oracle, w, inp, kept, kinds, topk=topk, key_block=key_block)
    res = run_layer(w, inp, dev, kept, kinds, topk=topk, topk_key_block=key_block)
    assert np.array_equal(res["topk_mask"], ref["topk_mask"])
    nbk = -(-w.N // key_block)
    pop = np.array([bin(int(x)).count("1") for x in res["topk_mask"].reshape(-1)])
    assert (pop == min(topk, nbk)).all()
    compare_layer(res, ref, label=f"topk-{w.name}")
    # the same call without the debug outputs
    fast = run_layer(w, inp, dev, kept, kinds, topk=topk, topk_key_block=key_block, dbg=False)
    compare_layer(fast, ref, label=f"topk-{w.name}-fast")
    assert np.array_equal(fast["topk_mask"], ref["topk_mask"])
    if topk >= nbk:                                      # every block kept: the dense layer
        dense = run_layer(w, inp, dev, [w.nb] * w.H, kinds)
        assert errors(res["out"], dense["out"])[1] < 5e-3   # two independently rounded bf16 results


@pytest.mark.parametrize("wi,key_block,topk", [(1, 64, 4), (7, 128, 2), (5, 64, 3), (0, 64, 2)],
                         ids=["N693-B2-kb64-k4", "N1170-kb128-k2", "T70-gt-block-k3", "N270-tail14-k2"])
def test_topk_mask_temporal_heads(oracle, wi, key_block, topk):
    """Top-K with temporal heads (App. A.1.1 order inside App. A.1.2): the key blocks of an odd head are runs of its
    location-major order, so its block means, its selection and the keys it attends to differ from the stored-order
    ones; mask bit for bit, output to the bf16 bar, ragged last key block included."""
    w = SMALL[wi]
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    assert kinds.any() and w.T > 1
    kept = [1] * w.H
    ref = _oracle_layer(oracle, w, inp, kept, kinds, topk=topk, key_block=key_block)
    ref_stored = _oracle_layer(oracle, w, inp, kept, np.zeros(w.H, dtype=np.uint8), topk=topk, key_block=key_block)
    assert not np.array_equal(ref["topk_mask"], ref_stored["topk_mask"])          # the order matters on these inputs
    res = run_layer(w, inp, dev, kept, kinds, topk=topk, topk_key_block=key_block)
    assert np.array_equal(res["topk_mask"], ref["topk_mask"])
    compare_layer(res, ref, label=f"topk-temporal-{w.name}")
    fast = run_layer(w, inp, dev, kept, kinds, topk=topk, topk_key_block=key_block, dbg=False)
    compare_layer(fast, ref, label=f"topk-temporal-{w.name}-fast")


@pytest.mark.parametrize("flags", [0, sb.SALAD_FLAG_UNFUSED_EPILOGUE], ids=["fused", "unfused"])
@pytest.mark.parametrize("wi", [1, 7, 0, 4], ids=["N693-B2", "N1170", "N270-tail14", "N512"])
def test_rotary_linear_branch(oracle, wi, flags):
    """RoPE inside the linear branch (Sec. 4.1; numerator rotated, normaliser not): the layer against the oracle,
    with a static scale large enough that the linear branch carries weight; zero angles reproduce the plain layer.
    fused: the attention kernel's epilogue rotates relu(Q) in registers; unfused: the separate apply kernel does."""
    w = SMALL[wi]
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [3] * w.H if w.nb >= 3 else [1] * w.H
    cs, sn = wl.rope_tables(w.T, w.Hh, w.W, w.d)
    rope_dev = (torch.from_numpy(cs).cuda(), torch.from_numpy(sn).cuda())
    ref = _oracle_layer(oracle, w, inp, kept, kinds, lam=20.0, rope=(cs, sn))
    ref_plain = _oracle_layer(oracle, w, inp, kept, kinds, lam=20.0)
    res = run_layer(w, inp, dev, kept, kinds, lam=20.0, rope=rope_dev, flags=flags)
    compare_layer(res, ref, label=f"rope-{w.name}")
    fast = run_layer(w, inp, dev, kept, kinds, lam=20.0, rope=rope_dev, flags=flags, dbg=False)
    assert np.array_equal(fast["out"], res["out"])
    if w.N > 1:
        assert errors(ref["o_linear"], ref_plain["o_linear"])[1] > 0.05          # the rotation is not a small effect
    one = torch.ones_like(rope_dev[0]); zero = torch.zeros_like(rope_dev[0])
    res0 = run_layer(w, inp, dev, kept, kinds, lam=20.0, rope=(one, zero), flags=flags)
    plain = run_layer(w, inp, dev, kept, kinds, lam=20.0, flags=flags)
    assert torch.equal(res0["out_t"], plain["out_t"])                            # identity rotation: the same bits


@pytest.mark.parametrize("w", PROJ_SHAPES, ids=lambda w: w.name)
def test_full_projection_with_rotary_linear_branch(oracle, w):
    """Alg. 1 "Proj" as a full matrix over the rotary linear branch (the paper's layer has both): the emit pass writes the
    rotated O_l, the GEMM projects it; small shapes with B = 2 and a ragged tail, against the oracle."""
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [3, 4, 3, 4][:w.H]
    D = w.H * w.d
    wp = wl.round_to_bf16((wl.normal(w.seed, "w_proj", (D, D)) / np.sqrt(D) * 8.0).astype(np.float32))
    wp_dev = torch.from_numpy(wp).cuda().to(torch.bfloat16)
    cs, sn = wl.rope_tables(w.T, w.Hh, w.W, w.d)
    rope_dev = (torch.from_numpy(cs).cuda(), torch.from_numpy(sn).cuda())
    res = run_layer(w, inp, dev, kept, kinds, head_scale=None, w_proj=wp_dev, rope=rope_dev, dbg=False)
    ref = _oracle_layer(oracle, w, inp, kept, kinds, w_proj=wp.astype(np.float64), rope=(cs, sn))
    ref_plain = _oracle_layer(oracle, w, inp, kept, kinds, w_proj=wp.astype(np.float64))
    assert errors(ref["out"], ref_plain["out"])[1] > 1e-2             # the rotation changes the projected branch
    compare_layer(res, ref, check_linear=False, label="proj+rope")


def test_wan13_480p_rotary_sampled(oracle):
    """The rotary linear branch at the headline size: full rotated state and sampled rows against the oracle."""
    w = wl.WAN13_480P
    say("480p-rope: generating inputs")
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [sb.salad_kept_from_sparsity(w.nb, w.sparsity)] * w.H
    cs, sn = wl.rope_tables(w.T, w.Hh, w.W, w.d)
    rope_dev = (torch.from_numpy(cs).cuda(), torch.from_numpy(sn).cuda())
    say("480p-rope: GPU call")
    res = run_layer(w, inp, dev, kept, kinds, rope=rope_dev)
    sel = wl.sample_blocks(w.nb, 4, w.seed)
    say(f"480p-rope: oracle on {len(sel)} query blocks per head")
    ref = _oracle_layer(oracle, w, inp, kept, kinds, sel=sel, rope=(cs, sn))
    compare_layer(res, ref, label="480p-rope")
    assert np.isfinite(res["out"]).all()


@pytest.mark.parametrize("grid,key_block,topk", [((10, 10, 20), 64, 5), ((10, 20, 20), 64, 4), ((7, 11, 13), 192, 6),
                                                 ((16, 16, 16), 64, 8), ((4, 33, 31), 64, 8)],
                         ids=["32-key-blocks-k5", "63-key-blocks-k4", "6-key-blocks-k6-all", "64-key-blocks-k8",
                              "64-key-blocks-ragged-k8"])
def test_topk_selection_kernel_instantiations(oracle, grid, key_block, topk):
    """Shapes that reach the other instantiations of the selection kernel (up to 32 and up to 64 key blocks, four
    and eight kept slots), a ragged everything (N = 2000, 4000, 1001) and the limits: 64 key blocks (bit 63 of the
    mask word) with 8 kept, N = 4096 and N = 4092 (last key block of 60 tokens)."""
    w = wl.small("topk-shapes", 1, 2, 128, *grid, "bf16", 0.5, seed=211 + topk)
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = np.zeros(w.H, dtype=np.uint8)
    kept = [1] * w.H
    ref = _oracle_layer(oracle, w, inp, kept, kinds, topk=topk, key_block=key_block)
    res = run_layer(w, inp, dev, kept, kinds, topk=topk, topk_key_block=key_block)
    assert np.array_equal(res["topk_mask"], ref["topk_mask"])
    compare_layer(res, ref, label=f"topk-N{w.N}-kb{key_block}-k{topk}")


def test_topk_rotary_dropping_together(oracle):
    """The widened pieces in one call: Top-K mask for the sparse branch, rotary linear branch, and branch dropping
    with a threshold between the two samples' dynamic scales (sample 0 keeps its branch, sample 1 loses it)."""
    w = SMALL[1]                                        # B = 2, H = 3, N = 693
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = np.zeros(w.H, dtype=np.uint8)
    kept = [1] * w.H
    cs, sn = wl.rope_tables(w.T, w.Hh, w.W, w.d)
    rope_dev = (torch.from_numpy(cs).cuda(), torch.from_numpy(sn).cuda())
    s = oracle.gate(inp["x_t"], inp["w_gate"], 0.0)
    tau = float(0.5 * (s.min() + s.max()))
    assert s.min() < tau < s.max()
    ref = _oracle_layer(oracle, w, inp, kept, kinds, lam=10.0, topk=3, key_block=128, rope=(cs, sn), drop_threshold=tau)
    res = run_layer(w, inp, dev, kept, kinds, lam=10.0, topk=3, topk_key_block=128, rope=rope_dev, drop_threshold=tau)
    assert res["dropped"].tolist() == ref["dropped"].tolist() and sorted(res["dropped"].tolist()) == [0, 1]
    assert np.array_equal(res["topk_mask"], ref["topk_mask"])
    compare_layer(res, ref, check_linear=False, label="topk+rope+drop")
    b_drop = int(np.argmax(ref["dropped"]))
    sparse_only = run_layer(w, inp, dev, kept, kinds, lam=0.0, topk=3, topk_key_block=128)["out_t"]
    assert torch.equal(res["out_t"][b_drop], sparse_only[b_drop])
    # the same call without the debug outputs
    fast = run_layer(w, inp, dev, kept, kinds, lam=10.0, topk=3, topk_key_block=128, rope=rope_dev, drop_threshold=tau, dbg=False)
    compare_layer(fast, ref, check_linear=False, label="topk+rope+drop-fast")
    assert torch.equal(fast["out_t"][b_drop], sparse_only[b_drop])


@pytest.mark.parametrize("topk,key_block", [(4, 64), (2, 128), (1, 64)], ids=["k4", "k2", "k1"])
def test_topk_merge_inside_the_apply_pass(oracle, topk, key_block):
    """Regrouped Top-K path without debug outputs, projection or rotation: the partial results of a query are merged
    by the linear-apply pass itself (fp32, one rounding of the sum).  Against the oracle, with one of the two samples
    pruned (Sec. 4.3): that sample must come out as the merge kernel writes it for lambda = 0, bit for bit, and the
    call with debug outputs (merge kernel, then the apply pass) must agree with the oracle as well."""
    w = SMALL[1]                                        # B = 2, H = 3, N = 693: three passes of 256 rows, ragged
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = np.zeros(w.H, dtype=np.uint8)
    kept = [1] * w.H
    s = oracle.gate(inp["x_t"], inp["w_gate"], 0.0)
    tau = float(0.5 * (s.min() + s.max()))
    ref = _oracle_layer(oracle, w, inp, kept, kinds, lam=10.0, topk=topk, key_block=key_block, drop_threshold=tau)
    ref_all = _oracle_layer(oracle, w, inp, kept, kinds, lam=10.0, topk=topk, key_block=key_block)
    fast = run_layer(w, inp, dev, kept, kinds, lam=10.0, topk=topk, topk_key_block=key_block, drop_threshold=tau, dbg=False)
    assert fast["dropped"].tolist() == ref["dropped"].tolist() and sorted(fast["dropped"].tolist()) == [0, 1]
    assert np.array_equal(fast["topk_mask"], ref["topk_mask"])
    compare_layer(fast, ref, check_linear=False, label="topk-merge-in-apply+drop")
    b_drop = int(np.argmax(ref["dropped"]))
    sparse_only = run_layer(w, inp, dev, kept, kinds, lam=0.0, topk=topk, topk_key_block=key_block, dbg=False)["out_t"]
    assert torch.equal(fast["out_t"][b_drop], sparse_only[b_drop])
    assert not torch.equal(fast["out_t"][1 - b_drop], sparse_only[1 - b_drop])
    # nobody pruned: both ways of merging against the oracle, and against each other (they differ by one bf16 rounding of O_s)
    fast_all = run_layer(w, inp, dev, kept, kinds, lam=10.0, topk=topk, topk_key_block=key_block, dbg=False)
    slow_all = run_layer(w, inp, dev, kept, kinds, lam=10.0, topk=topk, topk_key_block=key_block)
    e_fast = compare_layer(fast_all, ref_all, check_linear=False, label="topk-merge-in-apply")["out"]
    e_slow = compare_layer(slow_all, ref_all, label="topk-merge-kernel")["out"]
    assert e_fast[1] <= e_slow[1] * 1.05               # one rounding less cannot be less accurate
    assert errors(fast_all["out"], slow_all["out"])[1] < 5e-3


@pytest.fixture
def topk_variant():
    yield lambda v: sb.salad_tune("topk_variant", v)
    sb.salad_tune("topk_variant", 0)


def test_layer_call_under_graph_capture():
    """The layer call allocates nothing and never synchronises, so it can be captured into a HIP graph.
    Replays (with eager work and synchronisation in between) give the bits of the eager call."""
    w = SMALL[7]
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [4, 5, 4]
    eager = run_layer(w, inp, dev, kept, kinds, dbg=False)["out_t"].clone()
    grid = (w.T, w.Hh, w.W)
    row_ptr, col_idx = sb.salad_block_mask(*grid, w.block, kept)
    q, k, v = dev["q"], dev["k"], dev["v"]
    out = torch.zeros_like(q)
    ws = sb.Workspace(w.B, w.H, w.N, w.d, sb.SALAD_BF16, q.device)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        p, keep = sb.make_fwd_params(q, k, v, out, grid, row_ptr, col_idx, kinds, lam=w.lam, head_scale=dev["head_scale"],
                                     x_t=dev["x_t"], w_gate=dev["w_gate"], eps=w.eps, workspace=ws)
        sb.salad_fwd_call(p)
    for rep in range(3):
        out.fill_(float("nan"))                      # eager work between replays
        (dev["x_t"].float().sum()).item()            # ... and a synchronisation
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {rep} differs from the eager call"


def test_timing_modes_leave_results_alone():
    """Per-stage timing (mode 1), attention-only timing (mode 2) and no timing give the same bits; mode 2 reports
    the attention stage alone."""
    w = SMALL[7]
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [4, 5, 4]
    ref = run_layer(w, inp, dev, kept, kinds, dbg=False)["out_t"].clone()
    try:
        for mode in (1, 2):
            sb.salad_timing_read(reset=True)
            sb.salad_timing_enable(mode)
            outs = [run_layer(w, inp, dev, kept, kinds, dbg=False)["out_t"].clone() for _ in range(3)]
            sb.salad_timing_enable(0)
            kt = sb.salad_timing_read(reset=True)
            assert all(torch.equal(o, ref) for o in outs)
            assert kt.calls == 3 and kt.attn_ms > 0
            if mode == 1:
                assert kt.gate_ms > 0 and kt.state_ms > 0 and kt.finalize_ms > 0
            else:
                assert kt.gate_ms == 0 and kt.state_ms == 0 and kt.finalize_ms == 0 and kt.epilogue_ms == 0
    finally:
        sb.salad_timing_enable(0)
        sb.salad_timing_read(reset=True)


# ------------------------------------------------------------------- benchmark configurations

def _sampled_parity(oracle, w, nsel, label):
    say(f"{label}: generating inputs N={w.N} H={w.H}")
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [sb.salad_kept_from_sparsity(w.nb, w.sparsity)] * w.H
    say(f"{label}: GPU call, kept={kept[0]} of {w.nb}")
    res = run_layer(w, inp, dev, kept, kinds)
    sel = wl.sample_blocks(w.nb, nsel, w.seed)
    say(f"{label}: oracle on {len(sel)} query blocks per head")
    ref = _oracle_layer(oracle, w, inp, kept, kinds, sel=sel)
    assert np.array_equal(res["row_ptr"], ref["row_ptr"]) and np.array_equal(res["col_idx"], ref["col_idx"])
    assert np.abs(res["s"] - ref["s"]).max() < 2e-6
    compare_layer(res, ref, label=label)
    # properties that hold at any size: finite everywhere, every row written
    assert np.isfinite(res["out"]).all() and np.isfinite(res["o_sparse"]).all() and np.isfinite(res["o_linear"]).all()
    # the launch the benchmark times (no per-branch outputs: results leave through LDS as whole rows) gives the same
    # bits as the call above with its per-lane stores
    say(f"{label}: benchmark launch (no per-branch outputs)")
    fast = run_layer(w, inp, dev, kept, kinds, dbg=False)
    assert np.array_equal(fast["out"], res["out"])
    return res, ref, inp, dev, kinds, kept


def test_mid_config_sampled(oracle):
    _sampled_parity(oracle, wl.MID, 12, "mid")


def test_d64_large_tile_kernel_sampled(oracle):
    """bf16 d = 64 on the large-tile kernel at a size that fills the chip (N = 12480: 195 blocks, tail 0, 24 heads,
    odd heads temporal): sampled query blocks against the oracle, the benchmark launch bit-equal to the call with
    per-branch outputs, prebuilt visit lists bit-equal too, and the first-generation d = 64 kernel (the fallback,
    selected through the knob) within the same bars."""
    w = wl.small("d64-mid", 1, 24, 64, 8, 30, 52, "bf16", 0.75, seed=113)
    res, ref, inp, dev, kinds, kept = _sampled_parity(oracle, w, 10, "d64-mid")
    pre = run_layer(w, inp, dev, kept, kinds, dbg=False, prebuilt_lists=True)
    assert np.array_equal(pre["out"], res["out"])
    sb.salad_tune("attn_variant", 2)
    try:
        old = run_layer(w, inp, dev, kept, kinds)
    finally:
        sb.salad_tune("attn_variant", 0)
    compare_layer(old, ref, label="d64-mid/first-generation")


@pytest.mark.timeout(600)
def test_wan13_480p_90_sampled(oracle):
    """The headline configuration at full size, in the launch configuration the benchmark times; the oracle
    evaluates every one of the 512 query blocks of every head (all 393 120 output rows are compared), plus the
    full linear state and gate."""
    res, ref, inp, dev, kinds, kept = _sampled_parity(oracle, wl.WAN13_480P, wl.WAN13_480P.nb, "480p-90")
    Hs, Z = sb.salad_linear_state_fwd(dev["k"], dev["v"])
    torch.cuda.synchronize()
    assert errors(Hs.cpu().numpy().astype(np.float64), ref["Hs"])[1] < 2e-6
    assert errors(Z.cpu().numpy().astype(np.float64), ref["Z"])[1] < 2e-6


def test_wan13_480p_full_projection_sampled(oracle):
    """Alg. 1 "Proj" with the full D x D matrix at the headline size (H = 12, N = 32760: 128 row tiles of the
    projection GEMM, the last one with 248 rows), in the launch configuration the benchmark times; the oracle
    evaluates sampled query blocks of every head (first, last = tail, middle, seeded picks)."""
    w = wl.WAN13_480P
    say("480p-proj: generating inputs")
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = wl.head_kinds(w)
    kept = [sb.salad_kept_from_sparsity(w.nb, w.sparsity)] * w.H
    D = w.H * w.d
    wp = wl.round_to_bf16((wl.normal(w.seed, "w_proj", (D, D)) / np.sqrt(D)).astype(np.float32))
    wp_dev = torch.from_numpy(wp).cuda().to(torch.bfloat16)
    say("480p-proj: GPU call")
    res = run_layer(w, inp, dev, kept, kinds, head_scale=None, w_proj=wp_dev, dbg=False)
    sel = wl.sample_blocks(w.nb, 4, w.seed)
    say(f"480p-proj: oracle on {len(sel)} query blocks per head")
    ref = _oracle_layer(oracle, w, inp, kept, kinds, sel=sel, w_proj=wp.astype(np.float64))
    ref_ps = _oracle_layer(oracle, w, inp, kept, kinds, sel=sel)
    assert errors(ref["out"], ref_ps["out"])[1] > 1e-3                 # the projection changes the result
    compare_layer(res, ref, check_linear=False, label="480p-proj")
    assert np.isfinite(res["out"]).all()


def test_wan13_480p_topk_sampled(oracle):
    """Top-K mask at the headline size and sparsity: 40 key blocks of 832 tokens (13 blocks of 64; the last one
    312 tokens), 4 kept per query token = 90 % sparsity.  The full mask is compared bit for bit, the output on
    sampled query blocks."""
    w = wl.WAN13_480P
    say("480p-topk: generating inputs")
    inp = wl.make_inputs(w)
    dev = upload(w, inp)
    kinds = np.zeros(w.H, dtype=np.uint8)
    kept = [1] * w.H
    say("480p-topk: GPU call")
    res = run_layer(w, inp, dev, kept, kinds, topk=4, topk_key_block=832, dbg=False)
    sel = wl.sample_blocks(w.nb, 4, w.seed)
    say(f"480p-topk: oracle selection for every query, attention on {len(sel)} query blocks per head")
    ref = _oracle_layer(oracle, w, inp, kept, kinds, sel=sel, topk=4, key_block=832)
    assert np.array_equal(res["topk_mask"], ref["topk_mask"])
    compare_layer(res, ref, check_linear=False, label="480p-topk")
    assert np.isfinite(res["out"]).all()


@pytest.mark.timeout(600)
@pytest.mark.parametrize("case", ["list-too-long", "inexact-division"])
def test_long_sequence_takes_the_fallback_by_itself(oracle, case):
    """Shapes the large-tile kernel does not take, so that the dispatcher has to pick the 128-row kernel without being
    told (the tuning knob stays at automatic).  list-too-long: 6152 key blocks per head, more than the per-tile block
    list may hold in LDS.  inexact-division: N T >= 2^32, where the temporal order's multiply-high division by T is no
    longer exact (the list would fit).  One spatial and one temporal head, 5 kept blocks per row, ragged last block."""
    if case == "list-too-long":
        w = wl.small("long-seq", 1, 2, 128, 31, 100, 127, "bf16", 1.0 - 5.0 / 6152.0, seed=131)
        assert w.N == 393700 and w.nb == 6152 and w.N % 64 == 36
    else:
        w = wl.small("long-T", 1, 2, 128, 11078, 5, 7, "bf16", 1.0 - 5.0 / 6059.0, seed=132)
        assert w.N == 387730 and w.nb == 6059 and w.N % 64 == 18 and w.N * w.T >= 1 << 32
        assert ((w.nb + 63) & ~63) * 4 <= 24 * 1024
    assert sb.salad_kept_from_sparsity(w.nb, w.sparsity) == 5
    _sampled_parity(oracle, w, 8, w.name)


@pytest.mark.parametrize("rho", [0.0, 0.5, 0.75, 0.95])
def test_wan13_480p_sweep_sampled(oracle, rho):
    """The other points of the sparsity sweep at the 480p shape (same seeded inputs)."""
    w = wl.WAN13_480P.with_sparsity(rho)
    _sampled_parity(oracle, w, 4 if rho < 0.7 else 8, f"480p-{rho:g}")


@pytest.mark.timeout(900)
def test_wan14_720p_90_sampled(oracle):
    """Wan-14B-shaped 720p configuration: H=40, N=75600 (16-token tail), gate over D=5120."""
    _sampled_parity(oracle, wl.WAN14_720P, 4, "720p-90")
