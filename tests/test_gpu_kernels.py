"""Per-kernel parity of the HIP path against the fp64 oracle, through the C ABI (needs an MI355X)."""
import math

import numpy as np
import pytest
import torch

import paper_1806_00187_amd as A
from oracle import nmt_oracle as O
from tests.gpu_util import DEV, assert_close16, dev16, dev32, devi, f16, host, rel_l2

pytestmark = pytest.mark.gpu


def _drop(p, site, step, micro, seed, n_pos, uid=None):
    return dict(p=p, site=site, step=step, micro=micro, seed=seed, n_pos=n_pos, sent_uid=uid)


# ---- dropout masks: bit-exact ----------------------------------------------------------------
@pytest.mark.parametrize("p,n_pos,n_cols,B", [(0.3, 16, 64, 8), (0.1, 33, 1024, 5), (0.5, 7, 40, 3), (0.0, 4, 16, 2)])
def test_dropout_mask_bit_exact(p, n_pos, n_cols, B):
    seed, site, step, micro = (7 << 32) | 12345, 35, 4099, 3
    uid = np.arange(100, 100 + B)
    keep = torch.zeros(B * n_pos, n_cols, dtype=torch.uint8, device=DEV)
    A.nmt_op_dropout_mask(keep, B * n_pos, n_cols, _drop(p, site, step, micro, seed, n_pos, devi(uid)))
    want = O.dropout_keep(seed, site, step, micro, uid, n_pos, n_cols, p)
    assert (host(keep).astype(bool) == want).all()
    # default sentence ids = row index
    A.nmt_op_dropout_mask(keep, B * n_pos, n_cols, _drop(p, site, step, micro, seed, n_pos))
    want = O.dropout_keep(seed, site, step, micro, np.arange(B), n_pos, n_cols, p)
    assert (host(keep).astype(bool) == want).all()


# ---- GEMM -------------------------------------------------------------------------------------
GEMM_SHAPES = [(128, 128, 64), (200, 136, 72), (37, 1000, 64), (515, 264, 200), (3003, 1024, 1024), (256, 3072, 1024),
               (1, 8, 8), (130, 64, 4096), (136, 264, 3003),
               (4088, 3080, 200),   # enough 256 x 256 tiles for the large-tile kernel, ragged on every side
               (10240, 3328, 200), (25600, 2568, 72)]   # more tiles than compute units: resident work-groups walk over 2 and 4 tiles


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("mode", ["fwd", "dgrad", "wgrad"])
def test_gemm_matches_oracle(M, N, K, mode):
    rng = np.random.default_rng(M * 7 + N * 3 + K)
    a_t, b_t = {"fwd": (0, 0), "dgrad": (0, 1), "wgrad": (1, 1)}[mode]
    if a_t and M % 8:
        M = (M + 7) // 8 * 8           # a transposed operand's contiguous extent must be a multiple of 8
    Am = f16(rng.normal(size=(M, K)))            # logical A[m, k]
    Bm = f16(rng.normal(size=(N, K)) / math.sqrt(K))   # logical B[n, k]
    if (not a_t or not b_t) and K % 8:
        pytest.skip("direct operands need K % 8 == 0")
    dA = dev16(Am.T if a_t else Am)
    dB = dev16(Bm.T if b_t else Bm)
    dC = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
    A.nmt_op_gemm(dA, a_t, M if a_t else K, dB, b_t, N if b_t else K, dC, N, M, N, K)
    assert_close16(host(dC), Am @ Bm.T, f"gemm {mode} {M}x{N}x{K}")


@pytest.mark.parametrize("M,N,K", [(128, 128, 16), (200, 136, 72), (37, 1000, 66), (515, 264, 203), (1031, 2052, 1024)])
@pytest.mark.parametrize("mode", ["fwd", "dgrad", "wgrad"])
def test_fp32_comparison_gemm_matches_oracle(M, N, K, mode):
    """The benchmark-only fp32 product (fp32 matrix instructions) in the three operand layouts of a linear layer."""
    rng = np.random.default_rng(M + 3 * N + 7 * K)
    a_t, b_t = {"fwd": (0, 0), "dgrad": (0, 1), "wgrad": (1, 1)}[mode]
    r4 = lambda n: (n + 3) // 4 * 4
    Am, Bm = rng.normal(size=(M, K)).astype(np.float32), (rng.normal(size=(N, K)) / math.sqrt(K)).astype(np.float32)
    # leading dimensions are multiples of 4: pad the stored matrices' contiguous dimension
    def stored(X, t):
        Y = X.T if t else X
        out = np.zeros((Y.shape[0], r4(Y.shape[1])), dtype=np.float32)
        out[:, :Y.shape[1]] = Y
        return dev32(out), out.shape[1]
    dA, lda = stored(Am, a_t)
    dB, ldb = stored(Bm, b_t)
    ldc = r4(N)
    dC = torch.full((M, ldc), float("nan"), dtype=torch.float32, device=DEV)
    A.nmt_op_gemm_f32(dA, a_t, lda, dB, b_t, ldb, dC, ldc, M, N, K)
    got, want = host(dC)[:, :N], Am.astype(np.float64) @ Bm.astype(np.float64).T
    assert np.isfinite(got).all()
    assert np.abs(got - want).max() <= 2e-5 * max(1.0, np.abs(want).max()), (mode, M, N, K, np.abs(got - want).max())
    if K >= 66:     # the contraction cut into three pieces: the partial products add up to the same
        parts = torch.full((3 * M, ldc), float("nan"), dtype=torch.float32, device=DEV)
        A.nmt_op_gemm_f32(dA, a_t, lda, dB, b_t, ldb, parts, ldc, M, N, K, splits=3)
        got = host(parts).reshape(3, M, ldc)[:, :, :N].sum(axis=0)
        assert np.abs(got - want).max() <= 2e-5 * max(1.0, np.abs(want).max()), (mode, "3 pieces")


@pytest.mark.parametrize("M,N,K,splits", [(136, 264, 3003, 3), (256, 128, 8192, 0), (64, 64, 4500, 64), (1024, 512, 6000, 5),
                                            (2048, 2040, 1500, 3), (1024, 1024, 16384, 0)])  # the last two: large-tile kernel
def test_gemm_split_along_k_matches_oracle(M, N, K, splits):
    """Weight-gradient form (both operands stored [K, rows]) with the contraction cut into pieces."""
    rng = np.random.default_rng(M + N + K)
    Am, Bm = f16(rng.normal(size=(M, K))), f16(rng.normal(size=(N, K)) / math.sqrt(K))
    dC = torch.full((M, N + 8), float("nan"), dtype=torch.float16, device=DEV)
    part = torch.full((max(splits, 8) * M * N,), float("nan"), dtype=torch.float32, device=DEV)
    A.nmt_op_gemm_splitk(dev16(Am.T), 1, M, dev16(Bm.T), 1, N, dC, N + 8, M, N, K, part, splits)
    assert_close16(host(dC)[:, :N], Am @ Bm.T, f"split-k gemm {M}x{N}x{K}/{splits}")
    with pytest.raises(A.NmtError):
        A.nmt_op_gemm_splitk(dev16(Am.T), 1, M, dev16(Bm.T), 1, N, dC, N + 8, M, N, K, part[: M * N], 2)


def test_gemm_large_problem_with_a_small_tile_tail_keeps_epilogue_rows():
    """Enough rows for one full round of large tiles plus a remainder, which goes to a second launch
    with small tiles: bias, ReLU and the dropout counters of the remainder must be those of its rows."""
    rng = np.random.default_rng(17)
    n_pos, B = 50, 100
    M, N, K = B * n_pos, 3080, 64
    x, W, b = f16(rng.normal(size=(M, K))), f16(rng.normal(size=(N, K)) / 8), f16(rng.normal(size=N))
    add = f16(rng.normal(size=(M, N)))
    dC = dev16(add)
    drop = _drop(0.25, 50, 9, 1, 99, n_pos)
    A.nmt_op_gemm(dev16(x), 0, K, dev16(W), 0, K, dC, N, M, N, K, bias=dev16(b), relu=True, drop=drop, add=dC)
    keep = O.dropout_keep(99, 50, 9, 1, np.arange(B), n_pos, N, 0.25)
    want = np.maximum(O.linear_fwd(x, W, b), 0) * keep / (1 - float(np.float32(0.25))) + add
    assert_close16(host(dC), want, "bias+relu+dropout+add, 5000 rows")
    # input-gradient and weight-gradient forms of the same size
    dy = f16(rng.normal(size=(M, 256)))
    Wt = f16(rng.normal(size=(256, N)) / 16)           # stored [out=256, in=N]: dx = dy W
    dx = torch.zeros(M, N, dtype=torch.float16, device=DEV)
    A.nmt_op_gemm(dev16(dy), 0, 256, dev16(Wt), 1, N, dx, N, M, N, 256)
    assert_close16(host(dx), dy @ Wt, "dgrad, 5000 rows")
    xt = f16(rng.normal(size=(64, M)))                 # A stored [K, M]
    yt = f16(rng.normal(size=(64, N)) / 8)
    out = torch.zeros(M, N, dtype=torch.float16, device=DEV)
    A.nmt_op_gemm(dev16(xt), 1, M, dev16(yt), 1, N, out, N, M, N, 64)
    assert_close16(host(out), xt.T @ yt, "both operands transposed, 5000 rows")


def test_gemm_persistent_form_matches_oracle_and_the_tile_per_work_group_form():
    """Products of at least two large tiles per compute unit, no split along k and an epilogue that loads nothing per
    element run as one persistent work-group per compute unit that requests the next tile's first k-tiles before it
    stores the current one.  Ragged M, N and k; bias + ReLU and the k-major form against the oracle, then bias, ReLU and
    output scale bit for bit against the one-tile-per-work-group kernel (switch 0): both add the same products in the
    same order and round once."""
    rng = np.random.default_rng(29)
    n_pos, B = 40, 826
    M, N, K = B * n_pos + 8, 4104, 72            # 130 x 17 tiles; the last row and column of tiles are partial
    x, W, b = f16(rng.normal(size=(M, K))), f16(rng.normal(size=(N, K)) / 8), f16(rng.normal(size=N))
    dx, dW, db = dev16(x), dev16(W), dev16(b)
    dC = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
    A.nmt_op_gemm(dx, 0, K, dW, 0, K, dC, N, M, N, K, bias=db, relu=True)
    assert_close16(host(dC), np.maximum(O.linear_fwd(x, W, b), 0), "persistent, bias+relu")
    Wt = f16(rng.normal(size=(K, N)) / 8)        # input-gradient form: B stored [K, N]
    dWt = dev16(Wt)
    A.nmt_op_gemm(dx, 0, K, dWt, 1, N, dC, N, M, N, K)
    assert_close16(host(dC), x @ Wt, "persistent, k-major B")
    got = {}
    try:
        for mode in (0, 1):
            A.nmt_tuning("gemm_persist", mode)
            outs = []
            for kw in (dict(bias=db, relu=True), dict(bias=db), dict(relu=True), dict()):
                c = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
                A.nmt_op_gemm(dx, 0, K, dW, 0, K, c, N, M, N, K, **kw)
                outs.append(c)
                c = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
                A.nmt_op_gemm(dx, 0, K, dWt, 1, N, c, N, M, N, K, **kw)
                outs.append(c)
            got[mode] = outs
    finally:
        A.nmt_tuning("defaults")
    for a, b2 in zip(got[0], got[1]):
        assert torch.isfinite(a).all()
        assert torch.equal(a.view(torch.int16), b2.view(torch.int16))
    # contractions shorter than one k-tile, and not a multiple of it: the requests that run ahead into the
    # next tile then lie partly or wholly past k
    for K2 in (8, 40, 136):
        x2, W2 = f16(rng.normal(size=(M, K2))), f16(rng.normal(size=(N, K2)) / 4)
        A.nmt_op_gemm(dev16(x2), 0, K2, dev16(W2), 0, K2, dC, N, M, N, K2, bias=db)
        assert_close16(host(dC), O.linear_fwd(x2, W2, b), f"persistent, k={K2}")
        Wt2 = f16(rng.normal(size=(K2, N)) / 4)
        A.nmt_op_gemm(dev16(x2), 0, K2, dev16(Wt2), 1, N, dC, N, M, N, K2)
        assert_close16(host(dC), x2 @ Wt2, f"persistent, k-major B, k={K2}")


def test_gemm_tile_order_changes_no_bit():
    """The order in which work-groups take the tiles (rows walked in groups, runs of tiles per XCD, runs of
    (k-split, tile) pairs) only decides who computes what: for any group size every tile is written exactly
    once and holds the same bits.  Ragged 130 x 17 tiles (persistent and tile-per-work-group form) and a
    weight gradient cut along k."""
    rng = np.random.default_rng(31)
    M, N, K = 826 * 40 + 8, 4104, 72
    dx, dW = dev16(f16(rng.normal(size=(M, K)))), dev16(f16(rng.normal(size=(N, K)) / 8))
    Mw, Nw, Kw = 2048, 2040, 1500
    dAw, dBw = dev16(f16(rng.normal(size=(Kw, Mw)))), dev16(f16(rng.normal(size=(Kw, Nw)) / 32))
    part = torch.empty(3 * Mw * Nw, dtype=torch.float32, device=DEV)

    def run():
        outs = []
        for persist in (0, 1):
            A.nmt_tuning("gemm_persist", persist)
            c = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
            A.nmt_op_gemm(dx, 0, K, dW, 0, K, c, N, M, N, K)
            outs.append(c)
        c = torch.full((Mw, Nw), float("nan"), dtype=torch.float16, device=DEV)
        A.nmt_op_gemm_splitk(dAw, 1, Mw, dBw, 1, Nw, c, Nw, Mw, Nw, Kw, part, 3)
        outs.append(c)
        return outs

    try:
        ref = run()                                   # the built-in group size
        assert all(torch.isfinite(c).all() for c in ref)
        assert torch.equal(ref[0].view(torch.int16), ref[1].view(torch.int16))
        for group in (1, 3, 16, 200):                 # 200: more rows per group than there are tile rows
            A.nmt_tuning("gemm_group", group)
            for a, b in zip(ref, run()):
                assert torch.equal(a.view(torch.int16), b.view(torch.int16)), group
        A.nmt_tuning("defaults")
        # the tile shape does not change a bit either: every compiled shape forced in turn, in all three operand
        # layouts the step uses, with an epilogue, and large tiles chosen for a share of the chip
        Ms, Ns, Ks = 1000, 776, 264
        xa, xat = dev16(f16(rng.normal(size=(Ms, Ks)))), dev16(f16(rng.normal(size=(Ks, Ms))))
        wb, wbt = dev16(f16(rng.normal(size=(Ns, Ks)) / 8)), dev16(f16(rng.normal(size=(Ks, Ns)) / 8))
        bias = dev16(f16(rng.normal(size=Ns)))

        def shapes_run():
            outs = []
            for a, a_t, b, b_t in ((xa, 0, wb, 0), (xa, 0, wbt, 1), (xat, 1, wbt, 1)):
                c = torch.full((Ms, Ns), float("nan"), dtype=torch.float16, device=DEV)
                A.nmt_op_gemm(a, a_t, Ms if a_t else Ks, b, b_t, Ns if b_t else Ks, c, Ns, Ms, Ns, Ks, bias=None if a_t else bias, relu=not a_t)
                outs.append(c)
            return outs

        ref2 = shapes_run()
        assert all(torch.isfinite(c).all() for c in ref2)
        for tile in (1, 2, 3, 4, 5):
            A.nmt_tuning("gemm_tile", tile)
            for a, b in zip(ref2, shapes_run()):
                assert torch.equal(a.view(torch.int16), b.view(torch.int16)), ("tile", tile)
        A.nmt_tuning("gemm_tile", 0)
        A.nmt_tuning("gemm_share", 16)
        for a, b in zip(ref2 + ref, shapes_run() + run()):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), "share"
    finally:
        A.nmt_tuning("defaults")


def test_gemm_epilogues_match_oracle():
    rng = np.random.default_rng(5)
    M, N, K, n_pos = 3 * 50, 256, 64, 50
    x, W, b = f16(rng.normal(size=(M, K))), f16(rng.normal(size=(N, K)) / 8), f16(rng.normal(size=N))
    add = f16(rng.normal(size=(M, N)))
    dC = torch.zeros(M, N, dtype=torch.float16, device=DEV)
    # bias + relu + dropout (the feed-forward activation)
    drop = _drop(0.25, 50, 9, 1, 99, n_pos)
    A.nmt_op_gemm(dev16(x), 0, K, dev16(W), 0, K, dC, N, M, N, K, bias=dev16(b), relu=True, drop=drop)
    keep = O.dropout_keep(99, 50, 9, 1, np.arange(3), n_pos, N, 0.25)
    want = np.maximum(O.linear_fwd(x, W, b), 0) * keep / (1 - float(np.float32(0.25)))
    assert_close16(host(dC), want, "bias+relu+dropout")
    # bias + add (residual / gradient fan-in), output aliasing the addend
    dC.copy_(dev16(add))
    A.nmt_op_gemm(dev16(x), 0, K, dev16(W), 0, K, dC, N, M, N, K, bias=dev16(b), add=dC)
    assert_close16(host(dC), O.linear_fwd(x, W, b) + add, "bias+add in place")
    # ReLU backward mask
    hact = f16(np.maximum(rng.normal(size=(M, N)), 0))
    A.nmt_op_gemm(dev16(x), 0, K, dev16(W), 0, K, dC, N, M, N, K, relu_src=dev16(hact), mask_scale=1.25)
    assert_close16(host(dC), (x @ W.T) * (hact > 0) * 1.25, "relu backward mask")


def test_gemm_strided_operands_and_rejections():
    rng = np.random.default_rng(6)
    M, N, K = 96, 64, 32
    big = f16(rng.normal(size=(M, 3 * K)))
    W = f16(rng.normal(size=(N, K)) / 4)
    dbig = dev16(big)
    dC = torch.zeros(M, 2 * N, dtype=torch.float16, device=DEV)
    A.nmt_op_gemm(dbig[:, K:], 0, 3 * K, dev16(W), 0, K, dC[:, N:], 2 * N, M, N, K)
    assert_close16(host(dC)[:, N:], big[:, K:2 * K] @ W.T, "strided")
    assert (host(dC)[:, :N] == 0).all()
    with pytest.raises(A.NmtError):
        A.nmt_op_gemm(dbig, 0, 3 * K, dev16(W), 0, K, dC, 2 * N, M, 60, K)      # N not a multiple of 8
    with pytest.raises(A.NmtError):
        A.nmt_op_gemm(dbig, 0, 3 * K, dev16(W), 0, K, dC, 2 * N, 0, N, K)       # empty


# ---- attention --------------------------------------------------------------------------------
ATTN_CASES = [  # B, H, dh, Tq, Tk, causal
    (2, 4, 16, 16, 16, 1), (3, 2, 64, 33, 36, 0), (2, 2, 64, 45, 45, 1), (1, 2, 64, 256, 256, 1), (2, 1, 64, 130, 200, 0),
    (5, 3, 32, 7, 9, 0), (2, 2, 128, 40, 40, 1), (4, 2, 64, 1, 1, 1), (2, 2, 16, 100, 70, 0),
    (3, 5, 64, 20, 50, 0), (2, 3, 32, 64, 10, 0), (2, 2, 64, 64, 64, 1), (2, 2, 64, 100, 120, 0), (2, 2, 64, 96, 96, 1),
    (1, 2, 128, 70, 90, 0)]


def _attn_inputs(B, H, dh, Tq, Tk, causal, seed):
    rng = np.random.default_rng(seed)
    d = H * dh
    q, k, v = (f16(rng.normal(size=(B * T, d))) for T in (Tq, Tk, Tk))
    key_ids = rng.integers(4, 50, size=(B, Tk))
    for b in range(B):            # right padding of varying length; at least one real key
        npad = int(rng.integers(0, max(1, Tk // 2)))
        if npad:
            key_ids[b, Tk - npad:] = 1
    masked = np.broadcast_to((key_ids == 1)[:, None, :], (B, Tq, Tk)).copy()
    if causal:
        masked |= np.triu(np.ones((Tq, Tk), dtype=bool), k=1)[None]
    return q, k, v, key_ids, masked


@pytest.mark.parametrize("B,H,dh,Tq,Tk,causal", ATTN_CASES)
def test_attention_forward_and_backward_match_oracle(B, H, dh, Tq, Tk, causal):
    d = H * dh
    q, k, v, key_ids, masked = _attn_inputs(B, H, dh, Tq, Tk, causal, seed=B * 100 + Tq)
    o_ref, saved = O.attention_fwd(q, k, v, masked, B, Tq, Tk, H)
    # operands live side by side in one [N, 3d] buffer, as in the fused projection
    qkv_q = dev16(np.concatenate([q, np.zeros_like(q), np.zeros_like(q)], axis=1))
    kv = dev16(np.concatenate([k, v], axis=1))
    dO_np = f16(np.random.default_rng(9).normal(size=(B * Tq, d)))
    o = torch.zeros(B * Tq, d, dtype=torch.float16, device=DEV)
    lse = torch.zeros(H, B, Tq, dtype=torch.float32, device=DEV)  # head-major: [H, B*Tq]
    ids = devi(key_ids)
    A.nmt_op_attention_fwd(qkv_q, 3 * d, kv, 2 * d, kv[:, d:], 2 * d, o, d, lse, ids, 1, causal, B, H, dh, Tq, Tk)
    assert_close16(host(o), o_ref, "attention output", rel=3e-3, l2=1.5e-3)
    qh, kh, _, _ = saved
    a = qh @ kh.transpose(0, 1, 3, 2) / math.sqrt(dh)
    a = np.where(masked[:, None], -np.inf, a)
    mx = a.max(-1)
    lse_ref = mx + np.log(np.exp(a - mx[..., None]).sum(-1))
    assert np.abs(host(lse).transpose(1, 0, 2) - lse_ref).max() < 2e-3
    # backward, fed with the oracle's forward output rounded to fp16
    dq_ref, dk_ref, dv_ref = O.attention_bwd(dO_np, saved, B, Tq, Tk, H)
    dq = torch.zeros(B * Tq, d, dtype=torch.float16, device=DEV)
    dkv = torch.zeros(B * Tk, 2 * d, dtype=torch.float16, device=DEV)
    A.nmt_op_attention_bwd(qkv_q, 3 * d, kv, 2 * d, kv[:, d:], 2 * d, o, d, dev16(dO_np), d, lse, dq, d, dkv, 2 * d, dkv[:, d:], 2 * d,
                           ids, 1, causal, B, H, dh, Tq, Tk)
    got = host(dkv)
    for name, g, w in (("dq", host(dq), dq_ref), ("dk", got[:, :d], dk_ref), ("dv", got[:, d:], dv_ref)):
        assert np.isfinite(g).all(), name
        # (a single visible key gives an exactly zero score gradient: floor the denominator)
        err = np.linalg.norm(g - w) / max(np.linalg.norm(w), 1e-3 * math.sqrt(w.size))
        assert err < 4e-3, (name, err)


# ---- fused residual + dropout + LayerNorm -----------------------------------------------------------
@pytest.mark.parametrize("rows,n_pos,d,p", [(48, 16, 64, 0.1), (99, 33, 1024, 0.3), (70, 35, 512, 0.0), (26, 13, 2048, 0.2),
                                            (10, 5, 200, 0.5)])
def test_residual_layernorm_forward_and_backward_match_oracle(rows, n_pos, d, p):
    rng = np.random.default_rng(rows + d)
    sub, resid = f16(rng.normal(size=(rows, d))), f16(rng.normal(size=(rows, d)) * 2 + 0.5)
    gamma, beta = f16(1 + 0.3 * rng.normal(size=d)), f16(0.2 * rng.normal(size=d))
    dout = f16(rng.normal(size=(rows, d)))
    seed, site, step, micro = 42, 19, 77, 2
    drop = _drop(p, site, step, micro, seed, n_pos)
    keep = O.dropout_keep(seed, site, step, micro, np.arange(rows // n_pos), n_pos, d, p)
    scale = 1.0 / (1.0 - float(np.float32(p)))
    y = resid + sub * keep * scale
    want, saved = O.layernorm_fwd(y, gamma, beta, 1e-5)
    out = torch.zeros(rows, d, dtype=torch.float16, device=DEV)
    stats = torch.zeros(rows, 2, dtype=torch.float32, device=DEV)
    dsub, dres, dg, db = dev16(sub), dev16(resid), dev16(gamma), dev16(beta)
    A.nmt_op_residual_layernorm_fwd(dsub, dres, dg, db, out, stats, rows, d, 1e-5, drop)
    assert_close16(host(out), want, "layernorm forward")
    st = host(stats)
    assert np.abs(st[:, 0] - y.mean(1)).max() < 1e-5 * max(1.0, np.abs(y.mean(1)).max())
    assert np.abs(st[:, 1] * np.sqrt(y.var(1) + 1e-5) - 1).max() < 1e-5
    # backward
    dy_ref, dg_ref, db_ref = O.layernorm_bwd(dout, gamma, saved)
    dym_ref = dy_ref * keep * scale
    dy = torch.zeros(rows, d, dtype=torch.float16, device=DEV)
    dym = torch.zeros_like(dy)
    gg, gb, gbias = (torch.zeros(d, dtype=torch.float16, device=DEV) for _ in range(3))
    part = torch.zeros(A.nmt_op_layernorm_bwd_scratch(d), dtype=torch.float32, device=DEV)
    A.nmt_op_residual_layernorm_bwd(dev16(dout), dsub, dres, dg, stats, dy, dym if p > 0 else None, gg, gb, gbias, part, rows, d, drop)
    assert_close16(host(dy), dy_ref, "layernorm dy", rel=2e-3)
    if p > 0:
        assert_close16(host(dym), dym_ref, "layernorm masked dy", rel=2e-3)
    assert_close16(host(gg), dg_ref, "dgamma")
    assert_close16(host(gb), db_ref, "dbeta")
    assert_close16(host(gbias), dym_ref.sum(0), "dbias")


# ---- embedding ----------------------------------------------------------------------------------
@pytest.mark.parametrize("B,n_pos,d,V,p", [(8, 16, 64, 1000, 0.1), (5, 37, 1024, 32768, 0.3), (3, 9, 512, 264, 0.0)])
def test_embedding_forward_matches_oracle(B, n_pos, d, V, p):
    rng = np.random.default_rng(B + d)
    E = f16(rng.normal(size=(V, d)) * 0.05)
    ids = rng.integers(0, V, size=(B, n_pos))
    seed, site, step = 5, 1, 3
    x = torch.zeros(B * n_pos, d, dtype=torch.float16, device=DEV)
    A.nmt_op_embed_fwd(devi(ids), dev16(E), x, B * n_pos, d, V, _drop(p, site, step, 0, seed, n_pos))
    keep = O.dropout_keep(seed, site, step, 0, np.arange(B), n_pos, d, p)
    want = (math.sqrt(d) * E[ids.reshape(-1)] + np.tile(O.positional_encoding(n_pos, d), (B, 1))) * keep / (1 - float(np.float32(p)))
    assert_close16(host(x), want, "embedding forward")


@pytest.mark.parametrize("d,V,p,Ba,Sa,Bb,Sb", [(64, 1000, 0.1, 6, 11, 6, 9), (1024, 4096, 0.3, 6, 11, 6, 9), (128, 40000, 0.1, 40, 33, 37, 29),
                                               (64, 65536, 0.0, 3, 400, 5, 300)])
def test_embedding_backward_matches_oracle_and_is_deterministic(d, V, p, Ba, Sa, Bb, Sb):
    """The larger cases have ids whose positions fill several 64-entry blocks of the sorted list (sums
    carried over block borders), ids above 255 * 256 and more than one 1024-entry block per sort pass."""
    rng = np.random.default_rng(d)
    ids_a = rng.integers(4, V, size=(Ba, Sa))
    ids_b = rng.integers(4, V, size=(Bb, Sb))
    ids_a[:, :4] = 7            # a heavily repeated id, shared by both streams
    ids_b[:3, :] = 7
    ids_b[3:, -2:] = 1
    if Ba * Sa > 1000:
        ids_a[:, 5:12] = V - 1  # > 64 and > 192 occurrences: first, middle and last blocks of a carried sum
        ids_b[:, 3:6] = V - 3
        ids_a[1::2, 20:] = 300
    dxa, dxb = f16(rng.normal(size=(Ba * Sa, d))), f16(rng.normal(size=(Bb * Sb, d)))
    g0 = f16(rng.normal(size=(V, d)))
    da, db_ = _drop(p, 0, 5, 1, 77, Sa), _drop(p, 1, 5, 1, 77, Sb)
    ka = O.dropout_keep(77, 0, 5, 1, np.arange(Ba), Sa, d, p)
    kb = O.dropout_keep(77, 1, 5, 1, np.arange(Bb), Sb, d, p)
    want = g0.copy()
    sc = math.sqrt(d) / (1 - float(np.float32(p)))
    np.add.at(want, ids_a.reshape(-1), dxa * ka * sc)
    np.add.at(want, ids_b.reshape(-1), dxb * kb * sc)
    scratch = torch.zeros(A.nmt_op_embed_bwd_scratch(V, Ba * Sa + Bb * Sb, d), dtype=torch.int32, device=DEV)
    outs = []
    for _ in range(2):
        gE = dev16(g0)
        A.nmt_op_embed_bwd(devi(ids_a), dev16(dxa), Ba * Sa, da, devi(ids_b), dev16(dxb), Bb * Sb, db_, gE, d, V, scratch)
        outs.append(host(gE))
    assert (outs[0] == outs[1]).all()
    touched = np.zeros(V, dtype=bool)
    touched[ids_a.reshape(-1)] = True
    touched[ids_b.reshape(-1)] = True
    assert (outs[0][~touched] == g0[~touched]).all()            # untouched rows are left bit-identical
    assert_close16(outs[0], want, "embedding backward", rel=2e-3, l2=1e-3)


# ---- fused softmax + label-smoothed cross-entropy -------------------------------------------------
@pytest.mark.parametrize("rows,V,scale", [(128, 1000, 128.0), (37, 32768, 128.0), (9, 40000, 1.0), (16, 8, 4.0), (20, 2056, 2.0 ** 27)])
def test_softmax_xent_matches_oracle(rows, V, scale):
    rng = np.random.default_rng(rows + V)
    z = f16(rng.normal(size=(rows, V)) * 2)
    y = rng.integers(2, V, size=rows)
    y[rng.random(rows) < 0.2] = 1
    y[0] = 5
    loss_ref, n_ref, dz_ref = O.label_smoothed_nll(z, y, 1, 0.1)
    dz = dev16(z)
    row_loss = torch.zeros(rows, dtype=torch.float32, device=DEV)
    loss, ntok = torch.zeros(1, dtype=torch.float32, device=DEV), torch.zeros(1, dtype=torch.int32, device=DEV)
    A.nmt_op_softmax_xent(dz, devi(y), row_loss, rows, V, 1, 0.1, scale, loss, ntok)
    assert int(ntok.item()) == n_ref
    assert abs(loss.item() - loss_ref) / loss_ref < 1e-5
    got = host(dz)
    with np.errstate(over="ignore"):
        want16 = (dz_ref * scale).astype(np.float16).astype(np.float64)      # fp16 storage of the scaled gradient
    near_limit = np.abs(np.abs(dz_ref * scale) - 65520.0) < 0.01 * 65520.0     # fp32 vs fp64 may round either way here
    assert (np.isinf(got) == np.isinf(want16))[~near_limit].all()            # overflow happens in the same places
    fin = np.isfinite(want16) & np.isfinite(got)
    assert (got[y == 1] == 0).all()
    err = np.abs(got[fin] - (dz_ref * scale)[fin])
    assert (err <= 2e-3 * np.abs(dz_ref * scale)[fin] + scale * 2e-7).all()


# ---- column sums, accumulate, overflow check, Adam ----------------------------------------------------
@pytest.mark.parametrize("rows,cols", [(3003, 3072), (128, 64), (1, 8), (517, 4096)])
def test_colsum_matches_oracle(rows, cols):
    rng = np.random.default_rng(rows)
    x = f16(rng.normal(size=(rows, cols + 8)))
    dst = torch.zeros(cols, dtype=torch.float16, device=DEV)
    part = torch.zeros(A.nmt_op_colsum_scratch(cols), dtype=torch.float32, device=DEV)
    A.nmt_op_colsum(dev16(x), cols + 8, dst, part, rows, cols)
    assert_close16(host(dst), x[:, :cols].sum(0), "colsum")


@pytest.mark.parametrize("n", [8, 1000003, 4096])
def test_accumulate_is_exact(n):
    rng = np.random.default_rng(n)
    g1, g2 = f16(rng.normal(size=n) * 100), f16(rng.normal(size=n))
    acc = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    A.nmt_op_accumulate(dev16(g1), acc, n, True)
    assert (host(acc) == g1).all()
    A.nmt_op_accumulate(dev16(g2), acc, n, False)
    assert (host(acc) == (g1.astype(np.float32) + g2.astype(np.float32)).astype(np.float64)).all()
    ref = O.accumulate(O.accumulate(None, {"a": g1}, True), {"a": g2}, False)["a"]
    assert np.abs(host(acc) - ref).max() <= 1e-6 * np.abs(ref).max()


@pytest.mark.parametrize("n,poison", [(1000003, None), (1000003, (999999, np.inf)), (4096, (17, np.nan)), (64, (0, -np.inf)), (5, None)])
def test_check_overflow_flag_is_exact_and_unscales(n, poison):
    rng = np.random.default_rng(n)
    a = rng.normal(size=n).astype(np.float32) * 1000
    if poison:
        a[poison[0]] = poison[1]
    acc = dev32(a)
    flag = torch.full((1,), 7, dtype=torch.int32, device=DEV)
    A.nmt_op_check_overflow(acc, n, 1.0 / 1024.0, flag)
    ref_flag, ref = O.check_overflow({"a": a.astype(np.float64)}, 1.0 / 1024.0)
    assert int(flag.item()) == ref_flag == (1 if poison else 0)
    if not poison:
        assert (host(acc) == ref["a"]).all()          # power-of-two scaling is exact


def test_adam_matches_oracle_and_skips_on_flag():
    rng = np.random.default_rng(3)
    n = 100003
    w0 = f16(rng.normal(size=n) * 0.1)
    master, m, v = dev32(w0), torch.zeros(n, dtype=torch.float32, device=DEV), torch.zeros(n, dtype=torch.float32, device=DEV)
    w16 = dev16(w0)
    om, omm, ov = {"w": w0.copy()}, {"w": np.zeros(n)}, {"w": np.zeros(n)}
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    for t in range(1, 4):
        g = rng.normal(size=n).astype(np.float32)
        A.nmt_op_adam(master, m, v, dev32(g), w16, n, 5e-4, 0.9, 0.98, 1e-8, t, flag)
        ref16 = O.adam_step(om, omm, ov, {"w": g.astype(np.float64)}, 5e-4, 0.9, 0.98, 1e-8, t, 0)["w"]
        assert np.abs(host(master) - om["w"]).max() < 1e-6 * np.abs(om["w"]).max() + 1e-9
        assert rel_l2(host(m), omm["w"]) < 1e-6 and rel_l2(host(v), ov["w"]) < 1e-6
        assert (host(w16) == host(master).astype(np.float32).astype(np.float16).astype(np.float64)).all()
        assert rel_l2(host(w16), ref16) < 1e-3
    # the gradient's scale factor is applied as it is read: g * 1024 with factor 1/1024 is the same update, bit for bit
    g = rng.normal(size=n).astype(np.float32)
    twin = [t_.clone() for t_ in (master, m, v, w16)]
    A.nmt_op_adam(master, m, v, dev32(g), w16, n, 5e-4, 0.9, 0.98, 1e-8, 4, flag)
    A.nmt_op_adam(twin[0], twin[1], twin[2], dev32(g * np.float32(1024)), twin[3], n, 5e-4, 0.9, 0.98, 1e-8, 4, flag, grad_scale=1.0 / 1024)
    for a_, b_ in zip((master, m, v, w16), twin):
        assert (host(a_) == host(b_)).all()
    snap = [host(t_) for t_ in (master, m, v, w16)]
    flag.fill_(1)
    A.nmt_op_adam(master, m, v, dev32(rng.normal(size=n).astype(np.float32)), w16, n, 5e-4, 0.9, 0.98, 1e-8, 5, flag)
    for before, t_ in zip(snap, (master, m, v, w16)):
        assert (host(t_) == before).all()
