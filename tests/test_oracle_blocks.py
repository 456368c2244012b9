"""Pins for the oracle's building blocks: closed forms, invariants and library special cases."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import nmt_oracle as O


def test_softmax_rows_sum_to_one_and_masked_are_zero():
    rng = np.random.default_rng(0)
    a = rng.normal(size=(5, 7, 9)) * 10
    a[..., 3] = -np.inf
    p = O.softmax_rows(a)
    assert np.abs(p.sum(-1) - 1.0).max() < 1e-15
    assert (p[..., 3] == 0.0).all()


def test_attention_single_visible_key_returns_its_value():
    rng = np.random.default_rng(1)
    B, Tq, Tk, h, d = 2, 3, 5, 2, 8
    q, k, v = rng.normal(size=(B * Tq, d)), rng.normal(size=(B * Tk, d)), rng.normal(size=(B * Tk, d))
    masked = np.ones((B, Tq, Tk), dtype=bool)
    masked[:, :, 2] = False
    o, _ = O.attention_fwd(q, k, v, masked, B, Tq, Tk, h)
    want = np.repeat(v.reshape(B, Tk, d)[:, 2:3], Tq, axis=1).reshape(B * Tq, d)
    assert np.allclose(o, want, atol=1e-15)


def test_attention_matches_torch_sdpa():
    rng = np.random.default_rng(2)
    B, Tq, Tk, h, d = 2, 4, 6, 2, 8
    q, k, v = rng.normal(size=(B * Tq, d)), rng.normal(size=(B * Tk, d)), rng.normal(size=(B * Tk, d))
    masked = rng.random((B, Tq, Tk)) < 0.3
    masked[:, :, 0] = False
    o, _ = O.attention_fwd(q, k, v, masked, B, Tq, Tk, h)
    tq, tk, tv = (torch.tensor(x).reshape(B, -1, h, d // h).transpose(1, 2) for x in (q, k, v))
    ref = F.scaled_dot_product_attention(tq, tk, tv, attn_mask=~torch.tensor(masked)[:, None])
    ref = ref.transpose(1, 2).reshape(B * Tq, d).numpy()
    assert np.abs(o - ref).max() < 1e-12


def test_label_smoothing_closed_form_on_onehot_logits():
    V, eps, c = 50, 0.1, 3.7
    y = np.array([4, 9])
    z = np.zeros((2, V))
    z[np.arange(2), y] = c
    loss, n, dz = O.label_smoothed_nll(z, y, pad_id=1, eps=eps)
    want = math.log(math.exp(c) + V - 1) - (1 - eps + eps / V) * c
    assert n == 2 and abs(loss - 2 * want) < 1e-12
    assert np.abs(dz.sum(axis=1)).max() < 1e-15


def test_label_smoothing_uniform_logits_and_minimum():
    V = 37
    y = np.array([5])
    for eps in (0.0, 0.1, 0.4):
        loss, _, _ = O.label_smoothed_nll(np.zeros((1, V)), y, pad_id=1, eps=eps)
        assert abs(loss - math.log(V)) < 1e-12
    eps = 0.1
    q = np.full(V, eps / V)
    q[5] += 1 - eps
    loss, _, dz = O.label_smoothed_nll(np.log(q)[None, :], y, pad_id=1, eps=eps)
    assert abs(loss - (-(q * np.log(q)).sum())) < 1e-12       # the minimum is the entropy of q
    assert np.abs(dz).max() < 1e-15


def test_label_smoothing_matches_torch_and_ignores_padding():
    rng = np.random.default_rng(3)
    N, V, pad = 12, 23, 1
    z = rng.normal(size=(N, V)) * 3
    y = rng.integers(2, V, size=N)
    y[[2, 7]] = pad
    loss, n, dz = O.label_smoothed_nll(z, y, pad_id=pad, eps=0.1)
    zt = torch.tensor(z, requires_grad=True)
    ref = F.cross_entropy(zt, torch.tensor(y), ignore_index=pad, reduction="sum", label_smoothing=0.1)
    ref.backward()
    assert n == 10
    assert abs(loss - ref.item()) < 1e-10
    assert np.abs(dz - zt.grad.numpy()).max() < 1e-12
    assert (dz[[2, 7]] == 0).all()


def test_layernorm_identities_and_torch():
    rng = np.random.default_rng(4)
    N, d, eps = 6, 16, 1e-5
    y, g, b = rng.normal(size=(N, d)) * 2 + 1, rng.normal(size=d), rng.normal(size=d)
    out, saved = O.layernorm_fwd(y, np.ones(d), np.zeros(d), eps)
    var = y.var(axis=1)
    assert np.abs(out.mean(axis=1)).max() < 1e-15
    assert np.abs(out.var(axis=1) - var / (var + eps)).max() < 1e-12
    out, saved = O.layernorm_fwd(y, g, b, eps)
    yt, gt, bt = (torch.tensor(a, requires_grad=True) for a in (y, g, b))
    ref = F.layer_norm(yt, (d,), gt, bt, eps)
    assert np.abs(out - ref.detach().numpy()).max() < 1e-12
    dout = rng.normal(size=(N, d))
    ref.backward(torch.tensor(dout))
    dy, dg, db = O.layernorm_bwd(dout, g, saved)
    assert np.abs(dy - yt.grad.numpy()).max() < 1e-12
    assert np.abs(dg - gt.grad.numpy()).max() < 1e-12
    assert np.abs(db - bt.grad.numpy()).max() < 1e-12
    # the input gradient is orthogonal to the constant vector and to the normalised input
    assert np.abs(dy.sum(axis=1)).max() < 1e-12
    # (exactly so only without the variance floor, where mean(xhat^2) = 1)
    _, saved0 = O.layernorm_fwd(y, g, b, 0.0)
    dy0, _, _ = O.layernorm_bwd(dout, g, saved0)
    assert np.abs(dy0.sum(axis=1)).max() < 1e-12
    assert np.abs((dy0 * saved0[0]).sum(axis=1)).max() < 1e-12


def test_positional_encoding_values():
    pe = O.positional_encoding(5, 8)
    assert np.allclose(pe[0, 0::2], 0) and np.allclose(pe[0, 1::2], 1)
    assert abs(pe[3, 0] - math.sin(3.0)) < 1e-15 and abs(pe[3, 1] - math.cos(3.0)) < 1e-15
    assert abs(pe[2, 4] - math.sin(2.0 / 10000 ** (4 / 8))) < 1e-15
    assert abs(pe[2, 7] - math.cos(2.0 / 10000 ** (6 / 8))) < 1e-15


def test_linear_matches_definition():
    rng = np.random.default_rng(5)
    x, W, b, dy = rng.normal(size=(4, 3)), rng.normal(size=(5, 3)), rng.normal(size=5), rng.normal(size=(4, 5))
    y = O.linear_fwd(x, W, b)
    for i in range(4):
        for o in range(5):
            assert abs(y[i, o] - (sum(x[i, k] * W[o, k] for k in range(3)) + b[o])) < 1e-14
    dx, dW, db = O.linear_bwd(x, W, dy)
    xt, Wt, bt = (torch.tensor(a, requires_grad=True) for a in (x, W, b))
    F.linear(xt, Wt, bt).backward(torch.tensor(dy))
    assert np.allclose(dx, xt.grad.numpy()) and np.allclose(dW, Wt.grad.numpy()) and np.allclose(db, bt.grad.numpy())


def test_adam_closed_forms():
    rng = np.random.default_rng(6)
    g = {"w": rng.normal(size=7)}
    master, m, v = {"w": rng.normal(size=7)}, {"w": np.zeros(7)}, {"w": np.zeros(7)}
    w0 = master["w"].copy()
    lr, eps = 1e-3, 1e-8
    for t in range(1, 6):        # constant gradient: every step moves by lr * g / (|g| + eps)
        before = master["w"].copy()
        O.adam_step(master, m, v, g, lr, 0.9, 0.98, eps, t, flag=0)
        assert np.abs((master["w"] - before) + lr * g["w"] / (np.abs(g["w"]) + eps)).max() < 1e-12
    # overflow flag: nothing moves
    snap = (master["w"].copy(), m["w"].copy(), v["w"].copy())
    O.adam_step(master, m, v, g, lr, 0.9, 0.98, eps, 6, flag=1)
    assert (master["w"] == snap[0]).all() and (m["w"] == snap[1]).all() and (v["w"] == snap[2]).all()
    assert not (master["w"] == w0).all()


def test_adam_matches_torch_optimizer():
    rng = np.random.default_rng(7)
    w = rng.normal(size=9)
    master, m, v = {"w": w.copy()}, {"w": np.zeros(9)}, {"w": np.zeros(9)}
    wt = torch.tensor(w.copy(), requires_grad=True)
    opt = torch.optim.Adam([wt], lr=5e-4, betas=(0.9, 0.98), eps=1e-8)
    for t in range(1, 5):
        g = rng.normal(size=9)
        O.adam_step(master, m, v, {"w": g}, 5e-4, 0.9, 0.98, 1e-8, t, flag=0)
        wt.grad = torch.tensor(g)
        opt.step()
        assert np.abs(master["w"] - wt.detach().numpy()).max() < 1e-12


def test_lr_schedule_closed_form():
    peak = 5e-4
    assert abs(O.lr_schedule(1, peak) - peak / 4000) < 1e-18
    assert abs(O.lr_schedule(4000, peak) - peak) < 1e-18
    assert abs(O.lr_schedule(16000, peak) - peak / 2) < 1e-18
    assert O.lr_schedule(2000, peak) == pytest.approx(peak / 2)


def test_loss_scaler_trace():
    s = O.LossScaler(init_scale=128.0, window=2000)
    for i in range(1999):
        s.update(False)
    assert s.scale == 128.0 and s.clean == 1999
    s.update(False)
    assert s.scale == 256.0 and s.clean == 0          # doubled at exactly the 2000th clean update
    for i in range(700):
        s.update(False)
    s.update(True)
    assert s.scale == 128.0 and s.clean == 0          # halved, window restarts
    for i in range(1999):
        s.update(False)
    assert s.scale == 128.0
    s.update(False)
    assert s.scale == 256.0


def test_fp16_storage_boundary_and_overflow_predicate():
    g = O.to_fp16_storage({"a": np.array([65519.9, -65519.9, 65520.0, -65520.0, 1e-9])})["a"]
    assert np.isfinite(g[:2]).all() and g[0] == 65504.0
    assert np.isinf(g[2]) and np.isinf(g[3]) and g[3] < 0
    flag, _ = O.check_overflow({"a": np.array([1.0, 2.0])}, 0.5)
    assert flag == 0
    flag, _ = O.check_overflow({"a": np.array([1.0, np.inf])}, 0.5)
    assert flag == 1
    acc = O.accumulate({"a": np.array([np.inf])}, {"a": np.array([-np.inf])}, first=False)   # inf - inf
    assert O.check_overflow(acc, 1.0)[0] == 1
    flag, un = O.check_overflow({"a": np.array([3.0, -8.0])}, 0.25)
    assert (un["a"] == np.array([0.75, -2.0])).all()
