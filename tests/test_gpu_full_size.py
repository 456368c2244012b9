"""Parity at the benchmark's full sizes: Transformer-big on real sub-batches of the synthetic workload
(the shapes bench.py times), the 40000-word vocabulary with 5120-token sub-batches accumulated over
one update, the long-sequence tail on Transformer-base, and the dynamic-loss-scaling traces with a
forced overflow.  The oracle runs the same sub-batches on the host (seconds to a minute each); every
gradient tensor, the updated master weights and every skip decision are compared."""
import time

import numpy as np
import pytest

import nmt_inputs as I
from oracle import nmt_oracle as O
from paper_1806_00187_amd.session import Session, Trainer
from tests.gpu_util import host, record_parity, rel_l2
from tests.test_gpu_step import FP16, GRAD_TOL, LOSS_TOL, RAW, OracleStep, _check_grads, _oracle_cfg, check_master_weights, pass_gates

pytestmark = pytest.mark.gpu


def _zeros_like(P):
    return {k: np.zeros_like(v) for k, v in P.items()}


def _full_size_case(model_name, batch, loss_scale, what, lr=1e-3):
    """One sub-batch: loss, every gradient tensor, the overflow flag (also of the same step forced to
    overflow), then overflow check + Adam and the master weights."""
    import torch
    model = I.MODELS[model_name]
    weights = I.init_weights(seed=0, **model)
    cfg = _oracle_cfg(model)
    P16 = {k: v.astype(np.float64) for k, v in weights.items()}
    B, S = batch["src"].shape
    T = batch["tgt_in"].shape[1]
    t0 = time.time()
    ora = OracleStep(P16, cfg, batch, loss_scale, 7, 3)
    print(f"{model_name} (B,S,T)=({B},{S},{T}): oracle (both storage modes) took {time.time() - t0:.0f}s", flush=True)
    sess = Session(model, weights, max_sentences=B, max_len=256)
    try:
        db = sess.to_device(batch)
        sess.forward_loss(db, loss_scale, 7, 3)
        sess.backward()
        loss, ntok = float(sess.loss_sum.item()), int(sess.ntok.item())
        assert ntok == ora.ntok
        assert abs(loss - ora.loss) / ora.loss <= LOSS_TOL and abs(loss - ora.loss16) / ora.loss16 <= LOSS_TOL, (loss, ora.loss, ora.loss16)
        G, note = ora.with_decisions_of(pass_gates(sess, model, [batch])[0], what)
        g16_ref = O.to_fp16_storage(G)
        worst = _check_grads(sess, sess.g16, g16_ref, model["d_model"], f"{what}: g16",
                             {RAW: O.to_fp16_storage(ora.G), FP16: O.to_fp16_storage(ora.G16)}, note)
        print(f"{model_name}: loss {loss / ntok:.4f}/token (oracle {ora.loss / ora.ntok:.4f}), worst gradient rel-L2 {worst}", flush=True)
        flag_ref, g_ref = O.check_overflow(g16_ref, 1.0 / (loss_scale * ora.ntok))
        # the same step with the loss scaled up by 2^20 (the forced overflow of configuration 3)
        with np.errstate(over="ignore", invalid="ignore"):
            flag_forced_ref, _ = O.check_overflow(O.to_fp16_storage({k: v * 2.0 ** 20 for k, v in G.items()}), 1.0)
        del ora, G
        master = {k: v.copy() for k, v in P16.items()}
        O.adam_step(master, _zeros_like(P16), _zeros_like(P16), g_ref, lr, 0.9, 0.98, 1e-8, 1, flag_ref)
        del g_ref
        sess.accumulate(True)
        sess.check_overflow(1.0 / (loss_scale * ntok))
        assert int(sess.flag.item()) == flag_ref == 0
        sess.adam_step(lr, 1)
        check_master_weights(sess, master, f"{what}: master weights after one update")
        # overflow decision of the forced step; the skipped update leaves every buffer as it is
        before = [x.clone() for x in (sess.master, sess.m, sess.v, sess.w16)]
        sess.forward_loss(db, loss_scale * 2.0 ** 20, 7, 3)
        sess.backward()
        sess.accumulate(True)
        sess.check_overflow(1.0 / (loss_scale * 2.0 ** 20 * ntok))
        assert int(sess.flag.item()) == flag_forced_ref == 1
        sess.adam_step(lr, 2)
        torch.cuda.synchronize()
        for a, b in zip(before, (sess.master, sess.m, sess.v, sess.w16)):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
    finally:
        sess.close()


def test_transformer_big_sub_batch_matches_oracle():
    batch = I.workload_batches("big", which="median", count=1, n_sentences=50_000)[0]
    _full_size_case("big", batch, loss_scale=32.0, what="Transformer-big, one 3.5k-token sub-batch")


def test_transformer_big_40k_vocabulary_5k_token_sub_batch_matches_oracle():
    # the larger sub-batch (5120 tokens) and a vocabulary that is not a multiple of the GEMM tile (40000)
    batch = I.workload_batches("big40k", which="median", count=1, n_sentences=50_000)[0]
    assert batch["src"].shape[0] * max(batch["src"].shape[1], batch["tgt_in"].shape[1]) > 4000
    _full_size_case("big40k", batch, loss_scale=32.0, what="Transformer-big V=40000, one 5k-token sub-batch")


def test_transformer_base_long_sequences_match_oracle():
    # the longest bucket of the length distribution (sequences of ~250 tokens, few sentences)
    buckets, src_len, tgt_len, rng = I.make_buckets("base", 50_000)
    model = I.MODELS["base"]
    batch = I.fill_batch(buckets[-1], src_len, tgt_len, model["vocab"], rng)
    assert max(batch["src"].shape[1], batch["tgt_in"].shape[1]) > 200
    _full_size_case("base", batch, loss_scale=32.0, what="Transformer-base, longest sentences")


def test_big_40k_four_sub_batches_in_one_packed_pass_match_the_accumulated_oracle_update():
    """Configuration 5 as bench.py would run it: the 4 sub-batches (<= 5120 tokens each) of one update as ONE
    packed pass, then accumulate, overflow check and Adam -- against the oracle's update in the method's
    order (each sub-batch's gradient rounded to fp16, accumulated wide, unscaled, Adam)."""
    model = I.MODELS["big40k"]
    weights = I.init_weights(seed=0, **model)
    cfg = _oracle_cfg(model)
    P16 = {k: v.astype(np.float64) for k, v in weights.items()}
    batches = I.workload_batches("big40k", which="spread", count=4, n_sentences=50_000)
    loss_scale, step, lr = 16.0, 2, 1e-3
    what = "Transformer-big V=40000, 4 sub-batches as one packed pass"
    sess = Session(model, weights, max_sentences=max(b["src"].shape[0] for b in batches), max_len=256)
    try:
        (pk,) = sess.pack(batches)
        sess.forward_loss(pk, loss_scale, step)
        sess.backward()
        gates = pass_gates(sess, model, batches, packed=True)
        t0 = time.time()
        acc, raw, loss_ref, ntok_ref, notes = None, None, 0.0, 0, []
        for j, mb in enumerate(batches):
            ora = OracleStep(P16, cfg, mb, loss_scale, step, j, with_fp16=False)
            G, note = ora.with_decisions_of(gates[j], f"{what}: sub-batch {j}")
            notes.append(note)
            acc = O.accumulate(acc, O.to_fp16_storage(G), j == 0)          # the method's order: fp16 per sub-batch, summed wide
            raw = O.accumulate(raw, O.to_fp16_storage(ora.G), j == 0)
            loss_ref += ora.loss
            ntok_ref += ora.ntok
            del ora, G
        print(f"big40k, 4 sub-batches {[b['src'].shape for b in batches]}: oracle took {time.time() - t0:.0f}s", flush=True)
        flag_ref, g_ref = O.check_overflow(acc, 1.0 / (loss_scale * ntok_ref))
        master = {k: v.copy() for k, v in P16.items()}
        O.adam_step(master, _zeros_like(P16), _zeros_like(P16), g_ref, lr, 0.9, 0.98, 1e-8, 1, flag_ref)
        assert int(sess.ntok.item()) == ntok_ref == pk["n_tgt"]
        assert abs(float(sess.loss_sum.item()) - loss_ref) / loss_ref <= LOSS_TOL
        sess.accumulate(True)
        _check_grads(sess, sess.acc, acc, model["d_model"], f"{what}: accumulated gradient", {RAW: raw}, "; ".join(notes))
        del raw
        sess.check_overflow(1.0 / (loss_scale * ntok_ref))
        assert int(sess.flag.item()) == flag_ref == 0
        sess.adam_step(lr, 1)
        check_master_weights(sess, master, f"{what}: master weights")
    finally:
        sess.close()


def _scaler_trace(model_name, batches, forced_at, what, init_scale=128.0, peak_lr=1e-3):
    """len(batches) consecutive updates (one sub-batch each) with dynamic loss scaling from `init_scale`,
    update number `forced_at` (0-based) forced to overflow by a loss scale 2^20 times larger: overflow flags,
    loss scale, clean-update counter and Adam's step count must equal the oracle's after every update, and a
    skipped update must leave master weights, moments and fp16 weights bit-identical."""
    import torch
    model = I.MODELS[model_name]
    weights = I.init_weights(seed=0, **model)
    cfg = _oracle_cfg(model)
    P16 = {k: v.astype(np.float64) for k, v in weights.items()}
    master = {k: v.copy() for k, v in P16.items()}
    om, ov = _zeros_like(P16), _zeros_like(P16)
    ref_scaler = O.LossScaler(init_scale)
    sess = Session(model, weights, max_sentences=max(b["src"].shape[0] for b in batches), max_len=256)
    try:
        tr = Trainer(sess, peak_lr=peak_lr, warmup=4000, init_scale=init_scale)
        w_now, t_ref = P16, 1
        flags_gpu, flags_ref, margins = [], [], []
        t0 = time.time()
        for it, batch in enumerate(batches):
            override_gpu = tr.scale * 2.0 ** 20 if it == forced_at else None
            override_ref = ref_scaler.scale * 2.0 ** 20 if it == forced_at else None
            before = [x.clone() for x in (sess.master, sess.m, sess.v, sess.w16)]
            t_before = tr.t
            assert tr.t == t_ref
            lr_ref = O.lr_schedule(t_ref, peak_lr, 4000)
            assert abs(tr.lr() - lr_ref) <= 1e-15
            loss, ntok, flag = tr.step([sess.to_device(batch)], scale_override=override_gpu)
            with np.errstate(over="ignore", invalid="ignore"):
                out = O.train_update(w_now, master, om, ov, cfg, [batch], ref_scaler, t=t_ref, lr=lr_ref, scale_override=override_ref,
                                     storage="fp16")
            flags_gpu.append(flag)
            flags_ref.append(out["flag"])
            # how far the largest finite accumulated element is from the fp16 limit (a decision within a few
            # percent of 1 would be one both sides may legitimately take differently)
            finite = [np.abs(v[np.isfinite(v)]).max() for v in out["acc"].values() if np.isfinite(v).any()]
            margins.append(float(max(finite)) / 65504.0 if not out["flag"] else float("inf"))
            assert flag == out["flag"], (what, "update", it, "gpu", flags_gpu, "oracle", flags_ref, margins)
            assert (tr.scale, tr.clean) == (ref_scaler.scale, ref_scaler.clean), (what, it)
            assert ntok == out["n_tok"]
            if out["flag"]:
                torch.cuda.synchronize()
                for a, b in zip(before, (sess.master, sess.m, sess.v, sess.w16)):
                    assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), (what, "update", it, "moved although skipped")
                assert tr.t == t_before
            else:
                t_ref += 1
                w_now = out["w16"]
                assert abs(loss - out["loss_sum"]) / out["loss_sum"] <= LOSS_TOL, (what, it, loss, out["loss_sum"])
        print(f"{what}: {len(batches)} updates, oracle + GPU took {time.time() - t0:.0f}s; flags {flags_gpu}, final loss scale {tr.scale}, "
              f"largest |accumulated gradient| / 65504 per applied update: {[round(m, 3) for m in margins if np.isfinite(m)]}", flush=True)
        assert flags_gpu[forced_at] == 1 and sum(flags_gpu) >= 1
        check_master_weights(sess, master, f"{what}: master weights after {len(batches)} updates")
        return flags_gpu, tr.scale
    finally:
        sess.close()


def test_transformer_base_twenty_updates_with_one_forced_overflow_follow_the_oracle_trace():
    """Configuration 3's trace on Transformer-base: 20 consecutive updates, dynamic loss scaling from 2^7, update
    8 forced to overflow.  (Sub-batches of <= 1792 tokens so that the oracle's 20 updates fit the test's
    time; the full 3584-token shape is covered by the single-update tests above and the trace on
    Transformer-big below.)"""
    buckets, src_len, tgt_len, rng = I.make_buckets("base", 20_000)
    model = I.MODELS["base"]
    half = I.bucket_by_tokens(src_len, tgt_len, 1792)
    pick = rng.integers(0, len(half), size=20)
    batches = [I.fill_batch(half[i], src_len, tgt_len, model["vocab"], rng) for i in pick]
    _scaler_trace("base", batches, forced_at=7, what="Transformer-base, 20-update loss-scaling trace")


def test_transformer_big_three_updates_with_one_forced_overflow_follow_the_oracle_trace():
    """The same on Transformer-big at the full 3584-token sub-batch size: three updates, the second forced to overflow."""
    batches = I.workload_batches("big", which="random", count=3, n_sentences=50_000)
    _scaler_trace("big", batches, forced_at=1, what="Transformer-big, 3-update loss-scaling trace", init_scale=32.0)


def test_bench_configuration_one_packed_pass_equals_sub_batches_one_by_one():
    """The launch configuration bench.py times: Transformer-big, all 16 sub-batches of an update as one
    packed pass.  The oracle cannot run 53k tokens of the big model in test time, so this checks the
    property that holds at any size: the pass must give the loss, token count and gradient of the 16
    sub-batches processed one by one through the path the tests above pin to the oracle, up to the
    rounding of one fp16 store per sub-batch (the one-by-one gradients) versus one per pass."""
    model = I.MODELS["big"]
    weights = I.init_weights(seed=0, **model)
    batches = I.workload_batches("big_accum", which="random", count=16, n_sentences=50_000)
    loss_scale, step = 1.0, 5
    sess = Session(model, weights, max_sentences=max(b["src"].shape[0] for b in batches), max_len=256)
    try:
        loss_1, ntok_1 = 0.0, 0
        for j, b in enumerate(batches):
            sess.forward_loss(sess.to_device(b), loss_scale, step, j)
            sess.backward()
            sess.accumulate(j == 0)
            loss_1 += float(sess.loss_sum.item())
            ntok_1 += int(sess.ntok.item())
        ref = sess.named(sess.acc)
        ref = {k: v.astype(np.float64) for k, v in ref.items()}
        (pk,) = sess.pack(batches)
        sess.forward_loss(pk, loss_scale, step)
        sess.backward()
        assert int(sess.ntok.item()) == ntok_1 == pk["n_tgt"]
        assert abs(float(sess.loss_sum.item()) - loss_1) / loss_1 <= 1e-4
        gs = sess.grad_scale()
        assert gs == 0.125                  # 52.7k target positions: three doublings beyond 8191
        got = {k: v.astype(np.float64) / gs for k, v in sess.named(sess.g16).items()}
        d = model["d_model"]
        errs = {}
        for name, w in ref.items():
            g = got[name].astype(np.float64).reshape(w.shape)
            assert np.isfinite(g).all(), name
            if name.endswith(("bqkv", "bkv")):      # the key-bias part is zero in exact arithmetic: compare the rest
                key = slice(d, 2 * d) if name.endswith("bqkv") else slice(0, d)
                rest = np.ones(w.shape[0], dtype=bool)
                rest[key] = False
                g, w = g[rest], w[rest]
            errs[name] = rel_l2(g, w)
            assert errs[name] <= 5e-3, (name, errs[name])
        print("packed pass of 16 sub-batches vs one by one: worst gradient rel-L2", max(errs.items(), key=lambda t: t[1]), flush=True)
        sess.accumulate(True)               # divides the factor out again
        acc = sess.named(sess.acc)
        assert all(rel_l2(acc[k].astype(np.float64), got[k]) <= 1e-6 for k in ref)
        # the attention work lists (query tiles, sentences by length class) and the persistent form only choose
        # which work-groups start: the same pass with the kernels enumerating every (sentence, tile), one work
        # item per work-group, and the weight gradients on the caller's stream gives the same bits
        import torch
        import paper_1806_00187_amd as A
        g_lists = sess.g16.clone()
        loss_lists = float(sess.loss_sum.item())
        try:
            for name in ("worklists", "attn_persist"):
                A.nmt_tuning(name, 0)
            A.nmt_tuning("one_stream", 1)
            sess.forward_loss(pk, loss_scale, step)
            sess.backward()
            torch.cuda.synchronize()
        finally:
            A.nmt_tuning("defaults")
        assert float(sess.loss_sum.item()) == loss_lists
        assert torch.equal(sess.g16.view(torch.int16), g_lists.view(torch.int16))
    finally:
        sess.close()
