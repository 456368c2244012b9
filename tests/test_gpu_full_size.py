"""Parity at the benchmark's full sizes: Transformer-big on one real sub-batch of the synthetic
workload (the shape bench.py times), and the long-sequence tail on Transformer-base.  The fp64
oracle runs the same sub-batch on the host (about a minute for the big model), every gradient
tensor is compared."""
import time

import numpy as np
import pytest

import nmt_inputs as I
from oracle import nmt_oracle as O
from paper_1806_00187_amd.session import Session
from tests.test_gpu_step import GRAD_TOL, LOSS_TOL, _check_grads, _gate_allowance, _oracle_cfg

pytestmark = pytest.mark.gpu


def _full_size_case(model_name, batch, loss_scale, draws):
    model = I.MODELS[model_name]
    weights = I.init_weights(seed=0, **model)
    cfg = _oracle_cfg(model)
    P16 = {k: v.astype(np.float64) for k, v in weights.items()}
    B, S = batch["src"].shape
    T = batch["tgt_in"].shape[1]
    t0 = time.time()
    loss_ref, ntok_ref, cache = O.forward_loss(P16, cfg, batch["src"], batch["tgt_in"], batch["tgt_out"], training=True, step=7, micro=3)
    g_exact = O.backward(P16, cfg, cache, loss_scale)
    g16_ref = O.to_fp16_storage(g_exact)
    allow = _gate_allowance(P16, cfg, cache, loss_scale, g_exact, draws=draws)
    print(f"{model_name} (B,S,T)=({B},{S},{T}): oracle took {time.time() - t0:.0f}s", flush=True)
    flag_ref, _ = O.check_overflow(g16_ref, 1.0)
    # the same step with the loss scaled up by 2^20: gradients scale exactly (power of two)
    big = O.to_fp16_storage({k: v * 2.0 ** 20 for k, v in g_exact.items()})
    flag_forced_ref, _ = O.check_overflow(big, 1.0)
    del cache, big

    sess = Session(model, weights, max_sentences=B, max_len=256)
    db = sess.to_device(batch)
    sess.forward_loss(db, loss_scale, 7, 3)
    sess.backward()
    loss, ntok = float(sess.loss_sum.item()), int(sess.ntok.item())
    assert ntok == ntok_ref
    assert abs(loss - loss_ref) / loss_ref <= LOSS_TOL, (loss, loss_ref)
    worst = _check_grads(sess, sess.g16, g16_ref, model["d_model"], f"{model_name} g16", allow)
    print(f"{model_name}: loss {loss / ntok:.4f}/token (oracle {loss_ref / ntok_ref:.4f}), worst gradient rel-L2 {worst}", flush=True)
    sess.accumulate(True)
    sess.check_overflow(1.0 / (loss_scale * ntok))
    assert int(sess.flag.item()) == flag_ref == 0
    # overflow decision of the forced step
    sess.forward_loss(db, loss_scale * 2.0 ** 20, 7, 3)
    sess.backward()
    sess.accumulate(True)
    sess.check_overflow(1.0)
    assert int(sess.flag.item()) == flag_forced_ref == 1
    sess.close()


def test_transformer_big_sub_batch_matches_oracle():
    batch = I.workload_batches("big", which="median", count=1, n_sentences=50_000)[0]
    _full_size_case("big", batch, loss_scale=32.0, draws=2)


def test_transformer_base_long_sequences_match_oracle():
    # the longest bucket of the length distribution (sequences of ~250 tokens, few sentences)
    buckets, src_len, tgt_len, rng = I.make_buckets("base", 50_000)
    model = I.MODELS["base"]
    batch = I.fill_batch(buckets[-1], src_len, tgt_len, model["vocab"], rng)
    assert max(batch["src"].shape[1], batch["tgt_in"].shape[1]) > 200
    _full_size_case("base", batch, loss_scale=32.0, draws=2)
