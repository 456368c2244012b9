"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its host
logic (parameter layout, workspace sizing, scaler, schedule, argument validation) is right."""
import os
import re

import numpy as np
import pytest

import nmt_inputs as I
import paper_1806_00187_amd as A
from oracle import nmt_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _cfg(model, **kw):
    base = dict(enc_layers=model["enc_layers"], dec_layers=model["dec_layers"], d_model=model["d_model"],
                n_heads=model["n_heads"], d_ff=model["d_ff"], vocab=model["vocab"], pad_id=1, dropout=model.get("dropout", 0.0),
                act_dropout=0.0, label_smoothing=0.1, ln_eps=1e-5, seed=0, max_sentences=1024, max_len=256)
    base.update(kw)
    return base


def test_library_exports_every_declared_symbol():
    lib = A.load()
    header = open(os.path.join(ROOT, "include", "nmt.h")).read()
    declared = set(re.findall(r"\b(nmt_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(A.exported_symbols())


@pytest.mark.parametrize("name", ["tiny", "base", "big", "big40k"])
def test_parameter_layout_matches_the_model_description(name):
    model = I.MODELS[name]
    ctx = A.nmt_create(**_cfg(model))
    try:
        shapes = I.param_shapes(**model)
        assert A.nmt_param_tensors(ctx) == len(shapes)
        off = 0
        for i, (pname, shape) in enumerate(shapes):
            got = A.nmt_param_info(ctx, i)
            rows, cols = (shape if len(shape) == 2 else (1, shape[0]))
            assert got == (pname, off, rows, cols)
            assert off % 8 == 0
            off += rows * cols
        assert A.nmt_param_count(ctx) == off == I.param_count(**model)
    finally:
        A.nmt_destroy(ctx)


def test_big_model_has_the_papers_parameter_count():
    ctx = A.nmt_create(**_cfg(I.MODELS["big"]))
    assert round(A.nmt_param_count(ctx) / 1e6) == 210      # "210M parameters"
    A.nmt_destroy(ctx)


def test_workspace_grows_with_the_batch_and_rejects_bad_shapes():
    ctx = A.nmt_create(**_cfg(I.MODELS["tiny"], max_sentences=16, max_len=32))
    a, b = A.nmt_workspace_bytes(ctx, 8, 16, 16), A.nmt_workspace_bytes(ctx, 16, 32, 32)
    assert 0 < a < b
    for bad in ((0, 4, 4), (17, 4, 4), (4, 33, 4), (4, 4, 0)):
        with pytest.raises(A.NmtError):
            A.nmt_workspace_bytes(ctx, *bad)
    A.nmt_destroy(ctx)


@pytest.mark.parametrize("bad", [dict(d_model=60), dict(n_heads=3), dict(vocab=1001), dict(dropout=1.0), dict(max_len=4096),
                                 dict(d_ff=10), dict(pad_id=-1), dict(ln_eps=0.0), dict(attn_dropout=0.1)])
def test_create_rejects_invalid_configurations(bad):
    with pytest.raises(A.NmtError) as e:
        A.nmt_create(**_cfg(I.MODELS["tiny"], **bad))
    assert e.value.code == A.binding.NMT_EINVAL


def test_calls_out_of_order_fail_cleanly():
    ctx = A.nmt_create(**_cfg(I.MODELS["tiny"]))
    lib = A.load()
    assert lib.nmt_backward(ctx, None) == A.binding.NMT_ESTATE
    assert lib.nmt_accumulate(ctx, 1, None) == A.binding.NMT_EINVAL          # nothing bound
    assert b"not bound" in lib.nmt_last_error()
    A.nmt_destroy(ctx)


def test_scaler_matches_the_oracle_trace():
    rng = np.random.default_rng(0)
    ref = O.LossScaler(128.0, window=50)
    scale, clean = 128.0, 0
    for i in range(2000):
        ov = bool(rng.random() < 0.01)
        ref.update(ov)
        scale, clean = A.nmt_scaler_update(scale, clean, ov, 50)
        assert (scale, clean) == (ref.scale, ref.clean)
    with pytest.raises(A.NmtError):
        A.nmt_scaler_update(2.0 ** -14, 0, True, 50)


def test_paper_scaler_window():
    scale, clean = 128.0, 0
    for _ in range(1999):
        scale, clean = A.nmt_scaler_update(scale, clean, False)
    assert (scale, clean) == (128.0, 1999)
    assert A.nmt_scaler_update(scale, clean, False) == (256.0, 0)      # up after 2000 clean updates
    assert A.nmt_scaler_update(256.0, 77, True) == (128.0, 0)          # down on overflow


def test_lr_schedule_matches_the_oracle():
    for t in (1, 17, 3999, 4000, 4001, 16000, 10 ** 6):
        assert A.nmt_lr_schedule(t, 1e-3) == pytest.approx(O.lr_schedule(t, 1e-3), rel=1e-15)
    assert A.nmt_lr_schedule(4000, 5e-4) == 5e-4


def test_tuning_switches_accept_their_names_and_reject_others():
    for name, value in (("gemm_group", 3), ("gemm_persist", 0), ("attn_persist", 0), ("worklists", 0), ("one_stream", 1), ("gemm_share", 4), ("gemm_tile", 3), ("defaults", 0)):
        A.nmt_tuning(name, value)
    assert A.binding.tuning_value("gemm_share", 1) == 1 and A.binding.tuning_value("one_stream", 0) == 0   # "defaults" forgets what was set
    A.nmt_tuning("gemm_share", 2)
    assert A.binding.tuning_value("gemm_share", 1) == 2
    A.nmt_tuning("defaults")
    for name, value in (("gemm_group", 0), ("gemm_persist", 2), ("gemm_share", 0), ("gemm_share", 17), ("gemm_tile", 6), ("no_such_switch", 1)):
        with pytest.raises(A.NmtError) as e:
            A.nmt_tuning(name, value)
        assert e.value.code == A.binding.NMT_EINVAL


def test_loss_totals_need_a_forward_call():
    ctx = A.nmt_create(**_cfg(I.MODELS["tiny"]))
    lib = A.load()
    import ctypes as C
    buf = (C.c_float * 1)()
    cnt = (C.c_int32 * 1)()
    assert lib.nmt_accumulate_loss(ctx, 1, C.cast(buf, C.c_void_p), C.cast(cnt, C.c_void_p), None) == A.binding.NMT_ESTATE
    A.nmt_destroy(ctx)
