"""Helpers for the GPU parity tests."""
import numpy as np
import torch

DEV = "cuda:0"

# Every gradient / weight comparison against the oracle leaves its figures here; tests/conftest.py prints
# them at the end of the run (also under -q) and writes them to parity_summary.json in the run's output folder
# (NMT_TEST_OUTPUT_DIR, or the folder tests/conftest.py defaults to).
PARITY = []


def _digest(e):
    name, worst = max(e.items(), key=lambda t: t[1])
    vals = sorted(e.values())
    return {"worst": float(worst), "worst_tensor": name, "median": float(vals[len(vals) // 2]),
            "above_2e-2": {k: round(float(v), 5) for k, v in sorted(e.items()) if v > 2e-2}}


def record_parity(case, errs, also=None, note=None):
    """case: what was compared; errs: dict tensor name -> relative L2 error against the reference the test
    asserts on; also: dict label -> such a dict against other references (recorded, not asserted)."""
    rec = {"case": case, "tensors": len(errs), "asserted": _digest(errs)}
    for label, e in (also or {}).items():
        rec[label] = _digest(e)
    if note:
        rec["note"] = note
    PARITY.append(rec)


def dev16(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float16)).to(DEV)


def dev32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def devi(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.detach().cpu().numpy().astype(np.float64)


def rel_l2(got, want):
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30))


def f16(a):
    """Values after fp16 storage, as float64."""
    return np.asarray(a).astype(np.float16).astype(np.float64)


def assert_close16(got, want, what, rel=1.5e-3, l2=6e-4):
    """fp16-result check: relative L2 error of the whole tensor and an element-wise bound of a few
    fp16 ulps relative to max(|want|, tensor rms)."""
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.isfinite(got).all(), what
    e = rel_l2(got, want)
    assert e <= l2, (what, "rel l2", e)
    rms = float(np.sqrt((want ** 2).mean()))
    bound = rel * np.maximum(np.abs(want), rms) + 1e-7
    worst = float((np.abs(got - want) / bound).max())
    assert worst <= 1.0, (what, "worst element error / bound", worst)
