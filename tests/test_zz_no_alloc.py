"""The entry point that allocates nothing: column sums with the partial sums in the library's fixed device
array, against the entry point that takes a caller-provided scratch buffer (same kernels, so the bits
must be equal), on two calls in a row, the second with a smaller input, and the size limit."""
import numpy as np
import pytest
import torch

import paper_1806_00187_amd as A
from tests.gpu_util import DEV

pytestmark = pytest.mark.gpu


def _both(rows, cols, ld, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    src = (torch.randn(rows, ld, generator=g) * 3).to(torch.float16).to(DEV)
    part = torch.full((A.nmt_op_colsum_scratch(cols),), float("nan"), dtype=torch.float32, device=DEV)
    want = torch.full((cols,), float("nan"), dtype=torch.float16, device=DEV)
    got = torch.full((cols,), float("nan"), dtype=torch.float16, device=DEV)
    A.nmt_op_colsum(src, ld, want, part, rows, cols)
    A.nmt_op_colsum_static(src, ld, got, rows, cols)
    torch.cuda.synchronize()
    return got, want, src


def test_colsum_static_equals_colsum_on_two_calls_in_a_row_the_second_smaller():
    for rows, cols, ld, seed in ((5003, 4096, 4096, 1), (777, 1032, 1040, 2), (40000, 3072, 3072, 3), (9, 8, 8, 4)):
        got, want, src = _both(rows, cols, ld, seed)
        assert torch.isfinite(want).all()
        assert torch.equal(got.view(torch.int16), want.view(torch.int16)), (rows, cols)
        ref = src[:, :cols].double().sum(0).cpu().numpy()
        err = np.abs(got.double().cpu().numpy() - ref)
        assert (err <= 1e-3 * np.abs(ref) + 0.3).all(), (rows, cols, err.max())


def test_colsum_static_rejects_what_the_fixed_array_cannot_hold():
    src = torch.zeros(4, 4104, dtype=torch.float16, device=DEV)
    dst = torch.zeros(4104, dtype=torch.float16, device=DEV)
    with pytest.raises(A.NmtError) as e:
        A.nmt_op_colsum_static(src, 4104, dst, 4, 4104)
    assert e.value.code == A.NMT_EINVAL and "4096" in str(e.value)
