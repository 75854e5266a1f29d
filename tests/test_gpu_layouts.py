"""Freezes the register layouts the kernels are written against: the library's self-check runs
small integer matrix products through the documented MFMA operand / accumulator layouts, the
accumulator-as-operand reuse and the transposing LDS read; the same products are formed here in
numpy from the patterns the header states.  Everything is exact, so the comparison is too."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _expected():
    i = np.arange(32)[:, None]
    k16 = np.arange(16)[None, :]
    A1 = (37 * i + 11 * k16 + (i * k16) % 7) % 3 - 1                 # 32 x 16
    k = np.arange(16)[:, None]
    j = np.arange(32)[None, :]
    B1 = (29 * k + 13 * j + (k * j) % 5) % 5 - 2                     # 16 x 32
    C1 = A1 @ B1
    r = np.arange(32)[None, :]
    A2 = (17 * i + 7 * r + (i * r) % 11) % 7 - 3                     # 32 x 32
    C2 = A2 @ C1
    tr = np.empty((64, 4))
    for lane in range(64):
        q, ii = divmod(lane, 16)
        for t in range(4):
            tr[lane, t] = 64 * (4 * q + t) + 16 + ii
    return C1.astype(np.float64), C2.astype(np.float64), tr


@pytest.mark.parametrize("dtype_code", [0, 1])
def test_mfma_and_transposing_read_layouts(dtype_code):
    import torch
    from paper_2502_12784_amd import spark_layout_probe
    out = spark_layout_probe(dtype_code)
    torch.cuda.synchronize()
    out = out.cpu().numpy().astype(np.float64)
    C1, C2, tr = _expected()
    assert np.abs(C1).max() <= 32 and len(np.unique(C1)) > 20       # a real test pattern, exact in bf16
    assert np.array_equal(out[:1024].reshape(32, 32), C1)
    assert np.array_equal(out[1024:2048].reshape(32, 32), C2)
    assert np.array_equal(out[2048:].reshape(64, 4), tr)
