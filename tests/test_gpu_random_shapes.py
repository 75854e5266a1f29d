"""GPU parity on seeded random problems: batch, heads, both lengths, head size, dtype, mask,
dropout rate and tensor layout are drawn together, so that combinations no hand-written case
lists are exercised.  Every element of every output is compared with the oracle (same bar as
the other parity tests).  The draws are fixed by the seeds below.
"""
import math

import numpy as np
import pytest

from paper_2502_12784_amd import synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _draw(seed):
    r = np.random.default_rng(seed)
    # the paper's two head sizes for the first 40 seeds, any supported one afterwards
    d = int(r.choice([64, 128])) if seed < 3040 else 8 * int(r.integers(1, 17))
    dtype = [synth.F16, synth.BF16][int(r.integers(2))]
    causal = bool(r.integers(2))
    B, H = int(r.integers(1, 4)), int(r.integers(1, 5))
    Nq = int(r.choice([1, 2, 31, 32, 33, 63, 64, 65, 100, 127, 128, 129, 191, 200, 255, 256, 257, 300, 400, 511]))
    Nk = Nq if causal or r.integers(2) else int(r.choice([1, 7, 32, 64, 96, 130, 200, 257, 384, 500]))
    p = float(r.choice([0.0, 0.0, 0.1, 0.25, 0.5]))
    layout = str(r.choice(["bhnd", "bnhd", "padded"]))
    scale = float(r.choice([1.0 / math.sqrt(d), 0.05, 0.3]))
    return dict(B=B, H=H, Nq=Nq, Nk=Nk, d=d, dtype=dtype, causal=causal, p=p, layout=layout, scale=scale)


def _lay_out(t, layout):
    """The same [B,H,N,d] values in another memory layout (a view with other strides)."""
    import torch
    if layout == "bhnd":
        return t
    if layout == "bnhd":
        return t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    pad = torch.zeros(t.shape[:3] + (t.shape[3] + 16,), dtype=t.dtype, device=t.device)
    v = pad[..., :t.shape[3]]
    v.copy_(t)
    return v


@pytest.mark.parametrize("seed", list(range(3000, 3064)))
def test_random_problem(seed):
    import torch
    from paper_2502_12784_amd import spark_dropout_threshold, spark_mha_strided_bwd, spark_mha_strided_fwd
    c = _draw(seed)
    print(f"\n[random] seed={seed} {c}", flush=True)
    inp = synth.make_inputs(c["B"], c["H"], c["Nq"], c["d"], c["dtype"], seed=seed,
                            Nk=None if c["Nk"] == c["Nq"] else c["Nk"])
    Q, K, V, dO = (_lay_out(pu.to_device(inp[n], c["dtype"]), c["layout"]) for n in ("Q", "K", "V", "dO"))
    drop = (c["p"], seed * 7919 + 1, seed % 5)
    O, LSE = spark_mha_strided_fwd(Q, K, V, c["scale"], c["causal"], *drop)
    dQ, dK, dV = spark_mha_strided_bwd(Q, K, V, O, LSE, dO, c["scale"], c["causal"], *drop)
    torch.cuda.synchronize()
    gpu = {"O": O.contiguous(), "LSE": LSE, "dQ": dQ.contiguous(), "dK": dK.contiguous(), "dV": dV.contiguous()}
    thr = spark_dropout_threshold(c["p"])
    ref = pu.run_oracle(inp, c["dtype"], c["scale"], c["causal"],
                        dropout=None if thr == 0 else (thr, drop[1], drop[2]))
    m = pu.compare(gpu, ref, c["dtype"])
    print(f"[random] {m}", flush=True)
    pu.assert_within_tolerance(m, (seed, c))
