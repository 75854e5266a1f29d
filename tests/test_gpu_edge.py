"""GPU tests beyond plain parity: argument errors with real device buffers, odd scales, many
heads, a non-default stream, backward fed with the oracle's forward, reuse of caller buffers."""
import math

import numpy as np
import pytest

from paper_2502_12784_amd import synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu


def _dev_inputs(B, H, N, d, dtype, seed, sigma_qk=1.0):
    inp = synth.make_inputs(B, H, N, d, dtype, seed, sigma_qk=sigma_qk)
    return inp, {n: pu.to_device(inp[n], dtype) for n in inp}


@pytest.mark.parametrize("scale", [0.02, 0.3, 1.0])
@pytest.mark.parametrize("causal", [False, True])
def test_other_scales(scale, causal):
    B, H, N, d, dtype = 1, 2, 192, 64, synth.F16
    inp = synth.make_inputs(B, H, N, d, dtype, seed=515)
    gpu = pu.run_gpu(inp, dtype, scale, causal)
    ref = pu.run_oracle(inp, dtype, scale, causal)
    m = pu.compare(gpu, ref, dtype)
    print(f"\n[parity] scale={scale} causal={causal}: {m}", flush=True)
    pu.assert_within_tolerance(m, ("scale", scale, causal))


@pytest.mark.parametrize("dtype,d", [(synth.F16, 64), (synth.BF16, 128)])
def test_many_heads_and_batches(dtype, d):
    B, H, N = 3, 5, 160
    inp = synth.make_inputs(B, H, N, d, dtype, seed=77)
    gpu = pu.run_gpu(inp, dtype, 1.0 / math.sqrt(d), True)
    ref = pu.run_oracle(inp, dtype, 1.0 / math.sqrt(d), True)
    pu.assert_within_tolerance(pu.compare(gpu, ref, dtype), (B, H, N, d, dtype))


def test_peaked_softmax_moves_the_reference_often():
    """Logits with std 8: the running maximum jumps by more than the lazy-rescale threshold
    many times, so the rescale path of the online softmax is exercised."""
    B, H, N, d, dtype = 1, 2, 640, 64, synth.F16
    inp = synth.make_inputs(B, H, N, d, dtype, seed=9, sigma_qk=math.sqrt(8.0))
    gpu = pu.run_gpu(inp, dtype, 0.125, False)
    ref = pu.run_oracle(inp, dtype, 0.125, False)
    m = pu.compare(gpu, ref, dtype)
    print(f"\n[parity] peaked: {m}", flush=True)
    pu.assert_within_tolerance(m, "peaked")


@pytest.mark.parametrize("dtype,d,causal", [(synth.F16, 64, False), (synth.BF16, 128, True)])
def test_backward_on_oracle_forward(dtype, d, causal):
    """spark_mha_bwd alone, fed with the oracle's O (rounded to the storage type) and LSE:
    localises a backward error independently of the forward kernel."""
    import torch
    from paper_2502_12784_amd import spark_mha_bwd
    B, H, N = 1, 2, 320
    scale = 1.0 / math.sqrt(d)
    inp, dev = _dev_inputs(B, H, N, d, dtype, seed=4321)
    ref = pu.run_oracle(inp, dtype, scale, causal)
    O = pu.to_device(synth.round_to_bits(ref["O"].astype(np.float32), dtype), dtype)
    LSE = torch.from_numpy(ref["LSE"].astype(np.float32)).cuda()
    dQ, dK, dV = spark_mha_bwd(dev["Q"], dev["K"], dev["V"], O, LSE, dev["dO"], scale, causal)
    torch.cuda.synchronize()
    for name, g in (("dQ", dQ), ("dK", dK), ("dV", dV)):
        rel = np.linalg.norm(pu.to_f64(g) - ref[name]) / np.linalg.norm(ref[name])
        assert rel <= pu.TOL_REL_L2, (name, rel)


def test_non_default_stream_and_caller_buffers():
    """Work is enqueued on the stream that is current at the call; outputs and workspace the
    caller passes are used as they are, and calls can be repeated on them."""
    import torch
    from paper_2502_12784_amd import spark_mha_bwd, spark_mha_fwd
    from paper_2502_12784_amd.binding import _dtype_code, spark_mha_bwd_workspace_bytes
    B, H, N, d, dtype = 2, 2, 256, 128, synth.BF16
    scale = 1.0 / math.sqrt(d)
    inp, dev = _dev_inputs(B, H, N, d, dtype, seed=31)
    ref = pu.run_oracle(inp, dtype, scale, True)
    O = torch.full_like(dev["Q"], float("nan"))
    LSE = torch.full((B, H, N), float("nan"), dtype=torch.float32, device="cuda")
    dQ, dK, dV = (torch.full_like(dev["Q"], float("nan")) for _ in range(3))
    ws = torch.empty(spark_mha_bwd_workspace_bytes(B, H, N, d, _dtype_code(dev["Q"])), dtype=torch.uint8, device="cuda")
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        for _ in range(2):  # the second call overwrites the first one's results completely
            spark_mha_fwd(dev["Q"], dev["K"], dev["V"], scale, True, O=O, LSE=LSE)
            spark_mha_bwd(dev["Q"], dev["K"], dev["V"], O, LSE, dev["dO"], scale, True, dQ=dQ, dK=dK, dV=dV,
                          workspace=ws)
    st.synchronize()
    m = pu.compare({"O": O, "LSE": LSE, "dQ": dQ, "dK": dK, "dV": dV}, ref, dtype)
    pu.assert_within_tolerance(m, "stream")


def test_errors_leave_outputs_untouched():
    """Bad arguments with real device buffers: an error code comes back and nothing ran."""
    import torch
    from paper_2502_12784_amd import SparkError, load_library, spark_mha_bwd, spark_mha_fwd
    B, H, N, d, dtype = 1, 1, 128, 64, synth.F16
    _, dev = _dev_inputs(B, H, N, d, dtype, seed=5)
    lib = load_library()
    O = torch.full_like(dev["Q"], 7.0)
    LSE = torch.full((B, H, N), 7.0, dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    args = [dev["Q"].data_ptr(), dev["K"].data_ptr(), dev["V"].data_ptr(), O.data_ptr(), LSE.data_ptr()]
    assert lib.spark_mha_fwd(*args, B, H, N, 100, 0.125, 0, 0, st) == -2        # head dim
    assert lib.spark_mha_fwd(*args, B, H, N, d, -0.125, 0, 0, st) == -2       # scale
    assert lib.spark_mha_fwd(*args, B, H, N, d, 0.125, 0, 5, st) == -3        # dtype
    assert lib.spark_mha_fwd(args[0] + 2, *args[1:], B, H, N, d, 0.125, 0, 0, st) == -4  # alignment
    torch.cuda.synchronize()
    assert bool((O == 7.0).all()) and bool((LSE == 7.0).all())
    O, LSE = spark_mha_fwd(dev["Q"], dev["K"], dev["V"], 0.125, False)
    dQ = torch.full_like(dev["Q"], 7.0)
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(SparkError) as e:
        spark_mha_bwd(dev["Q"], dev["K"], dev["V"], O, LSE, dev["dO"], 0.125, False, dQ=dQ, workspace=small)
    assert e.value.status == -5
    torch.cuda.synchronize()
    assert bool((dQ == 7.0).all())


def test_bitwise_reproducible_d128():
    import torch
    inp = synth.make_inputs(1, 3, 700, 128, synth.BF16, 1234)
    a = pu.run_gpu(inp, synth.BF16, 0.09, True)
    b = pu.run_gpu(inp, synth.BF16, 0.09, True)
    for n in ("O", "LSE", "dQ", "dK", "dV"):
        assert torch.equal(a[n], b[n]), n
