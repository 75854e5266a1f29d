"""Helpers shared by the GPU parity tests: run the HIP path and the fp64 oracle on the same
seeded inputs and measure the differences.  (Test code: may import both sides.)"""
from __future__ import annotations

import json
import os

import numpy as np

import oracle
from paper_2502_12784_amd import synth

# Tolerances (fp16 / bf16 inputs): max-abs on O and LSE, relative L2 on the gradients.
#
# O.  Three figures are computed for every case and printed:
#   O_maxabs      raw max |O - O_ref|;
#   O_excess_ulp  max (|O - O_ref| - half_ulp_out(O_ref)): what is left once the unavoidable single
#                 rounding of the result to the 16-bit output type is set aside (up to |x| 2^-11 for
#                 fp16, up to |x| 2^-8 for bf16, which alone exceeds 2e-3 once |x| >= 0.5);
#   O_excess_op   the same with, in addition, the bound u * sum_j P_ij |V_jk| on what rounding P to the
#                 16-bit operand type of the second contraction (Sec. 3.2.2) can do to O_i (u = 2^-8
#                 for bf16's 8 significant bits; the oracle evaluates the sum exactly, a forward
#                 with |V|).
# Asserted:  fp16: O_excess_ulp <= 2e-3 (no operand term).  bf16: every element either meets that
# too, or meets O_excess_op <= 2e-3; the number of elements that needed the operand term is
# printed (O_needed_op) so that the looser reading is never used silently.
#
# Gradients: relative L2 per tensor, and a per-row check that one wrong row cannot hide in: for
# every (batch, head, row)  ||g_row - ref_row|| <= TOL_ROW * (||ref_row|| + ROW_FLOOR * rms row
# norm of the tensor), TOL_ROW = 2e-2 for fp16 and 5e-2 for bf16.  A row that is zero, stale or
# belongs to another row has an error of the order of its own norm: it fails unless its norm is
# below a tenth (fp16: a twentieth) of the typical row's.  The absolute part (ROW_FLOOR) is
# needed because the backward consumes the forward's 16-bit O: D = rowsum(dO o O) carries O's
# rounding, and in dS = P o (dP - D) that error does not shrink with the row.  The extreme case is
# causal row 0, whose exact dQ is zero (one key: dP = D); measured there: up to 0.047 x the rms
# row norm in bf16 (N = 4096, d = 128, with dropout), 0.002 in fp16.
TOL_ABS = 2e-3
TOL_REL_L2 = 1e-2
TOL_ROW = {synth.F16: 2e-2, synth.BF16: 5e-2}
ROW_FLOOR = 2.0


def half_ulp(x64: np.ndarray, dtype: str) -> np.ndarray:
    """Half a unit in the last place of the 16-bit output type at |x| (normal range)."""
    mant = 10 if dtype == synth.F16 else 7
    ax = np.abs(x64)
    min_exp = -14 if dtype == synth.F16 else -126
    e = np.floor(np.log2(np.maximum(ax, 2.0 ** min_exp)))
    return 0.5 * 2.0 ** (e - mant)


def to_device(bits: np.ndarray, dtype: str):
    import torch
    t = torch.from_numpy(bits.view(np.int16).copy()).cuda()
    return t.view(torch.float16 if dtype == synth.F16 else torch.bfloat16)


def to_f64(t) -> np.ndarray:
    import torch
    return t.detach().to(torch.float64).cpu().numpy()


def run_gpu(inp, dtype, scale, causal, dropout=None):
    """Forward then backward through the C ABI on the forward's own O and LSE.
    dropout: None or (p_drop, seed, offset) for the dropout entry points."""
    import torch
    from paper_2502_12784_amd import (spark_mha_bwd, spark_mha_cross_bwd, spark_mha_cross_fwd,
                                      spark_mha_dropout_bwd, spark_mha_dropout_fwd, spark_mha_fwd)
    Q, K, V, dO = (to_device(inp[n], dtype) for n in ("Q", "K", "V", "dO"))
    if dropout is not None:
        O, LSE = spark_mha_dropout_fwd(Q, K, V, scale, causal, *dropout)
        dQ, dK, dV = spark_mha_dropout_bwd(Q, K, V, O, LSE, dO, scale, causal, *dropout)
    elif K.shape != Q.shape:  # Nq != Nk: the cross-attention entry points
        O, LSE = spark_mha_cross_fwd(Q, K, V, scale, causal)
        dQ, dK, dV = spark_mha_cross_bwd(Q, K, V, O, LSE, dO, scale, causal)
    else:
        O, LSE = spark_mha_fwd(Q, K, V, scale, causal)
        dQ, dK, dV = spark_mha_bwd(Q, K, V, O, LSE, dO, scale, causal)
    torch.cuda.synchronize()
    return {"O": O, "LSE": LSE, "dQ": dQ, "dK": dK, "dV": dV}


def run_oracle(inp, dtype, scale, causal, heads=None, dropout=None):
    """Oracle on all heads, or on the flat head indices `heads` of [B,H,N,d] bit arrays.
    dropout: None or (threshold, seed, offset); the oracle draws the keep mask itself."""
    arrs = {}
    B, H, Nq, _ = inp["Q"].shape
    Nk = inp["K"].shape[2]
    keep, ks = None, 1.0
    if dropout is not None:
        thr, seed, offset = dropout
        keep = oracle.dropout_mask(B, H, Nq, Nk, seed, offset, thr)
        ks = 256.0 / (256 - thr)
        if heads is not None:
            keep = np.ascontiguousarray(keep.reshape(B * H, 1, Nq, Nk)[list(heads)])
    for n in ("Q", "K", "V", "dO"):
        a = inp[n]
        if heads is not None:
            B, H, N, d = a.shape
            a = a.reshape(B * H, 1, N, d)[list(heads)]
        arrs[n] = synth.bits_to_f64(a, dtype)
    # scale as the fp32 value the kernel receives
    s = float(np.float32(scale))
    ref = oracle.mha_bwd(arrs["Q"], arrs["K"], arrs["V"], arrs["dO"], s, causal, keep, ks)
    # bound on the effect of rounding P to the 16-bit operand type: u * P |V|
    # (bf16 only: fp16 cases are held to 2e-3 + half an output ulp without it)
    if dtype == synth.BF16:
        ref["O_operand_rounding"] = 2.0 ** -8 * oracle.mha_fwd(arrs["Q"], arrs["K"], np.abs(arrs["V"]), s,
                                                               causal, False, keep, ks)[0]
    return ref


def compare(gpu, ref, dtype, heads=None):
    """Return error measures; `heads` selects flat heads of the GPU tensors to match `ref`."""
    out = {"dtype": dtype}

    def pick(t):
        a = to_f64(t)
        if heads is not None:
            a = a.reshape((-1, 1) + a.shape[2:])[list(heads)]
        return a

    o_gpu, o_ref = pick(gpu["O"]), ref["O"]
    err = np.abs(o_gpu - o_ref)
    out["O_maxabs"] = float(err.max())
    over_ulp = err - half_ulp(o_ref, dtype)
    out["O_excess_ulp"] = float(over_ulp.max())
    out["O_excess_op"] = float((over_ulp - ref.get("O_operand_rounding", 0.0)).max())
    out["O_needed_op"] = int((over_ulp > TOL_ABS).sum())
    out["O_elems"] = int(err.size)
    out["LSE_maxabs"] = float(np.abs(pick(gpu["LSE"]) - ref["LSE"]).max())
    for n in ("dQ", "dK", "dV"):
        g, r = pick(gpu[n]), ref[n]
        rn = np.linalg.norm(r)
        if rn < 1e-9 * np.sqrt(r.size):
            # degenerate case with an exactly zero gradient (e.g. one key: dS = 0): compare the
            # RMS error with a unit-scale gradient instead of dividing by zero
            rn = np.sqrt(r.size)
            row_rms = np.sqrt(r.shape[-1])
        else:
            row_rms = rn / np.sqrt(r.size / r.shape[-1])
        out[n + "_relL2"] = float(np.linalg.norm(g - r) / rn)
        out[n + "_finite"] = bool(np.isfinite(g).all())
        row_err = np.linalg.norm(g - r, axis=-1)
        row_ref = np.linalg.norm(r, axis=-1)
        ratio = row_err / (row_ref + ROW_FLOOR * row_rms)
        out[n + "_row"] = float(ratio.max())
        worst = np.unravel_index(int(ratio.argmax()), ratio.shape)
        out[n + "_row_at"] = [int(x) for x in worst]  # (batch or sampled head, head, row)
        out[n + "_row_at_ref"] = float(row_ref[worst] / row_rms)  # that row's norm / rms row norm
        out[n + "_row_at_err"] = float(row_err[worst] / row_rms)
    log = os.environ.get("SPARK_PARITY_LOG")
    if log:
        with open(log, "a") as f:
            f.write(json.dumps(out) + "\n")
    return out


def assert_within_tolerance(m, label=""):
    if m["dtype"] == synth.F16:
        assert m["O_excess_ulp"] <= TOL_ABS, (label, m)
    else:
        assert m["O_excess_op"] <= TOL_ABS, (label, m)
        if m["O_needed_op"]:
            print("[parity] %s: %d of %d elements of O exceed 2e-3 + half an output ulp and are "
                  "within the bf16 operand-rounding bound" % (label, m["O_needed_op"], m["O_elems"]))
    assert m["LSE_maxabs"] <= TOL_ABS, (label, m)
    for n in ("dQ", "dK", "dV"):
        assert m[n + "_finite"], (label, m)
        assert m[n + "_relL2"] <= TOL_REL_L2, (label, m)
        assert m[n + "_row"] <= TOL_ROW[m["dtype"]], (label, m)
