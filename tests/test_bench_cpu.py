"""bench.py's host-side pieces that need no GPU: flop / byte accounting behind the tables, and the
rule that measured HBM traffic is quoted only while the kernel sources match the profile's digest."""
import os
import shutil

import pytest

import bench
from paper_2502_12784_amd import synth


def test_counted_flops_and_hbm_floor():
    w = synth.WORKLOADS["C4"]  # B=4 H=16 N=4096 d=128 causal
    assert w.fwd_flops == 4 * 4 * 16 * 4096 ** 2 * 128 / 2
    assert w.bwd_flops == 2.5 * w.fwd_flops
    t = 4 * 16 * 4096 * 128 * 2
    us, by = bench.hbm_floor_us(w, "fwd")
    assert by == 4 * t + 4 * 16 * 4096 * 4
    assert us == pytest.approx(by / 8e12 * 1e6)
    us_b, by_b = bench.hbm_floor_us(w, "bwd")
    assert by_b == 8 * t + 5 * 4 * 16 * 4096 * 4 and us_b > us


def test_config_table_figures():
    w = synth.WORKLOADS["C5"]
    k = {"fwd": 0.5, "bwd_dq": 0.75, "bwd_dkdv": 1.0}
    text = bench.config_table([("C5", w, 2.5, k)], "cmd")
    row = [l for l in text.splitlines() if l.startswith("C5")][0]
    cells = [c.split() for c in row.split("|")]
    assert float(cells[1][0]) == 500.0                                   # fwd us
    assert float(cells[1][1]) == pytest.approx(w.fwd_flops / 0.5e-3 / 1e12, abs=0.06)
    assert float(cells[2][0]) == 1750.0                                  # bwd us = dQ + dK/dV
    assert float(cells[3][1]) == pytest.approx((w.fwd_flops + w.bwd_flops) / 2.5e-3 / 1e12, abs=0.06)
    assert float(cells[3][2]) == pytest.approx(100 * (w.fwd_flops + w.bwd_flops) / 2.5e-3 / 1e12 / 2500, abs=0.06)


def test_traffic_is_quoted_only_for_matching_sources(tmp_path, monkeypatch):
    root = tmp_path
    csrc = root / "paper_2502_12784_amd" / "csrc"
    csrc.mkdir(parents=True)
    (csrc / "a.hpp").write_text("// kernel v1\n")
    (root / "profiles").mkdir()
    monkeypatch.setattr(bench, "ROOT", str(root))
    digest = bench.csrc_digest()
    (root / "profiles" / "hbm_traffic_C4.txt").write_text(
        "header\ncsrc_sha256: %s\nbwd_dkdv traffic_bytes_per_launch: 4.05e+08\n" % digest)
    assert bench.read_traffic("C4", "bwd_dkdv") == 4.05e8
    assert bench.read_traffic("C4", "fwd") is None          # no such line
    assert bench.read_traffic("C5", "bwd_dkdv") is None     # no such file
    (csrc / "a.hpp").write_text("// kernel v2\n")           # the kernels changed: the figure is stale
    assert bench.csrc_digest() != digest
    assert bench.read_traffic("C4", "bwd_dkdv") is None


def test_committed_traffic_profiles_carry_a_digest():
    prof = os.path.join(os.path.dirname(os.path.abspath(bench.__file__)), "profiles")
    for name in os.listdir(prof):
        if name.startswith("hbm_traffic_"):
            assert "csrc_sha256" in open(os.path.join(prof, name)).read(), name
