"""Compile the HIP sources into ``libspark_mha.so`` next to this file (gfx950 only)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libspark_mha.so")
SOURCES = [os.path.join(CSRC, "spark_mha.hip")]
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # a rule for the test machines: never let the compiler form packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + SOURCES + ["-o", tmp]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, LIB)
    return LIB


MIX_BENCH = os.path.join(HERE, "mix_floor_bench")


def build_mix_floor_bench() -> str:
    """The stand-alone microbenchmark csrc/mix_floor_bench.hip (what the instruction mix of each
    attention loop costs as a straight-line loop on this GPU); run the executable on the GPU."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    res = subprocess.run([hipcc] + flags + [os.path.join(CSRC, "mix_floor_bench.hip"), "-o", MIX_BENCH],
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    return MIX_BENCH


def device_assembly():
    """(assembly text, compiler remarks) of the library's device code; nothing is written next to
    the sources."""
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    with tempfile.TemporaryDirectory() as tmp:
        cmd = [hipcc] + flags + ["--cuda-device-only", "-S", "-Rpass-analysis=kernel-resource-usage"] + SOURCES
        res = subprocess.run(cmd + ["-o", os.path.join(tmp, "out.s")], stdout=subprocess.PIPE,
                             stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + res.stdout)
        return open(os.path.join(tmp, "out.s")).read(), res.stdout


def unguarded_lds_loads(asm: str):
    """Direct global->LDS loads in the assembly that are not immediately preceded by the s_nop 4 hazard
    guard (see BufView::load16_to_lds): the compiler cannot see those loads, so nothing else
    separates them from a VALU write of the scalar registers they read.  Returns the offending lines."""
    import re
    lines = [l.strip() for l in asm.split("\n") if l.startswith("\t") and not l.strip().startswith((".", ";"))]
    return [l for prev, l in zip(lines, lines[1:])
            if re.match(r"buffer_load_dword(x4)? .* lds", l) and prev != "s_nop 4"]


def kernel_resources() -> str:
    """Registers, scratch and occupancy of every kernel instantiation, from the compiler's own
    resource-usage remarks."""
    import re
    asm, remarks = device_assembly()

    class res:  # noqa: N801  (keeps the parsing below unchanged)
        stdout = remarks
    rows = []
    for block in re.split(r"remark: Function Name: ", res.stdout)[1:]:
        mangled = block.split()[0]
        m = re.match(r"_ZN5spark(\d+)", mangled)
        if not m:
            continue
        n = int(m.group(1))
        start = m.end()
        name, targs = mangled[start:start + n], mangled[start + n:]
        args = []
        if targs.startswith("I"):
            for tok in re.findall(r"DF16_|DF16b|Li\d+E|Lb[01]E", targs.split("EE")[0] + "E"):
                args.append({"DF16_": "fp16", "DF16b": "bf16"}.get(tok) or
                            (tok[2:-1] if tok[1] == "i" else ("yes" if tok[2] == "1" else "no")))
        get = lambda key: int(re.search(key + r": (\d+)", block).group(1))
        # scratch traffic inside the kernel body: count the spill instructions the assembly holds
        body = asm[asm.index(mangled + ":"):]
        body = body[:body.index("s_endpgm")]
        # ... and how many of them sit in an innermost loop that holds matrix instructions, i.e. in one
        # of the loops over tiles (the rest is prologue / epilogue code, run once per tile).  A loop is
        # a branch back to an earlier label; innermost = no other such range inside it.
        parts = re.split(r"\n(\.LBB[0-9_]+):", body)
        labels = ["entry"] + parts[1::2]
        blocks = [parts[0]] + parts[2::2]
        loops = []
        for i, bb in enumerate(blocks):
            for target in re.findall(r"s_c?branch\w* (\.LBB[0-9_]+)", bb):
                if target in labels and labels.index(target) <= i:
                    loops.append((labels.index(target), i))
        inner = [l for l in loops if not any(o != l and l[0] <= o[0] and o[1] <= l[1] for o in loops)]
        in_loops = sum(len(re.findall(r"scratch_(?:load|store)", bb)) for a, b in inner
                       if any("v_mfma" in x for x in blocks[a:b + 1]) for bb in blocks[a:b + 1])
        rows.append((name, ", ".join(args), get("VGPRs"), get("AGPRs"), get(r"ScratchSize \[bytes/lane\]"),
                     get(r"Occupancy \[waves/SIMD\]"), len(re.findall(r"scratch_(?:load|store)", body)), in_loops))
    out = ["Per-instantiation resources of libspark_mha.so for gfx950 (compiler remarks, -Rpass-analysis=kernel-resource-usage).",
           "command: python -m paper_2502_12784_amd.build --resources",
           "template arguments: element type, head-dimension tile D, causal, dropout[, waves per workgroup];",
           "scratch = bytes per lane of spill space; scratch instrs = scratch loads + stores in the kernel's code;",
           "in tile loops = those of them inside an innermost loop that holds matrix instructions (the loops over",
           "K/V or Q/dO tiles); the others are prologue / epilogue code that runs once per tile of the workgroup",
           "",
           "%-30s %-26s %5s %5s %8s %10s %14s %14s" % ("kernel", "template arguments", "VGPR", "AGPR", "scratch",
                                                      "waves/SIMD", "scratch instrs", "in tile loops")]
    for r in sorted(rows):
        out.append("%-30s %-26s %5d %5d %8d %10d %14d %14d" % r)
    return "\n".join(out) + "\n"


if __name__ == "__main__":
    import sys
    if "--resources" in sys.argv:
        print(kernel_resources(), end="")
    elif "--mix-bench" in sys.argv:
        print(build_mix_floor_bench())
    else:
        print(build_library(verbose=True))
