"""Compile the HIP sources for gfx950: csrc/ into paper_2603_05168_amd/libsbn.so (the layer) and bench_csrc/ into
paper_2603_05168_amd/libsbn_probe.so (ceiling probes of the benchmark, apart from the layer's library)."""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsbn.so")
PROBE_SRC = os.path.join(HERE, "bench_csrc")
PROBE_LIB = os.path.join(HERE, "libsbn_probe.so")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                      # quantizer arithmetic must round exactly as written
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(force: bool = True, verbose: bool = False) -> str:
    srcs = sources()
    probe_srcs = sorted(glob.glob(os.path.join(PROBE_SRC, "*.hip")))
    deps = srcs + probe_srcs + glob.glob(os.path.join(CSRC, "*.hpp")) + glob.glob(os.path.join(HERE, "..", "include", "*.h"))
    if not force and all(os.path.exists(l) and all(os.path.getmtime(l) >= os.path.getmtime(d) for d in deps) for l in (LIB, PROBE_LIB)):
        return LIB
    objs = []
    probe_objs = []
    procs = []
    for s in srcs + probe_srcs:
        o = s[:-4] + ".o"
        (probe_objs if s in probe_srcs else objs).append(o)
        cmd = ["hipcc", "-c"] + [f for f in FLAGS if f != "-shared"] + ["-o", o, s]
        procs.append((s, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for s, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            sys.stderr.write(f"--- {s}\n{out}\n")
        elif verbose and out.strip():
            sys.stderr.write(f"--- {s}\n{out}\n")
    if failed:
        raise RuntimeError("hipcc failed")
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, check=True)
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", PROBE_LIB] + probe_objs, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
