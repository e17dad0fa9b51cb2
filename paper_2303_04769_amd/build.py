"""Builds libsmall_hip.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsmall_hip.so")
PROBE_LIB = os.path.join(HERE, "libsmall_probe.so")       # the benchmark's matrix-rate probe, a library of its own
SOURCES = ["elementwise.hip", "window.hip", "window_rows.hip", "window_dpp.hip", "window_dpp_u8.hip", "pool_dpp_u8.hip", "quant_ends.hip", "pool_dpp.hip", "conv.hip", "conv_same.hip", "conv_pw.hip", "dwpw.hip", "dwpw_run.hip", "chain.hip", "resident.hip", "quant.hip", "table2.hip", "small_api.hip"]
# packed fp32 VALU ops are switched off for every device translation unit
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-gpu-rdc", "-Wall", "-Wno-unused-function", "-Wno-pass-failed",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# SMALL_RES_TIMING=1 in the environment builds the image-resident run with cycle stamps per layer and wave (read back by
# `bench.py --resident-timing`); the stamps cost a few store instructions per layer, so the default build has none.
if os.environ.get("SMALL_RES_TIMING"):
    FLAGS = FLAGS + ["-DSMALL_RES_TIMING"]


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build_lib(force=False, verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    # objects built with other flags (the timing build) are never mixed with this build's
    stamp = os.path.join(OBJ, "flags.txt")
    flags = " ".join(FLAGS)
    if not os.path.exists(stamp) or open(stamp).read() != flags:
        force = True
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    headers = [os.path.join(CSRC, "small_internal.h"), os.path.join(HERE, "..", "include", "small.h")]
    objs, procs = [], []
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ, src.replace(".hip", ".o"))
        objs.append(o)
        if force or _stale(o, [s] + headers):
            cmd = [hipcc] + FLAGS + ["-c", s, "-o", o]
            if verbose:
                print(" ".join(cmd), flush=True)
            procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = []
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if p.returncode:
            failed.append(f"{src}:\n{out}")
        elif verbose and out:
            print(out)
    if failed:
        raise RuntimeError("hipcc failed\n" + "\n".join(failed))
    with open(stamp, "w") as f:
        f.write(flags)
    if force or procs or _stale(LIB, objs):
        subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    probe_src = os.path.join(CSRC, "probe.hip")
    if force or _stale(PROBE_LIB, [probe_src, os.path.join(HERE, "..", "include", "small_probe.h")]):
        out = subprocess.run([hipcc] + FLAGS + ["-shared", probe_src, "-o", PROBE_LIB], stdout=subprocess.PIPE,
                             stderr=subprocess.STDOUT, text=True)
        if out.returncode:
            raise RuntimeError("hipcc failed\nprobe.hip:\n" + out.stdout)
    return LIB


if __name__ == "__main__":
    print(build_lib(force=True, verbose=True))
