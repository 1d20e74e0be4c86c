"""Build the HIP libraries (gfx950) in-tree with hipcc: libvarlen_attn.so, the attention library
(csrc/*.hip), and libva_probes.so, the benchmark's measurement aids (probes/*.hip)."""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
PROBES = os.path.join(HERE, "probes")
LIB = os.path.join(HERE, "libvarlen_attn.so")
PROBES_LIB = os.path.join(HERE, "libva_probes.so")
OBJ_DIR = os.path.join(HERE, "_build")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]

TARGETS = ((LIB, CSRC), (PROBES_LIB, PROBES))


def sources(src_dir=CSRC):
    return sorted(glob.glob(os.path.join(src_dir, "*.hip")))


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every .hip source and link both shared libraries; always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    procs = []
    objs = {lib: [] for lib, _ in TARGETS}
    for lib, src_dir in TARGETS:
        for src in sources(src_dir):
            obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
            objs[lib].append(obj)
            cmd = [hipcc, *FLAGS, "-I" + src_dir, *extra_flags, "-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines()
                        if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
        if p.returncode != 0:
            failed = True
            print(out, file=sys.stderr)
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    for lib, _ in TARGETS:
        subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs[lib], "-o", lib])
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
