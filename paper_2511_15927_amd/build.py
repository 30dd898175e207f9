"""Compile the HIP library for gfx950 into paper_2511_15927_amd/libbimamba.so (in-tree, hipcc)."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libbimamba.so")
# (d_state, lanes per chain) pairs the scan kernels are instantiated for
VARIANTS = ((4, 1), (8, 1), (16, 1), (16, 2), (16, 4), (32, 1), (32, 2), (32, 4), (64, 1), (64, 4), (128, 1), (128, 4))
# packed fp32 VALU forms are switched off for every kernel in this library
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument", "-I", os.path.join(ROOT, "include"),
         "-I", CSRC]
NOISE = "is not a recognized feature for this target"


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    log = "\n".join(l for l in r.stdout.splitlines() if NOISE not in l)
    if r.returncode != 0:
        raise RuntimeError("failed: " + " ".join(cmd) + "\n" + log[:4000])
    return log


def sources():
    return [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC))] + [os.path.join(ROOT, "include", "bimamba.h")]


def newest_dep(src, newest_all):
    """Modification time an object must beat: its source and the headers that source includes."""
    text = open(src).read()
    deps = [src, os.path.join(ROOT, "include", "bimamba.h")]
    for h in ("kernels.h", "launch.h", "ssd_kernels.h", "ssd_wide.h", "bwd_kernels.h"):
        if h in text or (h == "kernels.h"):
            deps.append(os.path.join(CSRC, h))
    return max(os.path.getmtime(p) for p in deps)


def build(force: bool = True, jobs: int = 8):
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(os.path.getmtime(p) for p in sources()):
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    units = [(os.path.join(CSRC, "bimamba_api.hip"), os.path.join(OBJ, "bimamba_api.o"), [])]
    for n, s in VARIANTS:
        units.append((os.path.join(CSRC, "scan_inst.hip"), os.path.join(OBJ, "scan_n%d_s%d.o" % (n, s)),
                      ["-DBM_N=%d" % n, "-DBM_S=%d" % s]))
    units.append((os.path.join(CSRC, "ssd_inst.hip"), os.path.join(OBJ, "ssd_inst.o"), []))
    units.append((os.path.join(CSRC, "bwd_inst.hip"), os.path.join(OBJ, "bwd_inst.o"), []))
    newest = max(os.path.getmtime(p) for p in sources())
    todo = [u for u in units if force or not os.path.exists(u[1]) or os.path.getmtime(u[1]) < newest_dep(u[0], newest)]
    cmds = [["hipcc"] + FLAGS + extra + ["-c", src, "-o", obj] for src, obj, extra in todo]
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(cmds)))) as ex:
        logs = list(ex.map(_run, cmds))
    logs.append(_run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + [u[1] for u in units]))
    out = "\n".join(l for l in logs if l.strip())
    if out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(force="--incremental" not in sys.argv))
