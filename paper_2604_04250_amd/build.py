"""Build libcawn.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libcawn.so")
# (the scan kernels' families are translation units of their own: they compile side by side)
SOURCES = ["cawn_fwd_plain.hip", "cawn_fwd_valve.hip", "cawn_fwd_ret.hip", "cawn_fwd_valve_ret.hip",
           "cawn_api.hip", "cawn_fwd.hip", "cawn_bwd.hip", "cawn_bwd_plain.hip", "cawn_bwd_valve.hip",
           "cawn_bwd_ret.hip", "cawn_bwd_hconv.hip", "cawn_bwd_hconv_valve.hip", "cawn_bwd_hconv_ret.hip"]
# The backward kernel is a persistent loop whose body fills its register budget (4 waves per SIMD).
# Hoisting loop-invariant copies of uniform values and addresses out of that loop costs ~10 VGPRs
# and a wave of occupancy; they are a few ALU ops per tile when left inside.
BWD_FLAGS = ["-mllvm", "-disable-machine-licm"]
FILE_FLAGS = {src: BWD_FLAGS for src in SOURCES if src.startswith("cawn_bwd_")}
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-ffp-contract=off", "-Wall", "-Wno-unused-function",
         # every atomic here is issued by one lane; the wave-level atomic combiner would only add a
         # read-back of the result right behind the atomic, i.e. a wait for its round trip
         "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build(verbose: bool = False, defines=(), out: str = OUT, objdir: str = CSRC) -> str:
    """Compile every translation unit (always: callers rebuild after a source change).
    `defines` (e.g. ["CAWN_NSTEP=4"]) and `out` let a tuning sweep build geometry variants."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    os.makedirs(objdir, exist_ok=True)

    def cc(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *FILE_FLAGS.get(src, []), *[f"-D{d}" for d in defines], "-c",
               os.path.join(CSRC, src), "-o", obj]
        # the compiler's per-kernel resource report (registers, scratch, occupancy) goes to a text
        # file beside the object; tests read it to catch a kernel that starts to spill
        cmd.insert(-4, "-Rpass-analysis=kernel-resource-usage")
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
        report, rest, in_remark, held = [], [], False, []
        for line in r.stderr.splitlines():
            if line.startswith("In file included from"):
                held.append(line)       # the include chain in front of a diagnostic: kept only if that is no remark
                continue
            if "[-Rpass-analysis=kernel-resource-usage]" in line:
                report.append(line)
                in_remark = True
                held = []
                continue
            rest += held
            held = []
            if in_remark and line.lstrip()[:1].isdigit() is False and "|" in line[:12] or \
                    in_remark and line.lstrip().split(" ", 1)[0].isdigit() and "|" in line[:12]:
                pass            # the source excerpt and caret under a remark
            else:
                rest.append(line)
                in_remark = False
        if rest:
            print("\n".join(rest), file=sys.stderr, flush=True)
        if r.returncode != 0:
            raise subprocess.CalledProcessError(r.returncode, cmd)
        with open(obj[:-2] + ".res.txt", "w") as f:
            for line in report:
                f.write(line.split("remark: ", 1)[-1].replace(" [-Rpass-analysis=kernel-resource-usage]", "").strip() + "\n")
        return obj

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 4)) as ex:
        objs = list(ex.map(cc, SOURCES))
    cmd = [hipcc, "-shared", "--offload-arch=gfx950", "-fno-gpu-rdc", "-o", out, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return out


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
