"""Compile the HIP sources under csrc/ for gfx950 into paper_2209_15427_amd/libmpq.so."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libmpq.so")

FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
         # keep the compiler from forming packed-fp32 instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


RESOURCES = os.path.join(OBJ, "kernel_resources.txt")


def _compile(name):
    """Compile one source; the compiler's per-kernel resource remarks (registers, scratch, occupancy)
    are kept, one line per kernel, for kernel_resources(); everything else it prints is passed on."""
    src = os.path.join(CSRC, name)
    obj = os.path.join(OBJ, name[:-4] + ".o")
    r = subprocess.run(["hipcc", *FLAGS, "-Rpass-analysis=kernel-resource-usage", "-c", src, "-o", obj],
                       stderr=subprocess.PIPE, text=True)
    rows, cur, rest, skip = [], None, [], 0
    for line in r.stderr.splitlines():
        if "[-Rpass-analysis=kernel-resource-usage]" in line:
            body = line.split("remark:", 1)[1].replace("[-Rpass-analysis=kernel-resource-usage]", "").strip()
            key, _, val = body.partition(":")
            if key == "Function Name":
                cur = {"file": name, "kernel": val.strip()}
                rows.append(cur)
                skip = 2                      # the source line and the caret that follow the first remark
            elif cur is not None:
                cur[key.strip()] = val.strip()
        elif skip > 0:
            skip -= 1
        else:
            rest.append(line)
    if rest:
        print("\n".join(rest))
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, r.args)
    return obj, rows


def kernel_resources():
    """[{file, kernel, VGPRs, AGPRs, scratch, occupancy}] of the last build, or None if there is none."""
    if not os.path.exists(RESOURCES):
        return None
    out = []
    for line in open(RESOURCES):
        f = line.rstrip("\n").split("\t")
        if len(f) == 6:
            out.append({"file": f[0], "kernel": f[1], "VGPRs": int(f[2]), "AGPRs": int(f[3]), "scratch": int(f[4]),
                        "occupancy": int(f[5])})
    return out


def build(jobs: int = 6) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        done = list(ex.map(_compile, sources()))
    objs = [o for o, _ in done]
    with open(RESOURCES, "w") as f:
        for _, rows in done:
            for r in rows:
                f.write("\t".join([r["file"], r["kernel"], r.get("VGPRs", "0"), r.get("AGPRs", "0"),
                                   r.get("ScratchSize [bytes/lane]", "0"), r.get("Occupancy [waves/SIMD]", "0")]) + "\n")
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-Wl,-z,defs", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    print(build())
