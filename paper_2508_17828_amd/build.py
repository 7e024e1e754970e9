"""Compile libtrim.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libtrim.so")
RESOURCES = os.path.join(HERE, "libtrim.resources.txt")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    # every rounding stays where the source puts it (survivor sets must be reproducible)
    "-ffp-contract=off", "-fno-fast-math",
    # no packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
    # per-kernel registers, spills and static LDS, checked below
    "-Rpass-analysis=kernel-resource-usage",
]

_FIELDS = (("VGPRs", "vgpr"), ("AGPRs", "agpr"), (r"ScratchSize \[bytes/lane\]", "scratch"),
           (r"Occupancy \[waves/SIMD\]", "waves"), ("SGPRs Spill", "sgpr_spill"),
           ("VGPRs Spill", "vgpr_spill"), (r"LDS Size \[bytes/block\]", "static_lds"))


def kernel_resources(remarks: str):
    """Parse the compiler's kernel-resource-usage remarks: {mangled name: {field: int}}."""
    out = {}
    for block in re.split(r"remark: Function Name: ", remarks)[1:]:
        name = block.split()[0]
        out[name] = {key: int(re.search(pat + r": (\d+)", block).group(1)) for pat, key in _FIELDS}
    return out


def _without_remarks(stderr: str):
    """The compiler's output less the resource remarks (with their source excerpts and include
    trails) and the host pass's note about the packed-fp32 feature."""
    out, pending, in_remark = [], [], False
    for line in stderr.splitlines():
        if "packed-fp32-ops" in line:
            continue
        if line.startswith("In file included from"):
            pending.append(line)
            in_remark = False
            continue
        if re.match(r"^\S.*:\d+:\d+: ", line):           # a diagnostic's first line
            in_remark = "remark:" in line
            if not in_remark:
                out += pending
            pending = []
        if not in_remark:
            out.append(line)
    return out


def check_resources(res) -> None:
    """The search kernels address their distance table from LDS address 0: none may carry
    static LDS in front of its dynamic area."""
    bad = [n for n, r in res.items() if "search_kernel" in n and r["static_lds"] != 0]
    if bad:
        raise RuntimeError("search kernels with static LDS (their table would not start at LDS "
                           "address 0): " + ", ".join(bad))


# The search kernel's instances: one object per (mode, result entries per lane, bits per code).
INSTANCES = ([(0, e, b, 0) for b in (8, 4) for e in (1, 2, 4, 16)] + [(1, 1, 8, 0), (1, 1, 4, 0)] +
             [(0, 1, 8, 1), (0, 1, 4, 1), (0, 1, 8, 2), (0, 1, 4, 2)])   # last: the lean (80-register) small-k kNN instances, for short and for long rows


def _compile(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    p = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    rest = _without_remarks(p.stderr)
    if rest:
        print("\n".join(rest), file=sys.stderr, flush=True)
    if p.returncode != 0:
        raise subprocess.CalledProcessError(p.returncode, cmd)
    return kernel_resources(p.stderr)


def build(verbose: bool = False, extra=()) -> str:
    """Compile the API translation unit and every group of search-kernel instances (in parallel),
    check the kernels' resources, link libtrim.so."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    cflags = [f for f in FLAGS if f != "-shared"] + list(extra) + ["-c"]
    jobs = [([hipcc] + cflags + ["-o", os.path.join(objdir, "trim_api.o"), os.path.join(CSRC, "trim_api.hip")])]
    for mode, e, bits, lean in INSTANCES:
        obj = os.path.join(objdir, f"search_m{mode}_e{e}_c{bits}_l{lean}.o")
        jobs.append([hipcc] + cflags + [f"-DTRIM_INST_MODE={mode}", f"-DTRIM_INST_E={e}",
                                        f"-DTRIM_INST_BITS={bits}", f"-DTRIM_INST_LEAN={lean}", "-o", obj,
                                        os.path.join(CSRC, "trim_search_inst.hip")])
    workers = max(1, min(len(jobs), int(os.environ.get("MAX_JOBS", os.cpu_count() or 4))))
    res = {}
    with ThreadPoolExecutor(max_workers=workers) as pool:
        for r in pool.map(lambda c: _compile(c, verbose), jobs):
            res.update(r)
    check_resources(res)
    tmp = OUT + ".tmp"
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + [j[j.index("-o") + 1] for j in jobs]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    os.replace(tmp, OUT)
    with open(RESOURCES, "w") as f:
        for name in sorted(res):
            f.write(name + " " + " ".join(f"{k}={v}" for k, v in res[name].items()) + "\n")
    return OUT


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
