"""Builds libsk.so (HIP kernels + host library) for gfx950 with hipcc, in-tree."""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libsk.so")
SOURCES = ["sk_kernels.hip", "sk_top2.hip", "sk_probe.hip", "sk_pool.cpp"]
HEADERS = ["sk_internal.h", os.path.join("..", "..", "include", "sk.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-FP32 instructions are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-result",
]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS]
    return any(os.path.exists(d) and os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every source into libsk.so.  Cross-compiles without a GPU."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + ["-Rpass-analysis=kernel-resource-usage", "-o", tmp] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd))
    try:
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + r.stdout + r.stderr)
        check_no_spills(r.stderr)
        os.replace(tmp, LIB)
    finally:
        if os.path.exists(tmp):          # a failed compile or a refused kernel leaves nothing behind
            os.unlink(tmp)
    return LIB


def check_no_spills(remarks: str) -> None:
    """The MFMA attention kernel counts its own outstanding vector-memory operations
    (s_waitcnt vmcnt(N) against the direct-to-LDS loads in flight).  Register spills would add
    scratch loads and stores to that count, so a build in which that kernel spills is refused."""
    name = None
    for line in remarks.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split()[0]
        elif name and "sk_attn_bf16" in name:
            for key in ("VGPRs Spill:", "ScratchSize [bytes/lane]:"):
                if key in line and int(line.split(key)[1].split()[0]) != 0:
                    raise RuntimeError("kernel %s uses scratch memory (%s); its hand-placed vmcnt waits assume none"
                                       % (name, line.split("remark:")[-1].strip()))


if __name__ == "__main__":
    print(build(verbose=True))


def build_host_check(driver_src: str, out: str) -> str:
    """Builds an executable from `driver_src` plus the library's sources with AddressSanitizer and
    UndefinedBehaviorSanitizer on the HOST pass only (the device code is compiled as always and never
    runs: the driver uses metadata-only pools).  The sanitizer runtime is linked into the executable,
    so it runs as it is, with no preloaded library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    san = []
    for f in ("-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"):
        san += ["-Xarch_host", f]
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-g", "-std=c++17"] + san + \
          ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-o", out, driver_src] + \
          [os.path.join(CSRC, s) for s in SOURCES]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc (sanitized host build) failed:\n" + r.stdout + r.stderr)
    return out
