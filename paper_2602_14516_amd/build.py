"""Build libampd.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libampd.so")
SOURCES = ["kernels.hip", "api.cpp", "api_host.cpp", "plan.cpp"]
HEADERS = ["kernels.h", "plan.h", "api_host.h", os.path.join(INCLUDE, "ampd.h")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES] + [h if os.path.isabs(h) else os.path.join(CSRC, h) for h in HEADERS]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 into libampd.so; returns its path."""
    if not force and not _stale():
        return LIB
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           # packed-fp32 VALU forms are kept out of the generated code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-x", "hip", "-I", INCLUDE, "-I", CSRC]
    cmd += [os.path.join(CSRC, f) for f in SOURCES]
    cmd += ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB


def kernel_resources() -> dict:
    """Registers, scratch and LDS of every kernel in kernels.hip, as the compiler reports them for gfx950
    (-Rpass-analysis=kernel-resource-usage; device code only, nothing is linked or written next to the sources)."""
    import re
    import tempfile
    with tempfile.TemporaryDirectory() as tmp:
        cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-I", INCLUDE, "-I", CSRC, "-c", "--cuda-device-only", "-Rpass-analysis=kernel-resource-usage",
               os.path.join(CSRC, "kernels.hip"), "-o", os.path.join(tmp, "kernels.o")]
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    out, name = {}, None
    for line in res.stdout.splitlines():
        m = re.search(r"remark:\s+(Function Name|VGPRs|AGPRs|TotalSGPRs|ScratchSize \[bytes/lane\]|VGPRs Spill|SGPRs Spill|"
                      r"LDS Size \[bytes/block\]|Occupancy \[waves/SIMD\]): (\S+)", line)
        if not m:
            continue
        if m.group(1) == "Function Name":
            name = m.group(2)
            out[name] = {}
        elif name is not None:
            out[name][m.group(1)] = int(m.group(2))
    return out


SCHED_LIB = os.path.join(HERE, "libampd_sched.so")
SCHED_SRC = os.path.join(CSRC, "sched.cpp")
SCHED_HDR = os.path.join(INCLUDE, "ampd_sched.h")


def build_sched(force: bool = False) -> str:
    """Compile the host-only scheduling library (no GPU code) with g++."""
    stale = (not os.path.exists(SCHED_LIB) or
             os.path.getmtime(SCHED_LIB) < max(os.path.getmtime(SCHED_SRC), os.path.getmtime(SCHED_HDR)))
    if force or stale:
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-Wall", "-I", INCLUDE,
                               SCHED_SRC, "-o", SCHED_LIB])
    return SCHED_LIB


HOST_SAN_LIB = os.path.join(HERE, "libampd_host_san.so")
SCHED_SAN_LIB = os.path.join(HERE, "libampd_sched_san.so")


def build_host_sanitized(address: bool = True):
    """Compile the host-only code (planner, argument validation and the entry points that never touch a GPU; the
    scheduling library) with g++ under the undefined-behaviour sanitizer and, unless address=False, the address
    sanitizer.  Returns (host library, scheduling library, sanitizer runtime to preload or None).  CPU only: the
    libraries hold no GPU code and export only the host-side entry points."""
    san = "address,undefined" if address else "undefined"
    flags = ["g++", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-Wall", f"-fsanitize={san}",
             "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-I", INCLUDE, "-I", CSRC]
    subprocess.check_call(flags + [os.path.join(CSRC, "api_host.cpp"), os.path.join(CSRC, "plan.cpp"), "-o", HOST_SAN_LIB])
    subprocess.check_call(flags + [SCHED_SRC, "-o", SCHED_SAN_LIB])
    runtime = None
    if address:
        runtime = subprocess.check_output(["g++", "-print-file-name=libasan.so"], text=True).strip()
        runtime = os.path.realpath(runtime)
    return HOST_SAN_LIB, SCHED_SAN_LIB, runtime


if __name__ == "__main__":
    print(build_sched(force=True))
    print(build(force=True, verbose=True))
