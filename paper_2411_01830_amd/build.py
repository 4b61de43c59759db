"""Compile the HIP/C++ sources into libfaastube.so next to this file (gfx950 only)."""
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfaastube.so")
SOURCES = ["ft_pool.cpp", "ft_plan.cpp", "ft_api.cpp", "ft_open.cpp", "ft_policy.cpp", "ft_store.cpp", "ft_paths.cpp", "ft_kernels.hip", "ft_static.hip"]
# packed fp32 code generation is switched off for every translation unit
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Wall", "-Wno-unused-result",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # The ticket draw is one lane's atomic whose result is needed a whole tile later.
         # LLVM's wave-aggregation of uniform atomics would read the result back at once
         # and stall the workgroup on the atomic's latency, so it is switched off.
         "-mllvm", "-amdgpu-atomic-optimizer-strategy=None"]


def hipcc():
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the engine has no CPU fallback")
    return exe


def check_registers(remarks):
    """A host-link workgroup and a pool->pool workgroup must fit on one CU together
    (one wavefront of each per SIMD, 512 registers per lane, allocated in eights):
    a job with both kinds of traffic runs the two kernels side by side, and a
    host-link workgroup that took a CU for itself would idle that CU's share of HBM.
    The limit checked is 480, not 512: builds whose two kernels added up to 488 and 496
    registers measured 1.2 % less of the host link beside pool->pool launches (large_mixed:
    99.6 -> 98.3 % of the measured peak), the build at 480 does not."""
    import re
    regs = {}
    name = None
    for line in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
            regs[name] = 0
        m = re.search(r"\b(VGPRs|AGPRs): (\d+)", line)
        if m and name and "Spill" not in line:
            regs[name] += int(m.group(2))
    up8 = lambda v: (v + 7) // 8 * 8
    per_class = {}
    for k, v in regs.items():
        m = re.search(r"ft_copy_kernelILb1ELi(\d)E", k)
        if m:
            per_class[int(m.group(1))] = up8(v)
    if sorted(per_class) != [0, 1, 2, 3]:
        raise RuntimeError(f"could not read the copy kernels' register counts: {regs}")
    for host in (0, 1):
        if per_class[host] + per_class[2] > 480:
            raise RuntimeError(f"copy kernels no longer fit one CU together: class {host} uses "
                               f"{per_class[host]} registers, pool->pool {per_class[2]}")
    if 2 * per_class[3] > 512:
        raise RuntimeError(f"two workgroups of the light pool->pool build no longer fit one CU: {per_class[3]} registers each")
    return per_class


def build(verbose=False):
    out_dir = os.path.join(HERE, "_build")
    os.makedirs(out_dir, exist_ok=True)
    objs = []
    for src in SOURCES:
        obj = os.path.join(out_dir, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc(), "-x", "hip", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if src == "ft_kernels.hip":
            cmd.insert(-4, "-Rpass-analysis=kernel-resource-usage")
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
        if res.returncode != 0:
            sys.stderr.write(res.stderr)
            raise RuntimeError(f"hipcc failed on {src}")
        if src == "ft_kernels.hip":
            per_class = check_registers(res.stderr)
            if verbose:
                print("registers per lane (host->pool, pool->host, pool->pool, pool->pool light):", per_class, flush=True)
        else:
            sys.stderr.write(res.stderr)
        objs.append(obj)
    cmd = [hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", LIB + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(LIB + ".tmp", LIB)
    return LIB


def build_native_tests(verbose=False):
    """tests/host/c_abi_stress: a C++ program that uses the library through include/faastube.h only."""
    root = os.path.dirname(HERE)
    src = os.path.join(root, "tests", "host", "c_abi_stress.cpp")
    exe = os.path.join(root, "tests", "host", "c_abi_stress")
    cmd = [hipcc(), "-x", "hip", "-O2", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", src, "-L" + HERE, "-lfaastube", "-Wl,-rpath,$ORIGIN/../../paper_2411_01830_amd", "-lpthread", "-o", exe + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stderr)
        raise RuntimeError("hipcc failed on c_abi_stress.cpp")
    os.replace(exe + ".tmp", exe)
    return exe


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
    print(build_native_tests(verbose="-v" in sys.argv))
