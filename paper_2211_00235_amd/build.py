"""Build the HIP library in-tree for gfx950 (hipcc cross-compiles without a GPU)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpe_mi355x.so")
SOURCES = ["pe_block.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-amdgpu-mfma-vgpr-form",      # MFMA accumulators in VGPRs: no AGPR<->VGPR copies around the softmax
         "-Wno-pass-failed", "-Wno-unused-result"]


def build(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode:
        lines = [l for l in (res.stdout + res.stderr).splitlines() if "packed-fp32-ops" not in l]
        print("\n".join(lines))
    if res.returncode:
        raise RuntimeError("hipcc failed building %s" % LIB)
    return LIB


def build_host_check(out, verbose=False):
    """Host-only exercise of the C ABI (tests/host_checks/abi_host_check.cpp) linked with the library's source, the
    HOST code instrumented with AddressSanitizer and UndefinedBehaviorSanitizer (the device code is compiled as
    usual and never run: the program calls nothing that needs a GPU)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    root = os.path.dirname(HERE)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined"]
    flags = [f for f in FLAGS if f not in ("-shared", "-fPIC", "-O3")] + ["-O1", "-g"]
    cmd = ([hipcc] + flags + san + [os.path.join(CSRC, s) for s in SOURCES] +
           [os.path.join(root, "tests", "host_checks", "abi_host_check.cpp"), "-o", out])
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode:
        print("\n".join(l for l in (res.stdout + res.stderr).splitlines() if "packed-fp32-ops" not in l))
    if res.returncode:
        raise RuntimeError("hipcc failed building %s" % out)
    return out


def build_attn_bench(out=None, verbose=False):
    """Stand-alone timing program of the attention kernels (csrc/bench/attn_bench.hip); returns its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = out or os.path.join(HERE, "attn_bench")
    flags = [f for f in FLAGS if f not in ("-shared", "-fPIC")] + ["-Wno-implicit-const-int-float-conversion"]
    cmd = [hipcc] + flags + [os.path.join(CSRC, "bench", "attn_bench.hip"), "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode:
        print("\n".join(l for l in (res.stdout + res.stderr).splitlines() if "packed-fp32-ops" not in l))
    if res.returncode:
        raise RuntimeError("hipcc failed building %s" % out)
    return out


def build_mem_probe(out=None, verbose=False):
    """Stand-alone read-bandwidth probe (csrc/bench/mem_probe.hip); returns its path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = out or os.path.join(HERE, "mem_probe")
    flags = [f for f in FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [hipcc] + flags + [os.path.join(CSRC, "bench", "mem_probe.hip"), "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode:
        print("\n".join(l for l in (res.stdout + res.stderr).splitlines() if "packed-fp32-ops" not in l))
    if res.returncode:
        raise RuntimeError("hipcc failed building %s" % out)
    return out


if __name__ == "__main__":
    import sys
    if "attn_bench" in sys.argv[1:]:
        print(build_attn_bench(verbose=True))
    elif "mem_probe" in sys.argv[1:]:
        print(build_mem_probe(verbose=True))
    else:
        print(build(verbose=True))
