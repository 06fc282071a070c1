"""Build libscalekv.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libscalekv.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep packed fp32 VALU ops out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + \
        glob.glob(os.path.join(HERE, "..", "include", "*.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source into one shared library.  Returns its path."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + sources() + ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB


# Measurement-only builds of the whole library with one ingredient of the pipelined attention
# kernel taken out (see attend_pipe.hip); written beside the real library under another name and
# only ever loaded when SCALEKV_LIBRARY names them (bench.py --attend-alone does that on request).
VARIANTS = {
    "no_softmax": ["-DSCALEKV_ABLATE_SOFTMAX"],
    "no_transfer": ["-DSCALEKV_ABLATE_TRANSFER"],
    "one_wg_per_cu": ["-DSCALEKV_ONE_WG_PER_CU"],
    "timeline": ["-DSCALEKV_TIMELINE"],
    # every grid walked backwards; results must be bit-identical (tests/test_gpu_wg_order.py)
    "reversed_order": ["-DSCALEKV_REVERSE_WG"],
    "timeline_no_transfer": ["-DSCALEKV_TIMELINE", "-DSCALEKV_ABLATE_TRANSFER"],
}


def variant_path(name: str) -> str:
    return os.path.join(HERE, f"libscalekv_{name}.so")


def build_variant(name: str) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + VARIANTS[name] + sources() + ["-o", variant_path(name)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr[-4000:])
    return variant_path(name)


SANITIZE_BIN = os.path.join(HERE, "sanitize_check")


def run_sanitized() -> str:
    """The whole library plus its driver (csrc/sanitize_main.cpp) as one executable whose HOST code
    is built with AddressSanitizer and UndefinedBehaviorSanitizer (device code is compiled as
    usual and never runs: the driver only exercises host-side checks and host-only routines, so
    no GPU is needed).  Returns the driver's output, raises if anything is reported."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    cmd = [hipcc] + flags + ["-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                             "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer"]
    cmd += sources() + [os.path.join(CSRC, "sanitize_main.cpp"), "-fsanitize=address", "-fsanitize=undefined",
                        "-o", SANITIZE_BIN]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc (sanitizer build) failed:\n" + res.stderr[-4000:])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([SANITIZE_BIN], capture_output=True, text=True, env=env, timeout=600)
    out = run.stdout + run.stderr
    if run.returncode != 0 or "runtime error" in out or "Sanitizer" in out:
        raise RuntimeError("the host-sanitizer build of the ABI layer reported a problem:\n" + out)
    return out


if __name__ == "__main__":
    import sys
    if "--sanitize" in sys.argv:
        print(run_sanitized().strip())
    elif "--variant" in sys.argv:
        for name in sys.argv[sys.argv.index("--variant") + 1:]:
            print(build_variant(name))
    else:
        print(build(force=True, verbose=True))
