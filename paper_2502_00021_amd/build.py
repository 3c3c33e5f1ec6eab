"""Compile libpxr.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpxr.so")
SOURCES = ["api.cpp", "conv_api.cpp", "pipeline.cpp", "scene.cpp", "render.hip", "kinematics.hip", "static_scratch.hip", "conv.hip", "peaks.hip", "selftest.hip"]

# -ffp-contract=off: the order and fusion of fp32 operations is part of the
# output contract (coverage is decided by integers derived from these floats),
# so fusions are written out as fmaf and the compiler must not add its own.
# packed-fp32-ops is switched off for the device pass (see the platform notes).
# The LDS counters are already bumped once per wavefront by hand (ballot + popcount, lane 0 adds); the
# compiler's own wave-aggregation of uniform atomic adds would wrap that single-lane add a second time.
# Machine-level loop-invariant code motion is off: it parks constants (zero vectors, literals) in vector registers
# across the render kernel's band loop, which the 1024-thread variants (64 registers per lane) then spill; with it
# off those variants need 61 registers and nothing else gets slower (measured on every workload).
HIPFLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
            "-fno-fast-math", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-mllvm", "-amdgpu-atomic-optimizer-strategy=None", "-mllvm", "-disable-machine-licm",
            "-Wall", "-Wextra", "-Wno-unused-parameter", "-x", "hip"]


def stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if os.path.isfile(os.path.join(CSRC, f))]
    deps.append(os.path.join(ROOT, "include", "pxr.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def build(force=True, verbose=False, extra=(), out=None):
    """Compile the library.  `out`: another file than the in-tree libpxr.so (profiling builds, see __main__)."""
    if out is None and not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPFLAGS, *extra, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", out or LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return out or LIB


if __name__ == "__main__":
    # Profiling builds of the render kernel (csrc/profiling/, never part of the library), written to a file of
    # their own and loaded with `bench.py --profile-lib FILE`:
    #   --define PXR_STOP_AFTER=k   the kernel returns after phase k = 0..5 (hardware counters of k minus those of
    #                               k - 1 are phase k's); the frames are NOT rendered
    #   --define PXR_PHASE_TIMING   the first wavefront of every workgroup notes the shader clock at each barrier
    #                               (read with `bench.py --phase-clocks`); add --define PXR_WAVE_ARRIVAL for the
    #                               arrival of every wavefront at every barrier (slower: two barriers per phase)
    import argparse

    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("--define", action="append", default=[], metavar="NAME[=VALUE]")
    ap.add_argument("--out", default=None, help="write the library here instead of in-tree")
    a = ap.parse_args()
    if a.define and not a.out:
        ap.error("a build with --define is a profiling build: give it a file of its own with --out")
    build(verbose=True, extra=["-D" + d for d in a.define] + (["-DPXR_PROFILING_BUILD"] if a.define else []), out=a.out)
