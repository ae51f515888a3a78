"""Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libvmsreplay.so")
SOURCES = ["vms_replay.hip", "vms_demo.hip", "vms_live.hip", "vms_peaks.hip"]
HEADERS = ["wave_hw.hpp", "wave_ops.hpp", "replay_plan.hpp", "replay_kernels.hpp", "replay_fine.hpp", "selftest.hpp", "../../include/vms_replay.h", "../../include/vms_live.h"]

# The replay loops branch on wave-uniform conditions only (whatever would switch lanes off is written
# with selects or kept in non-inlined functions).  With the option below LLVM leaves such regions as
# they are instead of rebuilding them around exec-mask style flow blocks: fewer branches per event.
HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-shared", "-fPIC", "-Wall",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-mllvm", "-structurizecfg-skip-uniform-regions=1",
               "-mllvm", "-align-all-nofallthru-blocks=6",      # branch targets on 64-byte lines: measured 2 % faster
               # one wavefront per SIMD and trace: schedule for latency (instruction-level parallelism inside the
               # wave), not for occupancy; measured 3 % (stitching) and 8 % (splitting kernel) faster
               "-mllvm", "-amdgpu-sched-strategy=max-ilp", "-mllvm", "-enable-post-misched=0",
               # no lifetime markers for locals: with them every `continue` out of a scope that holds a local
               # whose address was taken goes through a shared clean-up block and a switch on where to go next,
               # which LLVM does not thread away in these kernels (one flag test and two branches per event)
               "-Xclang", "-disable-lifetime-markers",
               "-Wno-inline-asm"]       # write_lane() names m0, which the compiler reserves but does not use here


def _stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS]
    return any(os.path.exists(d) and os.path.getmtime(d) > t for d in deps)


def build(force=False, save_temps_dir=None):
    """Build libvmsreplay.so next to this file; returns its path."""
    if not force and not _stale():
        return LIB
    srcs = [os.path.join(CSRC, s) for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    cmd = ["hipcc"] + HIPCC_FLAGS + ["-o", LIB] + srcs
    cwd = CSRC
    if save_temps_dir:
        os.makedirs(save_temps_dir, exist_ok=True)
        cmd.append("--save-temps")
        cwd = save_temps_dir
    r = subprocess.run(cmd, cwd=cwd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if out.strip():
        print(out)
    return LIB
