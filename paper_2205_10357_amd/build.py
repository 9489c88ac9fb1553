"""Build libsol_block.so in-tree with hipcc for gfx950 (no other target, no JIT cache)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsol_block.so")
PROBE = os.path.join(HERE, "loop_model.bin")
SOURCES = ["api.hip", "igemm.hip", "igemm_fast.hip", "igemm_panel.hip", "wgrad.hip", "wgrad_fast.hip", "smallc.hip", "direct_f32.hip", "glue.hip", "runtime.hip"]
HEADERS = ["common.h", "launch.h", "classes.h", "pack_tile.h", "reduce_rows.h", "sol_lds_tr.h", os.path.join("..", "..", "include", "sol_block.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fvisibility=hidden",
    # keep the compiler from forming packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-I", CSRC,
]


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every translation unit and link the shared library.  Returns its path."""
    hdrs = [os.path.join(CSRC, h) for h in HEADERS]
    objs = []
    procs = []
    for src in SOURCES:
        s = os.path.join(CSRC, src)
        o = os.path.join(CSRC, src.replace(".hip", ".o"))
        objs.append(o)
        if force or _stale(o, [s] + hdrs):
            cmd = [HIPCC] + FLAGS + ["-c", s, "-o", o]
            if verbose:
                print(" ".join(cmd))
            procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l]
        if p.returncode != 0:
            failed = True
            print(f"--- {src} failed ---\n" + "\n".join(lines), file=sys.stderr)
        elif verbose and lines:
            print(f"--- {src} ---\n" + "\n".join(lines))
    if failed:
        raise RuntimeError("hipcc failed")
    if force or procs or _stale(LIB, objs):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
        subprocess.run(cmd, check=True)
    # the stand-alone timing model of the slice loop (an executable of its own, not part of the library)
    probe_src = os.path.join(CSRC, "loop_model.hip")
    if force or _stale(PROBE, [probe_src]):
        cmd = [HIPCC, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", probe_src, "-o", PROBE]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            print("\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l), file=sys.stderr)
            raise RuntimeError("hipcc failed on loop_model.hip")
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
